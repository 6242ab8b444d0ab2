"""Thin ctypes binding over libmoe_lp.so (the C ABI declared in include/moe_lp.h).

Argument marshalling only: torch tensors supply device pointers and the current HIP
stream; every step of the path runs in the library's kernels.  There is no CPU
fallback: if the library is missing, `load()` raises.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_lp.so")
_lib = None

MOE_F32, MOE_BF16 = 0, 1
MOE_SCHED_CHUNKED, MOE_SCHED_LAYERED = 0, 1
MOE_W_DTYPE, MOE_W_MXFP4 = 0, 1
WEIGHT_FORMATS = {"": MOE_W_DTYPE, "dtype": MOE_W_DTYPE, "mxfp4": MOE_W_MXFP4}

EXPORTS = ["moe_workspace_bytes", "moe_create", "moe_destroy", "moe_router_topk", "moe_router_topk_noalloc", "moe_permute",
           "moe_grouped_ffn", "moe_grouped_ffn_mxfp4", "moe_combine", "moe_group_forward", "moe_num_layer_groups", "moe_layer_groups",
           "moe_stack_forward", "moe_read_counters", "moe_reset_counters",
           "moe_kernel_timing", "moe_read_kernel_timing", "moe_ffn_variant", "moe_set_ffn_variant",
           "moe_status_string"]

FFN_VARIANTS = {"auto": 0, "tile128": 1, "small": 2, "big": 3, "w4_tile64": 4, "w4_stream": 5}

KERNELS = {"router_logits": 0, "topk": 1, "permute": 2, "gate_up": 3, "down": 4, "combine": 5}


class MoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: moe_status {status} ({status_string(status)})")


class CConfig(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int32), ("E", ctypes.c_int32), ("K", ctypes.c_int32), ("I", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("renormalize", ctypes.c_int32), ("residual", ctypes.c_int32),
                ("weight_format", ctypes.c_int32), ("y_perm_f32", ctypes.c_int32),
                ("act_split", ctypes.c_int32)]


class CLayer(ctypes.Structure):
    _fields_ = [("w_router", ctypes.c_void_p), ("router_bias", ctypes.c_void_p),
                ("w_gate_up", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
                ("s_gate_up", ctypes.c_void_p), ("s_down", ctypes.c_void_p)]


class CSchedule(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("chunk", ctypes.c_int32)]


class CStackSchedule(ctypes.Structure):
    _fields_ = [("chunk", ctypes.c_int32), ("n_groups", ctypes.c_int32), ("granule", ctypes.c_int32)]


class CCounters(ctypes.Structure):
    _fields_ = [("expert_bytes", ctypes.c_uint64), ("router_bytes", ctypes.c_uint64),
                ("active_experts_total", ctypes.c_uint64), ("tokens_processed", ctypes.c_uint64),
                ("iterations", ctypes.c_uint32), ("layer_passes", ctypes.c_uint32)]


@dataclass
class Counters:
    expert_bytes: int
    router_bytes: int
    active_experts_total: int
    tokens_processed: int
    iterations: int
    layer_passes: int


def load():
    """Load the C-ABI library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(or paper_2510_08055_amd/build.py); the HIP library is required")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    L.moe_workspace_bytes.argtypes = [ctypes.POINTER(CConfig), i64, ctypes.POINTER(ctypes.c_size_t)]
    L.moe_create.argtypes = [ctypes.POINTER(CConfig), i64, vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
    L.moe_destroy.argtypes = [vp]
    L.moe_router_topk.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    L.moe_router_topk_noalloc.argtypes = [ctypes.POINTER(CConfig), vp, i64, vp, vp, vp, vp, vp]
    L.moe_permute.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    L.moe_grouped_ffn.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp]
    L.moe_grouped_ffn_mxfp4.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    L.moe_combine.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp]
    L.moe_group_forward.argtypes = [vp, ctypes.POINTER(CLayer), i32, vp, i64, vp, i64, CSchedule, vp, vp, vp]
    L.moe_num_layer_groups.argtypes = [i64, i32, i32]
    L.moe_layer_groups.argtypes = [i32, i32, ctypes.POINTER(i32)]
    L.moe_stack_forward.argtypes = [vp, ctypes.POINTER(CLayer), i32, vp, i64, vp, i64, CStackSchedule, vp, vp, vp]
    L.moe_read_counters.argtypes = [vp, ctypes.POINTER(CCounters), vp]
    L.moe_reset_counters.argtypes = [vp, vp]
    L.moe_kernel_timing.argtypes = [vp, ctypes.c_uint32]
    L.moe_read_kernel_timing.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64), vp]
    L.moe_ffn_variant.argtypes = [vp, i64]
    L.moe_ffn_variant.restype = ctypes.c_char_p
    L.moe_set_ffn_variant.argtypes = [vp, i32]
    L.moe_status_string.argtypes = [i32]
    L.moe_status_string.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("moe_ffn_variant", "moe_status_string"):
            getattr(L, name).restype = ctypes.c_int       # moe_status, or a count for moe_num_layer_groups
    _lib = L
    return L


def status_string(status: int) -> str:
    return load().moe_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise MoeError(status, what)


def moe_num_layer_groups(prompt_len: int, n_layers: int, granule: int = 512) -> int:
    """N_lg(L) = max(1, ceil(L / granule)), at most n_layers; 0 for invalid arguments (host arithmetic)."""
    return int(load().moe_num_layer_groups(int(prompt_len), int(n_layers), int(granule)))


def moe_layer_groups(n_layers: int, n_groups: int):
    """first_layer[0..n_groups]: group g holds layers first_layer[g] .. first_layer[g+1]-1."""
    out = (ctypes.c_int32 * (max(int(n_groups), 0) + 1))()
    _check(load().moe_layer_groups(int(n_layers), int(n_groups), out), "moe_layer_groups")
    return list(out)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the C ABI must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.bfloat16:
        return MOE_BF16
    if dt == torch.float32:
        return MOE_F32
    raise TypeError(f"unsupported dtype {dt}")


def workspace_bytes(H, E, K, I, dtype, max_tokens, renormalize=True, residual=True, weight_format="",
                    y_perm_f32=False, act_split=False) -> int:
    cfg = CConfig(H, E, K, I, _dtype_code(dtype), int(renormalize), int(residual), WEIGHT_FORMATS[weight_format],
                  int(y_perm_f32), int(act_split))
    out = ctypes.c_size_t(0)
    _check(load().moe_workspace_bytes(ctypes.byref(cfg), max_tokens, ctypes.byref(out)), "moe_workspace_bytes")
    return out.value


def moe_router_topk_noalloc(x, w_router, bias, K, renormalize=True, topk_idx=None, topk_w=None):
    """The router without a context or workspace (the library's static scratch holds the logits).  The outputs
    may be passed in, so that the call itself allocates nothing."""
    T, H = x.shape
    E = w_router.shape[0]
    cfg = CConfig(H, E, K, 8, _dtype_code(x.dtype), int(renormalize), 0, MOE_W_DTYPE, 0, 0)
    if topk_idx is None:
        topk_idx = torch.empty((T, K), dtype=torch.int32, device=x.device)
    if topk_w is None:
        topk_w = torch.empty((T, K), dtype=torch.float32, device=x.device)
    with torch.cuda.device(x.device):
        _check(load().moe_router_topk_noalloc(ctypes.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(bias), _ptr(topk_idx),
                                              _ptr(topk_w), _stream()), "moe_router_topk_noalloc")
    return topk_idx, topk_w


class Context:
    """A moe_ctx plus the torch-allocated workspace it lives on."""

    def __init__(self, H, E, K, I, dtype=torch.bfloat16, max_tokens=1024, renormalize=True, residual=True,
                 device="cuda:0", weight_format="", y_perm_f32=False, act_split=False):
        self.lib = load()
        self.H, self.E, self.K, self.I = H, E, K, I
        self.dtype = dtype
        self.max_tokens = max_tokens
        self.device = torch.device(device)
        self.weight_format = weight_format
        self.y_perm_dtype = torch.float32 if y_perm_f32 else dtype
        self.cfg = CConfig(H, E, K, I, _dtype_code(dtype), int(renormalize), int(residual),
                           WEIGHT_FORMATS[weight_format], int(y_perm_f32), int(act_split))
        n = ctypes.c_size_t(0)
        _check(self.lib.moe_workspace_bytes(ctypes.byref(self.cfg), max_tokens, ctypes.byref(n)),
               "moe_workspace_bytes")
        self.workspace = torch.empty(n.value + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self._ctx = ctypes.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.lib.moe_create(ctypes.byref(self.cfg), max_tokens, ctypes.c_void_p(base), n.value, _stream(),
                                       ctypes.byref(self._ctx)), "moe_create")

    def close(self):
        if self._ctx:
            self.lib.moe_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the five calls of the boundary, same names as the C ABI ----

    def moe_router_topk(self, x, w_router, bias=None):
        T = x.shape[0]
        idx = torch.empty((T, self.K), dtype=torch.int32, device=self.device)
        w = torch.empty((T, self.K), dtype=torch.float32, device=self.device)
        _check(self.lib.moe_router_topk(self._ctx, _ptr(x), T, _ptr(w_router), _ptr(bias), _ptr(idx), _ptr(w),
                                        _stream()), "moe_router_topk")
        return idx, w

    def moe_permute(self, x, topk_idx, want_x_perm=True):
        T = topk_idx.shape[0]
        A = T * self.K
        counts = torch.empty(self.E, dtype=torch.int32, device=self.device)
        offsets = torch.empty(self.E + 1, dtype=torch.int32, device=self.device)
        perm = torch.empty(A, dtype=torch.int32, device=self.device)
        inv = torch.empty(A, dtype=torch.int32, device=self.device)
        x_perm = torch.empty((A, self.H), dtype=self.dtype, device=self.device) if want_x_perm else None
        _check(self.lib.moe_permute(self._ctx, _ptr(x), _ptr(topk_idx), T, _ptr(counts), _ptr(offsets), _ptr(perm),
                                    _ptr(inv), _ptr(x_perm), _stream()), "moe_permute")
        return counts, offsets, perm, inv, x_perm

    def moe_grouped_ffn(self, x_perm, offsets, w_gate_up, w_down):
        A = x_perm.shape[0]
        y_perm = torch.empty((A, self.H), dtype=self.y_perm_dtype, device=self.device)
        _check(self.lib.moe_grouped_ffn(self._ctx, _ptr(x_perm), _ptr(offsets), A, _ptr(w_gate_up), _ptr(w_down),
                                        _ptr(y_perm), _stream()), "moe_grouped_ffn")
        return y_perm

    def moe_grouped_ffn_mxfp4(self, x_perm, offsets, w_gate_up, s_gate_up, w_down, s_down):
        A = x_perm.shape[0]
        y_perm = torch.empty((A, self.H), dtype=self.y_perm_dtype, device=self.device)
        _check(self.lib.moe_grouped_ffn_mxfp4(self._ctx, _ptr(x_perm), _ptr(offsets), A, _ptr(w_gate_up),
                                              _ptr(s_gate_up), _ptr(w_down), _ptr(s_down), _ptr(y_perm), _stream()),
               "moe_grouped_ffn_mxfp4")
        return y_perm

    def moe_combine(self, y_perm, inv_perm, topk_w, residual=None, out=None):
        T = topk_w.shape[0]
        y = out if out is not None else torch.empty((T, self.H), dtype=self.dtype, device=self.device)
        _check(self.lib.moe_combine(self._ctx, _ptr(y_perm), _ptr(inv_perm), _ptr(topk_w), _ptr(residual), T,
                                    _ptr(y), _stream()), "moe_combine")
        return y

    def pack_layers(self, layers: Sequence[dict]):
        """Host array of moe_layer structs from dicts of device tensors (kept alive by the caller)."""
        arr = (CLayer * len(layers))()
        for i, L in enumerate(layers):
            b = L.get("router_bias")
            sg, sd = L.get("s_gate_up"), L.get("s_down")
            arr[i] = CLayer(L["w_router"].data_ptr(), b.data_ptr() if b is not None else None,
                            L["w_gate_up"].data_ptr(), L["w_down"].data_ptr(),
                            sg.data_ptr() if sg is not None else None, sd.data_ptr() if sd is not None else None)
        return arr

    def moe_group_forward(self, layers, x_decode, x_prefill, schedule="layered", chunk=0, packed=None,
                          y_decode=None, y_prefill=None):
        D = 0 if x_decode is None else x_decode.shape[0]
        P = 0 if x_prefill is None else x_prefill.shape[0]
        arr = packed if packed is not None else self.pack_layers(layers)
        if y_decode is None:
            y_decode = torch.empty((D, self.H), dtype=self.dtype, device=self.device)
        if y_prefill is None:
            y_prefill = torch.empty((P, self.H), dtype=self.dtype, device=self.device)
        kind = {"chunked": MOE_SCHED_CHUNKED, "layered": MOE_SCHED_LAYERED}[schedule]
        _check(self.lib.moe_group_forward(self._ctx, arr, len(arr), _ptr(x_decode) if D else None, D,
                                          _ptr(x_prefill) if P else None, P, CSchedule(kind, int(chunk)),
                                          _ptr(y_decode) if D else None, _ptr(y_prefill) if P else None, _stream()),
               "moe_group_forward")
        return y_decode, y_prefill

    def moe_stack_forward(self, layers, x_decode, x_prefill, chunk=0, n_groups=0, granule=512, packed=None,
                          y_decode=None, y_prefill=None):
        D = 0 if x_decode is None else x_decode.shape[0]
        P = 0 if x_prefill is None else x_prefill.shape[0]
        arr = packed if packed is not None else self.pack_layers(layers)
        if y_decode is None:
            y_decode = torch.empty((D, self.H), dtype=self.dtype, device=self.device)
        if y_prefill is None:
            y_prefill = torch.empty((P, self.H), dtype=self.dtype, device=self.device)
        _check(self.lib.moe_stack_forward(self._ctx, arr, len(arr), _ptr(x_decode) if D else None, D,
                                          _ptr(x_prefill) if P else None, P,
                                          CStackSchedule(int(chunk), int(n_groups), int(granule)),
                                          _ptr(y_decode) if D else None, _ptr(y_prefill) if P else None, _stream()),
               "moe_stack_forward")
        return y_decode, y_prefill

    def moe_read_counters(self) -> Counters:
        c = CCounters()
        _check(self.lib.moe_read_counters(self._ctx, ctypes.byref(c), _stream()), "moe_read_counters")
        return Counters(c.expert_bytes, c.router_bytes, c.active_experts_total, c.tokens_processed, c.iterations,
                        c.layer_passes)

    def moe_reset_counters(self):
        _check(self.lib.moe_reset_counters(self._ctx, _stream()), "moe_reset_counters")

    def moe_kernel_timing(self, kernels=()):
        mask = 0
        for k in kernels:
            mask |= 1 << KERNELS[k]
        _check(self.lib.moe_kernel_timing(self._ctx, mask), "moe_kernel_timing")

    def moe_read_kernel_timing(self, kernel: str):
        """(total milliseconds, launches) of one timed kernel since moe_kernel_timing was set."""
        ms, n = ctypes.c_double(0), ctypes.c_int64(0)
        _check(self.lib.moe_read_kernel_timing(self._ctx, KERNELS[kernel], ctypes.byref(ms), ctypes.byref(n),
                                               _stream()), "moe_read_kernel_timing")
        return ms.value, n.value

    def moe_ffn_variant(self, T: int) -> str:
        return self.lib.moe_ffn_variant(self._ctx, T).decode()

    def moe_set_ffn_variant(self, variant="auto"):
        """Pin the grouped-GEMM kernel shape of this context (a name of FFN_VARIANTS, or the id)."""
        v = FFN_VARIANTS[variant] if isinstance(variant, str) else int(variant)
        _check(self.lib.moe_set_ffn_variant(self._ctx, v), "moe_set_ffn_variant")
