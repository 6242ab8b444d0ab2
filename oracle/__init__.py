"""CPU oracle of the MoE layer and of the chunked / layered schedules -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It wraps `moe_oracle.c` (plain fp64 C, built by `oracle/build.py`)
with numpy marshalling; it shares nothing with the GPU library and never
imports it.

Arrays are numpy: float64, float32, or uint16 holding bfloat16 bit patterns
(widened exactly to fp64 inside the C code).
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

F64, F32, BF16, MXFP4 = 0, 1, 2, 3
SCHED_CHUNKED, SCHED_LAYERED = 0, 1


class OracleError(RuntimeError):
    pass


class _Counters(ctypes.Structure):
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


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        L = ctypes.CDLL(_LIB_PATH)
        L.orc_round_bf16.restype = ctypes.c_double
        L.orc_round_bf16.argtypes = [ctypes.c_double]
        L.orc_round_f32.restype = ctypes.c_double
        L.orc_round_f32.argtypes = [ctypes.c_double]
        L.orc_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float64:
        return F64
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float64, float32 or uint16 (bf16 bits), not {a.dtype}")


def _c(a, dtype=None):
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what}: oracle error {rc} "
                          f"({ {1: 'bad argument', 2: 'non-finite logit', 3: 'allocation'}.get(rc, '?')})")


def _round(a, fmt):
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty_like(a)
    lib().orc_round_array(_p(a), ctypes.c_int64(a.size), int(fmt), _p(out))
    return out


def round_bf16(a):
    """Round float64 values to the nearest bfloat16 (ties to even); returns float64."""
    return _round(a, BF16)


def round_f32(a):
    """Round float64 values to the nearest binary32 (ties to even); returns float64."""
    return _round(a, F32)


def bf16_bits(a):
    """uint16 bit patterns of float64 values that are exactly representable in bfloat16 (e.g. round_bf16's)."""
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    assert (f.astype(np.float64) == a).all() and ((f.view(np.uint32) & 0xFFFF) == 0).all(), "not bfloat16 values"
    return (f.view(np.uint32) >> 16).astype(np.uint16)


def router_topk(x, w_router, bias, k, renormalize=True, want_logits=False, want_gap=False):
    """x [T,H], w_router [E,H], bias [E] float32 or None -> idx [T,k] int32, w [T,k] f64 (+ logits, gap)."""
    x, w_router = _c(x), _c(w_router)
    T, H = x.shape
    E = w_router.shape[0]
    assert w_router.shape == (E, H)
    b = None if bias is None else _c(bias, np.float32)
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    logits = np.zeros((T, E), dtype=np.float64) if want_logits else None
    gap = np.zeros((T,), dtype=np.float64) if want_gap else None
    rc = lib().orc_router_topk(_p(x), _dt(x), ctypes.c_int64(T), ctypes.c_int64(H), _p(w_router),
                               _dt(w_router), _p(b), E, k, int(bool(renormalize)),
                               _p(idx), _p(w), _p(logits), _p(gap))
    _check(rc, "router_topk")
    out = [idx, w]
    if want_logits:
        out.append(logits)
    if want_gap:
        out.append(gap)
    return tuple(out)


def permute(idx, E):
    """idx [T,k] int32 -> counts [E], offsets [E+1], perm [T*k], inv [T*k] (all int32)."""
    idx = _c(idx, np.int32)
    T, k = idx.shape
    counts = np.zeros(E, dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    perm = np.zeros(T * k, dtype=np.int32)
    inv = np.zeros(T * k, dtype=np.int32)
    rc = lib().orc_permute(_p(idx), ctypes.c_int64(T), k, E, _p(counts), _p(offsets), _p(perm), _p(inv))
    _check(rc, "permute")
    return counts, offsets, perm, inv


def mxfp4_dequant(codes, scales):
    """MXFP4 tensor -> float64: codes uint8 [..., n/2] (two FP4 E2M1 elements per byte, even element in the
    low nibble), scales uint8 [..., n/32] (E8M0, one per 32 consecutive elements)."""
    codes, scales = _c(codes, np.uint8), _c(scales, np.uint8)
    n = codes.size * 2
    assert scales.size * 32 == n
    out = np.zeros(n, dtype=np.float64)
    lib().orc_mxfp4_dequant(_p(codes), _p(scales), ctypes.c_int64(n), _p(out))
    return out.reshape(codes.shape[:-1] + (codes.shape[-1] * 2,))


def moe_layer(x, w_router, bias, w_gate_up, w_down, k, renormalize=True, residual=False, want_mag=False,
              s_gate_up=None, s_down=None):
    """One MoE layer.  x [T,H]; w_router [E,H]; w_gate_up [E,2I,H]; w_down [E,H,I].

    With s_gate_up / s_down given, the expert weights are MXFP4: w_gate_up uint8 [E,2I,H/2], s_gate_up
    uint8 [E,2I,H/32], w_down uint8 [E,H,I/2], s_down uint8 [E,H,I/32]; the router stays as it is.
    Returns y [T,H] f64 (unrounded), idx [T,k] int32, w [T,k] f64 (and, with want_mag, y_mag [T,H] =
    sum_j w_j |expert output| (+ |x|): the magnitude of the terms y is summed from).
    """
    x, w_router = _c(x), _c(w_router)
    T, H = x.shape
    E = w_router.shape[0]
    assert w_router.shape == (E, H)
    rdt = _dt(w_router)
    if s_gate_up is None:
        w_gate_up, w_down = _c(w_gate_up), _c(w_down)
        I = w_down.shape[2]
        assert w_gate_up.shape == (E, 2 * I, H) and w_down.shape == (E, H, I)
        wdt = rdt
        assert _dt(w_gate_up) == wdt and _dt(w_down) == wdt
        sgu = sd = None
    else:
        w_gate_up, w_down = _c(w_gate_up, np.uint8), _c(w_down, np.uint8)
        sgu, sd = _c(s_gate_up, np.uint8), _c(s_down, np.uint8)
        I = w_down.shape[2] * 2
        assert w_gate_up.shape == (E, 2 * I, H // 2) and w_down.shape == (E, H, I // 2)
        assert sgu.shape == (E, 2 * I, H // 32) and sd.shape == (E, H, I // 32)
        wdt = MXFP4
    b = None if bias is None else _c(bias, np.float32)
    y = np.zeros((T, H), dtype=np.float64)
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    mag = np.zeros((T, H), dtype=np.float64) if want_mag else None
    rc = lib().orc_moe_layer_q(_p(x), _dt(x), ctypes.c_int64(T), ctypes.c_int64(H), _p(w_router), rdt, _p(b),
                               _p(w_gate_up), _p(sgu), _p(w_down), _p(sd), wdt, E, k, ctypes.c_int64(I),
                               int(bool(renormalize)), int(bool(residual)), _p(y), _p(idx), _p(w), _p(mag))
    _check(rc, "moe_layer")
    if want_mag:
        return y, idx, w, mag
    return y, idx, w


def group_forward(layers, x_decode, x_prefill, k, schedule, chunk=0, renormalize=True, residual=True,
                  act_dtype=None, want_trace=False):
    """A contiguous layer group under `schedule` ("chunked" with `chunk`, or "layered").

    layers: list of dicts with w_router [E,H], router_bias ([E] float32 or None),
    w_gate_up [E,2I,H], w_down [E,H,I].  x_decode [D,H], x_prefill [P,H].
    act_dtype: format activations are rounded to between layers (default: that of x).
    Returns y_decode [D,H] f64, y_prefill [P,H] f64, Counters (and the routing trace).
    """
    n = len(layers)
    Wr = [_c(l["w_router"]) for l in layers]
    Wgu = [_c(l["w_gate_up"]) for l in layers]
    Wd = [_c(l["w_down"]) for l in layers]
    Bs = [None if l.get("router_bias") is None else _c(l["router_bias"], np.float32) for l in layers]
    E, H = Wr[0].shape
    I = Wd[0].shape[2]
    wdt = _dt(Wr[0])
    for a, b_, c_ in zip(Wr, Wgu, Wd):
        assert a.shape == (E, H) and b_.shape == (E, 2 * I, H) and c_.shape == (E, H, I)
        assert _dt(a) == wdt and _dt(b_) == wdt and _dt(c_) == wdt
    x_decode, x_prefill = _c(x_decode), _c(x_prefill)
    D, P = x_decode.shape[0], x_prefill.shape[0]
    if D and P:
        assert x_decode.dtype == x_prefill.dtype
    xsrc = x_decode if D else x_prefill
    xdt = _dt(xsrc)
    if act_dtype is None:
        act_dtype = xdt
    sched = {"chunked": SCHED_CHUNKED, "layered": SCHED_LAYERED}[schedule]
    VP = ctypes.c_void_p * n
    FP = ctypes.c_void_p * n
    wr_arr = VP(*[a.ctypes.data for a in Wr])
    gu_arr = VP(*[a.ctypes.data for a in Wgu])
    d_arr = VP(*[a.ctypes.data for a in Wd])
    b_arr = FP(*[None if b_ is None else b_.ctypes.data for b_ in Bs])
    y_decode = np.zeros((D, H), dtype=np.float64)
    y_prefill = np.zeros((P, H), dtype=np.float64)
    ctr = _Counters()
    trace = None
    if want_trace:
        step = P if (schedule == "layered" or P == 0) else chunk
        n_iter = 1 if P == 0 else -(-P // max(step, 1))
        trace = np.zeros(((n_iter * D + P) * n * k,), dtype=np.int32)
    rc = lib().orc_group_forward(wr_arr, b_arr, gu_arr, d_arr, wdt, n, ctypes.c_int64(H), E, k,
                                 ctypes.c_int64(I), int(bool(renormalize)), int(bool(residual)),
                                 int(act_dtype), _p(x_decode), ctypes.c_int64(D), _p(x_prefill),
                                 ctypes.c_int64(P), xdt, sched, ctypes.c_int64(chunk),
                                 _p(y_decode), _p(y_prefill), ctypes.byref(ctr), _p(trace))
    _check(rc, "group_forward")
    c = Counters(ctr.expert_bytes, ctr.router_bytes, ctr.active_experts_total, ctr.tokens_processed,
                 ctr.iterations, ctr.layer_passes)
    if want_trace:
        return y_decode, y_prefill, c, trace
    return y_decode, y_prefill, c


def num_layer_groups(prompt_len, n_layers, granule=512) -> int:
    """N_lg(L) = max(1, ceil(L / granule)), at most n_layers (0 for invalid arguments)."""
    return int(lib().orc_num_layer_groups(ctypes.c_int64(prompt_len), int(n_layers), ctypes.c_int64(granule)))


def layer_groups(n_layers, n_groups):
    """first[0..n_groups]: group g holds layers first[g] .. first[g+1]-1."""
    first = np.zeros(max(n_groups, 0) + 1, dtype=np.int32)
    _check(lib().orc_layer_groups(int(n_layers), int(n_groups), _p(first)), "layer_groups")
    return first


def stack_forward(layers, x_decode, x_prefill, k, chunk=0, n_groups=0, granule=512, renormalize=True,
                  residual=True, act_dtype=None):
    """A whole layer stack under the one-group-per-iteration rule, the prompt cut into slices of `chunk`
    tokens (0: one slice), each slice crossing n_groups layer groups (0: the group-count rule with `granule`).
    Arguments as for group_forward.  Returns y_decode [D,H] f64, y_prefill [P,H] f64, Counters.
    """
    n = len(layers)
    Wr = [_c(l["w_router"]) for l in layers]
    Wgu = [_c(l["w_gate_up"]) for l in layers]
    Wd = [_c(l["w_down"]) for l in layers]
    Bs = [None if l.get("router_bias") is None else _c(l["router_bias"], np.float32) for l in layers]
    E, H = Wr[0].shape
    I = Wd[0].shape[2]
    wdt = _dt(Wr[0])
    for a, b_, c_ in zip(Wr, Wgu, Wd):
        assert a.shape == (E, H) and b_.shape == (E, 2 * I, H) and c_.shape == (E, H, I)
        assert _dt(a) == wdt and _dt(b_) == wdt and _dt(c_) == wdt
    x_decode, x_prefill = _c(x_decode), _c(x_prefill)
    D, P = x_decode.shape[0], x_prefill.shape[0]
    if D and P:
        assert x_decode.dtype == x_prefill.dtype
    xdt = _dt(x_decode if D else x_prefill)
    if act_dtype is None:
        act_dtype = xdt
    VP = ctypes.c_void_p * n
    wr_arr = VP(*[a.ctypes.data for a in Wr])
    gu_arr = VP(*[a.ctypes.data for a in Wgu])
    d_arr = VP(*[a.ctypes.data for a in Wd])
    b_arr = VP(*[None if b_ is None else b_.ctypes.data for b_ in Bs])
    y_decode = np.zeros((D, H), dtype=np.float64)
    y_prefill = np.zeros((P, H), dtype=np.float64)
    ctr = _Counters()
    rc = lib().orc_stack_forward(wr_arr, b_arr, gu_arr, d_arr, wdt, n, ctypes.c_int64(H), E, k,
                                 ctypes.c_int64(I), int(bool(renormalize)), int(bool(residual)),
                                 int(act_dtype), _p(x_decode), ctypes.c_int64(D), _p(x_prefill),
                                 ctypes.c_int64(P), xdt, ctypes.c_int64(chunk), int(n_groups),
                                 ctypes.c_int64(granule), _p(y_decode), _p(y_prefill), ctypes.byref(ctr))
    _check(rc, "stack_forward")
    return y_decode, y_prefill, Counters(ctr.expert_bytes, ctr.router_bytes, ctr.active_experts_total,
                                         ctr.tokens_processed, ctr.iterations, ctr.layer_passes)
