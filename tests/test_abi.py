"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every symbol the
header declares, and rejects bad arguments with the documented status codes before any launch."""
import ctypes
import os
import re

import pytest
import torch

from paper_2510_08055_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe_lp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert binding.status_string(0) == "ok"
    assert len({binding.status_string(i) for i in range(8)}) == 8


def _ws(H=256, E=8, K=2, I=512, dtype=1, T=64, wfmt=0, yf32=0, split=0):
    lib = binding.load()
    cfg = binding.CConfig(H, E, K, I, dtype, 1, 1, wfmt, yf32, split)
    n = ctypes.c_size_t(0)
    return lib.moe_workspace_bytes(ctypes.byref(cfg), T, ctypes.byref(n)), n.value


def test_workspace_bytes_and_argument_errors():
    st, n = _ws()
    assert st == 0 and n > 0
    st2, n2 = _ws(T=128)
    assert st2 == 0 and n2 > n
    # the big buffers are accounted for: act [T*K, I] and y_perm [T*K, H] in bf16
    assert n >= 64 * 2 * (512 + 256) * 2
    assert _ws(K=9)[0] == 2          # K > E            -> MOE_ERR_SHAPE
    assert _ws(E=0)[0] == 2
    assert _ws(E=4096)[0] == 2
    assert _ws(T=0)[0] == 2
    assert _ws(T=2 ** 30)[0] == 2 and _ws(T=2 ** 62)[0] == 2      # T*K must fit 31 bits, whatever T (no wrap-around)
    assert _ws(T=2 ** 30 - 1)[0] == 0
    assert _ws(dtype=7)[0] == 3      # unknown dtype    -> MOE_ERR_DTYPE
    assert _ws(H=257)[0] == 4        # H % 8 != 0       -> MOE_ERR_ALIGN
    assert _ws(I=12)[0] == 4
    # 4-bit expert weights: bf16 activations only, H and I multiples of 64, 0/1 the only formats
    assert _ws(wfmt=1)[0] == 0
    assert _ws(wfmt=1, dtype=0)[0] == 3
    assert _ws(wfmt=1, H=96)[0] == 4 and _ws(wfmt=1, I=96)[0] == 4
    assert _ws(wfmt=2)[0] == 3
    # fp32 expert outputs and a split intermediate: more workspace; the split needs bf16 weights and fp32 outputs
    st3, n3 = _ws(yf32=1)
    st4, n4 = _ws(yf32=1, split=1)
    assert st3 == 0 and st4 == 0 and n3 >= n + 64 * 2 * 256 * 2 and n4 >= n3 + 64 * 2 * 512 * 2
    assert _ws(yf32=2)[0] == 3 and _ws(yf32=1, split=2)[0] == 3
    assert _ws(split=1)[0] == 3 and _ws(yf32=1, split=1, dtype=0)[0] == 3 and _ws(yf32=1, split=1, wfmt=1)[0] == 3
    lib = binding.load()
    assert lib.moe_workspace_bytes(None, 64, ctypes.byref(ctypes.c_size_t(0))) == 1   # MOE_ERR_NULL
    cfg = binding.CConfig(256, 8, 2, 512, 1, 1, 1)
    assert lib.moe_workspace_bytes(ctypes.byref(cfg), 64, None) == 1


def test_create_rejects_bad_arguments_before_touching_the_gpu():
    lib = binding.load()
    cfg = binding.CConfig(256, 8, 2, 512, 1, 1, 1)
    ctx = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x10000)      # never dereferenced: every call below fails its checks first
    assert lib.moe_create(ctypes.byref(cfg), 64, None, 1 << 30, None, ctypes.byref(ctx)) == 1
    assert lib.moe_create(ctypes.byref(cfg), 64, fake, 16, None, ctypes.byref(ctx)) == 5          # workspace
    assert lib.moe_create(ctypes.byref(cfg), 64, ctypes.c_void_p(0x10010), 1 << 30, None, ctypes.byref(ctx)) == 4
    bad = binding.CConfig(256, 8, 9, 512, 1, 1, 1)
    assert lib.moe_create(ctypes.byref(bad), 64, fake, 1 << 30, None, ctypes.byref(ctx)) == 2
    assert lib.moe_destroy(None) == 1
    assert lib.moe_router_topk(None, None, 4, None, None, None, None, None) == 1
    assert lib.moe_set_ffn_variant(None, 0) == 1


def test_router_topk_noalloc_rejects_bad_arguments_before_touching_the_gpu():
    lib = binding.load()
    cfg = binding.CConfig(256, 128, 8, 512, 1, 1, 1)
    fake = ctypes.c_void_p(0x10000)      # never dereferenced: every call below fails its checks first
    assert lib.moe_router_topk_noalloc(None, fake, 4, fake, None, fake, fake, None) == 1
    assert lib.moe_router_topk_noalloc(ctypes.byref(cfg), fake, -1, fake, None, fake, fake, None) == 2
    assert lib.moe_router_topk_noalloc(ctypes.byref(cfg), fake, 4097, fake, None, fake, fake, None) == 5   # 4097 * 128 logits
    assert lib.moe_router_topk_noalloc(ctypes.byref(cfg), fake, 2 ** 62, fake, None, fake, fake, None) == 5   # T * E overflows 64 bits
    assert lib.moe_router_topk_noalloc(ctypes.byref(cfg), None, 4, fake, None, fake, fake, None) == 1
    assert lib.moe_router_topk_noalloc(ctypes.byref(cfg), ctypes.c_void_p(0x10008), 4, fake, None, fake, fake, None) == 4
    assert lib.moe_router_topk_noalloc(ctypes.byref(cfg), None, 0, None, None, None, None, None) == 0      # no rows: a no-op
    bad = binding.CConfig(256, 8, 9, 512, 1, 1, 1)
    assert lib.moe_router_topk_noalloc(ctypes.byref(bad), fake, 4, fake, None, fake, fake, None) == 2


def test_group_count_rule_and_layer_groups_are_host_arithmetic():
    # Sec. 4.4: N_lg(L) = max(1, ceil(L / 512)): 8192 tokens -> 16 groups, 512 tokens -> 1 group
    assert binding.moe_num_layer_groups(8192, 48, 512) == 16
    assert binding.moe_num_layer_groups(512, 48, 512) == 1
    assert binding.moe_num_layer_groups(513, 48, 512) == 2
    assert binding.moe_num_layer_groups(0, 48, 512) == 1
    assert binding.moe_num_layer_groups(10 ** 9, 48, 512) == 48          # never more groups than layers
    assert binding.moe_num_layer_groups(-1, 48, 512) == 0 and binding.moe_num_layer_groups(1, 0, 512) == 0
    assert binding.moe_num_layer_groups(1, 48, 0) == 0
    assert binding.moe_layer_groups(48, 16) == list(range(0, 49, 3))
    assert binding.moe_layer_groups(10, 4) == [0, 3, 6, 8, 10]
    lib = binding.load()
    assert lib.moe_layer_groups(4, 2, None) == 1
    buf = (ctypes.c_int32 * 8)()
    assert lib.moe_layer_groups(4, 5, buf) == 2 and lib.moe_layer_groups(4, 0, buf) == 2


def test_stack_forward_rejects_bad_arguments_before_touching_the_gpu():
    lib = binding.load()
    sched = binding.CStackSchedule(0, 1, 0)
    assert lib.moe_stack_forward(None, None, 1, None, 0, None, 0, sched, None, None, None) == 1


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libmoe_lp.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_build_rejects_scratch_in_kernels_with_asynchronous_loads():
    """The build reads the compiler's resource remarks and refuses a stream / router kernel that spills."""
    from paper_2510_08055_amd import build
    ok = ("x.hip:1:1: remark: Function Name: _ZN3moe29grouped_gemm_w4_stream_kernelILb1ELb1EEEv [-Rpass-analysis]\n"
          "x.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis]\n"
          "x.hip:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis]\n")
    assert build._scratch_users(ok, ("grouped_gemm_w4_stream_kernel",)) == []
    bad = ok.replace("ScratchSize [bytes/lane]: 0", "ScratchSize [bytes/lane]: 836").replace("VGPRs Spill: 0", "VGPRs Spill: 2072")
    found = build._scratch_users(bad, ("grouped_gemm_w4_stream_kernel",))
    assert len(found) == 2 and "836" in found[0] and "2072" in found[1]
    other = bad.replace("grouped_gemm_w4_stream_kernel", "some_other_kernel")
    assert build._scratch_users(other, ("grouped_gemm_w4_stream_kernel",)) == []
    # the same remarks as the compiler words them when it also keeps its intermediate files (-save-temps)
    bad2 = ("remark: x.hip:202:0: Function Name: _ZN3moe29grouped_gemm_bf16_pipe_kernelILi8ELi256EEEv [-Rpass-analysis]\n"
            "remark: x.hip:202:0:     ScratchSize [bytes/lane]: 104 [-Rpass-analysis]\n"
            "remark: x.hip:202:0:     VGPRs Spill: 25 [-Rpass-analysis]\n")
    found = build._scratch_users(bad2, ("grouped_gemm_bf16_pipe_kernel",))
    assert len(found) == 2 and "104" in found[0] and "25" in found[1]


def test_build_rejects_m0_uses_outside_the_asm_issued_lds_loads():
    """The direct-to-LDS loads write M0 from inline asm; the build refuses assembly that touches M0 otherwise."""
    from paper_2510_08055_amd import build
    ok = ("\ts_add_i32 s17, s34, s9\n"
          "\ts_mov_b32 m0, s17\n"
          "\ts_nop 0\n"
          "\tglobal_load_lds_dwordx4 v[222:223], off\n"
          "\t;;#ASMEND\n"
          "\ts_mov_b32 m0, s4 ; comment\n"
          "\ts_nop 0\n"
          "\tglobal_load_lds_ushort v[2:3], off\n"
          "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]\n")
    assert build._foreign_m0_uses(ok) == []
    # the compiler's own forms: an add into M0, M0 as a source, a write that no LDS load follows
    assert len(build._foreign_m0_uses(ok.replace("s_mov_b32 m0, s17", "s_add_i32 m0, s37, s31"))) == 1
    assert len(build._foreign_m0_uses(ok + "\tv_readlane_b32 s3, v5, m0\n")) == 1
    assert len(build._foreign_m0_uses(ok.replace("\tglobal_load_lds_ushort v[2:3], off\n", "\tds_read_b32 v1, v2\n"))) == 1


def test_build_rejects_use_of_an_asynchronously_loaded_register_before_its_wait():
    """Row-map lookups are asm-issued loads awaited explicitly; the build scans the listing for early uses."""
    from paper_2510_08055_amd import build
    ok = ("_ZN3moe29grouped_gemm_bf16_pipe_kernelILi8EEEv:\n"
          "\tv_add_u32_e32 v13, 1, v2\n"
          "\t;;#ASMSTART\n"
          "\tglobal_load_dword v13, v[4:5], off\n"
          "\t;;#ASMEND\n"
          "\tv_add_u32_e32 v3, 1, v2\n"
          "\t;;#ASMSTART\n"
          "\ts_mov_b32 m0, s4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v[6:7], off\n"
          "\t;;#ASMEND\n"
          "\t;;#ASMSTART\n"
          "\ts_waitcnt vmcnt(1)\n"
          "\t;;#ASMEND\n"
          "\tv_max_i32_e32 v13, 0, v13\n")
    assert build._early_uses_of_async_loads(ok, "grouped_gemm_bf16_pipe_kernel") == []
    for early in ("\tv_mov_b32_e32 v20, v13\n", "\tscratch_store_dword off, v13, off\n", "\tv_pk_add_u16 v[12:13], v[2:3], v[2:3]\n"):
        bad = ok.replace("\tv_add_u32_e32 v3, 1, v2\n", early)
        found = build._early_uses_of_async_loads(bad, "grouped_gemm_bf16_pipe_kernel")
        assert len(found) == 1 and "v13" in found[0]
    # other functions of the file are not looked at
    assert build._early_uses_of_async_loads(bad.replace("pipe_kernel", "tile_kernel"), "grouped_gemm_bf16_pipe_kernel") == []
