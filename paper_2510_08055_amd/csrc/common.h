// Shared device/host helpers for the gfx950 MoE kernels (not used by the CPU oracle).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_lp.h"

namespace moe {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

constexpr int kWave = 64;
constexpr int kMaxExperts = 512;
constexpr int kMaxTopK = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest, ties to even, with the hardware conversion of gfx950 (v_cvt_pk_bf16_f32).
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float hw_float2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const hw_float2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hw_bf16x2_t));
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.0f) & 0xffffu); }

template <typename T> struct elem;
template <> struct elem<float> {
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct elem<bf16_t> {
    static __device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
    static __device__ __forceinline__ bf16_t from_f32(float v) { return f32_to_bf16(v); }
};

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// A batch of rows that lives in two buffers: rows [0, n0) in p0, the rest in p1 (row t - n0).  The
// layer-group driver reads the first layer's input straight from x_decode / x_prefill this way instead
// of copying the two pieces together first.
struct RowSrc {
    const void* p0;
    int64_t n0;
    const void* p1;
};
inline RowSrc single_src(const void* p) { return RowSrc{p, (int64_t)1 << 62, p}; }
template <typename T> __device__ __forceinline__ const T* row_ptr(const RowSrc& s, int64_t t, int64_t ld)
{
    return t < s.n0 ? static_cast<const T*>(s.p0) + t * ld : static_cast<const T*>(s.p1) + (t - s.n0) * ld;
}

// ---- launchers implemented in the .hip files; all return hipError_t from hipGetLastError() ----

// router.hip
hipError_t launch_router_logits(int dtype, RowSrc x, int64_t T, int H, const void* w_router, const float* bias,
                                int E, double* logits, int32_t* zero_buf, int zero_n, hipStream_t s);
// tile_hist (or NULL): [ceil(T*K / kPermTile), E] counters, already zero, that receive the expert histogram
hipError_t launch_topk(const double* logits, int64_t T, int E, int K, int renorm, int32_t* idx, float* w,
                       int32_t* tile_hist, hipStream_t s);

// permute.hip
constexpr int kPermTile = 8192;  // assignments per block of the permutation kernels
// hist_ready: tile_hist already holds the per-tile histograms (the top-k kernel counted them)
hipError_t launch_permute(const int32_t* idx, int64_t A, int E, int32_t* counts, int32_t* offsets,
                          int32_t* perm, int32_t* inv, int32_t* tile_hist, bool hist_ready,
                          unsigned long long* active_total, hipStream_t s);
hipError_t launch_fill_zero(void* p, int n_words, hipStream_t s);   // a fill kernel, not a memset node
hipError_t launch_gather_rows(int dtype, const void* x, const int32_t* perm, int K, int64_t A, int H,
                              void* x_perm, hipStream_t s);

// combine.hip
// y_perm_f32: y_perm holds float whatever dtype is
hipError_t launch_combine(int dtype, bool y_perm_f32, const void* y_perm, const int32_t* inv, const float* w,
                          bool has_residual, RowSrc residual, int64_t T, int K, int H, void* y0, int64_t rows0,
                          void* y1, hipStream_t s);

// ffn.hip
// x: [*, H]; row_map (or NULL): permuted row r reads x row row_map[r] / map_div; offsets [E+1].
// variant: a moe_ffn_variant_id (MOE_FFN_AUTO: chosen from the mean rows per expert); out_f32: y_perm is float;
// split: act is [A, 2I], every value a pair of bf16 (hi in column i, lo in column I + i); needs out_f32
hipError_t launch_ffn_gate_up(int dtype, int variant, bool split, RowSrc x, const int32_t* row_map, int map_div,
                              const int32_t* offsets, int64_t A, int E, int H, int I, const void* w_gate_up,
                              void* act, hipStream_t s);
hipError_t launch_ffn_down(int dtype, int variant, bool out_f32, bool split, const void* act, const int32_t* offsets,
                           int64_t A, int E, int H, int I, const void* w_down, void* y_perm, hipStream_t s);
const char* ffn_variant_name(int dtype, int variant, int64_t A, int E, int H, int I);

// Sets a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy of the code
// object).  `done` is the caller's per-kernel array of kMaxDevices flags.
constexpr int kMaxDevices = 16;
template <typename K> inline hipError_t ensure_lds_limit(K kern, size_t lds_bytes, bool* done)
{
    int d = 0;
    hipError_t e = hipGetDevice(&d);
    if (e != hipSuccess) return e;
    if (d < 0 || d >= kMaxDevices) return hipErrorInvalidDevice;
    if (done[d]) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes);
    if (e == hipSuccess) done[d] = true;
    return e;
}

// ffn_w4.hip: the same two GEMMs with MXFP4 expert weights (codes + scale bytes), bf16 activations
hipError_t launch_ffn_gate_up_w4(int variant, RowSrc x, const int32_t* row_map, int map_div, const int32_t* offsets,
                                 int64_t A, int E, int H, int I, const uint8_t* w_gate_up, const uint8_t* s_gate_up,
                                 void* act, hipStream_t s);
hipError_t launch_ffn_down_w4(int variant, bool out_f32, const void* act, const int32_t* offsets, int64_t A, int E, int H,
                              int I, const uint8_t* w_down, const uint8_t* s_down, void* y_perm, hipStream_t s);
const char* ffn_w4_variant_name(int variant, int64_t A, int E);

}  // namespace moe
