// Weighted un-permute and combine: a token's output is the mix of its K selected
// experts' outputs under the router's weights (Sec. 2.4), plus the residual stream.
// Pure bandwidth: one block per token, 16-byte loads of the K source rows, fp32
// accumulation in slot order, one rounding.
#include "common.h"

namespace moe {

template <typename T> struct pack16;   // 16 bytes of elements
template <> struct pack16<bf16_t> {
    static constexpr int N = 8;
    uint4 raw;
    __device__ __forceinline__ void unpack(float* f) const
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ void pack(const float* f)
    {
        raw.x = pack_bf16x2(f[0], f[1]);
        raw.y = pack_bf16x2(f[2], f[3]);
        raw.z = pack_bf16x2(f[4], f[5]);
        raw.w = pack_bf16x2(f[6], f[7]);
    }
};
template <> struct pack16<float> {
    static constexpr int N = 4;
    float4 raw;
    __device__ __forceinline__ void unpack(float* f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
    __device__ __forceinline__ void pack(const float* f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};

// y rows [0, rows0) go to y0, rows [rows0, T) to y1 (row t - rows0): lets the layer-group driver
// write decode rows and prefill rows to their separate output buffers without a copy.
// YT: element type of y_perm (T, or float when the context keeps the expert outputs in fp32).
template <typename T, typename YT>
__global__ __launch_bounds__(256) void combine_kernel(const YT* __restrict__ y_perm, const int32_t* __restrict__ inv,
                                                      const float* __restrict__ w, bool has_residual,
                                                      RowSrc residual, int K, int H, T* y0, int64_t rows0, T* y1)
{
    typedef pack16<T> P;
    typedef pack16<YT> PY;
    constexpr int NY = P::N / PY::N;      // 16-byte pieces of y_perm per 16 bytes of output (1, or 2 for fp32 under bf16)
    __shared__ int32_t s_row[kMaxTopK];
    __shared__ float s_w[kMaxTopK];
    const int64_t t = blockIdx.x;
    if (threadIdx.x < K) {
        // (entries are trusted to lie in [0, T K); the clamp keeps a bad one from becoming a wild address)
        const int32_t row = inv[t * K + threadIdx.x], last = (int32_t)gridDim.x * K - 1;
        s_row[threadIdx.x] = row < 0 ? 0 : (row > last ? last : row);
        s_w[threadIdx.x] = w[t * K + threadIdx.x];
    }
    __syncthreads();
    T* out = (t < rows0) ? (y0 + t * (int64_t)H) : (y1 + (t - rows0) * (int64_t)H);
    for (int c = threadIdx.x * P::N; c < H; c += 256 * P::N) {
        float acc[P::N], v[P::N];
#pragma unroll
        for (int i = 0; i < P::N; ++i) acc[i] = 0.f;
        for (int j = 0; j < K; ++j) {
            const YT* src = y_perm + (int64_t)s_row[j] * H + c;
#pragma unroll
            for (int h = 0; h < NY; ++h) {
                PY p;
                p.raw = *reinterpret_cast<const decltype(p.raw)*>(src + h * PY::N);
                p.unpack(v + h * PY::N);
            }
            const float wj = s_w[j];
#pragma unroll
            for (int i = 0; i < P::N; ++i) acc[i] = fmaf(wj, v[i], acc[i]);
        }
        if (has_residual) {
            P p;
            p.raw = *reinterpret_cast<const decltype(p.raw)*>(row_ptr<T>(residual, t, H) + c);
            p.unpack(v);
#pragma unroll
            for (int i = 0; i < P::N; ++i) acc[i] += v[i];
        }
        P o;
        o.pack(acc);
        *reinterpret_cast<decltype(o.raw)*>(out + c) = o.raw;
    }
}

hipError_t launch_combine(int dtype, bool y_perm_f32, const void* y_perm, const int32_t* inv, const float* w,
                          bool has_residual, RowSrc residual, int64_t T, int K, int H, void* y0, int64_t rows0, void* y1,
                          hipStream_t s)
{
    if (dtype == MOE_BF16 && y_perm_f32)
        combine_kernel<bf16_t, float><<<(unsigned)T, 256, 0, s>>>((const float*)y_perm, inv, w, has_residual, residual,
                                                                  K, H, (bf16_t*)y0, rows0, (bf16_t*)y1);
    else if (dtype == MOE_BF16)
        combine_kernel<bf16_t, bf16_t><<<(unsigned)T, 256, 0, s>>>((const bf16_t*)y_perm, inv, w, has_residual, residual,
                                                                   K, H, (bf16_t*)y0, rows0, (bf16_t*)y1);
    else
        combine_kernel<float, float><<<(unsigned)T, 256, 0, s>>>((const float*)y_perm, inv, w, has_residual, residual, K,
                                                                 H, (float*)y0, rows0, (float*)y1);
    return hipGetLastError();
}

}  // namespace moe
