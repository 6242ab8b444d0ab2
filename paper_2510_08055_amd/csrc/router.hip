// Router: fp64 logits on the f64 matrix cores, then a wavefront-level top-k with
// lowest-index tie-break and the softmax mixing weights (MoE router, Sec. 2.4).
//
// Logits are accumulated in fp64 so that the K selected experts and their order
// agree with an fp64 definition: products of two bf16 (or two fp32) values are
// exact in fp64 and the summation error (~1e-16 relative) is far below any
// realistic gap between neighbouring logits.  The reduction order of a token's
// logits depends only on H, never on the batch, so routing is batch-invariant:
// the chunked and the layered schedule route every token identically.
#include "common.h"

namespace moe {

typedef double double4_t __attribute__((ext_vector_type(4)));

// 8 consecutive elements widened to double.  load_async() issues the global load as inline asm, so that
// the compiler neither moves it nor waits for it: the caller waits with wait_loads<N>() (N = loads that may
// still be in flight), which also names the registers as in/out operands, so no use of them can be
// scheduled above the wait.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <typename T> struct vec8;
template <> struct vec8<bf16_t> {
    static constexpr int kLoads = 1;
    u32x4_t raw;
    __device__ __forceinline__ void load(const bf16_t* p) { raw = *reinterpret_cast<const u32x4_t*>(p); }
    __device__ __forceinline__ void load_async(const bf16_t* p)
    {
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(raw) : "v"(p) : "memory");
    }
    __device__ __forceinline__ void zero() { raw = u32x4_t{0, 0, 0, 0}; }
    __device__ __forceinline__ double get(int j) const
    {
        const uint32_t w = (j < 2) ? raw.x : (j < 4) ? raw.y : (j < 6) ? raw.z : raw.w;
        return (double)__uint_as_float((j & 1) ? (w & 0xffff0000u) : (w << 16));
    }
};
template <> struct vec8<float> {
    static constexpr int kLoads = 2;
    f32x4_t a, b;
    __device__ __forceinline__ void load(const float* p)
    {
        a = *reinterpret_cast<const f32x4_t*>(p);
        b = *reinterpret_cast<const f32x4_t*>(p + 4);
    }
    __device__ __forceinline__ void load_async(const float* p)
    {
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(a) : "v"(p) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, off offset:16" : "=v"(b) : "v"(p) : "memory");
    }
    __device__ __forceinline__ void zero() { a = b = f32x4_t{0.f, 0.f, 0.f, 0.f}; }
    __device__ __forceinline__ double get(int j) const
    {
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        return (double)v[j];
    }
};
template <int N> __device__ __forceinline__ void wait_loads(vec8<bf16_t>& x, vec8<bf16_t>& w)
{
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(x.raw), "+v"(w.raw) : "n"(N) : "memory");
}
template <int N> __device__ __forceinline__ void wait_loads(vec8<float>& x, vec8<float>& w)
{
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(x.a), "+v"(x.b), "+v"(w.a), "+v"(w.b) : "n"(N) : "memory");
}

// Drain of a ring of four operand buffers: waits for every load in flight and names ALL ring registers, so
// that none of them can be handed to another value while a look-ahead load may still land on it.
__device__ __forceinline__ void wait_ring(vec8<bf16_t> (&x)[4], vec8<bf16_t> (&w)[4])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(x[0].raw), "+v"(x[1].raw), "+v"(x[2].raw), "+v"(x[3].raw), "+v"(w[0].raw), "+v"(w[1].raw),
                   "+v"(w[2].raw), "+v"(w[3].raw)
                 :
                 : "memory");
}
__device__ __forceinline__ void wait_ring(vec8<float> (&x)[4], vec8<float> (&w)[4])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(x[0].a), "+v"(x[0].b), "+v"(x[1].a), "+v"(x[1].b), "+v"(x[2].a), "+v"(x[2].b), "+v"(x[3].a),
                   "+v"(x[3].b), "+v"(w[0].a), "+v"(w[0].b), "+v"(w[1].a), "+v"(w[1].b), "+v"(w[2].a), "+v"(w[2].b),
                   "+v"(w[3].a), "+v"(w[3].b)
                 :
                 : "memory");
}

// One block: a 16-token x 16-expert tile of logits with v_mfma_f64_16x16x4; its 4 waves split the
// hidden dimension (wave w takes the 32-wide k-chunks w, w+4, w+8, ...) and their partial tiles are
// added in wave order 0,1,2,3 through LDS, so the summation order of a logit is fixed by H alone.
// Lane l supplies row (l % 16) of both operands; its quarter q = l / 16 owns the 8 consecutive
// k-values [c*32 + q*8, c*32 + q*8 + 8) of chunk c and feeds them to 8 successive MFMAs (any fixed
// pairing of k-slots is a valid summation order).  The raw operands of the next chunks are fetched
// while the MFMAs of the current one run; many short waves per SIMD hide the rest of the latency.
// (32 x 32 tiles per block, each widened operand feeding two MFMAs, measured slower: a quarter as
// many blocks leaves a 20 % tail on 256 compute units, and the matrix pipe, not the loads, is the limit.)
constexpr int kRouterBufs = 4;      // (wait_ring names exactly four buffers)

template <typename T>
__global__ __launch_bounds__(256) void router_logits_kernel(RowSrc x, int64_t n_tok, int H,
                                                            const T* __restrict__ wr,
                                                            const float* __restrict__ bias, int E,
                                                            double* __restrict__ logits,
                                                            int32_t* __restrict__ zero_buf, int zero_n)
{
    __shared__ double part[3][4][64];   // partial tiles of waves 1..3: [wave-1][element v][lane]
    // side job of block (0,0): clear the per-tile expert histogram that the top-k kernel, next on the
    // stream, counts into (saves a separate fill launch)
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < zero_n; i += 256) zero_buf[i] = 0;
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int64_t t0 = (int64_t)blockIdx.x * 16;
    const int e0 = blockIdx.y * 16;
    const int64_t tr = (t0 + r < n_tok) ? (t0 + r) : (n_tok - 1);  // clamp: loads stay in bounds
    const int er = (e0 + r < E) ? (e0 + r) : (E - 1);
    const T* xp = row_ptr<T>(x, tr, H) + q * 8;
    const T* wp = wr + (int64_t)er * H + q * 8;

    double4_t acc = {0.0, 0.0, 0.0, 0.0};
    // Ring of kRouterBufs operand buffers: the raw operands of this wave's next kRouterBufs - 1 chunks are
    // in flight while the MFMAs of the current chunk run.  Loads and waits of the ring are explicit (the
    // compiler would otherwise sink the loads next to their uses and wait for all of them); the look-ahead
    // index is clamped to the wave's last whole chunk rather than tested, so the loop body is branch-free.
    vec8<T> xa[kRouterBufs], wa[kRouterBufs];
    auto multiply = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(xa[buf].get(j), wa[buf].get(j), acc, 0, 0, 0);
    };
    const int n_whole = H / 32;                                            // whole 32-wide chunks of a row
    const int mine = n_whole > wave ? (n_whole - wave + 3) / 4 : 0;         // of which this wave takes chunks wave, wave+4, ...
    auto fetch = [&](int buf, int i) {                                      // this wave's i-th chunk
        const int k0 = (wave + 4 * i) * 32;
        xa[buf].load_async(xp + k0);
        wa[buf].load_async(wp + k0);
    };
    constexpr int kPerChunk = 2 * vec8<T>::kLoads;                          // load instructions per chunk
    int i = 0;
    if (mine >= kRouterBufs) {
#pragma unroll
        for (int b = 0; b < kRouterBufs - 1; ++b) fetch(b, b);
        for (; i + kRouterBufs <= mine; i += kRouterBufs) {
#pragma unroll
            for (int b = 0; b < kRouterBufs; ++b) {
                const int ahead = i + b + kRouterBufs - 1;
                fetch((b + kRouterBufs - 1) % kRouterBufs, ahead < mine ? ahead : mine - 1);
                wait_loads<(kRouterBufs - 1) * kPerChunk>(xa[b], wa[b]);
                multiply(b);
            }
        }
        // the look-ahead loads of the last round are still in flight; they target ring registers
        wait_ring(xa, wa);
    }
    for (; i < mine; ++i) {        // the last few whole chunks, one at a time
        fetch(0, i);
        wait_loads<0>(xa[0], wa[0]);
        multiply(0);
    }
    if (H % 32 != 0 && wave == n_whole % 4) {      // the row's partial chunk: lanes past the end feed zeros
        const int k0 = n_whole * 32;
        if (k0 + q * 8 < H) {
            xa[0].load(xp + k0);
            wa[0].load(wp + k0);
        } else {
            xa[0].zero();
            wa[0].zero();
        }
        multiply(0);
    }
    if (wave > 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave - 1][v][lane] = acc[v];
    }
    __syncthreads();
    if (wave != 0) return;
    // D layout of the f64 16x16x4 MFMA: lane l, element v holds row 4*v + l/16 (token), column l % 16 (expert).
    const int e = e0 + r;
    if (e < E) {
        const double b = bias ? (double)bias[e] : 0.0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t t = t0 + v * 4 + q;
            const double z = ((acc[v] + part[0][v][lane]) + part[1][v][lane]) + part[2][v][lane];
            if (t < n_tok) logits[t * E + e] = z + b;
        }
    }
}

// (value, index) "greater" under the routing order: larger logit first, equal logits by lower index.
__device__ __forceinline__ bool before(double va, int ia, double vb, int ib)
{
    return va > vb || (va == vb && ia < ib);
}

// One wave per token (TPW tokens one after the other).  Lane l holds logits of experts l, l+64, ...;
// K rounds of a wave-wide arg-max, each removing the winner.  Lane j keeps the j-th winner and
// computes its weight.  The block also counts its assignments per (permutation tile, expert) in LDS
// and adds the non-zero bins to the global per-tile histogram: integer counts do not depend on the
// order of the atomics, and few experts (a skewed top-2 of 8) no longer serialise on one address.
constexpr int kTopkWaves = 8;
template <int NPL>
__global__ __launch_bounds__(kTopkWaves * 64) void topk_kernel(const double* __restrict__ logits, int64_t n_tok, int E,
                                                               int K, int renorm, int tpw, int32_t* __restrict__ idx,
                                                               float* __restrict__ w, int32_t* __restrict__ tile_hist)
{
    // a block's assignments (at most 8 waves x tpw tokens x K <= kPermTile) touch at most two tiles
    __shared__ int32_t hist[2][kMaxExperts];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int64_t tb0 = (int64_t)blockIdx.x * (kTopkWaves * tpw);
    const int64_t tile0 = tb0 * K / kPermTile;
    if (tile_hist) {
        for (int i = threadIdx.x; i < 2 * E; i += kTopkWaves * 64) hist[i / E][i % E] = 0;
        __syncthreads();
    }
    const double NEG = -__builtin_huge_val();
    for (int it = 0; it < tpw; ++it) {
        const int64_t t = tb0 + (int64_t)wave * tpw + it;
        if (t >= n_tok) break;
        double v[NPL];
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int e = lane + 64 * i;
            v[i] = (e < E) ? logits[t * E + e] : NEG;
        }
        double my_z = NEG;
        int my_e = 0;
        double z_max = 0.0;
        for (int j = 0; j < K; ++j) {
            double bv = v[0];
            int bi = 0;
#pragma unroll
            for (int i = 1; i < NPL; ++i)
                if (v[i] > bv) { bv = v[i]; bi = i; }
            int be = lane + 64 * bi;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const double ov = __shfl_xor(bv, off, 64);
                const int oe = __shfl_xor(be, off, 64);
                if (before(ov, oe, bv, be)) { bv = ov; be = oe; }
            }
            if (j == 0) z_max = bv;
            if (lane == j) { my_z = bv; my_e = be; }
            if ((be & 63) == lane) {
                const int slot = be >> 6;
#pragma unroll
                for (int i = 0; i < NPL; ++i)
                    if (i == slot) v[i] = NEG;
            }
        }
        // softmax numerator of the selected expert; denominator over all E unless renormalising
        double p = (lane < K) ? exp(my_z - z_max) : 0.0;
        double denom;
        if (renorm) {
            denom = p;
        } else {
            denom = 0.0;
#pragma unroll
            for (int i = 0; i < NPL; ++i) {
                const int e = lane + 64 * i;
                if (e < E) denom += exp(logits[t * E + e] - z_max);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) denom += __shfl_xor(denom, off, 64);
        if (lane < K) {
            idx[t * K + lane] = my_e;
            w[t * K + lane] = (float)(p / denom);
            if (tile_hist) atomicAdd(&hist[(t * K + lane) / kPermTile - tile0][my_e], 1);
        }
    }
    if (tile_hist) {
        __syncthreads();
        for (int i = threadIdx.x; i < 2 * E; i += kTopkWaves * 64) {
            const int c = hist[i / E][i % E];
            if (c) atomicAdd(&tile_hist[(tile0 + i / E) * E + i % E], c);
        }
    }
}

// ----------------------------------------------------------------------------------------------
// Top-k for K <= 16: one token per 16-lane row, four tokens per wave.  Lane c of a row holds the
// logits of experts c, c+16, c+32, ...; a round takes the lane's best, then an all-reduce over the
// row in four DPP steps (lane ^ 1, lane ^ 2, mirror within 8, mirror within 16: register-to-register
// moves, no LDS), under the same total order (logit desc, index asc), so every lane of the row ends
// with the same winner.  Lane j of the row keeps winner j.
// ----------------------------------------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
template <int CTRL> __device__ __forceinline__ double dpp_mov(double v)
{
    return __hiloint2double(dpp_mov<CTRL>(__double2hiint(v)), dpp_mov<CTRL>(__double2loint(v)));
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

template <int CTRL> __device__ __forceinline__ void row_best_step(double& bv, int& be)
{
    const double ov = dpp_mov<CTRL>(bv);
    const int oe = dpp_mov<CTRL>(be);
    if (before(ov, oe, bv, be)) { bv = ov; be = oe; }
}
template <int CTRL> __device__ __forceinline__ double row_sum_step(double v) { return v + dpp_mov<CTRL>(v); }

template <int NPL>   // logits per lane: experts c + 16 i, i < NPL
__global__ __launch_bounds__(kTopkWaves * 64) void topk_rows_kernel(const double* __restrict__ logits, int64_t n_tok,
                                                                    int E, int K, int renorm, int32_t* __restrict__ idx,
                                                                    float* __restrict__ w,
                                                                    int32_t* __restrict__ tile_hist)
{
    // a block's assignments (32 tokens x K <= 512) touch at most two permutation tiles
    __shared__ int32_t hist[2][kMaxExperts];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int c = lane & 15;
    const int64_t tb0 = (int64_t)blockIdx.x * (kTopkWaves * 4);
    const int64_t tile0 = tb0 * K / kPermTile;
    if (tile_hist) {
        for (int i = threadIdx.x; i < 2 * E; i += kTopkWaves * 64) hist[i / E][i % E] = 0;
        __syncthreads();
    }
    const int64_t t = tb0 + wave * 4 + (lane >> 4);
    const bool live = t < n_tok;
    const int64_t tl = live ? t : n_tok - 1;      // rows past the end work on a copy of the last token, store nothing
    const double NEG = -__builtin_huge_val();
    double v[NPL];
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
        const int e = c + 16 * i;
        v[i] = (e < E) ? logits[tl * E + e] : NEG;
    }
    double esum = 0.0;      // only without renormalisation: this lane's share of sum_e exp(z_e - z_max)
    double my_z = NEG, z_max = 0.0;
    int my_e = 0;
    for (int j = 0; j < K; ++j) {
        double bv = v[0];
        int be = c;
#pragma unroll
        for (int i = 1; i < NPL; ++i)
            if (v[i] > bv) { bv = v[i]; be = c + 16 * i; }     // equal values: the lower index stays
        row_best_step<kDppXor1>(bv, be);
        row_best_step<kDppXor2>(bv, be);
        row_best_step<kDppHalfMirror>(bv, be);
        row_best_step<kDppMirror>(bv, be);
        if (j == 0) {
            z_max = bv;
            if (!renorm) {
#pragma unroll
                for (int i = 0; i < NPL; ++i)
                    if (c + 16 * i < E) esum += exp(v[i] - z_max);
            }
        }
        if (c == j) { my_z = bv; my_e = be; }
        if ((be & 15) == c) {
            const int slot = be >> 4;
#pragma unroll
            for (int i = 0; i < NPL; ++i)
                if (i == slot) v[i] = NEG;
        }
    }
    const double p = (c < K) ? exp(my_z - z_max) : 0.0;
    double denom = renorm ? p : esum;
    denom = row_sum_step<kDppXor1>(denom);
    denom = row_sum_step<kDppXor2>(denom);
    denom = row_sum_step<kDppHalfMirror>(denom);
    denom = row_sum_step<kDppMirror>(denom);
    if (live && c < K) {
        idx[t * K + c] = my_e;
        w[t * K + c] = (float)(p / denom);
        if (tile_hist) atomicAdd(&hist[(t * K + c) / kPermTile - tile0][my_e], 1);
    }
    if (tile_hist) {
        __syncthreads();
        for (int i = threadIdx.x; i < 2 * E; i += kTopkWaves * 64) {
            const int cnt = hist[i / E][i % E];
            if (cnt) atomicAdd(&tile_hist[(tile0 + i / E) * E + i % E], cnt);
        }
    }
}


hipError_t launch_router_logits(int dtype, RowSrc x, int64_t T, int H, const void* w_router, const float* bias,
                                int E, double* logits, int32_t* zero_buf, int zero_n, hipStream_t s)
{
    dim3 grid((unsigned)((T + 15) / 16), (unsigned)((E + 15) / 16));
    if (dtype == MOE_BF16)
        router_logits_kernel<bf16_t><<<grid, 256, 0, s>>>(x, T, H, (const bf16_t*)w_router, bias, E, logits, zero_buf,
                                                          zero_n);
    else
        router_logits_kernel<float><<<grid, 256, 0, s>>>(x, T, H, (const float*)w_router, bias, E, logits, zero_buf,
                                                         zero_n);
    return hipGetLastError();
}

hipError_t launch_topk(const double* logits, int64_t T, int E, int K, int renorm, int32_t* idx, float* w,
                       int32_t* tile_hist, hipStream_t s)
{
    if (K <= 16) {
        const unsigned grid = (unsigned)((T + kTopkWaves * 4 - 1) / (kTopkWaves * 4));
        const int npl = (E + 15) / 16;
#define MOE_TOPK_ROWS(N) topk_rows_kernel<N><<<grid, kTopkWaves * 64, 0, s>>>(logits, T, E, K, renorm, idx, w, tile_hist)
        if (npl <= 1) MOE_TOPK_ROWS(1);
        else if (npl <= 2) MOE_TOPK_ROWS(2);
        else if (npl <= 4) MOE_TOPK_ROWS(4);
        else if (npl <= 8) MOE_TOPK_ROWS(8);
        else if (npl <= 16) MOE_TOPK_ROWS(16);
        else MOE_TOPK_ROWS(32);
#undef MOE_TOPK_ROWS
        return hipGetLastError();
    }
    // more than 16 winners per token: one token per wave, lane j keeps winner j
    const int tpw = T <= 2048 ? 1 : 4;
    const unsigned grid = (unsigned)((T + kTopkWaves * tpw - 1) / (kTopkWaves * tpw));
    const int npl = (E + 63) / 64;
    if (npl <= 1) topk_kernel<1><<<grid, kTopkWaves * 64, 0, s>>>(logits, T, E, K, renorm, tpw, idx, w, tile_hist);
    else if (npl <= 2) topk_kernel<2><<<grid, kTopkWaves * 64, 0, s>>>(logits, T, E, K, renorm, tpw, idx, w, tile_hist);
    else if (npl <= 4) topk_kernel<4><<<grid, kTopkWaves * 64, 0, s>>>(logits, T, E, K, renorm, tpw, idx, w, tile_hist);
    else topk_kernel<8><<<grid, kTopkWaves * 64, 0, s>>>(logits, T, E, K, renorm, tpw, idx, w, tile_hist);
    return hipGetLastError();
}

}  // namespace moe
