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


// ----------------------------------------------------------------------------------------------
// Two-pass router for bf16 inputs with renormalised weights: the same fp64 decisions for a fraction of
// the fp64 work.  The K selected experts, their order and their weights only need EXACT logits of the
// experts that can be among the K largest; which those are is settled with cheap approximate logits and
// a rigorous error bound.
//
// Pass A (router_screen_kernel): approximate logits f[t,e] on the bf16 matrix cores (fp32 accumulate).
// A product of two bf16 values is exact in fp32, so f differs from the exact logit z only by the
// roundings of the additions: |f - z| <= H u sum_h |x_h w_h| <= H u |x_t| |w_e| =: d[t,e] (u = 2^-23, twice
// the unit roundoff: holds for any order of the additions and for truncating adders; Cauchy-Schwarz for
// the second step; the squared norms come out of the same MFMA stream as the diagonals of x x^T and
// w w^T and are inflated for their own rounding; the bias adds its own term).  With L = the K-th
// largest of f - d over a token's experts, at least K experts have z >= L, so an expert with
// f + d < L is strictly below K others and cannot be selected: the rest, K plus a fraction of an
// expert per token at these logit spreads, are the token's candidates.
// Pass B (router_exact_topk_kernel): for the candidates only, the fp64 dot product with a summation
// order fixed by H alone (batch-invariant, as before), then the K largest under (logit desc, index asc)
// and their softmax weights, exactly as the full kernel computes them; per-tile expert histogram as
// in the top-k kernels.  Whatever the screen does, the decisions are those of the exact logits.
// ----------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_r __attribute__((ext_vector_type(8)));
typedef float float4_r __attribute__((ext_vector_type(4)));

constexpr int kScreenTokens = 16;      // tokens per block of pass A

template <int CT>   // expert column tiles (of 16) per wave: wave w owns tiles w, w + 4, ...
__global__ __launch_bounds__(256) void router_screen_kernel(RowSrc x, int64_t n_tok, int H,
                                                            const bf16_t* __restrict__ wr,
                                                            const float* __restrict__ bias, int E, int K,
                                                            int32_t* __restrict__ cand_cnt,
                                                            uint16_t* __restrict__ cand,
                                                            int32_t* __restrict__ zero_buf, int zero_n)
{
    constexpr int EP = CT * 64;                 // experts covered (padded)
    constexpr int NPL = EP / 16;                // values per lane in the selection phase
    extern __shared__ float sm[];               // lo [16][EP], hi [16][EP], xn2 [16], wn2 [EP]
    float* lo = sm;
    float* hi = sm + kScreenTokens * EP;
    float* xn2 = hi + kScreenTokens * EP;
    float* wn2 = xn2 + kScreenTokens;
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < zero_n; i += 256) zero_buf[i] = 0;
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int64_t t0 = (int64_t)blockIdx.x * kScreenTokens;
    const int64_t tr = (t0 + r < n_tok) ? (t0 + r) : (n_tok - 1);      // clamp: loads stay in bounds
    const bf16_t* xp = row_ptr<bf16_t>(x, tr, H) + q * 8;
    const bf16_t* wp[CT];
#pragma unroll
    for (int i = 0; i < CT; ++i) {
        const int e = (wave + 4 * i) * 16 + r;
        wp[i] = wr + (int64_t)(e < E ? e : E - 1) * H + q * 8;
    }
    float4_r acc[CT], gw[CT], gx = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < CT; ++i) {
        acc[i] = float4_r{0.f, 0.f, 0.f, 0.f};
        gw[i] = float4_r{0.f, 0.f, 0.f, 0.f};
    }
    // lane (r, q) feeds k-values [k0 + 8 q, k0 + 8 q + 8) of row r to both operands of a 16 x 16 x 32 MFMA
    const u32x4_t zero4 = {0, 0, 0, 0};
    for (int k0 = 0; k0 < H; k0 += 32) {
        const bool in = k0 + q * 8 < H;         // H is a multiple of 8: a lane's 8 values are in or out together
        const u32x4_t xr = in ? *reinterpret_cast<const u32x4_t*>(xp + k0) : zero4;
        u32x4_t wv[CT];
#pragma unroll
        for (int i = 0; i < CT; ++i) wv[i] = in ? *reinterpret_cast<const u32x4_t*>(wp[i] + k0) : zero4;
        const bf16x8_r xa = __builtin_bit_cast(bf16x8_r, xr);
        if (wave == 0) gx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, xa, gx, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < CT; ++i) {
            const bf16x8_r wb = __builtin_bit_cast(bf16x8_r, wv[i]);
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wb, acc[i], 0, 0, 0);
            gw[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, wb, gw[i], 0, 0, 0);
        }
    }
    // result layout: lane l, element v holds row 4 (l / 16) + v (first operand's row), column l % 16
    // squared norms: the diagonals of the two Gram tiles
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        if (4 * q + v == r) {
            if (wave == 0) xn2[r] = gx[v];
#pragma unroll
            for (int i = 0; i < CT; ++i) wn2[(wave + 4 * i) * 16 + r] = gw[i][v];
        }
    }
    __syncthreads();
    {
        const float NEGF = -__builtin_huge_valf();
        const float gamma = (float)H * 1.1920929e-7f;      // H * 2^-23
#pragma unroll
        for (int i = 0; i < CT; ++i) {
            const int e = (wave + 4 * i) * 16 + r;
            const float b = (bias && e < E) ? bias[e] : 0.f;
            const float nw = wn2[e];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 4 * q + v;
                const float f = acc[i][v] + b;
                // bound of |f - z|: the additions of the dot product (norms inflated by 2 % for their own
                // rounding), the addition of the bias, the roundings of the next two lines, and a floor
                const float d = 1.02f * gamma * __builtin_sqrtf(xn2[row] * nw) + 4.8e-7f * (fabsf(acc[i][v]) + fabsf(b)) + 1e-9f;
                lo[row * EP + e] = (e < E) ? f - d : NEGF;
                hi[row * EP + e] = (e < E) ? f + d : NEGF;
            }
        }
    }
    __syncthreads();
    // selection: one token per 16-lane row, 4 tokens per wave; lane c holds experts c, c + 16, ...
    const int c = r;
    const int row = wave * 4 + q;
    const int64_t t = t0 + row;
    const float NEGF = -__builtin_huge_valf();
    float v[NPL];
#pragma unroll
    for (int i = 0; i < NPL; ++i) v[i] = lo[row * EP + c + 16 * i];
    float L = NEGF;
    for (int j = 0; j < K; ++j) {
        float bv = v[0];
        int bi = 0;
#pragma unroll
        for (int i = 1; i < NPL; ++i)
            if (v[i] > bv) { bv = v[i]; bi = i; }
        int be = c + 16 * bi;
        // row-wide maximum of (value, expert): any fixed total order will do here, the K-th largest VALUE is what counts
        auto step = [&](float ov, int oe) {
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        };
        step(__builtin_bit_cast(float, dpp_mov<kDppXor1>(__builtin_bit_cast(int, bv))), dpp_mov<kDppXor1>(be));
        step(__builtin_bit_cast(float, dpp_mov<kDppXor2>(__builtin_bit_cast(int, bv))), dpp_mov<kDppXor2>(be));
        step(__builtin_bit_cast(float, dpp_mov<kDppHalfMirror>(__builtin_bit_cast(int, bv))), dpp_mov<kDppHalfMirror>(be));
        step(__builtin_bit_cast(float, dpp_mov<kDppMirror>(__builtin_bit_cast(int, bv))), dpp_mov<kDppMirror>(be));
        L = bv;
        if ((be & 15) == c) {
            const int slot = be >> 4;
#pragma unroll
            for (int i = 0; i < NPL; ++i)
                if (i == slot) v[i] = NEGF;
        }
    }
    // candidates: experts whose upper bound reaches L, listed by ascending expert index
    int n = 0;
    const int shift = q * 16;
    const unsigned below = (1u << c) - 1u;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
        const int e = c + 16 * i;
        const bool is = e < E && hi[row * EP + e] >= L;
        const unsigned m = (unsigned)((__ballot(is) >> shift) & 0xffffull);
        if (is && t < n_tok) cand[t * E + n + __popc(m & below)] = (uint16_t)e;
        n += __popc(m);
    }
    if (c == 0 && t < n_tok) cand_cnt[t] = n;
}

// Fixed-order sum over the 64 lanes of a wave (every lane ends with the same bits: a + b == b + a).
__device__ __forceinline__ double wave_sum(double v)
{
    v = row_sum_step<kDppXor1>(v);
    v = row_sum_step<kDppXor2>(v);
    v = row_sum_step<kDppHalfMirror>(v);
    v = row_sum_step<kDppMirror>(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// XC: 16-byte chunks of a row per lane held in registers as doubles (covers H <= 512 XC); 0: any H, the
// token's row is re-read and re-widened for every candidate.
template <int XC>
__global__ __launch_bounds__(kTopkWaves * 64) void router_exact_topk_kernel(
    RowSrc x, int64_t n_tok, int H, const bf16_t* __restrict__ wr, const float* __restrict__ bias, int E, int K, int tpw,
    const int32_t* __restrict__ cand_cnt, const uint16_t* __restrict__ cand, int32_t* __restrict__ idx,
    float* __restrict__ w, int32_t* __restrict__ tile_hist)
{
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
    const int n_chunks = H / 8;
    auto widen = [](const u32x4_t& raw, double* out) {
        const uint32_t d[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = (double)__uint_as_float(d[i] << 16);
            out[2 * i + 1] = (double)__uint_as_float(d[i] & 0xffff0000u);
        }
    };
    for (int it = 0; it < tpw; ++it) {
        const int64_t t = tb0 + (int64_t)wave * tpw + it;
        if (t >= n_tok) break;
        const bf16_t* xp = row_ptr<bf16_t>(x, t, H);
        constexpr int XR = XC > 0 ? XC : 1;
        double xd[XR][8];
        if (XC > 0) {
#pragma unroll
            for (int i = 0; i < XC; ++i) {
                const int ch = lane + 64 * i;
                u32x4_t raw = {0, 0, 0, 0};
                if (ch < n_chunks) raw = *reinterpret_cast<const u32x4_t*>(xp + ch * 8);
                widen(raw, xd[i]);
            }
        }
        const int cnt = __builtin_amdgcn_readfirstlane(cand_cnt[t]);
        double my_z = NEG;           // lane j < K: the j-th winner so far
        int my_e = 0x7fffffff;
        for (int base = 0; base < cnt; base += 64) {
            const int n_here = cnt - base < 64 ? cnt - base : 64;
            double new_z = NEG;      // lane s: the exact logit of candidate base + s
            int new_e = 0x7fffffff;
            for (int s = 0; s < n_here; ++s) {
                const int e = __builtin_amdgcn_readfirstlane((int)cand[t * E + base + s]);
                const bf16_t* wp = wr + (int64_t)e * H;
                double acc = 0.0;
                if (XC > 0) {
#pragma unroll
                    for (int i = 0; i < XC; ++i) {
                        const int ch = lane + 64 * i;
                        if (ch < n_chunks) {
                            double wd[8];
                            widen(*reinterpret_cast<const u32x4_t*>(wp + ch * 8), wd);
#pragma unroll
                            for (int j = 0; j < 8; ++j) acc = fma(xd[i][j], wd[j], acc);
                        }
                    }
                } else {
                    for (int ch = lane; ch < n_chunks; ch += 64) {
                        double xv[8], wd[8];
                        widen(*reinterpret_cast<const u32x4_t*>(xp + ch * 8), xv);
                        widen(*reinterpret_cast<const u32x4_t*>(wp + ch * 8), wd);
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc = fma(xv[j], wd[j], acc);
                    }
                }
                double z = wave_sum(acc);
                if (bias) z += (double)bias[e];
                if (lane == s) { new_z = z; new_e = e; }
            }
            // the K largest of (previous winners, new candidates): K rounds of a wave-wide arg-max
            double old_z = my_z;
            int old_e = my_e;
            my_z = NEG;
            my_e = 0x7fffffff;
            for (int j = 0; j < K; ++j) {
                double bv = new_z;
                int be = new_e;
                if (before(old_z, old_e, bv, be)) { bv = old_z; be = old_e; }
                const int mine = be;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    const double ov = __shfl_xor(bv, off, 64);
                    const int oe = __shfl_xor(be, off, 64);
                    if (before(ov, oe, bv, be)) { bv = ov; be = oe; }
                }
                if (lane == j) { my_z = bv; my_e = be; }
                if (be == mine && be != 0x7fffffff) {      // this lane held the winner: take it out
                    if (new_e == be) { new_z = NEG; new_e = 0x7fffffff; }
                    else { old_z = NEG; old_e = 0x7fffffff; }
                }
            }
        }
        // softmax over the K selected logits (renormalised weights)
        const double z_max = __shfl(my_z, 0, 64);
        const double p = (lane < K) ? exp(my_z - z_max) : 0.0;
        double denom = p;
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

bool router_two_pass_ok(int dtype, int renorm) { return dtype == MOE_BF16 && renorm != 0; }

hipError_t launch_router_two_pass(RowSrc x, int64_t T, int H, const void* w_router, const float* bias, int E, int K,
                                  int32_t* cand_cnt, uint16_t* cand, int32_t* idx, float* w, int32_t* tile_hist,
                                  int32_t* zero_buf, int zero_n, hipStream_t s)
{
    const bf16_t* wr = (const bf16_t*)w_router;
    const unsigned grid_a = (unsigned)((T + kScreenTokens - 1) / kScreenTokens);
    const int ct = (E + 63) / 64;      // column tiles per wave
#define MOE_SCREEN(N)                                                                                         \
    {                                                                                                          \
        const size_t lds = ((size_t)2 * kScreenTokens * (N) * 64 + kScreenTokens + (N) * 64) * sizeof(float); \
        static bool attr_set[kMaxDevices] = {};                                                                \
        hipError_t e = ensure_lds_limit(router_screen_kernel<N>, lds, attr_set);                              \
        if (e != hipSuccess) return e;                                                                         \
        router_screen_kernel<N><<<grid_a, 256, lds, s>>>(x, T, H, wr, bias, E, K, cand_cnt, cand, zero_buf, zero_n); \
    }
    if (ct <= 1) MOE_SCREEN(1)
    else if (ct <= 2) MOE_SCREEN(2)
    else if (ct <= 4) MOE_SCREEN(4)
    else MOE_SCREEN(8)
#undef MOE_SCREEN
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int tpw = T <= 2048 ? 1 : 4;
    const unsigned grid_b = (unsigned)((T + kTopkWaves * tpw - 1) / (kTopkWaves * tpw));
    const int xc = (H / 8 + 63) / 64;  // 16-byte chunks of a row per lane
#define MOE_EXACT(N) router_exact_topk_kernel<N><<<grid_b, kTopkWaves * 64, 0, s>>>(x, T, H, wr, bias, E, K, tpw, cand_cnt, cand, idx, w, tile_hist)
    if (xc <= 2) MOE_EXACT(2);
    else if (xc <= 4) MOE_EXACT(4);
    else if (xc <= 6) MOE_EXACT(6);
    else if (xc <= 8) MOE_EXACT(8);
    else MOE_EXACT(0);
#undef MOE_EXACT
    return hipGetLastError();
}

}  // namespace moe
