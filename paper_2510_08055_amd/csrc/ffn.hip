// Grouped expert FFN: per expert, gate_up GEMM with the SwiGLU epilogue fused, then the
// down GEMM (Sec. 2.1: FC layers with a SwiGLU non-linearity; Sec. 2.5: each expert's FC
// runs over the tokens routed to it and is memory-bound below the ridge point, compute-
// bound above it).  bf16 x bf16 -> fp32 on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Both operands are K-contiguous (activations [rows,K], weights [N,K]), which is exactly
// the MFMA operand layout: each lane feeds 8 consecutive k-values of one row.
#include "common.h"

namespace moe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;        // k-extent of one LDS stage
constexpr int kLdsStride = 72; // bf16 elements per LDS row: 64 + 8 pad -> 144 B, conflict-free 16 B reads

// ----------------------------------------------------------------------------------------------
// Work decomposition.  The launch grid is data-independent (an upper bound on the number of
// tiles); every block finds its own (expert, m-tile, n-tile) from the device-side offsets and
// blocks beyond the real tile count exit.  Experts without rows get no tile, so none of their
// weights is read.
//
// Hardware hands consecutive workgroup ids to the 8 XCDs round-robin.  Logical tile ids are
// therefore remapped so that each XCD walks one contiguous eighth of the logical order, and the
// logical order is expert-major, then n-tile, then m-tile: the m-tiles that share one weight
// tile run back to back on the same XCD (second and later reads hit that XCD's L2), and one
// expert's activation rows stay in the same L2 while its n-tiles stream by.
// ----------------------------------------------------------------------------------------------
struct TileCoord {
    int expert, row0, row_end, n_tile;
    bool valid;
};

__device__ __forceinline__ TileCoord find_tile(const int32_t* __restrict__ offsets, int E, int BM, int n_tiles)
{
    constexpr int EPL = kMaxExperts / 64;
    const int lane = lane_id();
    int off[EPL + 1];
#pragma unroll
    for (int i = 0; i <= EPL; ++i) {
        const int e = lane * EPL + i;
        off[i] = offsets[e <= E ? e : E];
    }
    int mt[EPL];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        mt[i] = (off[i + 1] - off[i] + BM - 1) / BM;
        sum += mt[i];
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    const int total_m = __shfl(incl, 63, 64);
    const long total = (long)total_m * n_tiles;
    const long chunk = (total + 7) / 8;
    const long slot = blockIdx.x / 8;
    const long logical = (long)(blockIdx.x % 8) * chunk + slot;
    TileCoord tc;
    tc.valid = (slot < chunk) && (logical < total);
    tc.expert = 0; tc.row0 = 0; tc.row_end = 0; tc.n_tile = 0;
    if (!tc.valid) return tc;
    // the lane whose experts contain the tile (tiles of an expert: mt_e * n_tiles, n-major)
    const unsigned long long hit = __ballot(logical < (long)incl * n_tiles);
    const int src = __ffsll((long long)hit) - 1;
    long rem = logical - (long)(incl - sum) * n_tiles;   // meaningful on lane src only
    int expert = 0, row0 = 0, row_end = 0, n_tile = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const long cnt = (long)mt[i] * n_tiles;
        if (rem >= 0 && rem < cnt) {
            expert = lane * EPL + i;
            n_tile = (int)(rem / mt[i]);
            row0 = off[i] + (int)(rem % mt[i]) * BM;
            row_end = off[i + 1];
            rem = -1;
        } else if (rem >= 0) {
            rem -= cnt;
        }
    }
    tc.expert = __shfl(expert, src, 64);
    tc.row0 = __shfl(row0, src, 64);
    tc.row_end = __shfl(row_end, src, 64);
    tc.n_tile = __shfl(n_tile, src, 64);
    return tc;
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// ----------------------------------------------------------------------------------------------
// LDS-tiled MFMA grouped GEMM.  256 threads = 4 waves arranged 2 (rows) x 2 (columns).
//   Out[r, n] = sum_k X[src(r), k] * W[e, n, k]                       (GATED = false)
//   Out[r, n] = silu(sum_k X.. * W[e, n, k]) * (sum_k X.. * W[e, N + n, k])   (GATED = true)
// GATED stages BN/2 gate rows and the matching BN/2 up rows so that each wave owns both halves
// of its output columns and the SwiGLU product is taken in registers.
// Global -> register -> LDS double buffering: the loads of stage s+1 are in flight while the
// MFMAs of stage s run.
// ----------------------------------------------------------------------------------------------
template <int BM, int BN, bool GATED>
__global__ __launch_bounds__(256) void grouped_gemm_bf16_kernel(
    const bf16_t* __restrict__ X, int ldx, const int32_t* __restrict__ row_map, int map_div,
    const int32_t* __restrict__ offsets, int E, const bf16_t* __restrict__ W, int64_t w_expert_stride, int N, int K,
    bf16_t* __restrict__ Out, int ldo)
{
    constexpr int NO = GATED ? BN / 2 : BN;          // output columns per block
    constexpr int TM = BM / 2 / 32;                  // 32-row MFMA tiles per wave
    constexpr int TNO = NO / 2 / 32;                 // 32-column output tiles per wave
    constexpr int TN = GATED ? 2 * TNO : TNO;        // MFMA column tiles per wave (gate tiles then up tiles)
    constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;
    constexpr int A_ELEMS = BM * kLdsStride, B_ELEMS = BN * kLdsStride;
    static_assert(TM >= 1 && TNO >= 1, "tile too small for a 2x2 wave grid of 32x32 MFMAs");

    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    auto ldsA = [&](int buf) { return lds + buf * (A_ELEMS + B_ELEMS); };
    auto ldsB = [&](int buf) { return lds + buf * (A_ELEMS + B_ELEMS) + A_ELEMS; };

    const int n_tiles = (N + NO - 1) / NO;
    const TileCoord tc = find_tile(offsets, E, BM, n_tiles);
    if (!tc.valid) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int n0 = tc.n_tile * NO;
    const bf16_t* We = W + (int64_t)tc.expert * w_expert_stride;

    // global source rows of this thread's 16-byte loads (fixed over the k-loop)
    const int ld_chunk = tid & 7, ld_row = tid >> 3;
    const bf16_t* a_src[A_LOADS];
    const bf16_t* b_src[B_LOADS];
#pragma unroll
    for (int p = 0; p < A_LOADS; ++p) {
        int r = tc.row0 + ld_row + 32 * p;
        if (r >= tc.row_end) r = tc.row_end - 1;            // ragged tail: re-read a valid row, result unused
        const int64_t src = row_map ? (int64_t)(row_map[r] / map_div) : (int64_t)r;
        a_src[p] = X + src * ldx + ld_chunk * 8;
    }
#pragma unroll
    for (int p = 0; p < B_LOADS; ++p) {
        const int rb = ld_row + 32 * p;
        int n;
        if (GATED) n = (rb < NO) ? (n0 + rb) : (n0 + rb - NO);
        else n = n0 + rb;
        if (n >= N) n = N - 1;
        if (GATED && rb >= NO) n += N;
        b_src[p] = We + (int64_t)n * K + ld_chunk * 8;
    }

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 a_reg[A_LOADS], b_reg[B_LOADS];
    auto load_stage = [&](int k0) {
        const bool in = (k0 + ld_chunk * 8) < K;
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            a_reg[p] = in ? *reinterpret_cast<const uint4*>(a_src[p] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            b_reg[p] = in ? *reinterpret_cast<const uint4*>(b_src[p] + k0) : make_uint4(0, 0, 0, 0);
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            *reinterpret_cast<uint4*>(ldsA(buf) + (ld_row + 32 * p) * kLdsStride + ld_chunk * 8) = a_reg[p];
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            *reinterpret_cast<uint4*>(ldsB(buf) + (ld_row + 32 * p) * kLdsStride + ld_chunk * 8) = b_reg[p];
    };

    // LDS rows this lane feeds to the MFMAs
    const int fr = lane & 31, fq = lane >> 5;
    int a_row[TM], b_row[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_row[i] = wm * (BM / 2) + i * 32 + fr;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        if (GATED) b_row[j] = (j < TNO) ? (wn * (NO / 2) + j * 32 + fr) : (NO + wn * (NO / 2) + (j - TNO) * 32 + fr);
        else b_row[j] = wn * (NO / 2) + j * 32 + fr;
    }

    const int nk = (K + kBK - 1) / kBK;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_stage((kt + 1) * kBK);
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8_t af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t*>(ldsA(buf) + a_row[i] * kLdsStride + kk * 16 + fq * 8);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8_t*>(ldsB(buf) + b_row[j] * kLdsStride + kk * 16 + fq * 8);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_stage(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator element v of a 32x32 tile: row (v/4)*8 + (lane/32)*4 + v%4, column lane%32.
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TNO; ++j) {
            const int col = n0 + wn * (NO / 2) + j * 32 + fr;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = tc.row0 + wm * (BM / 2) + i * 32 + (v >> 2) * 8 + fq * 4 + (v & 3);
                float val;
                if (GATED) val = silu_mul(acc[i][j][v], acc[i][j + TNO][v]);
                else val = acc[i][j][v];
                if (row < tc.row_end && col < N) Out[(int64_t)row * ldo + col] = f32_to_bf16(val);
            }
        }
    }
}

// ----------------------------------------------------------------------------------------------
// fp32 reference-precision path (small correctness workloads): one thread per output element.
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ int expert_of_row(const int32_t* __restrict__ offsets, int E, int r)
{
    int lo = 0, hi = E;   // largest e with offsets[e] <= r
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid] <= r) lo = mid; else hi = mid;
    }
    return lo;
}

template <bool GATED>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(const float* __restrict__ X, int ldx,
                                                               const int32_t* __restrict__ row_map, int map_div,
                                                               const int32_t* __restrict__ offsets, int E,
                                                               const float* __restrict__ W, int64_t w_expert_stride,
                                                               int N, int K, int64_t A, float* __restrict__ Out,
                                                               int ldo)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= A * N) return;
    const int r = (int)(g / N), n = (int)(g % N);
    const int e = expert_of_row(offsets, E, r);
    const int64_t src = row_map ? (int64_t)(row_map[r] / map_div) : (int64_t)r;
    const float* x = X + src * ldx;
    const float* w0 = W + (int64_t)e * w_expert_stride + (int64_t)n * K;
    float s0 = 0.f, s1 = 0.f;
    for (int k = 0; k < K; ++k) s0 = fmaf(x[k], w0[k], s0);
    if (GATED) {
        const float* w1 = w0 + (int64_t)N * K;
        for (int k = 0; k < K; ++k) s1 = fmaf(x[k], w1[k], s1);
        Out[(int64_t)r * ldo + n] = s0 / (1.0f + expf(-s0)) * s1;
    } else {
        Out[(int64_t)r * ldo + n] = s0;
    }
}

// ----------------------------------------------------------------------------------------------
template <int BM, int BN, bool GATED>
static hipError_t launch_bf16(const bf16_t* X, int ldx, const int32_t* row_map, int map_div, const int32_t* offsets,
                              int E, int64_t A, const bf16_t* W, int64_t w_expert_stride, int N, int K, bf16_t* Out,
                              int ldo, hipStream_t s)
{
    constexpr int NO = GATED ? BN / 2 : BN;
    const size_t lds_bytes = 2 * (size_t)(BM + BN) * kLdsStride * sizeof(bf16_t);
    auto kern = grouped_gemm_bf16_kernel<BM, BN, GATED>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t n_tiles = (N + NO - 1) / NO;
    const int64_t m_tiles_max = (A + BM - 1) / BM + (A < E ? A : E);   // sum_e ceil(m_e / BM) never exceeds this
    const int64_t grid = ((m_tiles_max * n_tiles + 7) / 8) * 8;
    kern<<<(unsigned)grid, 256, lds_bytes, s>>>(X, ldx, row_map, map_div, offsets, E, W, w_expert_stride, N, K, Out,
                                                ldo);
    return hipGetLastError();
}

hipError_t launch_ffn_gate_up(int dtype, const void* x, const int32_t* row_map, int map_div, const int32_t* offsets,
                              int64_t A, int E, int H, int I, const void* w_gate_up, void* act, hipStream_t s)
{
    if (dtype == MOE_BF16)
        return launch_bf16<128, 128, true>((const bf16_t*)x, H, row_map, map_div, offsets, E, A,
                                           (const bf16_t*)w_gate_up, (int64_t)2 * I * H, I, H, (bf16_t*)act, I, s);
    const unsigned grid = (unsigned)((A * I + 255) / 256);
    grouped_gemm_f32_kernel<true><<<grid, 256, 0, s>>>((const float*)x, H, row_map, map_div, offsets, E,
                                                       (const float*)w_gate_up, (int64_t)2 * I * H, I, H, A,
                                                       (float*)act, I);
    return hipGetLastError();
}

hipError_t launch_ffn_down(int dtype, const void* act, const int32_t* offsets, int64_t A, int E, int H, int I,
                           const void* w_down, void* y_perm, hipStream_t s)
{
    if (dtype == MOE_BF16)
        return launch_bf16<128, 128, false>((const bf16_t*)act, I, nullptr, 1, offsets, E, A, (const bf16_t*)w_down,
                                            (int64_t)H * I, H, I, (bf16_t*)y_perm, H, s);
    const unsigned grid = (unsigned)((A * H + 255) / 256);
    grouped_gemm_f32_kernel<false><<<grid, 256, 0, s>>>((const float*)act, I, nullptr, 1, offsets, E,
                                                        (const float*)w_down, (int64_t)H * I, H, I, A,
                                                        (float*)y_perm, H);
    return hipGetLastError();
}

const char* ffn_variant_name(int dtype, int64_t A, int E, int H, int I)
{
    (void)A; (void)E; (void)H; (void)I;
    return dtype == MOE_BF16 ? "grouped_gemm_bf16_kernel<128,128,gated>" : "grouped_gemm_f32_kernel<gated>";
}

}  // namespace moe
