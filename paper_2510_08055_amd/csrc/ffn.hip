// Grouped expert FFN: per expert, gate_up GEMM with the SwiGLU epilogue fused, then the
// down GEMM (Sec. 2.1: FC layers with a SwiGLU non-linearity; Sec. 2.5: each expert's FC
// runs over the tokens routed to it and is memory-bound below the ridge point, compute-
// bound above it).  bf16 x bf16 -> fp32 on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Both operands are K-contiguous (activations [rows,K], weights [N,K]), which is exactly
// the MFMA operand layout: each lane feeds 8 consecutive k-values of one row.
#include "ffn_tile.h"

namespace moe {

constexpr int kBK = 64;        // k-extent of one LDS stage
constexpr int kLdsStride = 72; // bf16 elements per LDS row: 64 + 8 pad -> 144 B, conflict-free 16 B reads

// ----------------------------------------------------------------------------------------------
// LDS-tiled MFMA grouped GEMM.  256 threads = 4 waves arranged 2 (rows) x 2 (columns).
//   Out[r, n] = sum_k X[src(r), k] * W[e, n, k]                       (GATED = false)
//   Out[r, n] = silu(sum_k X.. * W[e, n, k]) * (sum_k X.. * W[e, N + n, k])   (GATED = true)
// GATED stages BN/2 gate rows and the matching BN/2 up rows so that each wave owns both halves
// of its output columns and the SwiGLU product is taken in registers.
// Global -> register -> LDS double buffering: the loads of stage s+1 are in flight while the
// MFMAs of stage s run.
// ----------------------------------------------------------------------------------------------
// SPLIT (the intermediate held as a pair of bf16 values, value = hi + lo): the gated GEMM writes hi to
// column n and lo = bf16(value - hi) to column N + n of its output; the plain GEMM reads such rows
// (K = 2 * ldw k-values: the hi half, then the lo half) against weight rows of ldw values used twice.
template <int BM, int BN, bool GATED, typename OT, bool SPLIT>
__global__ __launch_bounds__(256) void grouped_gemm_bf16_kernel(
    RowSrc X, int ldx, const int32_t* __restrict__ row_map, int map_div,
    const int32_t* __restrict__ offsets, int E, const bf16_t* __restrict__ W, int64_t w_expert_stride, int N, int K,
    OT* __restrict__ Out, int ldo, int a_rows)
{
    const int ldw = (SPLIT && !GATED) ? K / 2 : K;      // k-values per weight row
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
    const TileCoord tc = find_tile<BM>(offsets, E, n_tiles, a_rows);
    if (!tc.valid) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: what depends on it stays in scalar registers
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
        // (a row map holds indices below a_rows; the clamp keeps a bad entry from becoming a wild address)
        int id = row_map ? row_map[r] : r;
        id = id < 0 ? 0 : (id < a_rows ? id : a_rows - 1);
        const int64_t src = row_map ? (int64_t)(id / map_div) : (int64_t)r;
        a_src[p] = row_ptr<bf16_t>(X, src, ldx) + ld_chunk * 8;
    }
#pragma unroll
    for (int p = 0; p < B_LOADS; ++p) {
        const int rb = ld_row + 32 * p;
        int n;
        if (GATED) n = (rb < NO) ? (n0 + rb) : (n0 + rb - NO);
        else n = n0 + rb;
        if (n >= N) n = N - 1;
        if (GATED && rb >= NO) n += N;
        b_src[p] = We + (int64_t)n * ldw + ld_chunk * 8;
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
        // second half of a split k-range: the same weight values again (ldw is a multiple of 8: a 16-byte
        // chunk lies in one half)
        const int kw = (k0 + ld_chunk * 8 >= ldw) ? k0 - ldw : k0;
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            b_reg[p] = in ? *reinterpret_cast<const uint4*>(b_src[p] + kw) : make_uint4(0, 0, 0, 0);
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
                if (SPLIT && GATED) val = opaque(val);
                if (row < tc.row_end && col < N) {
                    const OT hi = elem<OT>::from_f32(val);
                    Out[(int64_t)row * ldo + col] = hi;
                    if (SPLIT && GATED) Out[(int64_t)row * ldo + N + col] = elem<OT>::from_f32(val - elem<OT>::to_f32(hi));
                }
            }
        }
    }
}


// ----------------------------------------------------------------------------------------------
// Pipelined grouped GEMM: global -> LDS copies issued as direct-to-LDS loads
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions) into two rings of LDS
// slots, NSA stages of the activation rows and NSB stages of the weight rows, each stage PBK (64 or
// 32) k-values deep; one barrier per stage.  Used for both regimes of Sec. 2.5:
//   - weight streaming (few rows per expert): 64 x 128 tiles, 3 + 3 stages of 64 k-values (24 KB each);
//   - compute bound (hundreds of rows per expert): up to 256-row tiles with 64 k-values per stage, so
//     that every tile row asks for a whole 128-byte line per stage (fewer, larger requests measured
//     faster than 64-byte ones); 2 activation + 3 weight stages fill the 160 KB of LDS, the deeper
//     ring going to the operand that comes from HBM.
// NW waves arranged WM x WN; with 8 waves (2 per SIMD) one wave's barrier and LDS waits are covered
// by the other's MFMAs.
// One wave-level load moves 64 lanes x 16 B = 8 (or 16) whole tile rows into 1 KB of LDS.  LDS rows
// are unpadded (the hardware writes lanes contiguously), so bank conflicts on the 16-byte operand
// reads are avoided by an XOR swizzle applied on the SOURCE side: LDS chunk c of tile row r holds
// global 16-byte chunk c ^ swz(r).
// Row blocks (32 rows) of the m-tile that hold no real row are skipped by every wave.
// The k-order of the MFMAs is the same as in the other variants (bit-identical results).
// Requires K % PBK == 0.
// ----------------------------------------------------------------------------------------------
// OUT_F32: the output is stored as float (the down GEMM of a context that keeps y_perm in fp32).
// SPLIT: the intermediate is a pair of bf16 values, as in the kernel above.
// MAPPED: the rows come through a row map (the fused gather of the gate_up GEMM); without one the look-ups and
// their wait, a round trip to L2 at the start of every tile, are left out altogether.
template <int RBM, int BN, int WM, int NSA, int NSB, int PBK, int MINW, int NW, int ORD, bool GATED, bool OUT_F32,
          bool SPLIT, bool MAPPED>
__global__ __launch_bounds__(NW * 64, MINW) void grouped_gemm_bf16_pipe_kernel(
    RowSrc X, int ldx, const int32_t* __restrict__ row_map, int map_div,
    const int32_t* __restrict__ offsets, int E, const bf16_t* __restrict__ W, int64_t w_expert_stride, int N, int K,
    void* __restrict__ Out_, int ldo, int a_rows)
{
    static_assert(!(GATED && OUT_F32), "the intermediate of the gated GEMM is always held in the activation dtype");
    constexpr int BM = RBM * 32, WN = NW / WM;   // NW waves arranged WM (rows) x WN (columns)
    constexpr int NO = GATED ? BN / 2 : BN;     // output columns per block
    constexpr int TM = RBM / WM;                // row blocks per wave: rb = wm + WM * i
    constexpr int WNO = NO / WN;                // output columns per wave
    constexpr int TNO = WNO / 32;
    constexpr int TN = GATED ? 2 * TNO : TNO;
    constexpr int ROWB = PBK * 2;                       // bytes per LDS tile row
    constexpr int CPR = PBK / 8;                        // 16-byte chunks per row
    constexpr int RPL = 64 / CPR;                       // tile rows moved by one wave-level load (1 KB)
    constexpr int KS = PBK / 16;                        // MFMA k-slices per stage
    constexpr int A_LPW = BM / RPL / NW, B_LPW = BN / RPL / NW;   // load groups per wave and stage
    constexpr int LPS = A_LPW + B_LPW;                  // load instructions per thread and stage
    constexpr int A_SLOT = BM * ROWB, B_SLOT = BN * ROWB;   // bytes of one stage of either operand
    constexpr int B_BASE = NSA * A_SLOT;                // the weight ring follows the activation ring
    constexpr int NSMIN = NSA < NSB ? NSA : NSB, NSMAX = NSA < NSB ? NSB : NSA;
    static_assert(PBK == 64 || PBK == 32, "stage depth must be 64 or 32");
    static_assert(RBM % WM == 0 && TM <= 4 && TNO >= 1 && NSA >= 2 && NSB >= 2, "bad tile configuration");
    static_assert(ORD == 0 ? NSA == NSB : ORD == 1 ? (NSB >= NSA) : ORD == 2 ? (NSA >= NSB) : (NSA + 1 == NSB),
                  "the shallower ring loads first");
    // ORD 3: the activation ring is one stage shallower than the weight ring, and all activation loads of
    // stage g+NSA are issued at once, right behind the barrier at the end of step g that frees their slot
    // (before the last MFMAs of that step); only the weight loads are spread over the next step.  The
    // activation loads then have a whole step to land instead of half a step.
    constexpr bool A_EARLY = (ORD == 3);
    static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "tile rows must split evenly over the waves");
    // ORD 0-2: in a step the loads of activation stage g+NSA-1 are issued first, those of weight stage
    // g+NSB-1 after them; loads return in issue order, so when stage g+1 is needed the loads that may
    // still be in flight are the ones issued after activation stage g+1.  ORD 3: activation stage g+1 went
    // out behind the previous barrier, before the weight loads of step g, which are the B_LPW that may stay.
    constexpr int WAIT_MAIN = ORD == 3 ? B_LPW : (NSMIN - 2) * LPS + (NSA < NSB ? B_LPW : NSB < NSA ? A_LPW : 0);
    constexpr int WAIT_FIRST = (NSA - 2) * A_LPW;   // prologue: all weight stages, then the activation stages
    static_assert(WAIT_MAIN < 64 && WAIT_FIRST < 64, "vmcnt is a 6-bit counter");

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int n_tiles = (N + NO - 1) / NO;
    const TileCoord tc = find_tile<BM>(offsets, E, n_tiles, a_rows);
    if (!tc.valid) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: what depends on it stays in scalar registers
    const int wm = wave / WN, wn = wave % WN;
    const int n0 = tc.n_tile * NO;
    const bf16_t* We = W + (int64_t)tc.expert * w_expert_stride;
    const int rows_here = (tc.row_end - tc.row0) < BM ? (tc.row_end - tc.row0) : BM;
    const int rb_valid = (rows_here + 31) / 32;   // row blocks of this tile with at least one real row

    // ---- source addresses of this lane's loads: group g = wave + NW*p covers tile rows RPL*g .. RPL*g + RPL-1 ----
    // Order matters for the start-up latency: the row-map lookups are issued first, then (without waiting
    // for them) the weight addresses are formed and the weight stages of the prologue are put in flight,
    // and only then are the looked-up rows turned into activation addresses.
    const int l_row = lane / CPR, l_chunk = lane % CPR;
    const int nk_ = K / PBK;
    // stages per weight row: with a split intermediate the plain GEMM walks every weight row twice
    const int nk_w = (SPLIT && !GATED) ? nk_ / 2 : nk_;
    const int ldw = (SPLIT && !GATED) ? K / 2 : K;
    // The lookups are loads issued from inline asm, picked up after an explicit wait further down: a
    // lookup through the compiler would be waited for with vmcnt(0) (it does not know of the asm-issued
    // weight loads that follow), i.e. together with the first weight stages out of HBM.  Until that wait
    // the destination registers hold nothing; they are not touched in between.
    int32_t a_own[A_LPW], a_row_id[A_LPW];
#pragma unroll
    for (int p = 0; p < A_LPW; ++p) {
        int r = tc.row0 + (wave + NW * p) * RPL + l_row;
        if (r >= tc.row_end) r = tc.row_end - 1;
        a_own[p] = r;
        a_row_id[p] = 0;
        if (MAPPED) asm volatile("global_load_dword %0, %1, off" : "=v"(a_row_id[p]) : "v"(row_map + r) : "memory");
    }
    const bf16_t* b_src[B_LPW];
#pragma unroll
    for (int p = 0; p < B_LPW; ++p) {
        const int rb = (wave + NW * p) * RPL + l_row;
        int n;
        if (GATED) n = (rb < NO) ? (n0 + rb) : (n0 + rb - NO);
        else n = n0 + rb;
        if (n >= N) n = N - 1;
        if (GATED && rb >= NO) n += N;
        b_src[p] = We + (int64_t)n * ldw + ((l_chunk ^ swz<PBK>(rb)) << 3);
    }
    const uint32_t lds0 = lds_address(smem);
    auto issue_b = [&](int kt, int p) {
        const int kw = (SPLIT && !GATED && kt >= nk_w) ? kt - nk_w : kt;
        load_lds_16(b_src[p] + kw * PBK, lds0 + B_BASE + (kt % NSB) * B_SLOT + (wave + NW * p) * 1024);
    };
#pragma unroll
    for (int st = 0; st < NSB - 1; ++st)
        if (st < nk_)
#pragma unroll
            for (int p = 0; p < B_LPW; ++p) issue_b(st, p);
    if (MAPPED) {
        // the lookups came before the weight loads of the prologue: wait for them alone
        if (nk_ >= NSB - 1) wait_vmcnt<(NSB - 1) * B_LPW>();
        else wait_vmcnt<0>();
#pragma unroll
        for (int p = 0; p < A_LPW; ++p) {
            asm volatile("" : "+v"(a_row_id[p])::"memory");
            // a row map holds indices below a_rows; the clamp keeps a bad entry from becoming a wild address
            int32_t id = a_row_id[p] < 0 ? 0 : a_row_id[p];
            a_row_id[p] = id < a_rows ? id : a_rows - 1;
        }
    } else {
#pragma unroll
        for (int p = 0; p < A_LPW; ++p) a_row_id[p] = a_own[p];
    }
    const bf16_t* a_src[A_LPW];
#pragma unroll
    for (int p = 0; p < A_LPW; ++p) {
        const int tr = (wave + NW * p) * RPL + l_row;      // row inside the tile
        const int64_t src = MAPPED ? (int64_t)(a_row_id[p] / map_div) : (int64_t)a_row_id[p];
        a_src[p] = row_ptr<bf16_t>(X, src, ldx) + ((l_chunk ^ swz<PBK>(tr)) << 3);
    }
    // Loads of one stage, cut into KS parts that are issued in the shadow of the MFMAs of the KS
    // k-slices of the stage being multiplied: load p of the step (activation loads first) goes with
    // slice p * KS / LPS.
    // Lanes whose tile row lies past the tile's last row load nothing when that is safe: with NSA = 2 and
    // the activation loads issued first, no wait count includes an activation load, so it does not matter
    // whether a fully masked load instruction is issued or branched around.  The LDS rows they would have
    // filled feed only accumulator rows that are never stored.
    constexpr bool MASK_A = (NSA == 2 && (ORD == 1 || ORD == 3));
    bool a_live[A_LPW];
#pragma unroll
    for (int p = 0; p < A_LPW; ++p) a_live[p] = !MASK_A || ((wave + NW * p) * RPL + l_row) < rows_here;
    auto issue_a = [&](int kt, int p) {
        if (a_live[p])
            load_lds_16(a_src[p] + kt * PBK, lds0 + (kt % NSA) * A_SLOT + (wave + NW * p) * 1024);
    };
    // Load q of a step: ORD 0 alternates over the parts as A0 B0 | A1 B1 ..., ORD 1 issues the activation
    // loads first, ORD 2 the weight loads first; with ORD 3 a step's parts hold its weight loads only.
    auto load_is_a = [](int q) { return ORD == 2 ? q >= B_LPW : q < A_LPW; };
    auto load_idx = [](int q) { return ORD == 2 ? (q >= B_LPW ? q - B_LPW : q) : (q < A_LPW ? q : q - A_LPW); };
    auto load_part = [](int q) { return ORD == 0 ? q % KS : q * KS / LPS; };
    auto issue_part = [&](int g, int part, bool more_a, bool more_b) {
        if (A_EARLY) {
#pragma unroll
            for (int p = 0; p < B_LPW; ++p)
                if (p * KS / B_LPW == part && more_b) issue_b(g + NSB - 1, p);
            return;
        }
#pragma unroll
        for (int q = 0; q < LPS; ++q) {
            if (load_part(q) != part) continue;
            if (load_is_a(q)) {
                if (more_a) issue_a(g + NSA - 1, load_idx(q));
            } else {
                if (more_b) issue_b(g + NSB - 1, load_idx(q));
            }
        }
    };
    // ---- LDS byte offsets of the operand rows this lane feeds to the MFMAs ----
    const int fr = lane & 31, fq = lane >> 5;
    const int fsw = swz<PBK>(fr);     // the swizzle only looks at the low 4 row bits; row blocks are 32 rows
    int a_row[TM], b_row[TN], k_off[KS];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_row[i] = ((wm + WM * i) * 32 + fr) * ROWB;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int r;
        if (GATED) r = (j < TNO) ? (wn * WNO + j * 32 + fr) : (NO + wn * WNO + (j - TNO) * 32 + fr);
        else r = wn * WNO + j * 32 + fr;
        b_row[j] = B_BASE + r * ROWB;
    }
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) k_off[kk] = ((kk * 2 + fq) ^ fsw) << 4;

    // Software pipeline.  Global side: activation stages g+1 .. g+NSA-1 and weight stages g+1 ..
    // g+NSB-1 are in flight while stage g is multiplied (the weight ring may be one stage deeper: the
    // weights are what comes from HBM).  LDS side: the operand fragments of k-slice kk+1 are read while
    // the MFMAs of slice kk run; the last slice of a stage runs after the barrier that hands over the
    // next stage, under the reads of that stage's first slice.
    // The body is instantiated for the number TMV of row blocks this wave really has (0..TM), so the
    // hot loop is straight-line code; a wave with no row block still loads and synchronises.
    auto run = [&](auto tmv_const) {
        constexpr int TMV = decltype(tmv_const)::value;
        constexpr int TMA = TMV > 0 ? TMV : 1;
        float16_t acc[TMA][TN];
#pragma unroll
        for (int i = 0; i < TMA; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        bf16x8_t af[2][TMA], bfr[2][TN];
        auto read_frags = [&](int g, int kk, int set) {
            if (TMV == 0) return;
            const char* base_a = smem + (g % NSA) * A_SLOT;
            const char* base_b = smem + (g % NSB) * B_SLOT;
#pragma unroll
            for (int i = 0; i < TMV; ++i)
                af[set][i] = *reinterpret_cast<const bf16x8_t*>(base_a + a_row[i] + k_off[kk]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[set][j] = *reinterpret_cast<const bf16x8_t*>(base_b + b_row[j] + k_off[kk]);
        };
        auto mfma_set = [&](int set) {
#pragma unroll
            for (int i = 0; i < TMV; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    // weight rows as the MFMA's row operand, activation rows as its column operand: a lane then
                    // holds 4 consecutive OUTPUT COLUMNS of one output row, which the epilogue stores as 8 bytes
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][j], af[set][i], acc[i][j], 0, 0, 0);
        };

        // prologue: the weight stages are already in flight; the activation stages follow, and the first
        // wait lets through only the activation loads issued after stage 0's
#pragma unroll
        for (int st = 0; st < NSA - 1; ++st)
            if (st < nk_)
#pragma unroll
                for (int p = 0; p < A_LPW; ++p) issue_a(st, p);
        if (nk_ >= NSA - 1) wait_vmcnt<WAIT_FIRST>();
        else wait_vmcnt<0>();
        block_barrier();
        if (A_EARLY && NSA - 1 < nk_) {
#pragma unroll
            for (int p = 0; p < A_LPW; ++p) issue_a(NSA - 1, p);
        }
        read_frags(0, 0, 0);
        // One k-step.  MORE_A / MORE_B: activation stage g+NSA-1 / weight stage g+NSB-1 exists and is
        // loaded (in parts, between the MFMAs) into the slot stage g-1 used, free since the last
        // barrier.  NEXT: stage g+1 exists; it is waited for and handed over by the barrier before the
        // last slice of this stage is multiplied.
        // Ask the scheduler to issue the LDS reads and the global loads of a region one by one between
        // its MFMAs (they then execute in the shadow of the matrix pipe) instead of in a clump.
        auto interleave = [](int n_ds, int n_vmem, int n_mfma) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i < n_ds && i < n_mfma) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i < n_vmem && n_ds + i < n_mfma) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global load
                }
            }
        };
        auto parts_in = [&](int part, bool more_a, bool more_b) {
            int n = 0;
            if (A_EARLY) {
                for (int p = 0; p < B_LPW; ++p) n += (p * KS / B_LPW == part) && more_b;
                return n;
            }
            for (int q = 0; q < LPS; ++q)
                if (load_part(q) == part) n += load_is_a(q) ? more_a : more_b;
            return n;
        };
        auto step = [&](int g, auto more_a_c, auto more_b_c, auto next_c) {
            constexpr bool MORE_A = decltype(more_a_c)::value, MORE_B = decltype(more_b_c)::value;
            constexpr bool NEXT = decltype(next_c)::value;
#pragma unroll
            for (int kk = 0; kk < KS - 1; ++kk) {
                read_frags(g, kk + 1, (kk + 1) & 1);
                issue_part(g, kk, MORE_A, MORE_B);
                mfma_set(kk & 1);
                interleave(TMV > 0 ? TMV + TN : 0, parts_in(kk, MORE_A, MORE_B), TMV * TN);
            }
            issue_part(g, KS - 1, MORE_A, MORE_B);
            if (NEXT) {
                if (A_EARLY ? MORE_B : (MORE_A && MORE_B)) wait_vmcnt<WAIT_MAIN>();
                else wait_vmcnt<0>();        // the pipeline drains: wait for everything
                // all of this wave's reads of stage g have returned before its slots may be refilled
                wait_lds_reads();
                block_barrier();
                if (A_EARLY && MORE_A) {
#pragma unroll
                    for (int p = 0; p < A_LPW; ++p) issue_a(g + NSA, p);
                }
                read_frags(g + 1, 0, 0);
            }
            mfma_set((KS - 1) & 1);
            interleave(NEXT && TMV > 0 ? TMV + TN : 0, 0, TMV * TN);
        };
        using T = std::true_type;
        using F = std::false_type;
        const int n_main = nk_ - (NSMAX - 1) > 0 ? nk_ - (NSMAX - 1) : 0;   // steps that still start both loads
        int g = 0;
        for (; g < n_main; ++g) step(g, T{}, T{}, T{});
        for (; g < nk_ - 1; ++g) {
            // only the shallower ring may still have a stage to fetch
            if (!A_EARLY && NSA < NSB && g + NSA - 1 < nk_) step(g, T{}, F{}, T{});
            else if (NSB < NSA && g + NSB - 1 < nk_) step(g, F{}, T{}, T{});
            else step(g, F{}, F{}, T{});
        }
        step(g, F{}, F{}, F{});

        // Epilogue.  A lane holds, for output row fr of a row block, groups of 4 consecutive columns
        // (accumulator element v of tile (i, j): column (v/4)*8 + fq*4 + v%4); storing them directly
        // would scatter 8-byte pieces over 32 rows per instruction.  Each wave instead turns one row block
        // at a time (32 rows x WNO columns, at most 4 KB) through a private piece of LDS and writes it
        // out as whole 16-byte chunks, consecutive lanes along a row (64- or 128-byte runs per row).
        // The LDS used is an activation slot no stage occupies any more: stage nk-1, the last one, sits
        // in slot (nk-1) % NSA, and the readers of the other slots passed their barrier long ago, so no
        // block barrier is needed; a wave's own LDS operations execute in program order.
        constexpr int RB = TNO * 64;              // bytes of one row of the wave's output tile
        constexpr int CPRW = TNO * 4;             // 16-byte chunks per such row
        constexpr int REG = 32 * RB;              // bytes per wave
        constexpr int WPS = A_SLOT / REG;         // waves per free activation slot
        constexpr int RPI = 64 / CPRW;            // rows one wave-level 16-byte access covers
        static_assert(TNO <= 2 && WPS >= 1 && (NSA - 1) * WPS >= NW, "the epilogue staging does not fit the free slots");
        static_assert(!OUT_F32 || REG >= 4096, "a 32 x 32 float tile must fit the wave's staging piece");
        if (TMV > 0 && OUT_F32) {
            // float output: one 32 x 32 tile (4 KB: 32 rows of 8 16-byte chunks) at a time through the same
            // private piece of LDS; a lane's 4 consecutive columns are one chunk, chunk c of row r sits in
            // chunk slot c ^ (r & 7), and the tile goes out as 128-byte runs per row.
            float* Out = static_cast<float*>(Out_);
            char* epi = smem + ((nk_ + wave / WPS) % NSA) * A_SLOT + (wave % WPS) * REG;
#pragma unroll
            for (int i = 0; i < TMV; ++i) {
                const int64_t row_base = (int64_t)tc.row0 + (wm + WM * i) * 32;
#pragma unroll
                for (int j = 0; j < TNO; ++j) {
#pragma unroll
                    for (int a = 0; a < 4; ++a)
                        *reinterpret_cast<float4*>(epi + fr * 128 + (((a * 2 + fq) ^ (fr & 7)) << 4)) =
                            make_float4(acc[i][j][a * 4], acc[i][j][a * 4 + 1], acc[i][j][a * 4 + 2], acc[i][j][a * 4 + 3]);
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const int r = h * 8 + (lane >> 3), c = lane & 7;
                        const float4 v = *reinterpret_cast<const float4*>(epi + r * 128 + ((c ^ (r & 7)) << 4));
                        const int64_t row = row_base + r;
                        const int col = n0 + wn * WNO + j * 32 + c * 4;
                        if (row < tc.row_end && col < N)    // N is a multiple of 8: the 4 columns are in or out together
                            *reinterpret_cast<float4*>(Out + row * ldo + col) = v;
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
        } else if (TMV > 0) {
            bf16_t* Out = static_cast<bf16_t*>(Out_);
            char* epi = smem + ((nk_ + wave / WPS) % NSA) * A_SLOT + (wave % WPS) * REG;
            auto eswz = [](int r) { return (r >> (RB == 64 ? 2 : 1)) & (CPRW - 1); };
            constexpr int PARTS = (SPLIT && GATED) ? 2 : 1;      // the values, then what their bf16 rounding left over
#pragma unroll
            for (int i = 0; i < TMV; ++i) {
                if (GATED) {
#pragma unroll
                    for (int j = 0; j < TNO; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            acc[i][j][v] = silu_mul(acc[i][j][v], acc[i][j + TNO][v]);
                            if (SPLIT) acc[i][j][v] = opaque(acc[i][j][v]);
                        }
                }
#pragma unroll
                for (int part = 0; part < PARTS; ++part) {
#pragma unroll
                    for (int j = 0; j < TNO; ++j) {
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            float val[4];
#pragma unroll
                            for (int b = 0; b < 4; ++b) val[b] = acc[i][j][a * 4 + b];
                            const uint32_t p01 = pack_bf16x2(val[0], val[1]), p23 = pack_bf16x2(val[2], val[3]);
                            if (PARTS == 2 && part == 0) {      // keep the remainders for the second part
                                acc[i][j][a * 4 + 0] = val[0] - __uint_as_float(p01 << 16);
                                acc[i][j][a * 4 + 1] = val[1] - __uint_as_float(p01 & 0xffff0000u);
                                acc[i][j][a * 4 + 2] = val[2] - __uint_as_float(p23 << 16);
                                acc[i][j][a * 4 + 3] = val[3] - __uint_as_float(p23 & 0xffff0000u);
                            }
                            const int chunk = (j * 4 + a) ^ eswz(fr);
                            *reinterpret_cast<uint2*>(epi + fr * RB + chunk * 16 + fq * 8) = make_uint2(p01, p23);
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                    const int64_t row_base = (int64_t)tc.row0 + (wm + WM * i) * 32;
#pragma unroll
                    for (int h = 0; h < 32 / RPI; ++h) {
                        const int r = h * RPI + lane / CPRW, c = lane % CPRW;
                        const uint4 v = *reinterpret_cast<const uint4*>(epi + r * RB + ((c ^ eswz(r)) * 16));
                        const int64_t row = row_base + r;
                        const int col = n0 + wn * WNO + c * 8;
                        if (row < tc.row_end && col < N)    // N is a multiple of 8: a chunk is in or out as a whole
                            *reinterpret_cast<uint4*>(Out + row * ldo + part * N + col) = v;
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
    };

    // row blocks wm, wm + WM, ... below rb_valid belong to this wave
    const int tm_valid = (rb_valid - wm + WM - 1) / WM;
    if (TM >= 4 && tm_valid >= 4) run(std::integral_constant<int, (TM >= 4 ? 4 : 0)>{});
    else if (TM >= 3 && tm_valid >= 3) run(std::integral_constant<int, (TM >= 3 ? 3 : 0)>{});
    else if (TM >= 2 && tm_valid >= 2) run(std::integral_constant<int, (TM >= 2 ? 2 : 0)>{});
    else if (tm_valid >= 1) run(std::integral_constant<int, 1>{});
    else run(std::integral_constant<int, 0>{});
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
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(RowSrc X, int ldx,
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
    int id = row_map ? row_map[r] : r;
    id = id < 0 ? 0 : (id < A ? id : (int)A - 1);      // a bad map entry must not become a wild address
    const int64_t src = row_map ? (int64_t)(id / map_div) : (int64_t)r;
    const float* x = row_ptr<float>(X, src, ldx);
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
// Host side: variant choice and launches.  The host never sees the per-expert counts (they live on
// the device), so the variant is chosen from the mean rows per expert A/E; every variant is correct
// for any distribution of rows.
// ----------------------------------------------------------------------------------------------
enum Variant { V_TILE128 = 0, V_PIPE_SMALL, V_PIPE_BIG };

static Variant pick_variant(int variant, int64_t A, int E, int K)
{
    Variant v;
    const double mean_rows = (double)A / (double)E;
    if (mean_rows <= 64.0) v = V_PIPE_SMALL;   // weight streaming: 64 x 128 tiles, 3 stages of 64 k-values
    else v = V_PIPE_BIG;                       // up to 256-row tiles, 2 + 3 stages of 64 k-values
    if (variant == MOE_FFN_TILE128) v = V_TILE128;
    if (variant == MOE_FFN_PIPE_SMALL) v = V_PIPE_SMALL;
    if (variant == MOE_FFN_PIPE_BIG) v = V_PIPE_BIG;
    if (K % 64 != 0) v = V_TILE128;            // the pipelined kernels have no k-tail path
    return v;
}

template <int BM, int BN, bool GATED, typename OT, bool SPLIT>
static hipError_t launch_tile(RowSrc X, int ldx, const int32_t* row_map, int map_div, const int32_t* offsets,
                              int E, int64_t A, const bf16_t* W, int64_t w_expert_stride, int N, int K, void* Out,
                              int ldo, hipStream_t s)
{
    constexpr int NO = GATED ? BN / 2 : BN;
    const size_t lds_bytes = 2 * (size_t)(BM + BN) * kLdsStride * sizeof(bf16_t);
    auto kern = grouped_gemm_bf16_kernel<BM, BN, GATED, OT, SPLIT>;
    static bool attr_set[kMaxDevices] = {};
    hipError_t e = ensure_lds_limit(kern, lds_bytes, attr_set);
    if (e != hipSuccess) return e;
    const int64_t n_tiles = (N + NO - 1) / NO;
    const int64_t m_tiles_max = (A + BM - 1) / BM + (A < E ? A : E);   // sum_e ceil(m_e / BM) never exceeds this
    const int64_t grid = ((m_tiles_max * n_tiles + 7) / 8) * 8;
    if (grid >= ((int64_t)1 << 31)) return hipErrorInvalidValue;   // the device-side tile search counts in 32 bits
    kern<<<(unsigned)grid, 256, lds_bytes, s>>>(X, ldx, row_map, map_div, offsets, E, W, w_expert_stride, N, K,
                                                static_cast<OT*>(Out), ldo, (int)A);
    return hipGetLastError();
}

template <int RBM, int BN, int WM, int NSA, int NSB, int PBK, int MINW, int NW, int ORD, bool GATED, bool OUT_F32,
          bool SPLIT, bool MAPPED>
static hipError_t launch_pipe(RowSrc X, int ldx, const int32_t* row_map, int map_div, const int32_t* offsets,
                              int E, int64_t A, const bf16_t* W, int64_t w_expert_stride, int N, int K, void* Out,
                              int ldo, hipStream_t s)
{
    constexpr int BM = RBM * 32;
    constexpr int NO = GATED ? BN / 2 : BN;
    const size_t lds_bytes = ((size_t)NSA * BM + (size_t)NSB * BN) * PBK * 2;
    auto kern = grouped_gemm_bf16_pipe_kernel<RBM, BN, WM, NSA, NSB, PBK, MINW, NW, ORD, GATED, OUT_F32, SPLIT, MAPPED>;
    static bool attr_set[kMaxDevices] = {};
    hipError_t e = ensure_lds_limit(kern, lds_bytes, attr_set);
    if (e != hipSuccess) return e;
    const int64_t n_tiles = (N + NO - 1) / NO;
    const int64_t m_tiles_max = (A + BM - 1) / BM + (A < E ? A : E);
    const int64_t grid = ((m_tiles_max * n_tiles + 7) / 8) * 8;
    if (grid >= ((int64_t)1 << 31)) return hipErrorInvalidValue;   // the device-side tile search counts in 32 bits
    kern<<<(unsigned)grid, NW * 64, lds_bytes, s>>>(X, ldx, row_map, map_div, offsets, E, W, w_expert_stride, N, K, Out,
                                                ldo, (int)A);
    return hipGetLastError();
}

// K: k-extent of the GEMM (twice the weight rows' length when the plain GEMM reads a split intermediate)
template <bool GATED, bool OUT_F32, bool SPLIT>
static hipError_t launch_bf16(int variant, RowSrc X, int ldx, const int32_t* row_map, int map_div,
                              const int32_t* offsets, int E, int64_t A, const bf16_t* W, int64_t w_expert_stride,
                              int N, int K, void* Out, int ldo, hipStream_t s)
{
    // weight streaming: 64 x 128 tiles, 4 waves, 72 KB of LDS: two blocks share a compute unit, so one
    // block's prologue and epilogue are covered by the other's loads, and the many small tiles balance
    // well over the chip.  compute bound: 256 x 256 tiles, 8 waves (2 per SIMD: one wave's barrier and
    // LDS waits are covered by the other's MFMAs), 2 (rows) x 4 (columns).
    // (only the gate_up GEMM is ever called with a row map)
    const bool mapped = GATED && row_map != nullptr;
    if (!GATED && row_map != nullptr) return hipErrorInvalidValue;
    switch (pick_variant(variant, A, E, (SPLIT && !GATED) ? K / 2 : K)) {
        case V_PIPE_SMALL:
            if (mapped)
                return launch_pipe<2, 128, 2, 3, 3, 64, 2, 4, 0, GATED, OUT_F32, SPLIT, GATED>(X, ldx, row_map, map_div, offsets, E, A, W, w_expert_stride, N, K, Out, ldo, s);
            return launch_pipe<2, 128, 2, 3, 3, 64, 2, 4, 0, GATED, OUT_F32, SPLIT, false>(X, ldx, row_map, map_div, offsets, E, A, W, w_expert_stride, N, K, Out, ldo, s);
        case V_PIPE_BIG:
            if (mapped)
                return launch_pipe<8, 256, 2, 2, 3, 64, 2, 8, 3, GATED, OUT_F32, SPLIT, GATED>(X, ldx, row_map, map_div, offsets, E, A, W, w_expert_stride, N, K, Out, ldo, s);
            return launch_pipe<8, 256, 2, 2, 3, 64, 2, 8, 3, GATED, OUT_F32, SPLIT, false>(X, ldx, row_map, map_div, offsets, E, A, W, w_expert_stride, N, K, Out, ldo, s);
        default:
            if (OUT_F32)
                return launch_tile<128, 128, GATED, float, SPLIT>(X, ldx, row_map, map_div, offsets, E, A, W,
                                                                  w_expert_stride, N, K, Out, ldo, s);
            return launch_tile<128, 128, GATED, bf16_t, SPLIT>(X, ldx, row_map, map_div, offsets, E, A, W,
                                                               w_expert_stride, N, K, Out, ldo, s);
    }
}

hipError_t launch_ffn_gate_up(int dtype, int variant, bool split, RowSrc x, const int32_t* row_map, int map_div,
                              const int32_t* offsets, int64_t A, int E, int H, int I, const void* w_gate_up, void* act,
                              hipStream_t s)
{
    if (dtype == MOE_BF16) {
        if (split)      // act [A, 2I]: the values' bf16 roundings in columns [0, I), the remainders in [I, 2I)
            return launch_bf16<true, false, true>(variant, x, H, row_map, map_div, offsets, E, A, (const bf16_t*)w_gate_up,
                                                  (int64_t)2 * I * H, I, H, act, 2 * I, s);
        return launch_bf16<true, false, false>(variant, x, H, row_map, map_div, offsets, E, A, (const bf16_t*)w_gate_up,
                                               (int64_t)2 * I * H, I, H, act, I, s);
    }
    const unsigned grid = (unsigned)((A * I + 255) / 256);
    grouped_gemm_f32_kernel<true><<<grid, 256, 0, s>>>(x, H, row_map, map_div, offsets, E,
                                                       (const float*)w_gate_up, (int64_t)2 * I * H, I, H, A,
                                                       (float*)act, I);
    return hipGetLastError();
}

hipError_t launch_ffn_down(int dtype, int variant, bool out_f32, bool split, const void* act, const int32_t* offsets,
                           int64_t A, int E, int H, int I, const void* w_down, void* y_perm, hipStream_t s)
{
    if (dtype == MOE_BF16) {
        if (split)      // (a split intermediate comes with fp32 expert outputs)
            return launch_bf16<false, true, true>(variant, single_src(act), 2 * I, nullptr, 1, offsets, E, A,
                                                  (const bf16_t*)w_down, (int64_t)H * I, H, 2 * I, y_perm, H, s);
        if (out_f32)
            return launch_bf16<false, true, false>(variant, single_src(act), I, nullptr, 1, offsets, E, A,
                                                   (const bf16_t*)w_down, (int64_t)H * I, H, I, y_perm, H, s);
        return launch_bf16<false, false, false>(variant, single_src(act), I, nullptr, 1, offsets, E, A,
                                                (const bf16_t*)w_down, (int64_t)H * I, H, I, y_perm, H, s);
    }
    const unsigned grid = (unsigned)((A * H + 255) / 256);
    grouped_gemm_f32_kernel<false><<<grid, 256, 0, s>>>(single_src(act), I, nullptr, 1, offsets, E,
                                                        (const float*)w_down, (int64_t)H * I, H, I, A,
                                                        (float*)y_perm, H);
    return hipGetLastError();
}

const char* ffn_variant_name(int dtype, int variant, int64_t A, int E, int H, int I)
{
    (void)I;
    if (dtype != MOE_BF16) return "grouped_gemm_f32_kernel<gated>";
    switch (pick_variant(variant, A, E, H)) {
        case V_PIPE_SMALL: return "grouped_gemm_bf16_pipe_kernel<2,128,2,3,3,64,2,4,0,gated>";
        case V_PIPE_BIG: return "grouped_gemm_bf16_pipe_kernel<8,256,2,2,3,64,2,8,3,gated>";
        default: return "grouped_gemm_bf16_kernel<128,128,gated>";
    }
}

}  // namespace moe
