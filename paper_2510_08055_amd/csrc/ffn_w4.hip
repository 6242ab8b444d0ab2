// Grouped expert FFN with 4-bit expert weights (MXFP4) and bf16 activations.
//
// The paper's broader validation (Table 7) runs a model whose expert weights are fp4; what changes for
// the MoE layer is the bytes per expert, hence where the ridge of Sec. 2.5 lies: a decode-heavy batch
// streams 17/32 of a byte per weight instead of 2.  The format is the published OCP Microscaling MXFP4:
// FP4 E2M1 elements, two per byte (even element in the low nibble), one E8M0 scale byte (2^(s-127)) per
// 32 consecutive elements along k.  A dequantised weight is exactly representable in bf16, so the GEMM
// is the bf16 MFMA GEMM of ffn.hip on weights widened on the fly (v_cvt_scalef32_pk_bf16_fp4).
//
// Two kernel shapes.  The first, for batches with more than 96 rows per expert on average: 64-row x
// 256-weight-row tiles, 4 waves side by side along the weight rows (each widens and multiplies its own
// 64 weight rows against the tile's one or two 32-row blocks), 64 k-values per stage; activation rows
// come through a 2-stage LDS ring as in ffn.hip.  The packed weight rows and their scale bytes are
// fetched for TWO stages at a time (64 bytes of codes and 4 scale bytes per row) into a ring of 3 such
// double stages: the layer is bound by the number of memory requests, not their bytes, when every row
// contributes 32 + 2 bytes per stage (measured: 2.7x slower).  72 KB of LDS: two blocks share a compute
// unit.  The second, the weight-streaming shape for decode-heavy batches, is described further down.
// In both, within a 64-wide stage lane (row, q) feeds k-block q (32 values) to four successive MFMAs, 8
// values each, and the activation fragments follow the same k assignment; stages and MFMAs run in the
// same ascending order, so the two shapes produce bit-identical results and a chunked and a layered pass
// may pick different ones.
#include "ffn_tile.h"

namespace moe {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int kW4Rows = 64, kW4BN = 256, kW4Waves = 4, kW4K = 64;
constexpr int kW4NSA = 2, kW4NSB = 3;     // activation stages; weight DOUBLE stages (two stages each)

// Loads that may still be in flight while the wave goes on: the pipeline keeps count of the load
// instructions it has issued and of the last one each stage needs, so the wait is exact in the start-up
// and drain steps as well.  s_waitcnt takes an immediate: the count is rounded down to the next value in the tree.
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    if (n >= 10) {
        if (n >= 16) {
            if (n >= 20) wait_vmcnt<20>();
            else if (n >= 18) wait_vmcnt<18>();
            else wait_vmcnt<16>();
        } else {
            if (n >= 14) wait_vmcnt<14>();
            else if (n >= 12) wait_vmcnt<12>();
            else wait_vmcnt<10>();
        }
    } else {
        if (n >= 4) {
            if (n >= 8) wait_vmcnt<8>();
            else if (n >= 6) wait_vmcnt<6>();
            else wait_vmcnt<4>();
        } else {
            if (n >= 3) wait_vmcnt<3>();
            else if (n >= 2) wait_vmcnt<2>();
            else if (n >= 1) wait_vmcnt<1>();
            else wait_vmcnt<0>();
        }
    }
}

// 8 FP4 values (one dword) times the block's scale -> 8 bf16, in k order.
__device__ __forceinline__ bf16x8_t widen_fp4x8(uint32_t v, float scale)
{
    const bf16x2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(v, scale, 0);
    const bf16x2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(v, scale, 1);
    const bf16x2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(v, scale, 2);
    const bf16x2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(v, scale, 3);
    return bf16x8_t{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// E8M0 scale byte -> float 2^(s - 127); s = 0 is 2^-127, a subnormal float.
__device__ __forceinline__ float e8m0_to_float(uint32_t s) { return __uint_as_float(s ? s << 23 : 0x00400000u); }

// The same for byte SH / 8 of a word, in three instructions: the byte is moved into the exponent field
// in place, and 2^-127 = 0x00400000 exceeds the result only when the byte is 0.  (Written as a compare
// and select the compiler extracts the byte twice, with three constants moved into registers per use.)
template <int SH> __device__ __forceinline__ float e8m0_byte_to_float(uint32_t word)
{
    uint32_t bits = (SH <= 23 ? word << (23 - SH) : word >> (SH - 23)) & 0x7f800000u, out;
    asm("v_max_u32 %0, %1, %2" : "=v"(out) : "s"(0x00400000u), "v"(bits));
    return __uint_as_float(out);
}

//   Out[r, n] = sum_k X[src(r), k] * W[e, n, k]                                        (GATED = false)
//   Out[r, n] = silu(sum_k X.. * W[e, n, k]) * (sum_k X.. * W[e, N + n, k])            (GATED = true)
// W: packed codes [E][rows][K/2] bytes, S: scales [E][rows][K/32] bytes; rows = N (or 2N when GATED).
// Requires K % 64 == 0.
// OUT_F32: the output is stored as float (down GEMM of a context that keeps y_perm in fp32).
template <bool GATED, bool OUT_F32>
__global__ __launch_bounds__(kW4Waves * 64, 2) void grouped_gemm_w4_kernel(
    RowSrc X, int ldx, const int32_t* __restrict__ row_map, int map_div, const int32_t* __restrict__ offsets, int E,
    const uint8_t* __restrict__ W, const uint8_t* __restrict__ S, int64_t rows_per_expert, int N, int K,
    void* __restrict__ Out_, int ldo, int a_rows)
{
    static_assert(!(GATED && OUT_F32), "the intermediate of the gated GEMM is always bf16");
    constexpr int BM = kW4Rows, BN = kW4BN, NW = kW4Waves, NSA = kW4NSA, NSB = kW4NSB, PBK = kW4K;
    constexpr int WN = NW;                      // the waves sit side by side along the weight rows
    constexpr int TM = BM / 32;                 // every wave multiplies all row blocks of the tile
    constexpr int NO = GATED ? BN / 2 : BN;     // output columns per block
    constexpr int WNO = NO / WN;                // output columns per wave
    constexpr int TNO = WNO / 32;
    constexpr int TN = GATED ? 2 * TNO : TNO;
    constexpr int A_ROWB = PBK * 2, A_SLOT = BM * A_ROWB;        // 128-byte activation rows, 8 KB per stage
    constexpr int B_ROWB = PBK, B_SLOT = BN * B_ROWB;            // 64 bytes of codes per weight row and DOUBLE stage
    constexpr int S_SLOT = BN * 4;                               // 4 scale bytes per weight row and double stage
    constexpr int SW_STAGES = 8, SW_SLOT = BN * 16;              // or, for rows of 16+ scale bytes: 16 per 8 stages
    constexpr int A_LPW = BM / 8 / NW;                           // activation loads per wave and stage (8 rows each)
    constexpr int B_LPW = BN / 16 / NW;                          // code loads per wave and double stage (16 rows each)
    constexpr int B_BASE = NSA * A_SLOT, S_BASE = B_BASE + NSB * B_SLOT;   // the scale area: max(NSB * S_SLOT, 2 * SW_SLOT)
    static_assert(A_LPW == 2 && B_LPW == 4 && TNO >= 1 && TM == 2, "tile configuration");
    static_assert((NSA - 1) * A_LPW + (NSB - 1) * (B_LPW + 1) + 2 <= 20, "wait_vmcnt_at_most covers up to 20 loads in flight");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const uint32_t ldsb = lds_address(smem);    // LDS byte address of the block's dynamic shared memory

    const int n_tiles = (N + NO - 1) / NO;
    const TileCoord tc = find_tile<BM>(offsets, E, n_tiles, a_rows);
    if (!tc.valid) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave-uniform: the load bookkeeping stays in scalar registers
    const int wn = wave;
    const int n0 = tc.n_tile * NO;
    const int nk = K / PBK;
    const int64_t row_bytes = K / 2, row_scales = K / 32;
    const uint8_t* We = W + (int64_t)tc.expert * rows_per_expert * row_bytes;
    const uint8_t* Se = S + (int64_t)tc.expert * rows_per_expert * row_scales;

    // ---- source addresses ----
    // activations: load p of this wave covers tile rows (wave + NW p) * 8 .. + 7, lane = (row, 16-byte chunk)
    const int a_lrow = lane >> 3, a_chunk = lane & 7;
    int32_t a_row_id[A_LPW];
#pragma unroll
    for (int p = 0; p < A_LPW; ++p) {
        int r = tc.row0 + (wave + NW * p) * 8 + a_lrow;
        if (r >= tc.row_end) r = tc.row_end - 1;
        int id = row_map ? row_map[r] : r;
        a_row_id[p] = id < 0 ? 0 : (id < a_rows ? id : a_rows - 1);      // a bad map entry must not become a wild address
    }
    // weights: the wave's load covers tile rows wave * 32 .. + 31, lane = (row, 16-byte MX block of the stage)
    auto weight_row = [&](int rb) {       // tile row -> row of the expert's weight matrix
        int n;
        if (GATED) n = (rb < NO) ? (n0 + rb) : (n0 + rb - NO);
        else n = n0 + rb;
        if (n >= N) n = N - 1;
        if (GATED && rb >= NO) n += N;
        return n;
    };
    // Code load p of this wave covers tile rows (wave + NW p) * 16 .. + 15, lane = (row, 16-byte MX block of
    // the double stage); LDS block slot c of tile row r holds block c ^ bswz(r), so that the 16-byte operand
    // reads of consecutive rows (64 bytes apart) spread over the banks.
    auto bswz = [](int r) { return (r >> 2) & 3; };
    const uint8_t* b_src[B_LPW];
    bool b_first_half[B_LPW];     // this lane's block lies in the first stage of the double stage
#pragma unroll
    for (int p = 0; p < B_LPW; ++p) {
        const int rb = (wave + NW * p) * 16 + (lane >> 2);
        const int blk = (lane & 3) ^ bswz(rb);
        b_src[p] = We + (int64_t)weight_row(rb) * row_bytes + blk * 16;
        b_first_half[p] = blk < 2;
    }
    // Scales: wave w covers tile rows 64 w .. 64 w + 63, one row per lane, the 4 scale bytes of a
    // double stage as one (2-byte-aligned) dword.  When K is an odd number of stages the last double stage
    // has only 2 scale bytes left in the row: the dword is then taken 2 bytes earlier (or, for K = 64, the
    // load is 2 bytes wide), so that nothing past the row is read.
    // Rows with at least 16 scale bytes (K >= 512) fetch them 16 at a time instead, one load per row and 8
    // stages, into a ring of two such chunks; a chunk that would run past the row starts 16 bytes before
    // the row's end.  (Every row costs a memory request however few bytes it asks for, and the scales
    // were half of the requests.)
    const bool wide_scales = row_scales >= 16;
    const int n_chunks = (nk + SW_STAGES - 1) / SW_STAGES;
    auto chunk_start = [&](int c) {      // first scale byte of chunk c within the row
        const int b = c * 16;
        return b + 16 <= (int)row_scales ? b : (int)row_scales - 16;
    };
    const uint8_t* s_src = Se + (int64_t)weight_row(wave * 64 + lane) * row_scales;
    const int n_double = (nk + 1) / 2;
    const bool odd_tail = (nk & 1) != 0;

    int issued = 0;                    // load instructions this wave has issued
    int last_b[NSB], last_a[NSA];      // `issued` right after the last load of the (double) stage in each ring slot
    auto issue_b = [&](int d) {        // double stage d = stages 2d and 2d + 1
        const uint32_t bs = ldsb + B_BASE + (d % NSB) * B_SLOT;
        const bool tail = odd_tail && d == n_double - 1;
#pragma unroll
        for (int p = 0; p < B_LPW; ++p)
            if (!tail || b_first_half[p]) load_lds<16>(b_src[p] + (int64_t)d * B_ROWB, bs + (wave + NW * p) * 1024);
        issued += B_LPW;     // (every wave has lanes on both sides of the tail mask, so both loads are always issued)
        if (!wide_scales) {
            const uint32_t dst = ldsb + S_BASE + (d % NSB) * S_SLOT + wave * 256;
            if (!tail) load_lds<4>(s_src + d * 4, dst);
            else if (row_scales >= 4) load_lds<4>(s_src + row_scales - 4, dst);
            else load_lds<2>(s_src, dst);
            issued += 1;
        }
#pragma unroll
        for (int i = 0; i < NSB; ++i)
            if (i == d % NSB) last_b[i] = issued;
    };
    int last_s[2] = {0, 0};
    auto issue_s = [&](int c) {        // wide scale chunk c = stages 8c .. 8c + 7
        load_lds<16>(s_src + chunk_start(c), ldsb + S_BASE + (c & 1) * SW_SLOT + wave * 1024);
        issued += 1;
        if (c & 1) last_s[1] = issued;
        else last_s[0] = issued;
    };
#pragma unroll
    for (int i = 0; i < NSB; ++i) last_b[i] = 0;
#pragma unroll
    for (int i = 0; i < NSA; ++i) last_a[i] = 0;
    // the weight stages of the prologue go in flight while the row-map lookups return
    if (wide_scales) issue_s(0);
#pragma unroll
    for (int d = 0; d < NSB - 1; ++d)
        if (d < n_double) issue_b(d);
    const bf16_t* a_src[A_LPW];
#pragma unroll
    for (int p = 0; p < A_LPW; ++p) {
        const int tr = (wave + NW * p) * 8 + a_lrow;
        const int64_t src = row_map ? (int64_t)(a_row_id[p] / map_div) : (int64_t)a_row_id[p];
        a_src[p] = row_ptr<bf16_t>(X, src, ldx) + ((a_chunk ^ swz<64>(tr)) << 3);
    }
    // A load whose 8 tile rows all lie past the tile's last row is left out (a decode batch puts a
    // handful of rows into a 64-row tile; with 4-bit weights the activation tile would otherwise be most
    // of the requests); within a load, lanes past the last row are masked.  The choice is uniform over
    // the wave and counted, so the wait counts stay exact.  LDS rows never loaded feed only accumulator
    // rows that are never stored.
    const int tile_rows = (tc.row_end - tc.row0) < BM ? (tc.row_end - tc.row0) : BM;
    auto issue_a = [&](int kt) {
#pragma unroll
        for (int p = 0; p < A_LPW; ++p) {
            if ((wave + NW * p) * 8 >= tile_rows) continue;
            if ((wave + NW * p) * 8 + a_lrow < tile_rows)
                load_lds<16>(a_src[p] + kt * PBK, ldsb + (kt % NSA) * A_SLOT + (wave + NW * p) * 1024);
            issued += 1;
        }
#pragma unroll
        for (int i = 0; i < NSA; ++i)
            if (i == kt % NSA) last_a[i] = issued;
    };
#pragma unroll
    for (int st = 0; st < NSA - 1; ++st)
        if (st < nk) issue_a(st);

    // ---- LDS offsets of the operand rows this lane feeds to the MFMAs ----
    const int fr = lane & 31, fq = lane >> 5;
    const int fsw = swz<64>(fr);
    const int a_off = fr * A_ROWB;                 // row block i: + i * 32 * A_ROWB
    int b_off[TN], s_row[TN], b_sw[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int r;
        if (GATED) r = (j < TNO) ? (wn * WNO + j * 32 + fr) : (NO + wn * WNO + (j - TNO) * 32 + fr);
        else r = wn * WNO + j * 32 + fr;
        b_off[j] = r * B_ROWB;          // + the block's slot, which depends on the stage's half
        b_sw[j] = bswz(r);
        s_row[j] = r;
    }
    const bool two_blocks = tile_rows > 32;        // the tile's second 32-row block holds rows

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    for (int g = 0; g < nk; ++g) {
        const int d = g >> 1, half = g & 1;
        // stage g has landed when at most the loads issued after its last one are still in flight
        int need = 0;
#pragma unroll
        for (int i = 0; i < NSA; ++i)
            if (i == g % NSA) need = last_a[i];
#pragma unroll
        for (int i = 0; i < NSB; ++i)
            if (i == d % NSB && last_b[i] > need) need = last_b[i];
        const int sc_chunk = g / SW_STAGES;
        if (wide_scales && last_s[sc_chunk & 1] > need) need = last_s[sc_chunk & 1];
        wait_vmcnt_at_most(issued - need);
        block_barrier();       // every wave's part of stage g is in LDS; every wave is done reading stage g-1
        if (g + NSA - 1 < nk) issue_a(g + NSA - 1);                            // into the slot stage g-1 used
        if (half == 0 && d + NSB - 1 < n_double) issue_b(d + NSB - 1);         // into the slot double stage d-1 used
        if (wide_scales && g % SW_STAGES == 0 && sc_chunk + 1 < n_chunks) issue_s(sc_chunk + 1);   // slot of chunk c-1
        {
            const char* a_base = smem + (g % NSA) * A_SLOT + a_off;
            const char* bs_base = smem + B_BASE + (d % NSB) * B_SLOT;
            // where this stage's two scale bytes of a row sit: in the 16-byte chunk, or in the double stage's
            // dword (a clamped tail dword holds them in its upper half)
            const char* ss_base = wide_scales ? smem + S_BASE + (sc_chunk & 1) * SW_SLOT + (2 * g - chunk_start(sc_chunk))
                                              : smem + S_BASE + (d % NSB) * S_SLOT +
                                                    ((odd_tail && d == n_double - 1 && row_scales >= 4) ? 2 : half * 2);
            const int s_mul = wide_scales ? 4 : 1;     // rows are 16 bytes apart in a chunk, 4 in a dword slot
            bf16x8_t af[TM][4];
            u32x4_t bq[TN];
            float sc[TN];
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                af[0][j4] = *reinterpret_cast<const bf16x8_t*>(a_base + (((fq * 4 + j4) ^ fsw) << 4));
                if (two_blocks)
                    af[1][j4] = *reinterpret_cast<const bf16x8_t*>(a_base + 32 * A_ROWB + (((fq * 4 + j4) ^ fsw) << 4));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                bq[j] = *reinterpret_cast<const u32x4_t*>(bs_base + b_off[j] + (((half * 2 + fq) ^ b_sw[j]) << 4));
                sc[j] = e8m0_to_float(*reinterpret_cast<const uint8_t*>(ss_base + s_row[j] * 4 * s_mul + fq));
            }
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    // weight rows as the MFMA's row operand: a lane ends up with 4 consecutive output columns
                    const bf16x8_t wv = widen_fp4x8(bq[j][j4], sc[j]);
                    acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, af[0][j4], acc[0][j], 0, 0, 0);
                    if (two_blocks) acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, af[1][j4], acc[1][j], 0, 0, 0);
                }
            wait_lds_reads();   // this wave's reads of stage g have returned before it reaches the next barrier
        }
    }

    // accumulator element v of tile (i, j): output row 32 i + fr, column (v/4)*8 + fq*4 + v%4
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i == 1 && !two_blocks) break;
        const int64_t row = (int64_t)tc.row0 + i * 32 + fr;
#pragma unroll
        for (int j = 0; j < TNO; ++j) {
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int col = n0 + wn * WNO + j * 32 + a * 8 + fq * 4;
                float val[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (GATED) val[b] = silu_mul(acc[i][j][a * 4 + b], acc[i][j + TNO][a * 4 + b]);
                    else val[b] = acc[i][j][a * 4 + b];
                }
                if (row < tc.row_end && col < N) {  // N is a multiple of 8: the 4 columns are in or out together
                    if (OUT_F32)
                        *reinterpret_cast<float4*>(static_cast<float*>(Out_) + row * ldo + col) =
                            make_float4(val[0], val[1], val[2], val[3]);
                    else
                        *reinterpret_cast<uint2*>(static_cast<bf16_t*>(Out_) + row * ldo + col) =
                            make_uint2(pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3]));
                }
            }
        }
    }
}

// ----------------------------------------------------------------------------------------------
// The weight-streaming shape for decode-heavy batches (on average at most 96 rows per expert).
//
// With 4-bit weights a 64-value stage is 32 bytes of a weight row: fetched stage by stage (or two
// stages at a time) every 128-byte line of the weights is requested several times, a few stages
// apart, and a row whose start is not line-aligned (1440-byte rows: every row but one in four)
// straddles lines on top of that.  Measured on 128 experts x 5760 x 2880: 1.5x the weight bytes
// cross the fabric and the kernel stays at 0.37 of the HBM peak.  Here every weight row is fetched
// in whole, ALIGNED 128-byte lines: line L of a row holds the row's bytes [128 L - phase, 128 L -
// phase + 128), phase = (row address) mod 128, a multiple of 32, so a stage's 32 bytes never cross a
// line and stage s of a row of class c = phase / 32 lies in line (c + s) / 4 at 32-byte slot
// (c + s) % 4.  A row keeps two lines in LDS; when it moves on to line L - 1 (top of stage
// 4 (L - 1) - c) the line slot it has just left takes line L, four stages ahead of its first use.
// Rows of different classes turn over at different stages, so in the common case (row bytes an odd
// multiple of 32) a quarter of the rows fetches a line at every stage and the traffic is even.
//
// 32 x 256 tiles, 8 waves, each with its own 32 weight rows: a wave fetches the lines of its own
// rows, so only the activation tile is shared between waves.  The per-stage work of a wave is small
// (4 MFMAs behind 16 conversions) and the stage is a chain of dependent waits, so the kernel lives on
// the number of waves per SIMD (4) and on the length of that chain: every instruction on it costs.
// The load schedule is therefore fixed, with nothing to keep count of.  Every stage issues the same
// loads: [the activations of stage g + 3,] then line ((c + g) / 4) + 1 of the rows whose class c has
// (c + g) % 4 = 0; the start-up issues what stages -3, -2, -1 would have.  Past a row's end the rule
// fetches the row's last line once more (into the line slot the row has left for good), past the
// last stage the activation load repeats the last stage into a free slot: harmless and served by
// the caches, and the loads in flight at the top of a stage are always the same, so the wait count
// is a constant (row bytes an odd multiple of 32: one line load per stage) or one of four (else).
// Loads return in order, so the wait for the activations of stage g also covers every line issued
// before them: the activation ring (4 stages) runs as far ahead as the lines do.  The scale bytes
// never touch LDS: a lane needs one byte per stage for its weight row and holds them in registers
// (128 bytes of the row at a time).  For the gated GEMM waves 0-3 hold the gate rows and waves 4-7
// the matching up rows; the up accumulators cross through LDS once, after the last stage.  80 KB of
// LDS, two blocks per compute unit.
// ----------------------------------------------------------------------------------------------
constexpr int kS4Rows = 32, kS4NSA = 4, kS4Waves = 8;

// 16 bytes into registers without a compiler-inserted wait: the value may be used only after an explicit
// wait that covers the load, followed by settle().
__device__ __forceinline__ u32x4_t load_u32x4_async(const uint8_t* p)
{
    u32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
    return v;
}
__device__ __forceinline__ void settle(u32x4_t& v) { asm volatile("" : "+v"(v)::"memory"); }

// ODD: the row bytes are an odd multiple of 32 (the four line loads of a wave have the four classes).
// (second launch bound: waves per SIMD; two blocks of 8 waves per compute unit = 4)
template <bool GATED, bool ODD, bool OUT_F32>
__global__ __launch_bounds__(kS4Waves * 64, 4) void grouped_gemm_w4_stream_kernel(
    RowSrc X, int ldx, const int32_t* __restrict__ row_map, int map_div, const int32_t* __restrict__ offsets, int E,
    const uint8_t* __restrict__ W, const uint8_t* __restrict__ S, int64_t rows_per_expert, int N, int K,
    void* __restrict__ Out_, int ldo, int a_rows)
{
    static_assert(!(GATED && OUT_F32), "the intermediate of the gated GEMM is always bf16");
    constexpr int BM = kS4Rows, BN = kW4BN, NW = kS4Waves, NSA = kS4NSA, PBK = kW4K;
    constexpr int NO = GATED ? BN / 2 : BN;     // output columns per block
    constexpr int A_ROWB = PBK * 2, A_SLOT = BM * A_ROWB;        // 128-byte activation rows, 4 KB per stage
    constexpr int B_SLOT = BN * 128;                             // one 128-byte line of every weight row
    constexpr int B_BASE = NSA * A_SLOT;
    constexpr int B_LPW = BN / 8 / NW;                           // line loads per wave to cover its rows once (8 rows each)
    static_assert(BM == 32 && BN == 32 * NW && B_LPW == 4 && NSA == 4, "tile configuration");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const uint32_t ldsb = lds_address(smem);    // LDS byte address of the block's dynamic shared memory

    const int n_tiles = (N + NO - 1) / NO;
    const TileCoord tc = find_tile<BM>(offsets, E, n_tiles, a_rows);
    if (!tc.valid) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave-uniform: what depends on it stays in scalar registers
    const int n0 = tc.n_tile * NO;
    const int nk = K / PBK;
    const int64_t row_bytes = K / 2, row_scales = K / 32;
    const uint8_t* We = W + (int64_t)tc.expert * rows_per_expert * row_bytes;
    const uint8_t* Se = S + (int64_t)tc.expert * rows_per_expert * row_scales;
    const uint8_t* W_last = W + (int64_t)E * rows_per_expert * row_bytes - 16;     // last 16 bytes of the codes
    const uint8_t* S_end = S + (int64_t)E * rows_per_expert * row_scales;

    // activations: waves 0..3 fetch tile rows wave * 8 .. + 7, lane = (row, 16-byte chunk)
    const int a_lrow = lane >> 3, a_chunk = lane & 7;
    const int tile_rows = tc.row_end - tc.row0;     // 1 .. 32
    const bool a_loader = wave * 8 < tile_rows;     // (false for waves 4..7); a load whose rows all lie past the tile's last row is left out
    int32_t a_row_id, a_own;
    {
        int r = tc.row0 + wave * 8 + a_lrow;
        if (r >= tc.row_end) r = tc.row_end - 1;
        a_own = r;
        // fetched without a compiler-tracked wait: the weight loads below go out while it is in flight, and
        // the explicit wait in front of its first use leaves exactly those outstanding.  The load is issued
        // in every case (without a row map it reads a valid dummy word, offsets[0], and the result is
        // ignored): a conditional load would be an asm output merged with an earlier value, i.e. a register
        // copy that the compiler may place behind the load.
        const int32_t* src = row_map ? row_map + r : offsets;
        asm volatile("global_load_dword %0, %1, off" : "=v"(a_row_id) : "v"(src) : "memory");
    }

    // Tile row t -> row of the expert's weight matrix.  A row past the matrix (ragged last n-tile) is
    // replaced by the last real row with the same index mod 4, which has the same line phase; what it
    // produces is never stored.
    auto weight_row = [&](int t) {
        const bool up = GATED && t >= NO;
        int n = n0 + (up ? t - NO : t);
        if (n >= N) n -= ((n - N) / 4 + 1) * 4;
        return up ? n + N : n;
    };
    // Line loads: load k of this wave covers its 8 rows 32 wave + 4 i + q_k, i = lane / 8: rows 4 apart start
    // a multiple of 128 bytes apart, so they share a class.  When the row bytes are an odd multiple of 32
    // the four residues q have four different classes and q_k is the residue of class k (load k has class
    // k, known at compile time); otherwise q_k = k.  The instruction's 8 lines are LDS rows 8 (4 wave +
    // k) .. + 7; LDS chunk x of a row holds the line's chunk x ^ sw(row), sw chosen so that 16 lanes
    // reading the chunks of their stage (which differ between classes) fall into 16 different bank
    // groups.
    const int rb32 = (int)(row_bytes >> 5) & 3;
    const int c0 = __builtin_amdgcn_readfirstlane(
        (int)((uintptr_t)(We + (int64_t)weight_row(32 * wave) * row_bytes) >> 5) & 3);     // class of residue 0
    auto line_sw = [&](int t) {
        const int i = (t >> 2) & 7, q = t & 3;
        const int xq = ODD ? 0 : (rb32 == 2 ? (q >> 1) : q);
        return ((i >> 1) & 1) | (xq << 1);
    };
    const uint8_t* b_src[B_LPW];       // this lane's 16 bytes of line 0
    int cls[B_LPW], lmax[B_LPW];       // the load's class (wave-uniform; = k when ODD) and its rows' last line
    bool clamp_any = false;            // some address this wave will ask for lies outside W (wave-uniform)
#pragma unroll
    for (int k = 0; k < B_LPW; ++k) {
        const int q = ODD ? ((k - c0) * rb32) & 3 : k;     // rb32 is its own inverse mod 4
        const int t = 32 * wave + 4 * (lane >> 3) + q;
        const uint8_t* row = We + (int64_t)weight_row(t) * row_bytes;
        const int phase = (int)((uintptr_t)row & 127);
        b_src[k] = row - phase + (((lane & 7) ^ line_sw(t)) << 4);
        cls[k] = ODD ? k : __builtin_amdgcn_readfirstlane(phase >> 5);
        lmax[k] = (cls[k] + nk - 1) >> 2;
        // the first line may begin in front of W, the last one may end behind it
        clamp_any = clamp_any || __ballot(b_src[k] < W || b_src[k] + (int64_t)lmax[k] * 128 > W_last) != 0;
    }
    // ODD: the four loads of a lane differ by the same amount in every lane ((q_k - q_0) rows and the
    // difference of the two line phases: the stand-in rows of a ragged tile keep their distance as well),
    // so one address and three scalar offsets do, which frees six registers.
    const uint8_t* b_lane = b_src[0];
    int k_off[B_LPW];
#pragma unroll
    for (int k = 0; k < B_LPW; ++k) k_off[k] = ODD ? __builtin_amdgcn_readfirstlane((int)(b_src[k] - b_src[0])) : 0;
    auto line_addr = [&](int k, int L) {
        return ODD ? b_lane + (k_off[k] + L * 128) : b_src[k] + (int64_t)L * 128;
    };
    // this lane's operand row: tile row 32 wave + fr, k-half fq of every stage
    const int fr = lane & 31, fq = lane >> 5;
    const int t_own = 32 * wave + fr;
    const int wr_own = weight_row(t_own);
    const int k_own = ODD ? (c0 + rb32 * (fr & 3)) & 3 : (fr & 3);     // the load that fetches this row
    const int b_off = ((wave * 4 + k_own) * 8 + (fr >> 2)) * 128;
    const int b_sw = line_sw(t_own);
    const int b_cls = ODD ? k_own : (int)((uintptr_t)(We + (int64_t)wr_own * row_bytes) >> 5) & 3;
    const uint8_t* s_src = Se + (int64_t)wr_own * row_scales;     // both k-halves of a row fetch the same scale bytes
    // A row's scale bytes are fetched 128 at a time (64 stages; the whole row when K <= 4096) as up to 8
    // 16-byte pieces: neighbouring rows then touch the lines they share at the same moment, whereas
    // piecemeal fetches of 16 bytes every 8 stages brought each line in several times.  A lane keeps the 8
    // bytes of a piece that belong to its k-half (byte u of them is the scale of stage 8 piece + u).
    const int s_row_pieces = (int)((row_scales + 15) / 16);     // 16-byte pieces that hold bytes of the row
    int s_over = 0;                    // bytes by which the row's LAST piece would pass the end of S: it is fetched that much earlier
    {
        const int over = (int)(s_src + (int64_t)s_row_pieces * 16 - S_end);
        s_over = over > 0 ? over : 0;
    }
    uint32_t s_lo[8], s_hi[8], s_cur_lo = 0, s_cur_hi = 0;
    auto fetch_piece = [&](int piece) {
        return load_u32x4_async(s_src + piece * 16 - (piece == s_row_pieces - 1 ? s_over : 0));
    };
    auto keep_piece = [&](u32x4_t v, int piece, uint32_t& lo_out, uint32_t& hi_out) {
        settle(v);
        if (piece == s_row_pieces - 1 && s_over > 0) {      // the row's last piece started s_over bytes early
            uint64_t lo = (uint64_t)v[0] | ((uint64_t)v[1] << 32);
            uint64_t hi = (uint64_t)v[2] | ((uint64_t)v[3] << 32);
            const int sh = s_over * 8;
            if (sh >= 64) {
                lo = hi >> (sh - 64);
                hi = 0;
            } else {
                lo = (lo >> sh) | (hi << (64 - sh));
                hi >>= sh;
            }
            v = u32x4_t{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
        }
        const uint32_t sel = fq ? 0x07050301u : 0x06040200u;      // bytes fq, fq + 2, fq + 4, fq + 6 of a dword pair
        lo_out = __builtin_amdgcn_perm(v[1], v[0], sel);
        hi_out = __builtin_amdgcn_perm(v[3], v[2], sel);
    };

    // ---- the fixed load schedule ----
    const bf16_t* a_src = nullptr;
    // the loads of (pseudo-)stage g, g >= -3: activations of stage g + 3 into the slot stage g - 1 used, then
    // the lines that come due
    auto issue_stage = [&](int g, int a_slot) {
        if (a_loader) {
            const int kt = g + NSA - 1 < nk ? g + NSA - 1 : nk - 1;
            if (wave * 8 + a_lrow < tile_rows)
                load_lds<16>(a_src + kt * PBK, ldsb + a_slot * A_SLOT + wave * 1024);
        }
#pragma unroll
        for (int k = 0; k < B_LPW; ++k) {
            if (ODD ? ((k + g) & 3) != 0 : ((cls[k] + g) & 3) != 0) continue;
            const int L = ((cls[k] + g) >> 2) + 1;
            // past the row's last line the load repeats that line (it has just been fetched: no memory
            // traffic), still into the slot the rule names, which the row has left for good
            const int Lsrc = L < lmax[k] ? L : lmax[k];
            const uint8_t* a = line_addr(k, Lsrc);
            if (clamp_any) {      // only the wave that holds the last rows of W: a branch, not a select on every load
                asm volatile("");
                a = a > W_last ? W_last : a;
            }
            load_lds<16>(a, ldsb + B_BASE + (L & 1) * B_SLOT + (wave * B_LPW + k) * 1024);
        }
    };
    // Loads in flight at the top of stage g that stage g does not need: the lines of stages g-3, g-2, g-1
    // and the activations of stages g-2, g-1.
    int lines_at[4];                   // line loads of a stage = r (mod 4)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        lines_at[r] = 0;
#pragma unroll
        for (int k = 0; k < B_LPW; ++k) lines_at[r] += ((cls[k] + r) & 3) == 0;
    }
    auto wait_for_stage = [&](int r) {     // r = g mod 4, a compile-time constant where it is called
        if (ODD) {
            // 3 line loads may be in flight for every wave; a wave that fetches activations could leave its
            // last 2 activation loads in flight as well (5), but the stricter count costs nothing (the
            // lines run four stages ahead, and three would do) and saves a branch in every stage
            wait_vmcnt<3>();
        } else {
            const int n = lines_at[(r + 1) & 3] + lines_at[(r + 2) & 3] + lines_at[(r + 3) & 3] + (a_loader ? 2 : 0);
            wait_vmcnt_at_most(n);
        }
    };

    // ---- start-up: scale bytes, line 0 of every row, then what stages -3, -2, -1 would issue ----
    // the first 8 pieces, until the row-map lookup below has returned (a row with fewer pieces fetches its
    // last one again: with conditional loads the compiler treats the eight values as one 32-register tuple
    // and copies it around)
    u32x4_t s_raw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s_raw[i] = fetch_piece(i < s_row_pieces ? i : s_row_pieces - 1);
#pragma unroll
    for (int k = 0; k < B_LPW; ++k) {
        const uint8_t* a = line_addr(k, 0);
        if (clamp_any) {
            a = a < W ? W : a;
            a = a > W_last ? W_last : a;
        }
        load_lds<16>(a, ldsb + B_BASE + (wave * B_LPW + k) * 1024);
    }
    {
        // the row-map load and the scale pieces came before the 4 line loads: wait for them, cut the pieces
        // down to this lane's bytes
        wait_vmcnt<B_LPW>();
        asm volatile("" : "+v"(a_row_id)::"memory");
        {      // a row map holds indices below a_rows; the clamp keeps a bad entry from becoming a wild address
            int32_t id = a_row_id < 0 ? 0 : a_row_id;
            id = id < a_rows ? id : a_rows - 1;
            a_row_id = row_map ? id : a_own;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) keep_piece(s_raw[i], i < s_row_pieces ? i : s_row_pieces - 1, s_lo[i], s_hi[i]);
        const int tr = wave * 8 + a_lrow;
        const int64_t src = row_map ? (int64_t)(a_row_id / map_div) : (int64_t)a_row_id;
        a_src = row_ptr<bf16_t>(X, src, ldx) + ((a_chunk ^ swz<64>(tr)) << 3);
    }
    issue_stage(-3, 0);
    issue_stage(-2, 1);
    issue_stage(-1, 2);

    // activation fragment j4 of this lane's token row: LDS offset inside a stage's slot (the slot's own
    // offset is a constant of the unrolled step and goes into the instruction)
    // (LDS addresses as integers in the LDS address space: the compiler then folds the slot into the
    // instruction's offset field instead of adding the array's base at every read)
    typedef __attribute__((address_space(3))) const bf16x8_t lds_bf16x8_t;
    typedef __attribute__((address_space(3))) const u32x4_t lds_u32x4_t;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t*)smem;
    uint32_t a_rd[4];
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4) a_rd[j4] = lds0 + fr * A_ROWB + (((fq * 4 + j4) ^ swz<64>(fr)) << 4);
    const uint32_t b_rd = lds0 + B_BASE + b_off;
    const uint32_t b_rd_odd = b_rd + ((fq ^ (b_sw & 1)) << 4);
    // token columns past the tile's rows are never stored: their lanes skip the activation reads (with a
    // handful of rows per expert most of the LDS read traffic would be for nothing; reading them anyway
    // measured 3 % slower)
    const bool a_reader = fr < ((tile_rows + 7) & ~7);

    float16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    bf16x8_t af[4];
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4)
#pragma unroll
        for (int v = 0; v < 8; ++v) af[j4][v] = (__bf16)0.f;

    for (int g0 = 0; g0 < nk; g0 += 8) {
        const int chunk = g0 >> 3;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int g = g0 + u;
            if (g >= nk) break;
            wait_for_stage(u & 3);
            block_barrier();       // every wave's part of stage g is in LDS; every wave is done reading stage g-1
            if (u == 0) {          // the scale bytes of stages g0 .. g0 + 7: piece g0 / 8 of the row
                if (chunk > 0 && (chunk & 7) == 0) {
                    // K > 4096: the next 128 scale bytes, two pieces at a time, each pair awaited on the spot
                    // (once per 64 stages; everything issued earlier lands as well, which the fixed wait
                    // counts of the next stages allow for)
#pragma unroll
                    for (int i = 0; i < 8; i += 2) {
                        const int last = s_row_pieces - 1;
                        const int p0 = chunk + i < last ? chunk + i : last;
                        const int p1 = chunk + i + 1 < last ? chunk + i + 1 : last;
                        u32x4_t t0 = fetch_piece(p0), t1 = fetch_piece(p1);
                        wait_vmcnt<0>();
                        keep_piece(t0, p0, s_lo[i], s_hi[i]);
                        keep_piece(t1, p1, s_lo[i + 1], s_hi[i + 1]);
                    }
                }
                switch (chunk & 7) {
                    case 0: s_cur_lo = s_lo[0]; s_cur_hi = s_hi[0]; break;
                    case 1: s_cur_lo = s_lo[1]; s_cur_hi = s_hi[1]; break;
                    case 2: s_cur_lo = s_lo[2]; s_cur_hi = s_hi[2]; break;
                    case 3: s_cur_lo = s_lo[3]; s_cur_hi = s_hi[3]; break;
                    case 4: s_cur_lo = s_lo[4]; s_cur_hi = s_hi[4]; break;
                    case 5: s_cur_lo = s_lo[5]; s_cur_hi = s_hi[5]; break;
                    case 6: s_cur_lo = s_lo[6]; s_cur_hi = s_hi[6]; break;
                    default: s_cur_lo = s_lo[7]; s_cur_hi = s_hi[7]; break;
                }
            }
            // the operand reads go out first (the weight piece before the activation fragments: the conversions
            // start from it), the loads of this stage are issued while they return
            // stage g of this lane's row: 32-byte piece (b_cls + g) % 4 of the line in slot ((b_cls + g) / 4) % 2
            uint32_t b_addr;
            if (ODD) {      // (the swizzle only touches the 16-byte half: folded into b_rd_odd; one multiply puts
                            // the piece at bits 5-6 and the slot at bit 15)
                static_assert(B_SLOT == 1 << 15, "the slot bit");
                b_addr = b_rd_odd + ((((uint32_t)(b_cls + u) & 7u) * 0x2020u) & 0x8060u);
            } else {
                const int tt = b_cls + g;
                const int y = ((tt & 3) << 1) | fq;
                b_addr = b_rd + ((tt >> 2) & 1) * B_SLOT + ((y ^ b_sw) << 4);
            }
            const u32x4_t bq = *(lds_u32x4_t*)(uintptr_t)b_addr;
            if (a_reader) {
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4)
                    af[j4] = *(lds_bf16x8_t*)(uintptr_t)(a_rd[j4] + (u & 3) * A_SLOT);
            }
            issue_stage(g, (u + NSA - 1) & 3);
            const uint32_t s_word = (u & 4) ? s_cur_hi : s_cur_lo;
            const float sc = (u & 3) == 0   ? e8m0_byte_to_float<0>(s_word)
                             : (u & 3) == 1 ? e8m0_byte_to_float<8>(s_word)
                             : (u & 3) == 2 ? e8m0_byte_to_float<16>(s_word)
                                            : e8m0_byte_to_float<24>(s_word);
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                // weight rows as the MFMA's row operand: a lane ends up with 4 consecutive output columns
                bf16x8_t wv = widen_fp4x8(bq[j4], sc);
                // This wave's reads of stage g must have returned before it reaches the next barrier.  The wait
                // hangs on the last widened operand: placed after the loop it would have no data dependence
                // on the conversions and the scheduler would hoist it above them, so that they waited for
                // the activation fragments as well as for the weight piece they need.
                if (j4 == 3) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wv)::"memory");
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, af[j4], acc, 0, 0, 0);
            }
        }
    }
    // The line and activation loads of the last stages are still in flight; nothing reads them, but the
    // accumulator exchange below writes LDS, and a block must not end with loads into LDS outstanding.
    wait_vmcnt<0>();

    // accumulator element v: output row fr, column (v/4)*8 + fq*4 + v%4 of the wave's 32 columns
    if (GATED) {
        // The up waves hand their accumulators to the gate waves through their own weight rows in LDS (no
        // other wave reads those, and every line fetched into them has been used): 4 KB per wave, quad a of
        // lane l at a * 1024 + l * 16.
        char* xch = smem + B_BASE + wave * 4 * 1024;
        if (wave >= 4) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<float4*>(xch + a * 1024 + lane * 16) =
                    make_float4(acc[a * 4], acc[a * 4 + 1], acc[a * 4 + 2], acc[a * 4 + 3]);
            wait_lds_reads();
        }
        block_barrier();
        if (wave >= 4) return;
    }
    const int64_t row = (int64_t)tc.row0 + fr;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int col = n0 + (wave & (GATED ? 3 : 7)) * 32 + a * 8 + fq * 4;
        float val[4];
        if (GATED) {
            const float4 up = *reinterpret_cast<const float4*>(smem + B_BASE + (wave + 4) * 4 * 1024 + a * 1024 + lane * 16);
            val[0] = silu_mul(acc[a * 4 + 0], up.x);
            val[1] = silu_mul(acc[a * 4 + 1], up.y);
            val[2] = silu_mul(acc[a * 4 + 2], up.z);
            val[3] = silu_mul(acc[a * 4 + 3], up.w);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b) val[b] = acc[a * 4 + b];
        }
        if (row < tc.row_end && col < N) {  // N is a multiple of 8: the 4 columns are in or out together
            if (OUT_F32)
                *reinterpret_cast<float4*>(static_cast<float*>(Out_) + row * ldo + col) =
                    make_float4(val[0], val[1], val[2], val[3]);
            else
                *reinterpret_cast<uint2*>(static_cast<bf16_t*>(Out_) + row * ldo + col) =
                    make_uint2(pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3]));
        }
    }
}

// Which kernel shape a launch uses: the streaming shape up to 96 rows per expert on average.  Its
// 32-row tiles re-read (from L2) and re-widen the weights once per 32 rows, which a prefill-heavy batch
// pays for: measured on 32 experts x 5760 x 2880 the two shapes are level at 40 rows per expert, the
// streaming shape 3 % ahead at 72, 5 % behind at 136 and 13 % behind at 264.
bool w4_use_stream(int variant, int64_t A, int E)
{
    if (variant == MOE_FFN_W4_TILE64) return false;
    if (variant == MOE_FFN_W4_STREAM) return true;
    return A <= (int64_t)96 * E;
}

template <bool GATED, bool OUT_F32>
hipError_t launch_w4(int variant, RowSrc X, int ldx, const int32_t* row_map, int map_div, const int32_t* offsets, int E,
                     int64_t A, const uint8_t* W, const uint8_t* S, int64_t rows_per_expert, int N, int K, void* Out,
                     int ldo, hipStream_t s)
{
    constexpr int NO = GATED ? kW4BN / 2 : kW4BN;
    // the streaming kernel takes a row's address mod 128 for a multiple of 32 (the callers check it)
    if ((reinterpret_cast<uintptr_t>(W) & 31u) != 0) return hipErrorInvalidValue;
    const bool stream = w4_use_stream(variant, A, E);
    const int tile_rows = stream ? kS4Rows : kW4Rows;
    const size_t lds_bytes = stream ? (size_t)kS4NSA * kS4Rows * kW4K * 2 + (size_t)2 * kW4BN * 128
                                    : (size_t)kW4NSA * kW4Rows * kW4K * 2 + (size_t)kW4NSB * kW4BN * kW4K +
                                          2 * kW4BN * 16;   // scale area: max(3 dword slots, 2 chunk slots)
    const bool odd = ((K / 2) >> 5) & 1;     // row bytes an odd multiple of 32
    auto kern = stream ? (odd ? grouped_gemm_w4_stream_kernel<GATED, true, OUT_F32>
                              : grouped_gemm_w4_stream_kernel<GATED, false, OUT_F32>)
                       : grouped_gemm_w4_kernel<GATED, OUT_F32>;
    static bool attr_set[3][kMaxDevices] = {};
    const int which = stream ? (odd ? 2 : 1) : 0;
    hipError_t e = ensure_lds_limit(kern, lds_bytes, attr_set[which]);
    if (e != hipSuccess) return e;
    const int64_t n_tiles = (N + NO - 1) / NO;
    const int64_t m_tiles_max = (A + tile_rows - 1) / tile_rows + (A < E ? A : E);
    const int64_t grid = ((m_tiles_max * n_tiles + 7) / 8) * 8;
    if (grid >= ((int64_t)1 << 31)) return hipErrorInvalidValue;   // the device-side tile search counts in 32 bits
    kern<<<(unsigned)grid, (stream ? kS4Waves : kW4Waves) * 64, lds_bytes, s>>>(X, ldx, row_map, map_div, offsets, E, W, S, rows_per_expert, N, K,
                                                          Out, ldo, (int)A);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_gate_up_w4(int variant, RowSrc x, const int32_t* row_map, int map_div, const int32_t* offsets,
                                 int64_t A, int E, int H, int I, const uint8_t* w_gate_up, const uint8_t* s_gate_up,
                                 void* act, hipStream_t s)
{
    return launch_w4<true, false>(variant, x, H, row_map, map_div, offsets, E, A, w_gate_up, s_gate_up, (int64_t)2 * I, I,
                                  H, act, I, s);
}

hipError_t launch_ffn_down_w4(int variant, bool out_f32, const void* act, const int32_t* offsets, int64_t A, int E, int H,
                              int I, const uint8_t* w_down, const uint8_t* s_down, void* y_perm, hipStream_t s)
{
    if (out_f32)
        return launch_w4<false, true>(variant, single_src(act), I, nullptr, 1, offsets, E, A, w_down, s_down, (int64_t)H, H,
                                      I, y_perm, H, s);
    return launch_w4<false, false>(variant, single_src(act), I, nullptr, 1, offsets, E, A, w_down, s_down, (int64_t)H, H, I,
                                   y_perm, H, s);
}

const char* ffn_w4_variant_name(int variant, int64_t A, int E)
{
    return w4_use_stream(variant, A, E) ? "grouped_gemm_w4_stream_kernel<gated>" : "grouped_gemm_w4_kernel<gated>";
}

}  // namespace moe
