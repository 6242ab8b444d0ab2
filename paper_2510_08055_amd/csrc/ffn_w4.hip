// Grouped expert FFN with 4-bit expert weights (MXFP4) and bf16 activations.
//
// The paper's broader validation (Table 7) runs a model whose expert weights are fp4; what changes for
// the MoE layer is the bytes per expert, hence where the ridge of Sec. 2.5 lies: a decode-heavy batch
// streams 17/32 of a byte per weight instead of 2.  The format is the published OCP Microscaling MXFP4:
// FP4 E2M1 elements, two per byte (even element in the low nibble), one E8M0 scale byte (2^(s-127)) per
// 32 consecutive elements along k.  A dequantised weight is exactly representable in bf16, so the GEMM
// is the bf16 MFMA GEMM of ffn.hip on weights widened on the fly (v_cvt_scalef32_pk_bf16_fp4).
//
// One kernel shape, the weight-streaming one: 64-row x 256-weight-row tiles, 4 waves side by side along
// the weight rows (each widens and multiplies its own 64 weight rows against the tile's one or two
// 32-row blocks: widening the weights is the ALU work of a decode batch, so it is spread over all four
// SIMDs), 64 k-values per stage; activation rows come through a 2-stage LDS ring as in ffn.hip.  The packed weight
// rows and their scale bytes are fetched for TWO stages at a time (64 bytes of codes and 4 scale bytes
// per row) into a ring of 3 such double stages: the layer is bound by the number of memory requests,
// not their bytes, when every row contributes 32 + 2 bytes per stage (measured: 2.7x slower).  72 KB of
// LDS: two blocks share a compute unit.
// Within a 64-wide stage lane (row, q) feeds k-block q (32 values) to four successive MFMAs, 8 values
// each; the activation fragments follow the same k assignment.  Any fixed assignment is a valid
// summation order; this kernel is the only 4-bit variant, so every schedule sees the same one.
#include "ffn_tile.h"

namespace moe {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int kW4Rows = 64, kW4BN = 256, kW4Waves = 4, kW4K = 64;
constexpr int kW4NSA = 2, kW4NSB = 3;     // activation stages; weight DOUBLE stages (two stages each)

// Loads that may still be in flight while the wave goes on: the pipeline keeps count of the load
// instructions it has issued and of the last one each stage needs, so the wait is exact in the start-up
// and drain steps as well.  s_waitcnt takes an immediate: the count is rounded down to an even number.
__device__ __forceinline__ void wait_vmcnt_at_most(int n)
{
    if (n >= 20) wait_vmcnt<20>();
    else if (n >= 18) wait_vmcnt<18>();
    else if (n >= 16) wait_vmcnt<16>();
    else if (n >= 14) wait_vmcnt<14>();
    else if (n >= 12) wait_vmcnt<12>();
    else if (n >= 10) wait_vmcnt<10>();
    else if (n >= 8) wait_vmcnt<8>();
    else if (n >= 6) wait_vmcnt<6>();
    else if (n >= 4) wait_vmcnt<4>();
    else if (n >= 2) wait_vmcnt<2>();
    else wait_vmcnt<0>();
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

//   Out[r, n] = sum_k X[src(r), k] * W[e, n, k]                                        (GATED = false)
//   Out[r, n] = silu(sum_k X.. * W[e, n, k]) * (sum_k X.. * W[e, N + n, k])            (GATED = true)
// W: packed codes [E][rows][K/2] bytes, S: scales [E][rows][K/32] bytes; rows = N (or 2N when GATED).
// Requires K % 64 == 0.
template <bool GATED>
__global__ __launch_bounds__(kW4Waves * 64, 2) void grouped_gemm_w4_kernel(
    RowSrc X, int ldx, const int32_t* __restrict__ row_map, int map_div, const int32_t* __restrict__ offsets, int E,
    const uint8_t* __restrict__ W, const uint8_t* __restrict__ S, int64_t rows_per_expert, int N, int K,
    bf16_t* __restrict__ Out, int ldo)
{
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

    const int n_tiles = (N + NO - 1) / NO;
    const TileCoord tc = find_tile<BM>(offsets, E, n_tiles);
    if (!tc.valid) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
        a_row_id[p] = row_map ? row_map[r] : r;
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
        char* bs = smem + B_BASE + (d % NSB) * B_SLOT;
        const bool tail = odd_tail && d == n_double - 1;
#pragma unroll
        for (int p = 0; p < B_LPW; ++p)
            if (!tail || b_first_half[p])
                __builtin_amdgcn_global_load_lds((glb_ptr_t*)(b_src[p] + (int64_t)d * B_ROWB),
                                                 (lds_ptr_t*)(bs + (wave + NW * p) * 1024), 16, 0, 0);
        issued += B_LPW;     // (every wave has lanes on both sides of the tail mask, so both loads are always issued)
        if (!wide_scales) {
            lds_ptr_t* dst = (lds_ptr_t*)(smem + S_BASE + (d % NSB) * S_SLOT + wave * 256);
            if (!tail) __builtin_amdgcn_global_load_lds((glb_ptr_t*)(s_src + d * 4), dst, 4, 0, 0);
            else if (row_scales >= 4) __builtin_amdgcn_global_load_lds((glb_ptr_t*)(s_src + row_scales - 4), dst, 4, 0, 0);
            else __builtin_amdgcn_global_load_lds((glb_ptr_t*)s_src, dst, 2, 0, 0);
            issued += 1;
        }
#pragma unroll
        for (int i = 0; i < NSB; ++i)
            if (i == d % NSB) last_b[i] = issued;
    };
    int last_s[2] = {0, 0};
    auto issue_s = [&](int c) {        // wide scale chunk c = stages 8c .. 8c + 7
        __builtin_amdgcn_global_load_lds((glb_ptr_t*)(s_src + chunk_start(c)),
                                         (lds_ptr_t*)(smem + S_BASE + (c & 1) * SW_SLOT + wave * 1024), 16, 0, 0);
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
                __builtin_amdgcn_global_load_lds((glb_ptr_t*)(a_src[p] + kt * PBK),
                                                 (lds_ptr_t*)(smem + (kt % NSA) * A_SLOT + (wave + NW * p) * 1024), 16, 0,
                                                 0);
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
                if (row < tc.row_end && col < N)    // N is a multiple of 8: the 4 columns are in or out together
                    *reinterpret_cast<uint2*>(Out + row * ldo + col) =
                        make_uint2(pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3]));
            }
        }
    }
}

template <bool GATED>
hipError_t launch_w4(RowSrc X, int ldx, const int32_t* row_map, int map_div, const int32_t* offsets, int E, int64_t A,
                     const uint8_t* W, const uint8_t* S, int64_t rows_per_expert, int N, int K, bf16_t* Out, int ldo,
                     hipStream_t s)
{
    constexpr int NO = GATED ? kW4BN / 2 : kW4BN;
    const size_t lds_bytes = (size_t)kW4NSA * kW4Rows * kW4K * 2 + (size_t)kW4NSB * kW4BN * kW4K + 2 * kW4BN * 16;   // scale area: max(3 dword slots, 2 chunk slots)
    auto kern = grouped_gemm_w4_kernel<GATED>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t n_tiles = (N + NO - 1) / NO;
    const int64_t m_tiles_max = (A + kW4Rows - 1) / kW4Rows + (A < E ? A : E);
    const int64_t grid = ((m_tiles_max * n_tiles + 7) / 8) * 8;
    if (grid >= ((int64_t)1 << 31)) return hipErrorInvalidValue;   // the device-side tile search counts in 32 bits
    kern<<<(unsigned)grid, kW4Waves * 64, lds_bytes, s>>>(X, ldx, row_map, map_div, offsets, E, W, S, rows_per_expert, N, K,
                                                          Out, ldo);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ffn_gate_up_w4(RowSrc x, const int32_t* row_map, int map_div, const int32_t* offsets, int64_t A, int E,
                                 int H, int I, const uint8_t* w_gate_up, const uint8_t* s_gate_up, void* act,
                                 hipStream_t s)
{
    return launch_w4<true>(x, H, row_map, map_div, offsets, E, A, w_gate_up, s_gate_up, (int64_t)2 * I, I, H,
                           (bf16_t*)act, I, s);
}

hipError_t launch_ffn_down_w4(const void* act, const int32_t* offsets, int64_t A, int E, int H, int I,
                              const uint8_t* w_down, const uint8_t* s_down, void* y_perm, hipStream_t s)
{
    return launch_w4<false>(single_src(act), I, nullptr, 1, offsets, E, A, w_down, s_down, (int64_t)H, H, I,
                            (bf16_t*)y_perm, H, s);
}

}  // namespace moe
