// Pieces shared by the grouped-GEMM kernels (bf16 weights in ffn.hip, 4-bit weights in ffn_w4.hip):
// the device-side tile search, the SwiGLU epilogue function and the helpers of the direct-to-LDS
// software pipeline.
#pragma once
#include <type_traits>

#include "common.h"

namespace moe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

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
    int expert, row0, row_end, n_tile;   // rows [row0, row_end) of the permuted batch belong to this tile
    bool valid;
};

// An expert with m rows is cut into ceil(m / BM) m-tiles of (nearly) equal size, each a whole number of
// 32-row blocks: 1032 rows and BM = 256 give 224+224+224+192+168 rather than 4 x 256 + 8, so no block
// streams a whole weight tile for a handful of rows.
// (The host bounds the grid so that the tile count fits 31 bits.)
// Offsets are trusted to be a non-decreasing sequence in [0, max_rows]; they are clamped to that range and
// negative counts to zero all the same, so that offsets gone wrong (a caller's bug, an uninitialised buffer)
// give wrong results inside the output's rows, never a store outside them.
template <int BM>
__device__ __forceinline__ TileCoord find_tile(const int32_t* __restrict__ offsets, int E, int n_tiles, int max_rows)
{
    constexpr int EPL = kMaxExperts / 64;
    const int lane = lane_id();
    int off[EPL + 1];
#pragma unroll
    for (int i = 0; i <= EPL; ++i) {
        const int e = lane * EPL + i;
        const int o = offsets[e <= E ? e : E];
        off[i] = o < 0 ? 0 : (o > max_rows ? max_rows : o);
    }
    int mt[EPL];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const int cnt = off[i + 1] > off[i] ? off[i + 1] - off[i] : 0;
        mt[i] = (cnt + BM - 1) / BM;
        sum += mt[i];
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    const int total = __shfl(incl, 63, 64) * n_tiles;
    const int chunk = (total + 7) / 8;
    const int slot = blockIdx.x / 8;
    const int logical = (int)(blockIdx.x % 8) * chunk + slot;
    TileCoord tc;
    tc.valid = __builtin_amdgcn_readfirstlane((slot < chunk) && (logical < total)) != 0;   // uniform: no divergent join below
    tc.expert = 0; tc.row0 = 0; tc.row_end = 0; tc.n_tile = 0;
    if (!tc.valid) return tc;
    // the lane whose experts contain the tile (tiles of an expert: mt_e * n_tiles, n-major), then the
    // expert among that lane's EPL; the one division happens after the choice
    const unsigned long long hit = __ballot(logical < incl * n_tiles);
    const int src = __ffsll((long long)hit) - 1;
    int rem = logical - (incl - sum) * n_tiles;   // meaningful on lane src only
    int s_e = 0, s_lo = 0, s_hi = 0, s_mt = 1, s_rem = 0;
    bool found = false;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const int cnt = mt[i] * n_tiles;
        const bool here = !found && rem < cnt;
        if (here) {
            s_e = lane * EPL + i;
            s_lo = off[i];
            s_hi = off[i + 1];
            s_mt = mt[i];
            s_rem = rem;
            found = true;
        }
        rem -= cnt;
    }
    s_e = __shfl(s_e, src, 64);
    s_lo = __shfl(s_lo, src, 64);
    s_hi = __shfl(s_hi, src, 64);
    s_mt = __shfl(s_mt, src, 64);
    s_rem = __shfl(s_rem, src, 64);
    const int n_tile = s_rem / s_mt;
    const int t = s_rem - n_tile * s_mt;
    const int rb = (s_hi - s_lo + 31) / 32;                 // 32-row blocks of this expert
    const int per = (rb + s_mt - 1) / s_mt;                 // row blocks per tile
    int row0 = s_lo + t * per * 32;
    int row_end = row0 + per * 32;
    if (row_end > s_hi) row_end = s_hi;
    if (row0 > row_end) row0 = row_end;                     // cannot happen: per * (mt - 1) < rb
    // the same in every lane: handed out as scalars, so that what the kernels derive from them (base
    // addresses, row counts, the bookkeeping of the load pipeline) stays in scalar registers
    tc.expert = __builtin_amdgcn_readfirstlane(s_e);
    tc.row0 = __builtin_amdgcn_readfirstlane(row0);
    tc.row_end = __builtin_amdgcn_readfirstlane(row_end);
    tc.n_tile = __builtin_amdgcn_readfirstlane(n_tile);
    return tc;
}

// silu(g) * u with silu(g) = g / (1 + e^-g); hardware exp2 and reciprocal (1 ulp each), far inside the
// rounding of the bf16 (or the tolerance of the fp32) result.
__device__ __forceinline__ float silu_mul(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// The value as it stands in a register: the compiler can no longer fuse the multiplication that produced it
// into a later subtraction (fp contraction would make `v - round(v)` depend on where it is compiled).
__device__ __forceinline__ float opaque(float v)
{
    asm volatile("" : "+v"(v));
    return v;
}

typedef __attribute__((address_space(3))) void lds_ptr_t;
typedef __attribute__((address_space(1))) const void glb_ptr_t;

// Waits and barriers of the software pipeline are inline asm with a memory clobber: the compiler must
// not move LDS reads or the direct-to-LDS loads across them (the bare s_barrier intrinsic is not a
// memory barrier for the optimiser, and __syncthreads() would drain every load still in flight).
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds_reads() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// One wave-level direct-to-LDS load: lane i's BYTES bytes from `src` land at LDS byte address lds_base + BYTES i
// (lds_base is wave-uniform and travels in M0).  Issued from inline asm on purpose.  The compiler's
// wait-count pass takes the builtin form for an access to both global memory and LDS, and while it
// believes one to be in flight (it never sees the explicit vmcnt waits above, so: always) it turns
// every LDS wait into lgkmcnt(0): an MFMA that needs the fragments read one k-slice ago then also waits
// for the reads just issued for the next slice.  With the asm form the waits carry the exact count.
// The kernels that use it must not leave anything else in M0 (nothing in them does: LDS instructions
// need no M0 on this target).
template <int BYTES> __device__ __forceinline__ void load_lds(const void* src, uint32_t lds_base)
{
    static_assert(BYTES == 16 || BYTES == 4 || BYTES == 2, "direct-to-LDS loads move 16, 4 or 2 bytes per lane");
    if (BYTES == 16)
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_base) : "memory");
    else if (BYTES == 4)
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(lds_base) : "memory");
    else
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_ushort %0, off" ::"v"(src), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void load_lds_16(const void* src, uint32_t lds_base) { load_lds<16>(src, lds_base); }
// LDS byte address of a pointer into the block's dynamic shared memory
__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(lds_ptr_t*)p;
}

// Source-side swizzle of a tile row: which LDS 16-byte chunk slot holds global chunk c of row r is
// c ^ swz(r).  Chosen so that the 16-byte operand reads of 8 (and of 16) consecutive rows fall into
// distinct bank groups whether the LDS serves 128 or 256 bytes per clock.
template <int PBK> __device__ __forceinline__ int swz(int r)
{
    if (PBK == 64) return (r & 7) ^ ((r >> 3) & 1);
    return ((r >> 1) & 3) ^ ((r >> 3) & 1);
}

}  // namespace moe
