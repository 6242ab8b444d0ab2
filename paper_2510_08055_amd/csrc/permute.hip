// Token permutation: per-expert histogram, prefix sum and a STABLE rank of every
// assignment, so that the tokens routed to each expert (Sec. 3.1) form a contiguous,
// deterministically ordered batch: order = (expert, token, slot).
//
// Counting uses LDS integer atomics (order-free, hence deterministic).  The rank of an
// assignment inside its expert comes from an ordered scan, never from "claim a slot"
// atomics: tile prefix (from the per-tile histograms) + wave prefix + a running per-wave
// counter + the rank among equal experts inside one 64-wide chunk (ballot matching).
#include "common.h"

namespace moe {

// Expert ids are trusted to lie in [0, E); clamping keeps a corrupt id from indexing outside LDS.
__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

constexpr int kPermThreads = 1024;                       // 16 waves
constexpr int kPermWaves = kPermThreads / 64;
constexpr int kPermRounds = kPermTile / kPermThreads;    // 64-wide chunks per wave
static_assert(kPermRounds * kPermThreads == kPermTile, "tile must be a whole number of rounds");

// Pass 1 (only when there is more than one tile): tile_hist[tile][e].
__global__ __launch_bounds__(kPermThreads) void permute_hist_kernel(const int32_t* __restrict__ idx, int64_t A,
                                                                    int E, int32_t* __restrict__ tile_hist)
{
    __shared__ int32_t hist[kMaxExperts];
    for (int e = threadIdx.x; e < E; e += kPermThreads) hist[e] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kPermTile;
    for (int i = threadIdx.x; i < kPermTile; i += kPermThreads) {
        const int64_t f = base + i;
        if (f < A) atomicAdd(&hist[clamp_expert(idx[f], E)], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kPermThreads) tile_hist[(int64_t)blockIdx.x * E + e] = hist[e];
}

// Pass 2: every block derives the global offsets (all tiles' histograms are tiny) and the
// start of its own tile inside each expert, then ranks and scatters its assignments.
// With a single tile the block builds the histogram itself and pass 1 is skipped.
__global__ __launch_bounds__(kPermThreads) void permute_scatter_kernel(
    const int32_t* __restrict__ idx, int64_t A, int E, int n_tiles, const int32_t* __restrict__ tile_hist,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
    int32_t* __restrict__ inv, unsigned long long* __restrict__ active_total)
{
    __shared__ int32_t total[kMaxExperts];              // assignments per expert, whole batch
    __shared__ int32_t start[kMaxExperts];              // first permuted row of this tile inside expert e
    __shared__ int32_t wave_cnt[kPermWaves][kMaxExperts];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = blockIdx.x;
    const int64_t base = (int64_t)tile * kPermTile;

    for (int e = tid; e < E; e += kPermThreads) {
        total[e] = 0;
        start[e] = 0;
    }
    for (int i = tid; i < kPermWaves * kMaxExperts; i += kPermThreads) (&wave_cnt[0][0])[i] = 0;
    __syncthreads();
    if (n_tiles == 1) {
        for (int i = tid; i < kPermTile; i += kPermThreads)
            if (base + i < A) atomicAdd(&total[clamp_expert(idx[base + i], E)], 1);
    } else {
        for (int e = tid; e < E; e += kPermThreads) {
            int tot = 0, before = 0;
            for (int t = 0; t < n_tiles; ++t) {
                const int h = tile_hist[(int64_t)t * E + e];
                tot += h;
                if (t < tile) before += h;
            }
            total[e] = tot;
            start[e] = before;
        }
    }
    __syncthreads();
    // exclusive scan over experts by wave 0: lane l owns experts [l*8, l*8+8)
    if (wave == 0) {
        int loc[kMaxExperts / 64];
        int sum = 0;
#pragma unroll
        for (int i = 0; i < kMaxExperts / 64; ++i) {
            const int e = lane * (kMaxExperts / 64) + i;
            loc[i] = (e < E) ? total[e] : 0;
            sum += loc[i];
        }
        int incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        int run = incl - sum;
        int act = 0;
#pragma unroll
        for (int i = 0; i < kMaxExperts / 64; ++i) {
            const int e = lane * (kMaxExperts / 64) + i;
            if (e < E) {
                start[e] += run;
                if (tile == 0) {
                    counts[e] = loc[i];
                    offsets[e] = run;
                }
                act += (loc[i] > 0);
            }
            run += loc[i];
        }
        if (tile == 0) {
            if (lane == 63) offsets[E] = incl;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) act += __shfl_xor(act, off, 64);
            if (lane == 0 && active_total) atomicAdd(active_total, (unsigned long long)act);
        }
    }
    __syncthreads();

    // Rank inside the wave's 512-assignment region, chunk by chunk in index order.
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    int my_e[kPermRounds], my_rank[kPermRounds];
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    // all of this thread's expert ids are fetched up front: one memory latency, not one per round
#pragma unroll
    for (int r = 0; r < kPermRounds; ++r) {
        const int64_t f = base + (int64_t)wave * (kPermRounds * 64) + r * 64 + lane;
        my_e[r] = (f < A) ? clamp_expert(idx[f], E) : -1;
    }
#pragma unroll
    for (int r = 0; r < kPermRounds; ++r) {
        const bool valid = my_e[r] >= 0;
        const int e = valid ? my_e[r] : 0;
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const uint64_t bal = __ballot(valid && bit);
            peers &= bit ? bal : ~bal;
        }
        if (valid) {
            my_rank[r] = wave_cnt[wave][e] + __popcll(peers & lt_mask);
        } else {
            my_rank[r] = 0;
        }
        // wave_cnt[wave] is private to this wave and a wave's LDS operations execute in program order,
        // so the update below cannot overtake the reads above: no block barrier inside the rounds.
        __builtin_amdgcn_wave_barrier();
        if (valid && (63 - __clzll(peers)) == lane) wave_cnt[wave][e] += __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // wave_cnt[w][e] becomes the first permuted row of wave w's assignments to expert e: this tile's
    // start inside the expert plus the counts of the waves in front (one pass per expert, instead of
    // every assignment adding up the waves in front of it)
    for (int e = tid; e < E; e += kPermThreads) {
        int c[kPermWaves];
#pragma unroll
        for (int wv = 0; wv < kPermWaves; ++wv) c[wv] = wave_cnt[wv][e];
        int run = start[e];
#pragma unroll
        for (int wv = 0; wv < kPermWaves; ++wv) {
            wave_cnt[wv][e] = run;
            run += c[wv];
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kPermRounds; ++r) {
        const int e = my_e[r];
        if (e < 0) continue;
        const int pos = wave_cnt[wave][e] + my_rank[r];
        const int64_t f = base + (int64_t)wave * (kPermRounds * 64) + r * 64 + lane;
        perm[pos] = (int32_t)f;
        inv[f] = pos;
    }
}

template <typename VT>
__global__ __launch_bounds__(256) void gather_rows_kernel(const VT* __restrict__ x, const int32_t* __restrict__ perm,
                                                          int K, int64_t A, int vec_per_row, VT* __restrict__ out)
{
    const int64_t r = blockIdx.x;
    if (r >= A) return;
    const int64_t src = perm[r] / K;
    const VT* s = x + src * vec_per_row;
    VT* d = out + r * vec_per_row;
    for (int i = threadIdx.x; i < vec_per_row; i += 256) d[i] = s[i];
}

hipError_t launch_permute(const int32_t* idx, int64_t A, int E, int32_t* counts, int32_t* offsets, int32_t* perm,
                          int32_t* inv, int32_t* tile_hist, bool hist_ready, unsigned long long* active_total,
                          hipStream_t s)
{
    const int n_tiles = (int)((A + kPermTile - 1) / kPermTile);
    if (n_tiles > 1 && !hist_ready) {
        permute_hist_kernel<<<n_tiles, kPermThreads, 0, s>>>(idx, A, E, tile_hist);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    permute_scatter_kernel<<<n_tiles, kPermThreads, 0, s>>>(idx, A, E, n_tiles, tile_hist, counts, offsets, perm,
                                                            inv, active_total);
    return hipGetLastError();
}

// Zeroes n 32-bit words.  In place of hipMemsetAsync wherever a caller may be capturing the stream into a
// HIP graph (memset nodes have replayed wrongly on this platform).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, int n)
{
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i < n) p[i] = 0u;
}

hipError_t launch_fill_zero(void* p, int n_words, hipStream_t s)
{
    if (n_words <= 0) return hipSuccess;
    fill_zero_kernel<<<(unsigned)((n_words + 255) / 256), 256, 0, s>>>(static_cast<uint32_t*>(p), n_words);
    return hipGetLastError();
}

hipError_t launch_gather_rows(int dtype, const void* x, const int32_t* perm, int K, int64_t A, int H, void* x_perm,
                              hipStream_t s)
{
    const int row_bytes = H * (dtype == MOE_BF16 ? 2 : 4);
    gather_rows_kernel<uint4><<<(unsigned)A, 256, 0, s>>>((const uint4*)x, perm, K, A, row_bytes / 16,
                                                          (uint4*)x_perm);
    return hipGetLastError();
}

}  // namespace moe
