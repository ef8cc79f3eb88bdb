// Dispatch stage: stable counting sort of slice->expert assignments (the grouping of paper
// Section 3.4), with an optional per-expert capacity, plus the load statistics of Eq. 2 and
// of the ELE metric (Section 4).
//
// Three kernels over chunks of kDispChunk consecutive assignment ids a = n*k + j:
//   1. histogram   block_counts[b][e] = # assignments of chunk b bound for expert e
//   2. scan        per expert, exclusive prefix over chunks (in place) -> rank of a chunk's first
//                  assignment inside its expert; totals -> counts_raw, counts, offsets
//   3. scatter     stable rank of every assignment inside its chunk, final row, perm / inv;
//                  one extra block computes the load statistics from the counts
// When the table of step 1 is small (the headline has 512 chunks x 32 experts) step 2 is folded into
// step 3: every scatter block sums the table itself, which is cheaper than a latency-bound launch.
// Stability needs ranks in ascending a.  A block walks its chunk in rounds of 256 consecutive
// ids; inside a wavefront the rank among equal experts comes from ballots (one per bit of the
// expert id gives every lane the mask of lanes holding the same expert), across wavefronts and
// rounds from a small LDS table scanned in (round, wavefront) order.
#include "common.h"

namespace slicemoe {

__device__ __forceinline__ unsigned long long same_expert_mask(int e, bool valid, int nbits)
{
    unsigned long long m = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long bal = __ballot(valid && bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

__global__ __launch_bounds__(kDispThreads) void dispatch_hist_kernel(
    const int32_t *__restrict__ idx, int Na, int E, int nbits, int32_t *__restrict__ block_counts)
{
    __shared__ int cnt[64];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    if (tid < 64) cnt[tid] = 0;
    __syncthreads();
    const int base = blockIdx.x * kDispChunk;
    int ex[kDispItems];
#pragma unroll
    for (int i = 0; i < kDispItems; ++i) {
        const int a = base + i * kDispThreads + tid;
        ex[i] = a < Na ? clamp_expert(idx[a], E) : -1;
    }
#pragma unroll
    for (int i = 0; i < kDispItems; ++i) {
        const bool valid = ex[i] >= 0;
        const int e = valid ? ex[i] : 0;
        const unsigned long long m = same_expert_mask(e, valid, nbits);
        const unsigned long long below = m & ((1ull << lane) - 1ull);
        if (valid && below == 0) atomicAdd(&cnt[e], __popcll(m));
    }
    __syncthreads();
    if (tid < E) block_counts[(size_t)blockIdx.x * E + tid] = cnt[tid];
}

// Load statistics of a routed batch from the per-expert counts: one wavefront, lane e owns
// expert e (E <= 64), sums by cross-lane reduction.
//   stats[0] = CV^2 (population variance; the capacity loss of Eq. 2 divided by alpha)
//   stats[1] = ELE = -sum load_e log load_e / log E (Section 4)     stats[2] = dropped fraction
//   stats[3] = CV^2 with the sample variance
__device__ __forceinline__ double wave_sum(double v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ void load_stats_wave(int raw, int kept_e, bool have, int E, float *__restrict__ stats)
{
    const double c = have ? (double)raw : 0.0;
    const double sum = wave_sum(c);
    const double kept = wave_sum(have ? (double)kept_e : 0.0);
    const double mean = sum / E;
    const double dl = have ? c - mean : 0.0;
    const double ss = wave_sum(dl * dl);
    const double l = (have && raw > 0) ? c / sum : 1.0;
    const double ent = wave_sum(-l * (double)logf((float)l));
    if ((threadIdx.x & 63) == 0) {
        stats[0] = mean > 0 ? (float)(ss / E / (mean * mean)) : 0.f;
        stats[1] = E > 1 ? (float)(ent / (double)logf((float)E)) : 1.f;
        stats[2] = sum > 0 ? (float)(1.0 - kept / sum) : 0.f;
        stats[3] = (mean > 0 && E > 1) ? (float)(ss / (E - 1) / (mean * mean)) : 0.f;
    }
}

// One block of 1024 threads walks the [nblocks][E] table in tiles of kScanTile entries staged in
// LDS (coalesced 16-byte loads and stores; the table is tiny, the kernel is latency-bound, so every
// global access is issued in one batch and every scan is a wavefront shuffle scan).  Inside a tile,
// thread (seg, e) with e = tid % Epow2 owns a contiguous run of chunks of expert e and sums it; the
// nseg <= 64 segment sums of an expert are then re-read segment-fastest, so that they sit in
// consecutive lanes, and scanned with shuffles on top of the running total carried from the previous
// tiles; finally each thread rewrites its run as exclusive prefixes.
constexpr int kScanTileMax = 32768;   // table entries per tile at most: 128 KiB of LDS (the headline table is 16384)

__device__ __forceinline__ int group_inclusive_scan(int v, int pos, int width)
{
    for (int o = 1; o < width; o <<= 1) {
        const int t = __shfl_up(v, o);
        if (pos >= o) v += t;
    }
    return v;
}

__global__ __launch_bounds__(1024) void dispatch_scan_kernel(
    int32_t *__restrict__ block_counts, int nblocks, int E, int Epow2, long long capacity,
    int32_t *__restrict__ counts_raw, int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int tile_entries)
{
    extern __shared__ __align__(16) int tile[];   // [tile_entries]
    __shared__ int seg_sum[1024];
    __shared__ int carry[64];
    const int tid = threadIdx.x;
    const int nseg = min(64, 1024 / Epow2);       // power of two: a segment group never straddles a wavefront
    // tile passes: expert fastest (consecutive lanes touch consecutive LDS words)
    const int e = tid % Epow2;
    const int seg = tid / Epow2;
    const bool active = e < E && seg < nseg;
    // scan of the segment sums: segment fastest (an expert's sums sit in consecutive lanes)
    const int e2 = tid / nseg;
    const int seg2 = tid % nseg;
    const bool active2 = e2 < E;
    const int chunks_per_tile = tile_entries / E;    // whole chunks only
    if (tid < 64) carry[tid] = 0;

    for (int c0 = 0; c0 < nblocks; c0 += chunks_per_tile) {
        const int nc = min(chunks_per_tile, nblocks - c0);
        const long long first = (long long)c0 * E;            // entry index of the tile start
        const int n_entries = nc * E;
        const bool vec = ((first & 3) == 0);                  // 16-byte pieces need an aligned tile start
        __syncthreads();   // previous tile fully written back, carry visible
        if (vec) {
            for (int i = tid * 4; i < n_entries; i += 1024 * 4) {
                if (i + 4 <= n_entries) *(int4 *)(tile + i) = *(const int4 *)(block_counts + first + i);
                else for (int q = i; q < n_entries; ++q) tile[q] = block_counts[first + q];
            }
        } else {
            for (int i = tid; i < n_entries; i += 1024) tile[i] = block_counts[first + i];
        }
        __syncthreads();
        const int per = (nc + nseg - 1) / nseg;
        const int b0 = seg * per;
        const int b1 = min(nc, b0 + per);
        int s = 0;
        if (active)
            for (int b = b0; b < b1; ++b) s += tile[b * E + e];
        if (active) seg_sum[seg * Epow2 + e] = s;
        __syncthreads();
        {
            const int v = active2 ? seg_sum[seg2 * Epow2 + e2] : 0;
            const int incl = group_inclusive_scan(v, seg2, nseg);
            const int base = active2 ? carry[e2] : 0;
            __syncthreads();                                   // everyone has read seg_sum and carry
            if (active2) seg_sum[seg2 * Epow2 + e2] = base + incl - v;   // exclusive prefix of the segment
            if (active2 && seg2 == nseg - 1) carry[e2] = base + incl;
        }
        __syncthreads();
        if (active) {
            int run = seg_sum[seg * Epow2 + e];
            for (int b = b0; b < b1; ++b) {
                const int t = tile[b * E + e];
                tile[b * E + e] = run;
                run += t;
            }
        }
        __syncthreads();
        if (vec) {
            for (int i = tid * 4; i < n_entries; i += 1024 * 4) {
                if (i + 4 <= n_entries) *(int4 *)(block_counts + first + i) = *(const int4 *)(tile + i);
                else for (int q = i; q < n_entries; ++q) block_counts[first + q] = tile[q];
            }
        } else {
            for (int i = tid; i < n_entries; i += 1024) block_counts[first + i] = tile[i];
        }
    }
    __syncthreads();
    if (tid < 64) {   // one wavefront: lane x owns expert x
        const int raw = tid < E ? carry[tid] : 0;
        const int c = (capacity >= 0 && raw > capacity) ? (int)capacity : raw;
        const int incl = group_inclusive_scan(c, tid, 64);
        if (tid < E) {
            counts_raw[tid] = raw;
            counts[tid] = c;
            offsets[tid] = incl - c;
        }
        if (tid == E - 1) offsets[E] = incl;
    }
}

// FUSED = false: `table` holds the exclusive per-expert prefixes written by dispatch_scan_kernel and the
// per-expert offsets come from `offsets`.
// FUSED = true (small tables, E a power of two >= 4): there is no scan kernel.  `table` holds the raw
// per-chunk counts; every block sums the whole table (coalesced 16-byte loads, all in flight at once) into
// the per-expert totals and into the prefix of its own chunk, derives counts and offsets itself, and block 0
// writes counts_raw / counts / offsets for the stages that follow.  Reading nchunks * E ints per block is
// cheaper than a separate latency-bound launch as long as the table is small.
template <bool FUSED>
__global__ __launch_bounds__(kDispThreads) void dispatch_scatter_kernel(
    const int32_t *__restrict__ idx, int Na, int E, int nbits, long long capacity,
    const int32_t *__restrict__ table, int32_t *__restrict__ offsets,
    int32_t *__restrict__ perm, int32_t *__restrict__ inv, int nchunks, int32_t *__restrict__ counts_raw,
    int32_t *__restrict__ counts, float *__restrict__ stats /* may be null */)
{
    constexpr int kWaves = kDispThreads / 64;
    __shared__ int wcnt[kDispItems][kWaves][64];
    __shared__ int s_pre[64];      // FUSED: rank of this chunk's first assignment inside each expert
    __shared__ int s_off[65];      // FUSED: per-expert offsets
    const int tid = threadIdx.x;
    const bool stats_block = (int)blockIdx.x == nchunks;   // one extra block: the load statistics, off everyone's critical path
    if constexpr (FUSED) {
        __shared__ int part[2][kDispThreads][4];
        const int n_entries = nchunks * E;              // a multiple of 4, and 4 * kDispThreads is a multiple of E:
        int tot[4] = {0, 0, 0, 0}, pre[4] = {0, 0, 0, 0};   // a thread always sees the same four experts
        for (int flat = tid * 4; flat < n_entries; flat += kDispThreads * 4) {
            const int4 v = *(const int4 *)(table + flat);
            const bool before = (flat >> nbits) < (int)blockIdx.x;   // chunk index of this piece
            tot[0] += v.x; tot[1] += v.y; tot[2] += v.z; tot[3] += v.w;
            if (before) { pre[0] += v.x; pre[1] += v.y; pre[2] += v.z; pre[3] += v.w; }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            part[0][tid][q] = tot[q];
            part[1][tid][q] = pre[q];
        }
        __syncthreads();
        int raw = 0, mine = 0;
        if (tid < E) {   // the threads t with (4 t) % E == 4 (tid / 4) hold expert tid in component tid % 4
            const int step = E / 4;
            for (int t = tid / 4; t < kDispThreads; t += step) {
                raw += part[0][t][tid & 3];
                mine += part[1][t][tid & 3];
            }
        }
        if (tid < 64) {   // one wavefront: lane x owns expert x
            const int c = (capacity >= 0 && raw > capacity) ? (int)capacity : raw;
            const int incl = group_inclusive_scan(tid < E ? c : 0, tid, 64);
            if (tid < E) {
                s_pre[tid] = mine;
                s_off[tid] = incl - c;
                if (blockIdx.x == 0) {
                    counts_raw[tid] = raw;
                    counts[tid] = c;
                    offsets[tid] = incl - c;
                }
            }
            if (tid == E - 1) {
                s_off[E] = incl;
                if (blockIdx.x == 0) offsets[E] = incl;
            }
            if (stats_block && stats) load_stats_wave(raw, c, tid < E, E, stats);
        }
        if (stats_block) return;
    } else {
        if (stats_block) {
            if (stats && tid < 64) load_stats_wave(tid < E ? counts_raw[tid] : 0, tid < E ? counts[tid] : 0, tid < E, E, stats);
            return;
        }
    }
    const int lane = tid & 63;
    const int wave = tid >> 6;
    for (int i = tid; i < kDispItems * kWaves * 64; i += kDispThreads) (&wcnt[0][0][0])[i] = 0;
    __syncthreads();

    const int base = blockIdx.x * kDispChunk;
    int ex[kDispItems];
    int rk[kDispItems];
#pragma unroll
    for (int i = 0; i < kDispItems; ++i) {
        const int a = base + i * kDispThreads + tid;
        ex[i] = a < Na ? clamp_expert(idx[a], E) : -1;
    }
#pragma unroll
    for (int i = 0; i < kDispItems; ++i) {
        const bool valid = ex[i] >= 0;
        const int e = valid ? ex[i] : 0;
        const unsigned long long m = same_expert_mask(e, valid, nbits);
        const int below = __popcll(m & ((1ull << lane) - 1ull));
        rk[i] = below;
        if (valid && below == 0) wcnt[i][wave][e] = __popcll(m);
    }
    __syncthreads();
    if (tid < E) {
        int run = FUSED ? s_pre[tid] : table[(size_t)blockIdx.x * E + tid];
        for (int i = 0; i < kDispItems; ++i)
            for (int w = 0; w < kWaves; ++w) {
                const int t = wcnt[i][w][tid];
                wcnt[i][w][tid] = run;
                run += t;
            }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kDispItems; ++i) {
        const int e = ex[i];
        if (e < 0) continue;
        const int a = base + i * kDispThreads + tid;
        const int rank = wcnt[i][wave][e] + rk[i];
        if (capacity < 0 || rank < capacity) {
            const int row = (FUSED ? s_off[e] : offsets[e]) + rank;
            perm[row] = a;
            inv[a] = row;
        } else {
            inv[a] = -1;
        }
    }
}

hipError_t launch_dispatch(const slicemoe_config &c, const int32_t *idx, int32_t *counts_raw,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                           int32_t *block_counts, float *stats, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    const int nblocks = (int)((Na + kDispChunk - 1) / kDispChunk);
    int nbits = 0;
    while ((1 << nbits) < c.E) ++nbits;
    const int Epow2 = 1 << nbits;
    const long long cap = slicemoe_capacity(&c);
    if (nblocks > 0) dispatch_hist_kernel<<<nblocks, kDispThreads, 0, s>>>(idx, (int)Na, c.E, nbits, block_counts);
    // small table and a power-of-two expert count: every scatter block scans the table itself
    const bool fused = nblocks > 0 && c.E >= 4 && Epow2 == c.E && (long long)nblocks * c.E <= 32768;
    if (fused) {
        dispatch_scatter_kernel<true><<<nblocks + (stats ? 1 : 0), kDispThreads, 0, s>>>(
            idx, (int)Na, c.E, nbits, cap, block_counts, offsets, perm, inv, nblocks, counts_raw, counts, stats);
        return hipGetLastError();
    }
    {
        long long want = (long long)nblocks * c.E;
        int tile_entries = (int)(want < 1024 ? 1024 : (want > kScanTileMax ? kScanTileMax : (want + 3) / 4 * 4));
        const int lds_cap = (max_lds_per_block() - 8 * 1024) / 4;
        if (tile_entries > lds_cap) tile_entries = lds_cap / 4 * 4;
        if (tile_entries < c.E) return hipErrorInvalidValue;
        hipError_t err = hipFuncSetAttribute((const void *)dispatch_scan_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                             tile_entries * 4);
        if (err != hipSuccess) return err;
        dispatch_scan_kernel<<<1, 1024, (size_t)tile_entries * 4, s>>>(block_counts, nblocks, c.E, Epow2, cap, counts_raw,
                                                                     counts, offsets, tile_entries);
    }
    if (nblocks > 0 || stats)
        dispatch_scatter_kernel<false><<<nblocks + (stats ? 1 : 0), kDispThreads, 0, s>>>(
            idx, (int)Na, c.E, nbits, cap, block_counts, offsets, perm, inv, nblocks, counts_raw, counts, stats);
    return hipGetLastError();
}

// ---- load statistics on their own (Eq. 2 statistic, ELE of Section 4) ---------------------
__global__ __launch_bounds__(64) void load_stats_kernel(const int32_t *__restrict__ counts_raw,
                                                        const int32_t *__restrict__ counts, int E,
                                                        float *__restrict__ stats)
{
    const int x = threadIdx.x;
    const bool have = x < E;
    load_stats_wave(have ? counts_raw[x] : 0, have ? counts[x] : 0, have, E, stats);
}

hipError_t launch_load_stats(const slicemoe_config &c, const int32_t *counts_raw, const int32_t *counts,
                             float *stats, hipStream_t s)
{
    load_stats_kernel<<<1, 64, 0, s>>>(counts_raw, counts, c.E, stats);
    return hipGetLastError();
}

}  // namespace slicemoe
