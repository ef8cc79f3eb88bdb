// Dispatch stage: stable counting sort of slice->expert assignments (the grouping of paper
// Section 3.4), with an optional per-expert capacity, plus the load statistics of Eq. 2 and
// of the ELE metric (Section 4).
//
// Three kernels over chunks of kDispChunk consecutive assignment ids a = n*k + j:
//   1. histogram   block_counts[b][e] = # assignments of chunk b bound for expert e
//   2. scan        per expert (one wavefront each), exclusive prefix over chunks (in place) -> rank of a
//                  chunk's first assignment inside its expert; totals -> counts_raw, counts
//   3. scatter     offsets from the counts, stable rank of every assignment inside its chunk, final
//                  row, perm / inv; one extra block computes the load statistics from the counts
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

__device__ __forceinline__ int group_inclusive_scan(int v, int pos, int width)
{
    for (int o = 1; o < width; o <<= 1) {
        const int t = __shfl_up(v, o);
        if (pos >= o) v += t;
    }
    return v;
}

// The columns of the [nblocks][E] table are independent: one block per expert, so that the experts spread over the
// CUs (a lane's loads are a whole table row apart; what bounds the kernel is the rate of such scattered requests of
// one CU and their latency: 67 us for Large's 4096 x 64 table with eight experts per block, 33 us with one wavefront
// per expert).  Thread `seg` owns a contiguous run of chunks of the expert: it sums the run, the run sums are scanned
// (shuffles inside a wavefront, a small LDS table across), and the thread rewrites its run as exclusive prefixes.
// The expert's total goes to counts_raw and, capped, to counts; the scatter kernel turns the counts into offsets.
constexpr int kScanWaves = 16, kScanSegs = kScanWaves * 64;
__global__ __launch_bounds__(kScanSegs) void dispatch_scan_kernel(
    int32_t *__restrict__ table, int nblocks, int E, long long capacity, int32_t *__restrict__ counts_raw,
    int32_t *__restrict__ counts)
{
    __shared__ int wave_total[kScanWaves];
    const int seg = threadIdx.x, lane = seg & 63, wave = seg >> 6;
    const int e = (int)blockIdx.x;   // < E by the launch
    const int per = (nblocks + kScanSegs - 1) / kScanSegs;
    const int b0 = min(nblocks, seg * per), b1 = min(nblocks, b0 + per);
    int s = 0;
    for (int b = b0; b < b1; ++b) s += table[(size_t)b * E + e];
    const int incl = group_inclusive_scan(s, lane, 64);
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int run = incl - s, total = 0;
    for (int w = 0; w < kScanWaves; ++w) {
        if (w < wave) run += wave_total[w];
        total += wave_total[w];
    }
    for (int b = b0; b < b1; ++b) {
        const int t = table[(size_t)b * E + e];
        table[(size_t)b * E + e] = run;
        run += t;
    }
    if (seg == 0) {
        counts_raw[e] = total;
        counts[e] = (capacity >= 0 && total > capacity) ? (int)capacity : total;
    }
}

// FUSED = false: `table` holds the exclusive per-expert prefixes and counts_raw / counts the totals written by
// dispatch_scan_kernel; every block derives the per-expert offsets from the counts and block 0 writes them out.
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
    __shared__ int s_off[65];      // per-expert offsets
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
        if (tid < 64) {   // one wavefront: lane x owns expert x
            const int c = tid < E ? counts[tid] : 0;
            const int incl = group_inclusive_scan(c, tid, 64);
            if (tid < E) {
                s_off[tid] = incl - c;
                if (blockIdx.x == 0) offsets[tid] = incl - c;
            }
            if (tid == E - 1) {
                s_off[E] = incl;
                if (blockIdx.x == 0) offsets[E] = incl;
            }
            if (stats_block && stats) load_stats_wave(tid < E ? counts_raw[tid] : 0, c, tid < E, E, stats);
        }
        if (stats_block) return;
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
            const int row = s_off[e] + rank;
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
    dispatch_scan_kernel<<<c.E, kScanSegs, 0, s>>>(block_counts, nblocks, c.E, cap, counts_raw, counts);
    // without any assignment the one block launched is the statistics block, which also writes the (zero) offsets
    dispatch_scatter_kernel<false><<<nblocks + ((stats || nblocks == 0) ? 1 : 0), kDispThreads, 0, s>>>(
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
