// Dispatch stage: stable counting sort of slice->expert assignments (the grouping of paper
// Section 3.4), with an optional per-expert capacity, plus the load statistics of Eq. 2 and
// of the ELE metric (Section 4).
//
// Assignment ids a = n*k + j are cut into chunks of `chunk` consecutive ids.  The work is
//   1. histogram   table[e][c] = # assignments of chunk c bound for expert e (expert-major: the row of an expert is
//                  contiguous, `stride` ints apart).  Either dispatch_hist_kernel, or the router kernel, which holds
//                  the selected experts in registers anyway and writes the same table from its epilogue; then this
//                  stage reads the routing table only once.
//   2. scan        exclusive prefix over the chunks of every expert (the rank of a chunk's first assignment inside its
//                  expert) and the per-expert totals -> counts_raw, counts.
//   3. scatter     offsets from the counts, stable rank of every assignment inside its chunk, final row, perm / inv;
//                  one extra block computes the load statistics from the counts.
// When the table is small (the headline has 512 chunks x 32 experts) step 2 is folded into step 3: every scatter
// block sums the table itself, with coalesced 16-byte loads that are in flight together with the block's loads of the
// routing table, which is cheaper than a third latency-bound launch.  What that costs is the table's bytes times the
// number of blocks through every CU's memory pipeline, so such a table holds 16-bit counts and a scatter block covers
// several of its chunks.
// Stability needs ranks in ascending a.  A block walks its chunk in rounds of 256 consecutive ids; inside a wavefront
// the rank among equal experts comes from ballots (one per bit of the expert id gives every lane the mask of lanes
// holding the same expert), across wavefronts and rounds from a small LDS table scanned in (round, wavefront) order.
#include <mutex>

#include "common.h"

namespace slicemoe {

constexpr int kDispWaves = kDispThreads / 64;
constexpr int kHistThreads = 256;

// Table chunks of the stage entry point: 1024 assignments, more for batches beyond 4096 of those.  A scatter block
// covers about 2048 assignments (one wavefront per SIMD of a CU doing eight rounds: the rank computation is a few
// dozen vector instructions per round, so the work wants to be spread over every SIMD of the chip), i.e. `group`
// chunks of the table, at most kDispMaxItems rounds of kDispThreads ids.
DispatchGeom dispatch_geometry(long long Na, int E, int chunk)
{
    DispatchGeom g;
    if (chunk > 0) {
        g.chunk = chunk;
    } else {
        g.chunk = 1024;
        while (g.chunk < kDispThreads * kDispMaxItems && (Na + g.chunk - 1) / g.chunk > 4096) g.chunk *= 2;
    }
    g.nchunks = (int)((Na + g.chunk - 1) / g.chunk);
    g.stride = (g.nchunks + 7) / 8 * 8;
    if (g.stride == 0) g.stride = 8;
    // small table: a scatter block reads it with at most 16 loads per lane (a row of 128 chunks per load of a
    // quarter-wavefront, 16 rows per pass): up to 2048 chunks of 16 experts, 512 of 64
    g.fused = g.nchunks > 0 && (long long)((g.stride + 127) / 128) * ((E + 15) / 16) <= 16;
    g.group = 2048 / g.chunk;
    if (g.group < 1) g.group = 1;
    g.blocks = (g.nchunks + g.group - 1) / g.group;
    return g;
}

size_t dispatch_table_bytes(const DispatchGeom &g, int E) { return align_up((size_t)g.stride * E * sizeof(int32_t), 256); }

// Lanes of the wavefront that hold the same expert as this lane, as the two words of a 64-bit mask: one ballot per
// bit of the expert id.
struct LaneMask {
    uint32_t lo, hi;
};
__device__ __forceinline__ LaneMask same_expert_mask(int e, bool valid, int nbits)
{
    const unsigned long long all = __ballot(valid);
    LaneMask m = {(uint32_t)all, (uint32_t)(all >> 32)};
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long bal = __ballot(valid && bit);
        const uint32_t flip = bit ? 0u : ~0u;   // lanes without the bit want the complement
        m.lo &= (uint32_t)bal ^ flip;
        m.hi &= (uint32_t)(bal >> 32) ^ flip;
    }
    return m;
}
// set bits of the mask in lanes below this one / in all lanes
__device__ __forceinline__ int count_below(LaneMask m) { return (int)__builtin_amdgcn_mbcnt_hi(m.hi, __builtin_amdgcn_mbcnt_lo(m.lo, 0u)); }
__device__ __forceinline__ int count_all(LaneMask m) { return __popc(m.lo) + __popc(m.hi); }

// Cross-lane moves inside a row of 16 lanes as data-parallel-primitive modifiers of an ordinary move (no LDS round
// trip).  Lanes whose source does not exist read zero.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppQuadShr1 = 0x90;       // quad_perm [0,0,1,2]: lane i of a quad reads lane i-1 (lane 0 itself)
constexpr int kDppQuadShr2 = 0x44;       // quad_perm [0,1,0,1]: lane i of a quad reads lane i-2 (lanes 0, 1 themselves)
constexpr int kDppRowHalfMirror = 0x141; // lane i of a half-row of 8 reads lane 7-i
constexpr int kDppRowMirror = 0x140;     // lane i of a row reads lane 15-i
// sum over the 4 lanes of a quad / the 16 lanes of a row, in every lane of it
__device__ __forceinline__ int quad_sum(int v)
{
    v += dpp_move<kDppQuadSwap1>(v);
    v += dpp_move<kDppQuadSwap2>(v);
    return v;
}
__device__ __forceinline__ int row_sum(int v)
{
    v = quad_sum(v);
    v += dpp_move<kDppRowHalfMirror>(v);
    v += dpp_move<kDppRowMirror>(v);
    return v;
}
// inclusive prefix sum over the 4 lanes of a quad (w = lane % 4)
__device__ __forceinline__ int quad_inclusive_scan(int v, int w)
{
    const int a = dpp_move<kDppQuadShr1>(v);
    v += w >= 1 ? a : 0;
    const int b = dpp_move<kDppQuadShr2>(v);
    v += w >= 2 ? b : 0;
    return v;
}

__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

__global__ __launch_bounds__(kHistThreads) void dispatch_hist_kernel(
    const int32_t *__restrict__ idx, int Na, int E, int nbits, int chunk, int stride, void *__restrict__ table, bool narrow)
{
    __shared__ int cnt[64];
    const int tid = threadIdx.x;
    if (tid < 64) cnt[tid] = 0;
    __syncthreads();
    const long long base = (long long)blockIdx.x * chunk;
    for (int r0 = 0; r0 < chunk; r0 += 4 * kHistThreads) {   // four rounds of ids requested at a time
        int ev[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = r0 + i * kHistThreads;
            const long long a = base + r + tid;
            ev[i] = (r + tid < chunk && a < Na) ? idx[a] : 0;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = r0 + i * kHistThreads;
            const long long a = base + r + tid;
            const bool valid = r + tid < chunk && a < Na;
            const int e = valid ? clamp_expert(ev[i], E) : 0;
            const LaneMask m = same_expert_mask(e, valid, nbits);
            if (valid && count_below(m) == 0) atomicAdd(&cnt[e], count_all(m));
        }
    }
    __syncthreads();
    if (tid < E) {
        if (narrow) {
            uint16_t *row = (uint16_t *)table + (size_t)tid * stride;
            row[blockIdx.x] = (uint16_t)cnt[tid];
            if (blockIdx.x == gridDim.x - 1)   // the padding of a row of 16-bit counts reads as zero
                for (int c = (int)gridDim.x; c < stride; ++c) row[c] = 0;
        } else {
            ((int32_t *)table)[(size_t)tid * stride + blockIdx.x] = cnt[tid];
        }
    }
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

__device__ __forceinline__ int wave_sum(int v)
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

// Large tables: one block per expert walks that expert's row (contiguous memory).  Thread `seg` owns a run of
// consecutive chunks: it sums the run, the run sums are scanned (shuffles inside a wavefront, a small LDS table
// across), and the thread rewrites its run as exclusive prefixes.  The expert's total goes to counts_raw and, capped,
// to counts; the scatter kernel turns the counts into offsets.
constexpr int kScanWaves = 16, kScanSegs = kScanWaves * 64;
__global__ __launch_bounds__(kScanSegs) void dispatch_scan_kernel(
    int32_t *__restrict__ table, int nchunks, int stride, long long capacity, int32_t *__restrict__ counts_raw,
    int32_t *__restrict__ counts)
{
    __shared__ int wave_total[kScanWaves];
    const int seg = threadIdx.x, lane = seg & 63, wave = seg >> 6;
    const int e = (int)blockIdx.x;   // < E by the launch
    int32_t *row = table + (size_t)e * stride;
    const int per = (nchunks + kScanSegs - 1) / kScanSegs;
    const int b0 = min(nchunks, seg * per), b1 = min(nchunks, b0 + per);
    constexpr int kRun = 8;   // runs up to this long are held in registers: one round trip to memory, not one per chunk
    int vals[kRun];
    int s = 0;
    if (per <= kRun) {
#pragma unroll
        for (int i = 0; i < kRun; ++i) vals[i] = b0 + i < b1 ? row[b0 + i] : 0;
#pragma unroll
        for (int i = 0; i < kRun; ++i) s += vals[i];
    } else {
        for (int b = b0; b < b1; ++b) s += row[b];
    }
    const int incl = group_inclusive_scan(s, lane, 64);
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int run = incl - s, total = 0;
    for (int w = 0; w < kScanWaves; ++w) {
        if (w < wave) run += wave_total[w];
        total += wave_total[w];
    }
    if (per <= kRun) {
#pragma unroll
        for (int i = 0; i < kRun; ++i) {
            if (b0 + i < b1) row[b0 + i] = run;
            run += vals[i];
        }
    } else {
        for (int b = b0; b < b1; ++b) {
            const int t = row[b];
            row[b] = run;
            run += t;
        }
    }
    if (seg == 0) {
        counts_raw[e] = total;
        counts[e] = (capacity >= 0 && total > capacity) ? (int)capacity : total;
    }
}

// A scatter block (four wavefronts) covers `group` consecutive chunks of the table: bchunk = group * chunk assignment
// ids, walked in rounds of 256.
// FUSED = false: the rows of `table` (int32) hold the exclusive per-expert prefixes and counts_raw / counts the totals
// written by dispatch_scan_kernel.
// FUSED = true (small tables): there is no scan kernel and `table` holds the raw per-chunk counts as 16-bit values (a
// chunk has at most 4096 assignments; the padding of a row is zero).  Every block sums the whole table itself: a
// quarter-wavefront per expert row (16 lanes x 16 bytes = 128 chunks per load, every load of a row in flight at
// once), 16 rows per pass, into the expert's total and the prefix of the block's first chunk.  The eight counts of a
// piece are added as packed pairs; only the one piece of a row that straddles the block's first chunk is taken apart.
// Either way every block derives counts and offsets itself and block 0 writes counts_raw / counts / offsets for the
// stages that follow.  ITEMS: rounds the block may walk; `items` of them are in use.
template <bool FUSED, int ITEMS>
__global__ __launch_bounds__(kDispThreads) void dispatch_scatter_kernel(
    const int32_t *__restrict__ idx, int Na, int E, int nbits, long long capacity, int chunk, int group, int items,
    const void *__restrict__ table_, int stride, int nchunks, int nblocks, int32_t *__restrict__ offsets,
    int32_t *__restrict__ perm, int32_t *__restrict__ inv, int32_t *__restrict__ counts_raw,
    int32_t *__restrict__ counts, float *__restrict__ stats /* may be null */)
{
    __shared__ int wcnt[ITEMS][kDispWaves][64];
    __shared__ int s_tot[64];      // per-expert totals
    __shared__ int s_pre[64];      // rank of this block's first assignment inside each expert
    __shared__ int s_off[65];      // per-expert offsets
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int me = (int)blockIdx.x;
    const bool stats_block = me == nblocks;   // one extra block: the load statistics, off everyone's critical path
    const int first = stats_block ? nchunks : me * group;   // first table chunk of this block
    const int bchunk = group * chunk;

    // this block's part of the routing table, requested before anything else
    const int base = me * bchunk;   // < Na + bchunk: fits an int because Na < 2^31 - 2^12 is checked by the launcher
    int ex[ITEMS];
    unsigned have = 0;   // bit i: round i holds an assignment for this thread
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int r = i * kDispThreads + tid;
        const bool valid = i < items && !stats_block && r < bchunk && base + r < Na;
        ex[i] = valid ? idx[base + r] : 0;
        have |= valid ? 1u << i : 0u;
    }

    // FUSED: the table, at most 16 pieces per lane (a quarter-wavefront per expert row, 16 rows per pass, the passes
    // and the pieces of a row flattened into one sequence), requested right behind the routing table and summed only
    // after the ranks below, which need the routing table alone
    const int gl = lane & 15;
    const int pieces = stride / 8;                   // 16-byte pieces (8 chunks) per row, at most 256
    const int per_row = (pieces + 15) / 16;           // pieces of a row per lane
    const int n_loads = FUSED ? per_row * ((E + 15) / 16) : 0;   // <= 16 by the limits of the fused path
    uint4 v[16];
    if constexpr (FUSED) {
        const uint16_t *table = (const uint16_t *)table_;
        int q = 0, it = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (j < n_loads) {
                const int e = min(q * 16 + wave * 4 + (lane >> 4), E - 1);
                v[j] = ((const uint4 *)(table + (size_t)e * stride))[min(gl + 16 * it, pieces - 1)];
                if (++it == per_row) {
                    it = 0;
                    ++q;
                }
            }
        }
    } else {
        const int32_t *table = (const int32_t *)table_;
        if (tid < E) {
            s_tot[tid] = counts_raw[tid];
            s_pre[tid] = stats_block ? 0 : table[(size_t)tid * stride + first];
        }
    }

    // ranks inside the wavefront: one ballot per bit of the expert id, the rounds side by side so that their chains
    // of dependent vector -> scalar -> vector steps overlap.  The wavefront first clears its own rows of the table of
    // counts (LDS executes the operations of one wavefront in order, so no barrier is needed in between).
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
        if (i < items) wcnt[i][wave][lane] = 0;
    LaneMask m[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool valid = (have >> i) & 1u;
        ex[i] = valid ? clamp_expert(ex[i], E) : -1;
        const unsigned long long all = __ballot(valid);
        m[i].lo = (uint32_t)all;
        m[i].hi = (uint32_t)(all >> 32);
    }
    for (int b = 0; b < nbits; ++b) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool bit = ex[i] >= 0 && ((ex[i] >> b) & 1);
            const unsigned long long bal = __ballot(bit);
            const uint32_t flip = ((ex[i] >> b) & 1) ? 0u : ~0u;   // lanes without the bit want the complement
            m[i].lo &= (uint32_t)bal ^ flip;
            m[i].hi &= (uint32_t)(bal >> 32) ^ flip;
        }
    }
    int rk[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        rk[i] = count_below(m[i]);
        if (i < items && ex[i] >= 0 && rk[i] == 0) wcnt[i][wave][ex[i]] = count_all(m[i]);
    }

    if constexpr (FUSED) {
        // the one piece of a row that straddles the block's first chunk: its leading `first % 8` counts precede it
        const int pfull = first >> 3, lead = first & 7;
        uint32_t lead_mask[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) lead_mask[h] = lead >= 2 * h + 2 ? 0xFFFFFFFFu : (lead == 2 * h + 1 ? 0x0000FFFFu : 0u);
        int q = 0, it = 0, tot = 0, pre = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (j < n_loads) {
                const int p = gl + 16 * it;
                // eight 16-bit counts added as packed pairs (two sums of four, below 2^16 each)
                const uint32_t pairs = v[j].x + v[j].y + v[j].z + v[j].w;
                const uint32_t lead_pairs = (v[j].x & lead_mask[0]) + (v[j].y & lead_mask[1]) + (v[j].z & lead_mask[2]) +
                                            (v[j].w & lead_mask[3]);
                const int sum = (int)(pairs & 0xFFFFu) + (int)(pairs >> 16);
                const int lead_sum = (int)(lead_pairs & 0xFFFFu) + (int)(lead_pairs >> 16);
                tot += p < pieces ? sum : 0;
                pre += p < pfull ? sum : (p == pfull ? lead_sum : 0);
                if (++it == per_row) {   // the row is complete: reduce over its 16 lanes
                    tot = row_sum(tot);
                    pre = row_sum(pre);
                    const int e = q * 16 + wave * 4 + (lane >> 4);
                    if (e < E && gl == 0) {
                        s_tot[e] = tot;
                        s_pre[e] = pre;
                    }
                    tot = pre = 0;
                    it = 0;
                    ++q;
                }
            }
        }
    }
    __syncthreads();

    if (tid < 64) {   // one wavefront: lane x owns expert x
        const int raw = tid < E ? s_tot[tid] : 0;
        const int c = FUSED ? ((capacity >= 0 && raw > capacity) ? (int)capacity : raw) : (tid < E ? counts[tid] : 0);
        const int incl = group_inclusive_scan(c, tid, 64);
        if (tid < E) {
            s_off[tid] = incl - c;
            if (me == 0) {
                offsets[tid] = incl - c;
                if (FUSED) {
                    counts_raw[tid] = raw;
                    counts[tid] = c;
                }
            }
        }
        if (tid == E - 1) {
            s_off[E] = incl;
            if (me == 0) offsets[E] = incl;
        }
        if (stats_block && stats) load_stats_wave(raw, c, tid < E, E, stats);
    }
    if (stats_block) return;
    {   // exclusive prefix over (round, wavefront) of every expert's counts, starting from the block's own rank: four
        // threads per expert, one per wavefront column, walking the rounds; then a scan across the four
        const int e = tid >> 2, w = tid & 3;
        int vals[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) vals[i] = i < items ? wcnt[i][w][e] : 0;
        // the order is (round, wavefront): an entry's prefix is everything of earlier rounds plus the earlier
        // wavefronts of its own round
        int run = s_pre[e];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int incl = quad_inclusive_scan(vals[i], w);
            if (i < items) wcnt[i][w][e] = run + incl - vals[i];
            run += quad_sum(vals[i]);
        }
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        if (i >= items) continue;
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

template <bool FUSED>
static void run_scatter(int grid, hipStream_t s, const int32_t *idx, int Na, int E, int nbits, long long cap,
                        const DispatchGeom &g, const void *table, int32_t *offsets, int32_t *perm, int32_t *inv,
                        int32_t *counts_raw, int32_t *counts, float *stats)
{
    const int items = (g.group * g.chunk + kDispThreads - 1) / kDispThreads;
    if (items <= 4)
        dispatch_scatter_kernel<FUSED, 4><<<grid, kDispThreads, 0, s>>>(idx, Na, E, nbits, cap, g.chunk, g.group, items, table, g.stride,
                                                                        g.nchunks, g.blocks, offsets, perm, inv, counts_raw, counts, stats);
    else if (items <= 8)
        dispatch_scatter_kernel<FUSED, 8><<<grid, kDispThreads, 0, s>>>(idx, Na, E, nbits, cap, g.chunk, g.group, items, table, g.stride,
                                                                        g.nchunks, g.blocks, offsets, perm, inv, counts_raw, counts, stats);
    else
        dispatch_scatter_kernel<FUSED, 16><<<grid, kDispThreads, 0, s>>>(idx, Na, E, nbits, cap, g.chunk, g.group, items, table, g.stride,
                                                                         g.nchunks, g.blocks, offsets, perm, inv, counts_raw, counts, stats);
}

// table_chunk = 0: the histogram is computed here, in chunks of this stage's own choice.  table_chunk > 0: `table`
// already holds it in chunks of table_chunk assignments (the router wrote it, in the entry width dispatch_geometry
// names for that chunk size).
hipError_t launch_dispatch(const slicemoe_config &c, const int32_t *idx, int32_t *counts_raw,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                           int32_t *table, float *stats, hipStream_t s, int table_chunk)
{
    const long long Na = (long long)c.T * c.S * c.k;
    const DispatchGeom g = dispatch_geometry(Na, c.E, table_chunk);
    if ((g.group * g.chunk + kDispThreads - 1) / kDispThreads > kDispMaxItems) return hipErrorInvalidValue;
    if (Na > 0x7FFFFFFFll - kDispThreads * kDispMaxItems) return hipErrorInvalidValue;   // ids one block past the end stay ints
    int nbits = 0;
    while ((1 << nbits) < c.E) ++nbits;
    const long long cap = slicemoe_capacity(&c);
    if (g.nchunks > 0 && table_chunk == 0)
        dispatch_hist_kernel<<<g.nchunks, kHistThreads, 0, s>>>(idx, (int)Na, c.E, nbits, g.chunk, g.stride, table, g.fused);
    if (g.fused) {   // small table: every scatter block sums it itself
        run_scatter<true>(g.blocks + (stats ? 1 : 0), s, idx, (int)Na, c.E, nbits, cap, g, table, offsets, perm, inv, counts_raw,
                          counts, stats);
        return hipGetLastError();
    }
    dispatch_scan_kernel<<<c.E, kScanSegs, 0, s>>>(table, g.nchunks, g.stride, cap, counts_raw, counts);
    // without any assignment the one block launched is the statistics block, which also writes the (zero) offsets
    run_scatter<false>(g.blocks + ((stats || g.blocks == 0) ? 1 : 0), s, idx, (int)Na, c.E, nbits, cap, g, table, offsets, perm,
                       inv, counts_raw, counts, stats);
    return hipGetLastError();
}

// ---- the dispatch for callers that cannot allocate -------------------------------------------
// Same kernels, with the per-chunk histogram table in a fixed array of the library's own device image instead of a
// caller's workspace.  Every GPU holds its own copy of the array at its own address: the address is looked up once
// per device, with that device current, and from then on that pointer -- never the array's name, which in host code
// is only a handle for the lookup -- is what the kernels are given.
constexpr size_t kStaticTableInts = 262144;   // 1 MiB
static __device__ __align__(256) int32_t scratch[kStaticTableInts];

static hipError_t static_table(int32_t **out)
{
    static std::mutex mu;
    static int32_t *ptr[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        ptr[dev] = (int32_t *)p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

bool dispatch_static_fits(const slicemoe_config &c)
{
    const DispatchGeom g = dispatch_geometry((long long)c.T * c.S * c.k, c.E, 0);
    return (size_t)g.stride * c.E <= kStaticTableInts;
}

// The table is written in full by the histogram kernel before anything reads it, so nothing has to be cleared; calls
// that overlap on one GPU (two streams) would share it and race.
hipError_t launch_dispatch_static(const slicemoe_config &c, const int32_t *idx, int32_t *counts_raw, int32_t *counts,
                                  int32_t *offsets, int32_t *perm, int32_t *inv, hipStream_t s)
{
    if (!dispatch_static_fits(c)) return hipErrorInvalidValue;
    int32_t *table = nullptr;
    const hipError_t e = static_table(&table);
    if (e != hipSuccess) return e;
    return launch_dispatch(c, idx, counts_raw, counts, offsets, perm, inv, table, nullptr, s, 0);
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
