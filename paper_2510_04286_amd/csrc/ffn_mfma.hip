// Grouped expert FFN on the matrix cores (the "fused batched GEMM" of paper Section 3.4, with
// the expert of Section 3.1 and the input weighting of Eq. 1), bf16 inputs, fp32 accumulation.
//
//   y[r, :] = GELU(p_r * (x_r W1[e]) + b1[e]) W2[e] + b2[e]          (p (x W1) == (p x) W1)
//
// One launch covers all experts; the per-expert row ranges come from offsets[] on the device.
// A wavefront owns a unit of 32*NSUB stacked rows and the whole hidden width.  Per 32-wide
// hidden tile it runs GEMM1 (K = ds), applies bias / p / GELU to its 16 accumulators per lane
// and feeds them straight into GEMM2 as the B operand (see mfma.h): the [rows, He] hidden
// activations never exist in memory.  x rows are gathered through perm[] by the loads
// themselves (each lane reads the 16-byte pieces of its own row from h); loads for the next
// unit are issued before the current one is computed.  Weights come pre-packed in fragment
// order and are staged in LDS.  y is written as fp16 (three more mantissa bits than the bf16
// storage type, so the rounding of h' after the k-sum stays the only significant one); the two
// half-wavefronts exchange registers so that every lane stores whole 16-byte pieces of a row.
//
// Two variants:
//   resident  a whole expert (W1, W2, biases) fits in LDS (ds = 64, He = 256: 65 KiB).  One
//             block of 8 wavefronts per CU; stacked rows are split evenly over the blocks
//             regardless of expert boundaries; a block re-stages weights (asynchronous
//             global->LDS loads, overlapped with the first row gather) only when its range
//             crosses into another expert, and its wavefronts run independently in between.
//   streamed  larger experts (ds = 128, He = 512: 256 KiB): a block walks tiles of one expert
//             and streams the weights through LDS in chunks of hidden tiles, per row tile.
#include "mfma.h"

namespace slicemoe {

typedef _Float16 half_t;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// GELU(z) = z * Phi(z) with Phi(z) ~ 0.5 + zc * P(zc^2), zc = clamp(z, -3.5, 3.5), P a degree-5
// minimax polynomial: |Phi error| < 1.8e-4, i.e. a relative error of GELU well below the bf16
// rounding (2^-9) applied to the result.  Horner steps with literal coefficients are the cheapest
// VALU form on gfx950; no transcendental instruction is needed.
__device__ __forceinline__ float gelu_poly(float z)
{
    const float zc = __builtin_amdgcn_fmed3f(z, -3.5f, 3.5f);
    const float w = zc * zc;
    float P = -7.907663110e-07f;
    P = fmaf(P, w, 3.767626183e-05f);
    P = fmaf(P, w, -7.603790386e-04f);
    P = fmaf(P, w, 8.699680533e-03f);
    P = fmaf(P, w, -6.477227479e-02f);
    P = fmaf(P, w, 3.982652909e-01f);
    return z * fmaf(zc, P, 0.5f);
}

template <int DS, int NSUB> struct RowUnit {
    bf16x8 xb[NSUB][DS / 16];
    float p[NSUB];
    int row[NSUB];  // -1: no row
};

// Issue the gather of one unit: lane j of each 32-row sub-tile reads its row's K pieces.
template <int DS, int NSUB>
__device__ __forceinline__ void gather_rows(RowUnit<DS, NSUB> &u, const int (&a)[NSUB], const int (&row)[NSUB],
                                            const bf16_t *__restrict__ x, const float *__restrict__ pk, int k, int g)
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const bool valid = row[sub] >= 0;
        u.row[sub] = row[sub];
        u.p[sub] = valid ? pk[a[sub]] : 0.f;
        const long long n = a[sub] / k;
        const uint4 *xp = (const uint4 *)(x + n * DS);
#pragma unroll
        for (int ks = 0; ks < DS / 16; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (valid) v = xp[ks * 2 + g];
            u.xb[sub][ks] = __builtin_bit_cast(bf16x8, v);
        }
    }
}

// All hidden tiles [ht0, ht0 + nht) staged at w1s / w2s (tile hl at fragment offset hl): GEMM1,
// activation, GEMM2 accumulation into yacc.
template <int DS, int NSUB>
__device__ __forceinline__ void ffn_hidden_tiles(const RowUnit<DS, NSUB> &u, f32x16 (&yacc)[NSUB][DS / 32],
                                                 const uint4 *__restrict__ w1s, const uint4 *__restrict__ w2s,
                                                 const float *__restrict__ b1s, int ht0, int nht, int lane, int g)
{
    constexpr int KS = DS / 16;
    constexpr int OT = DS / 32;
    for (int hl = 0; hl < nht; ++hl) {
        f32x16 acc[NSUB];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[sub][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a1 = __builtin_bit_cast(bf16x8, w1s[(hl * KS + ks) * 64 + lane]);
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) acc[sub] = mfma_bf16(a1, u.xb[sub][ks], acc[sub]);
        }
        f32x4 bq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) bq[q] = *(const f32x4 *)(b1s + (ht0 + hl) * 32 + 8 * q + 4 * g);
        bf16x8 hb[NSUB][2];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float z = fmaf(acc[sub][r], u.p[sub], bq[r >> 2][r & 3]);
                hb[sub][r >> 3][r & 7] = (__bf16)gelu_poly(z);
            }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                const bf16x8 a2 = __builtin_bit_cast(bf16x8, w2s[((hl * 2 + s) * OT + ot) * 64 + lane]);
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) yacc[sub][ot] = mfma_bf16(a2, hb[sub][s], yacc[sub][ot]);
            }
    }
}

__device__ __forceinline__ uint32_t pack_half2(float a, float b)
{
    f16x2 v;
    v[0] = (half_t)a;
    v[1] = (half_t)b;
    return __builtin_bit_cast(uint32_t, v);
}

// y rows as fp16.  Per output tile a lane holds features 8q + 4g + (0..3) of its own row, i.e. half
// of each 16-byte piece; lanes j and j + 32 trade halves (v_permlane32_swap) so that lane (j, g)
// ends up with the whole pieces q = 2*qp + g and stores them with one 16-byte write each.
template <int DS, int NSUB>
__device__ __forceinline__ void store_rows(const RowUnit<DS, NSUB> &u, const f32x16 (&yacc)[NSUB][DS / 32],
                                           const float *__restrict__ b2s, half_t *__restrict__ y, int g)
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        half_t *yr = y + (size_t)(u.row[sub] < 0 ? 0 : u.row[sub]) * DS;
#pragma unroll
        for (int ot = 0; ot < DS / 32; ++ot)
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) {
                uint32_t lo[2], hi[2];  // lo: piece q = 2qp, hi: piece q = 2qp + 1 (this lane's half of each)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int q = 2 * qp + t;
                    const f32x4 bb = *(const f32x4 *)(b2s + ot * 32 + 8 * q + 4 * g);
                    const uint32_t d0 = pack_half2(yacc[sub][ot][4 * q + 0] + bb[0], yacc[sub][ot][4 * q + 1] + bb[1]);
                    const uint32_t d1 = pack_half2(yacc[sub][ot][4 * q + 2] + bb[2], yacc[sub][ot][4 * q + 3] + bb[3]);
                    if (t == 0) {
                        lo[0] = d0;
                        lo[1] = d1;
                    } else {
                        hi[0] = d0;
                        hi[1] = d1;
                    }
                }
                // after the swaps: lanes 0-31 hold (own lo, partner's lo) = piece 2qp; lanes 32-63 hold
                // (partner's hi, own hi) = piece 2qp + 1, both in feature order
                const auto s0 = __builtin_amdgcn_permlane32_swap(lo[0], hi[0], false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(lo[1], hi[1], false, false);
                if (u.row[sub] >= 0) {
                    const uint4 v = make_uint4(s0[0], s1[0], s0[1], s1[1]);
                    *(uint4 *)(yr + ot * 32 + 8 * (2 * qp + g)) = v;
                }
            }
    }
}

template <int DS, int NSUB>
__device__ __forceinline__ void zero_acc(f32x16 (&yacc)[NSUB][DS / 32])
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int ot = 0; ot < DS / 32; ++ot)
#pragma unroll
            for (int r = 0; r < 16; ++r) yacc[sub][ot][r] = 0.f;
}

// Asynchronous copy of n16 16-byte pieces from global memory to LDS by the whole block: each
// wavefront-level instruction moves 1 KiB (lane i -> dst + 16*i) without passing through registers.
// The caller waits (vmcnt) and synchronises before reading.
template <int THREADS>
__device__ __forceinline__ void async_copy_to_lds(const uint4 *__restrict__ src, uint4 *dst, int n16, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    for (int c = wave; c < n16 / 64; c += THREADS / 64)
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)(src + c * 64 + lane),
                                         (void __attribute__((address_space(3))) *)(dst + c * 64), 16, 0, 0);
}

// ------------------------------------------------------------------------------ resident
constexpr int kResThreads = 512;
constexpr int kResWaves = kResThreads / 64;

template <int DS, int NSUB>
__global__ __launch_bounds__(kResThreads, 2) void ffn_resident_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const char *__restrict__ experts, size_t e_stride, size_t off_w1,
    size_t off_w2, size_t off_b1, size_t off_b2, int He, int E, int k, half_t *__restrict__ y)
{
    constexpr int KS = DS / 16;
    constexpr int OT = DS / 32;
    constexpr int U = 32 * NSUB;  // rows per wavefront unit
    const int HT = He / 32;

    extern __shared__ __align__(16) char lds[];
    uint4 *w1s = (uint4 *)lds;                                // [HT][KS][64] fragments
    uint4 *w2s = w1s + (size_t)HT * KS * 64;                  // [HT][2][OT][64] fragments
    float *b1s = (float *)(w2s + (size_t)HT * 2 * OT * 64);   // [He]
    float *b2s = b1s + He;                                    // [DS]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 31;
    const int g = lane >> 5;

    // lane e keeps the end of expert e's row range: expert lookups are one ballot, not a chain of loads
    const int off_hi = offsets[min(lane + 1, E)];
    const int n_kept = __shfl(off_hi, E - 1);

    // even split of the kept rows over the blocks, in whole units
    const int units_total = (n_kept + U - 1) / U;
    const int units_per_block = (units_total + gridDim.x - 1) / gridDim.x;
    const long long r_begin = (long long)blockIdx.x * units_per_block * U;
    const int r_end = (int)min((long long)n_kept, r_begin + (long long)units_per_block * U);

    int r = (int)min(r_begin, (long long)n_kept);
    while (r < r_end) {
        const int e = __popcll(__ballot(lane < E && off_hi <= r));
        const int seg_end = min(__shfl(off_hi, e), r_end);
        const char *ew = experts + (size_t)e * e_stride;

        // units of this segment: unit q covers rows r + q*U ..., this wavefront takes q = wave, wave+8, ...
        const int nunits = (seg_end - r + U - 1) / U;
        auto unit_rows = [&](int q, int (&row)[NSUB]) {
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) {
                const int rr = r + q * U + sub * 32 + j;
                row[sub] = (q < nunits && rr < seg_end) ? rr : -1;
            }
        };
        auto load_perm = [&](const int (&row)[NSUB], int (&a)[NSUB]) {
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) a[sub] = row[sub] >= 0 ? perm[row[sub]] : 0;
        };
        // row indices of the first two units go out first, the weight copy overlaps their latency
        int row_c[NSUB], a_c[NSUB], row_n[NSUB], a_n[NSUB];
        unit_rows(wave, row_c);
        load_perm(row_c, a_c);
        unit_rows(wave + kResWaves, row_n);
        load_perm(row_n, a_n);

        __syncthreads();  // everyone is done with the previous expert's weights
        async_copy_to_lds<kResThreads>((const uint4 *)(ew + off_w1), w1s, HT * KS * 64, tid);
        async_copy_to_lds<kResThreads>((const uint4 *)(ew + off_w2), w2s, HT * 2 * OT * 64, tid);
        {
            const float *gb1 = (const float *)(ew + off_b1);
            const float *gb2 = (const float *)(ew + off_b2);
            for (int i = tid; i < He; i += kResThreads) b1s[i] = gb1[i];
            for (int i = tid; i < DS; i += kResThreads) b2s[i] = gb2[i];
        }
        RowUnit<DS, NSUB> cur;
        gather_rows<DS, NSUB>(cur, a_c, row_c, x, pk, k, g);
        __builtin_amdgcn_s_waitcnt(0);  // the asynchronous copies have landed
        __syncthreads();

        for (int q = wave; q < nunits; q += kResWaves) {
            // next unit's rows (indices arrived during the previous unit), indices of the one after
            RowUnit<DS, NSUB> nxt;
            gather_rows<DS, NSUB>(nxt, a_n, row_n, x, pk, k, g);
            unit_rows(q + 2 * kResWaves, row_n);
            load_perm(row_n, a_n);

            f32x16 yacc[NSUB][OT];
            zero_acc<DS, NSUB>(yacc);
            ffn_hidden_tiles<DS, NSUB>(cur, yacc, w1s, w2s, b1s, 0, HT, lane, g);
            store_rows<DS, NSUB>(cur, yacc, b2s, y, g);
            cur = nxt;
        }
        r = seg_end;
    }
}

// ------------------------------------------------------------------------------ streamed
constexpr int kFfnThreads = 256;
constexpr int kFfnWaves = kFfnThreads / 64;

template <int DS, int NSUB>
__global__ __launch_bounds__(kFfnThreads) void ffn_streamed_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const char *__restrict__ experts, size_t e_stride, size_t off_w1,
    size_t off_w2, size_t off_b1, size_t off_b2, int He, int E, int k, int hc, half_t *__restrict__ y)
{
    constexpr int KS = DS / 16;
    constexpr int OT = DS / 32;
    constexpr int TM = kFfnWaves * NSUB * 32;
    const int HT = He / 32;
    const int nchunks = HT / hc;

    extern __shared__ __align__(16) char lds[];
    uint4 *w1s = (uint4 *)lds;                                     // [hc][KS][64] fragments
    uint4 *w2s = w1s + (size_t)hc * KS * 64;                       // [hc][2][OT][64] fragments
    float *b1s = (float *)(w2s + (size_t)hc * 2 * OT * 64);        // [He]
    float *b2s = b1s + He;                                         // [DS]
    int *tile_prefix = (int *)(b2s + DS);                          // [E+1]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 31;
    const int g = lane >> 5;

    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            tile_prefix[e] = run;
            run += (offsets[e + 1] - offsets[e] + TM - 1) / TM;
        }
        tile_prefix[E] = run;
    }
    __syncthreads();
    const int total = tile_prefix[E];
    const int per_block = (total + gridDim.x - 1) / gridDim.x;
    const int t_begin = blockIdx.x * per_block;
    const int t_end = min(total, t_begin + per_block);

    int cur_e = -1;
    int e = 0;
    for (int t = t_begin; t < t_end; ++t) {
        while (tile_prefix[e + 1] <= t) ++e;
        const int row_begin = offsets[e] + (t - tile_prefix[e]) * TM;
        const int row_end = offsets[e + 1];
        const char *ew = experts + (size_t)e * e_stride;
        const bool new_expert = e != cur_e;

        int row[NSUB], a[NSUB];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            const int rr = row_begin + (wave * NSUB + sub) * 32 + j;
            row[sub] = rr < row_end ? rr : -1;
            a[sub] = row[sub] >= 0 ? perm[rr] : 0;
        }
        RowUnit<DS, NSUB> cur;
        gather_rows<DS, NSUB>(cur, a, row, x, pk, k, g);

        f32x16 yacc[NSUB][OT];
        zero_acc<DS, NSUB>(yacc);
        for (int ch = 0; ch < nchunks; ++ch) {
            __syncthreads();  // everyone is done with the previous contents
            async_copy_to_lds<kFfnThreads>((const uint4 *)(ew + off_w1) + (size_t)ch * hc * KS * 64, w1s, hc * KS * 64, tid);
            async_copy_to_lds<kFfnThreads>((const uint4 *)(ew + off_w2) + (size_t)ch * hc * 2 * OT * 64, w2s,
                                           hc * 2 * OT * 64, tid);
            if (new_expert && ch == 0) {
                const float *gb1 = (const float *)(ew + off_b1);
                const float *gb2 = (const float *)(ew + off_b2);
                for (int i = tid; i < He; i += kFfnThreads) b1s[i] = gb1[i];
                for (int i = tid; i < DS; i += kFfnThreads) b2s[i] = gb2[i];
            }
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            ffn_hidden_tiles<DS, NSUB>(cur, yacc, w1s, w2s, b1s, ch * hc, hc, lane, g);
        }
        cur_e = e;
        store_rows<DS, NSUB>(cur, yacc, b2s, y, g);
    }
}

struct FfnPlan {
    bool resident;
    int hc;
    size_t lds;
};

// Whole expert resident in LDS when it fits in half of a CU's LDS, else hidden tiles per chunk.
static FfnPlan plan_ffn(int ds, int He, int E)
{
    const int HT = He / 32, KS = ds / 16, OT = ds / 32;
    const size_t frag_per_ht = (size_t)(KS + 2 * OT) * 1024;  // bytes of W1+W2 fragments per hidden tile
    const size_t dev_max = (size_t)max_lds_per_block();
    FfnPlan p;
    const size_t resident_bytes = frag_per_ht * HT + (size_t)(He + ds) * 4;
    if (ds == 64 && resident_bytes <= 78 * 1024 && resident_bytes <= dev_max) {
        p.resident = true;
        p.hc = HT;
        p.lds = resident_bytes;
        return p;
    }
    // a streamed block needs the whole register file of its CU anyway, so chunks may take most of the LDS
    const size_t fixed = (size_t)(He + ds + E + 1) * 4 + 64;
    const size_t want = 140 * 1024;
    const size_t budget = dev_max < want ? dev_max : want;
    p.resident = false;
    p.hc = 1;
    for (int c = HT; c >= 1; --c)
        if (HT % c == 0 && frag_per_ht * c + fixed <= budget) {
            p.hc = c;
            break;
        }
    p.lds = frag_per_ht * p.hc + fixed;
    return p;
}

template <int DS, int NSUB>
static hipError_t run_ffn(const slicemoe_config &c, const FfnPlan &pl, const void *h, const float *p,
                          const int32_t *offsets, const int32_t *perm, const void *packed, void *y,
                          hipStream_t s)
{
    const PackedLayout L = packed_layout(c);
    const long long Na = (long long)c.T * c.S * c.k;
    const char *experts = (const char *)packed + L.experts;
    hipError_t err;
    if constexpr (DS == 64) {
        if (pl.resident) {
            constexpr int U = 32 * NSUB;
            long long blocks = (long long)num_compute_units();
            const long long max_blocks = (Na + U - 1) / U;
            if (blocks > max_blocks) blocks = max_blocks;
            auto kern = ffn_resident_kernel<DS, NSUB>;
            err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds);
            if (err != hipSuccess) return err;
            kern<<<(int)blocks, kResThreads, pl.lds, s>>>((const bf16_t *)h, p, offsets, perm, experts, L.e_stride,
                                                          L.e_w1, L.e_w2, L.e_b1, L.e_b2, c.He, c.E, c.k, (half_t *)y);
            return hipGetLastError();
        }
    }
    constexpr int TM = kFfnWaves * NSUB * 32;
    const long long max_tiles = (Na + TM - 1) / TM + c.E;
    long long blocks = (long long)num_compute_units() * (pl.lds <= 78 * 1024 ? 2 : 1);
    if (blocks > max_tiles) blocks = max_tiles;
    auto kern = ffn_streamed_kernel<DS, NSUB>;
    err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds);
    if (err != hipSuccess) return err;
    kern<<<(int)blocks, kFfnThreads, pl.lds, s>>>((const bf16_t *)h, p, offsets, perm, experts, L.e_stride, L.e_w1,
                                                  L.e_w2, L.e_b1, L.e_b2, c.He, c.E, c.k, pl.hc, (half_t *)y);
    return hipGetLastError();
}

hipError_t launch_ffn_mfma(const slicemoe_config &c, const void *h, const float *p,
                           const int32_t *offsets, const int32_t *perm, const void *packed,
                           void *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    if (Na == 0) return hipSuccess;
    const int ds = c.d / c.S;
    const FfnPlan pl = plan_ffn(ds, c.He, c.E);
    if (ds == 64) return run_ffn<64, 2>(c, pl, h, p, offsets, perm, packed, y, s);
    return run_ffn<128, 2>(c, pl, h, p, offsets, perm, packed, y, s);
}

}  // namespace slicemoe
