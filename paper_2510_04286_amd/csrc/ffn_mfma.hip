// Grouped expert FFN on the matrix cores (the "fused batched GEMM" of paper Section 3.4, with
// the expert of Section 3.1 and the input weighting of Eq. 1), bf16 inputs, fp32 accumulation.
//
//   y[r, :] = GELU(p_r * (x_r W1[e]) + b1[e]) W2[e] + b2[e]          (p (x W1) == (p x) W1)
//
// One launch covers all experts.  Work unit: a tile of TM stacked rows of one expert; tiles are
// enumerated on device from offsets[] (expert-major), each block takes a contiguous range of
// tiles, so a block changes expert rarely and re-stages weights only then.  A wavefront owns
// 32*NSUB rows and the whole hidden width; per 32-wide hidden tile it runs GEMM1 (K = ds),
// applies bias/p/GELU to the 16 accumulators per lane, and feeds them straight into GEMM2 as the
// B operand (see mfma.h) -- the [rows, He] hidden activations never exist in memory.
// Expert weights come pre-packed in fragment order and are staged in LDS: all of them when
// they fit (ds = 64, He = 256: 64 KiB + biases), otherwise in chunks of hidden tiles per row tile.
// The gather of x rows through perm[] is done by the loads themselves: a lane reads the
// 16-byte pieces of its own row directly from h in HBM.
#include "mfma.h"

namespace slicemoe {

constexpr int kFfnThreads = 256;
constexpr int kFfnWaves = kFfnThreads / 64;

// tanh-form GELU written as z * sigmoid(2*sqrt(2/pi)*(z + 0.044715 z^3)); exp2 and rcp are single
// hardware instructions.  |error| vs the erf form < 5e-4, below the bf16 rounding applied next.
__device__ __forceinline__ float gelu_fast(float z)
{
    const float c1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    const float c3 = c1 * 0.044715f;
    const float t = z * fmaf(c3, z * z, c1);
    const float e = __builtin_amdgcn_exp2f(t);
    return z * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int DS, int NSUB>
__global__ __launch_bounds__(kFfnThreads) void ffn_mfma_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const char *__restrict__ experts, size_t e_stride, size_t off_w1,
    size_t off_w2, size_t off_b1, size_t off_b2, int He, int E, int k, int hc, float *__restrict__ y)
{
    constexpr int KS = DS / 16;  // K-steps of GEMM1
    constexpr int OT = DS / 32;  // output tiles of GEMM2
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

        // ---- gather this wavefront's rows: B fragments of GEMM1 straight from h
        bf16x8 xb[NSUB][KS];
        float pr[NSUB];
        int row[NSUB];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            row[sub] = row_begin + (wave * NSUB + sub) * 32 + j;
            const bool valid = row[sub] < row_end;
            int a = 0;
            if (valid) a = perm[row[sub]];
            pr[sub] = valid ? pk[a] : 0.f;
            const long long n = a / k;
            const uint4 *xp = (const uint4 *)(x + n * DS);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (valid) v = xp[ks * 2 + g];
                xb[sub][ks] = __builtin_bit_cast(bf16x8, v);
            }
            if (!valid) row[sub] = -1;
        }

        f32x16 yacc[NSUB][OT];
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int r = 0; r < 16; ++r) yacc[sub][ot][r] = 0.f;

        for (int ch = 0; ch < nchunks; ++ch) {
            if (new_expert || nchunks > 1) {
                __syncthreads();  // everyone is done with the previous contents
                const uint4 *g1 = (const uint4 *)(ew + off_w1) + (size_t)ch * hc * KS * 64;
                const uint4 *g2 = (const uint4 *)(ew + off_w2) + (size_t)ch * hc * 2 * OT * 64;
                for (int i = tid; i < hc * KS * 64; i += kFfnThreads) w1s[i] = g1[i];
                for (int i = tid; i < hc * 2 * OT * 64; i += kFfnThreads) w2s[i] = g2[i];
                if (new_expert && ch == 0) {
                    const float *gb1 = (const float *)(ew + off_b1);
                    const float *gb2 = (const float *)(ew + off_b2);
                    for (int i = tid; i < He; i += kFfnThreads) b1s[i] = gb1[i];
                    for (int i = tid; i < DS; i += kFfnThreads) b2s[i] = gb2[i];
                }
                __syncthreads();
            }
            for (int hl = 0; hl < hc; ++hl) {
                const int ht = ch * hc + hl;
                // ---- GEMM1: 32 hidden features x (NSUB*32) rows, K = DS
                f32x16 acc[NSUB];
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[sub][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a1 = __builtin_bit_cast(bf16x8, w1s[(hl * KS + ks) * 64 + lane]);
#pragma unroll
                    for (int sub = 0; sub < NSUB; ++sub) acc[sub] = mfma_bf16(a1, xb[sub][ks], acc[sub]);
                }
                // ---- bias, Eq. 1 weight, GELU, round to bf16: B fragments of GEMM2
                f32x4 bq[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) bq[q] = *(const f32x4 *)(b1s + ht * 32 + 8 * q + 4 * g);
                bf16x8 hb[NSUB][2];
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float z = fmaf(acc[sub][r], pr[sub], bq[r >> 2][r & 3]);
                        hb[sub][r >> 3][r & 7] = (__bf16)gelu_fast(z);
                    }
                // ---- GEMM2: accumulate this hidden tile into the ds outputs
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int ot = 0; ot < OT; ++ot) {
                        const bf16x8 a2 = __builtin_bit_cast(bf16x8, w2s[((hl * 2 + s) * OT + ot) * 64 + lane]);
#pragma unroll
                        for (int sub = 0; sub < NSUB; ++sub)
                            yacc[sub][ot] = mfma_bf16(a2, hb[sub][s], yacc[sub][ot]);
                    }
            }
        }
        cur_e = e;

        // ---- y rows (fp32): lane holds, per output tile, features 8q + 4g + (0..3) of its own row
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            if (row[sub] < 0) continue;
            float *yr = y + (size_t)row[sub] * DS;
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c0 = ot * 32 + 8 * q + 4 * g;
                    const f32x4 bb = *(const f32x4 *)(b2s + c0);
                    f32x4 v;
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[c] = yacc[sub][ot][4 * q + c] + bb[c];
                    *(f32x4 *)(yr + c0) = v;
                }
        }
    }
}

struct FfnPlan {
    int nsub, hc;
    size_t lds;
};

// Pick rows per wavefront and hidden tiles per LDS chunk.
static FfnPlan plan_ffn(int ds, int He, int E)
{
    const int HT = He / 32, KS = ds / 16, OT = ds / 32;
    const size_t frag_per_ht = (size_t)(KS + 2 * OT) * 1024;  // bytes of W1+W2 fragments per hidden tile
    const size_t fixed = (size_t)(He + ds + E + 1) * 4 + 64;
    FfnPlan p;
    p.nsub = 2;
    const size_t dev_max = (size_t)max_lds_per_block();
    // two blocks per CU when a whole expert fits in half of the LDS; a ds = 128 block needs the
    // whole register file of its CU anyway, so its chunks may take most of the LDS
    const size_t budget_resident = dev_max < 72 * 1024 ? dev_max : 72 * 1024;
    const size_t want_stream = ds > 64 ? 140 * 1024 : 64 * 1024;
    const size_t budget_stream = dev_max < want_stream ? dev_max : want_stream;
    if (frag_per_ht * HT + fixed <= budget_resident) {
        p.hc = HT;
    } else {
        p.hc = 1;
        for (int c = HT; c >= 1; --c)
            if (HT % c == 0 && frag_per_ht * c + fixed <= budget_stream) {
                p.hc = c;
                break;
            }
    }
    p.lds = frag_per_ht * p.hc + fixed;
    return p;
}

template <int DS, int NSUB>
static hipError_t run_ffn(const slicemoe_config &c, const FfnPlan &pl, const void *h, const float *p,
                          const int32_t *offsets, const int32_t *perm, const void *packed, float *y,
                          hipStream_t s)
{
    const PackedLayout L = packed_layout(c);
    const long long Na = (long long)c.T * c.S * c.k;
    constexpr int TM = kFfnWaves * NSUB * 32;
    const long long max_tiles = (Na + TM - 1) / TM + c.E;
    const int blocks_per_cu = pl.lds <= 80 * 1024 ? 2 : 1;
    long long blocks = (long long)num_compute_units() * blocks_per_cu;
    if (blocks > max_tiles) blocks = max_tiles;
    auto kern = ffn_mfma_kernel<DS, NSUB>;
    hipError_t err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds);
    if (err != hipSuccess) return err;
    kern<<<(int)blocks, kFfnThreads, pl.lds, s>>>((const bf16_t *)h, p, offsets, perm,
                                                  (const char *)packed + L.experts, L.e_stride, L.e_w1, L.e_w2,
                                                  L.e_b1, L.e_b2, c.He, c.E, c.k, pl.hc, y);
    return hipGetLastError();
}

hipError_t launch_ffn_mfma(const slicemoe_config &c, const void *h, const float *p,
                           const int32_t *offsets, const int32_t *perm, const void *packed,
                           float *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    if (Na == 0) return hipSuccess;
    const int ds = c.d / c.S;
    const FfnPlan pl = plan_ffn(ds, c.He, c.E);
    if (ds == 64) return run_ffn<64, 2>(c, pl, h, p, offsets, perm, packed, y, s);
    return run_ffn<128, 2>(c, pl, h, p, offsets, perm, packed, y, s);
}

}  // namespace slicemoe
