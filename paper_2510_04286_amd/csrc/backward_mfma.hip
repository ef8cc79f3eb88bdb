// Matrix-core backward of the expert stage for slice widths 64, 96 and 128 and any hidden width that is a multiple
// of 32: the recomputed pre-activations, dL/dz, dL/dx, dL/dp and the expert weight gradients of the backward
// pass described in backward.hip, on v_mfma_f32_32x32x16_bf16.  Two kernels per width (the weights kernel of the wide
// slices, further down, is the only one whose wavefronts exchange anything):
//
//   bwd_rows_mfma_kernel     the forward's layout: a lane owns one stacked row (see mfma.h).  Per 32-row unit and
//                            32-wide hidden tile: u = W1^T x and da = W2 dy (weight fragment = A operand, row
//                            fragment = B), then per lane z = p u + b1, dz = da gelu'(z), and dx += W1 (p dz) with
//                            p dz fed from the accumulator registers as the B operand, exactly like the forward's
//                            second GEMM.  dL/dp = sum over the hidden units of dz u is a per-lane sum plus one
//                            exchange with lane ^ 32.  Writes dL/dx of the rows (fp32) and dL/dp.
//   bwd_weights_mfma_kernel  the transposed layout, because the weight gradients contract over ROWS, which the
//                            layout above keeps on lanes.  Swapping the operands of an MFMA transposes its result:
//                            with the row fragment as A and the weight fragment as B the accumulators come out as
//                            lane = hidden unit, registers = 16 of the 32 rows.  There z, the activation a1 and
//                            p dz are formed for the wavefront's own hidden tile, rounded to bf16 pairs (register
//                            pairs are row pairs: the contraction slots), and dW2 += a1^T dy, dW1 += x^T (p dz) are
//                            two MFMA pairs per 32 slice features.  The x and dy operands of those (lane = slice
//                            feature, slots = rows) are the row fragments transposed by an MFMA against an
//                            identity fragment, which is exact.  A block is one wavefront per hidden tile walking
//                            the rows of one chunk of one expert; each wavefront stores its 32 x 64 pieces of dW1
//                            and dW2 into the chunk's slot, which the reduction kernel of backward.hip adds up.
//
// Precision: u, da, z, the activation and its derivative in fp32 (erf by the five-term rational approximation of
// Abramowitz & Stegun 7.1.26, absolute error 1.5e-7, sharing its exponential with the density); the operands of the
// second-stage matrix instructions (p dz, a1) enter as two-term bf16 splits (hi + lo, 16 significant bits, one
// matrix instruction per term against exact bf16 data), so the results are of fp32 grade.  The kernels are bound by
// vector instructions, not by the matrix pipe, so the second term costs little.
#include "bwd_mfma.h"

namespace slicemoe {

constexpr int kBmDS = 64;
constexpr int kBmKS = kBmDS / 16;
constexpr int kBmOT = kBmDS / 32;
constexpr int kBmRowThreads = 768;   // rows kernel: 12 wavefronts of <= 168 registers
constexpr int kBmRowWaves = kBmRowThreads / 64;

// Backward copies of one expert's weights in fragment order (bytes from the start of the expert's block).
//   w1f  [HT][KS][64]      W1 fragments as the forward packs them: lane (i, g), slot m: W1[16ks + 8g + m][32ht + i]
//   w2r  [HT][KS][64]      rows of W2: lane (i, g), slot m: W2[32ht + i][16ks + 8g + m]
//   w1c  [HT][2][OT][64]   W1 with the hidden units as contraction slots in accumulator order:
//                          lane (i, g), slot m: W1[32ot + i][32ht + chain_feature(s, g, m)]
//   b1   [He] fp32
struct BwdPacked {
    size_t w1f, w2r, w1c, b1, stride;
};
static BwdPacked bwd_packed_layout(int ds, int He)
{
    BwdPacked L;
    const size_t frag = (size_t)ds * He * 2;
    L.w1f = 0;
    L.w2r = frag;
    L.w1c = 2 * frag;
    L.b1 = 3 * frag;
    L.stride = align_up(3 * frag + (size_t)He * 4, 256);
    return L;
}

// One thread per fragment (or bias value) of one job; see bwd_mfma.h for the layouts.
__device__ __forceinline__ void pack_layer1_item(const BwdPackJob &J, long long f)
{
    const int KS = J.K / 16;
    const long long per = (long long)(J.N / 32) * KS * 64;
    const int mat = (int)(f / per);
    long long r = f - (long long)mat * per;
    const int lane = (int)(r % 64);
    r /= 64;
    const int ks = (int)(r % KS), nt = (int)(r / KS);
    const int i = lane & 31, g = lane >> 5;
    const bf16_t *src = J.src + (size_t)mat * J.src_stride;
    const int col = 32 * nt + i;
    uint32_t v[4];
    for (int m = 0; m < 8; m += 2) {
        const int k0 = 16 * ks + 8 * g + m;
        const uint32_t lo = (k0 < J.Kv && col < J.Nv) ? src[(size_t)k0 * J.rs + (size_t)col * J.cs] : 0;
        const uint32_t hi = (k0 + 1 < J.Kv && col < J.Nv) ? src[(size_t)(k0 + 1) * J.rs + (size_t)col * J.cs] : 0;
        v[m / 2] = lo | (hi << 16);
    }
    *(uint4 *)(J.dst + (size_t)mat * J.dst_stride + (size_t)(f - (long long)mat * per) * 16) = make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ void pack_chain_item(const BwdPackJob &J, long long f)
{
    const int HT = J.K / 32, NT = J.N / 32;
    const long long per = (long long)HT * 2 * NT * 64;
    const int mat = (int)(f / per);
    long long r = f - (long long)mat * per;
    const int lane = (int)(r % 64);
    r /= 64;
    const int nt = (int)(r % NT);
    r /= NT;
    const int s = (int)(r % 2), ht = (int)(r / 2);
    const int i = lane & 31, g = lane >> 5;
    const bf16_t *src = J.src + (size_t)mat * J.src_stride;
    const int col = 32 * nt + i;
    uint32_t v[4];
    for (int m = 0; m < 8; m += 2) {
        uint32_t pr[2];
        for (int c = 0; c < 2; ++c) {
            const int kk = 32 * ht + chain_feature(s, g, m + c);
            bf16_t w = (kk < J.Kv && col < J.Nv) ? src[(size_t)kk * J.rs + (size_t)col * J.cs] : (bf16_t)0;
            if (J.kind == kPackChainF16) {   // bf16 values convert exactly unless tiny (rounded) or beyond the fp16 range (clamped)
                const _Float16 hv = (_Float16)fminf(fmaxf(bf16_to_f32(w), -65504.f), 65504.f);
                w = __builtin_bit_cast(bf16_t, hv);
            }
            pr[c] = w;
        }
        v[m / 2] = pr[0] | (pr[1] << 16);
    }
    *(uint4 *)(J.dst + (size_t)mat * J.dst_stride + (size_t)(f - (long long)mat * per) * 16) = make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ void pack_bias_item(const BwdPackJob &J, long long t)
{
    // K = values per matrix, N = padded count
    const int mat = (int)(t / J.N), i = (int)(t - (long long)mat * J.N);
    ((float *)(J.dst + (size_t)mat * J.dst_stride))[i] = i < J.K ? bf16_to_f32(J.src[(size_t)mat * J.src_stride + i]) : 0.f;
}

__global__ void bwd_pack_jobs_kernel(BwdPackJobs jobs)
{
    long long f = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    for (int q = 0; q < jobs.count; ++q) {   // the jobs' items are numbered one job after the other
        const BwdPackJob &J = jobs.job[q];
        if (f < J.items) {
            if (J.kind == kPackLayer1) pack_layer1_item(J, f);
            else if (J.kind == kPackBias) pack_bias_item(J, f);
            else pack_chain_item(J, f);
            return;
        }
        f -= J.items;
    }
}

BwdPackJob bwd_pack_job(int kind, const void *src, int K, int Kv, int N, int Nv, size_t rs, size_t cs, size_t src_stride,
                        char *dst, size_t dst_stride, int nmat)
{
    BwdPackJob J;
    J.kind = kind;
    J.src = (const bf16_t *)src;
    J.K = K; J.Kv = Kv; J.N = N; J.Nv = Nv;
    J.rs = rs; J.cs = cs; J.src_stride = src_stride;
    J.dst = dst; J.dst_stride = dst_stride;
    if (kind == kPackLayer1) J.items = (long long)nmat * (N / 32) * (K / 16) * 64;
    else if (kind == kPackBias) J.items = (long long)nmat * N;
    else J.items = (long long)nmat * (K / 32) * 2 * (N / 32) * 64;
    return J;
}

hipError_t bwd_pack_launch(const BwdPackJobs &jobs, hipStream_t s)
{
    long long total = 0;
    for (int q = 0; q < jobs.count; ++q) total += jobs.job[q].items;
    if (total == 0) return hipSuccess;
    bwd_pack_jobs_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(jobs);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ rows kernel
template <int HT>
__global__ __launch_bounds__(kBmRowThreads) void bwd_rows_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, const char *__restrict__ packed,
    size_t e_stride, size_t off_w2r, size_t off_w1c, size_t off_b1, int E, int k,
    float *__restrict__ dxrow, float *__restrict__ dpk)
{
    extern __shared__ __align__(16) char lds[];
    const uint4 *w1f = (const uint4 *)lds;
    const uint4 *w2r = (const uint4 *)(lds + off_w2r);
    const uint4 *w1c = (const uint4 *)(lds + off_w1c);
    const float *b1s = (const float *)(lds + off_b1);

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_kept = offsets[E];
    const int units_total = (n_kept + 31) / 32;
    const int units_per_block = (units_total + (int)gridDim.x - 1) / (int)gridDim.x;
    const long long r_begin = (long long)blockIdx.x * units_per_block * 32;
    const int r_end = (int)min((long long)n_kept, r_begin + (long long)units_per_block * 32);

    int r = (int)min(r_begin, (long long)n_kept);
    while (r < r_end) {
        int e = 0;
        while (e + 1 < E && offsets[e + 1] <= r) ++e;   // uniform over the block
        const int seg_end = min(offsets[e + 1], r_end);
        __syncthreads();   // everyone is done with the previous expert's weights
        stage_bytes(packed + (size_t)e * e_stride, lds, e_stride, tid, kBmRowThreads);
        __syncthreads();

        const int nunits = (seg_end - r + 31) / 32;
        for (int q = wave; q < nunits; q += kBmRowWaves) {
            const int row = r + q * 32 + j;
            const bool valid = row < seg_end;
            const int a = perm[valid ? row : r];
            const long long n = a / k;
            const float p = valid ? pk[a] : 0.f;
            const uint4 *xr = (const uint4 *)(x + n * kBmDS), *gr = (const uint4 *)(dout + n * kBmDS);
            bf16x8 xb[kBmKS], gb[kBmKS];
#pragma unroll
            for (int ks = 0; ks < kBmKS; ++ks) {
                xb[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);
                gb[ks] = __builtin_bit_cast(bf16x8, gr[2 * ks + g]);
            }
            f32x16 dx[kBmOT];
#pragma unroll
            for (int ot = 0; ot < kBmOT; ++ot)
#pragma unroll
                for (int i = 0; i < 16; ++i) dx[ot][i] = 0.f;
            float dp = 0.f;
#pragma unroll 1
            for (int ht = 0; ht < HT; ++ht) {
                f32x16 u, da;
#pragma unroll
                for (int i = 0; i < 16; ++i) u[i] = da[i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < kBmKS; ++ks) {
                    u = mfma_bf16(__builtin_bit_cast(bf16x8, w1f[(ht * kBmKS + ks) * 64 + lane]), xb[ks], u);
                    da = mfma_bf16(__builtin_bit_cast(bf16x8, w2r[(ht * kBmKS + ks) * 64 + lane]), gb[ks], da);
                }
                uint32_t hb[8], lb[8];
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const f32x4 bb = *(const f32x4 *)(b1s + ht * 32 + 8 * qq + 4 * g);
                    float pdz[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int i = 4 * qq + c;
                        const float z = fmaf(p, u[i], bb[c]);
                        float dens;
                        const float cdf = normal_cdf_pdf(z, &dens);
                        const float dz = da[i] * fmaf(z, dens, cdf);
                        dp = fmaf(dz, u[i], dp);
                        pdz[c] = p * dz;
                    }
                    split_bf16x2(pdz[0], pdz[1], hb[2 * qq], lb[2 * qq]);
                    split_bf16x2(pdz[2], pdz[3], hb[2 * qq + 1], lb[2 * qq + 1]);
                }
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const bf16x8 bh = __builtin_bit_cast(bf16x8, make_uint4(hb[4 * s], hb[4 * s + 1], hb[4 * s + 2], hb[4 * s + 3]));
                    const bf16x8 bl = __builtin_bit_cast(bf16x8, make_uint4(lb[4 * s], lb[4 * s + 1], lb[4 * s + 2], lb[4 * s + 3]));
#pragma unroll
                    for (int ot = 0; ot < kBmOT; ++ot) {
                        const bf16x8 wf = __builtin_bit_cast(bf16x8, w1c[((ht * 2 + s) * kBmOT + ot) * 64 + lane]);
                        dx[ot] = mfma_bf16(wf, bl, dx[ot]);   // small term first
                        dx[ot] = mfma_bf16(wf, bh, dx[ot]);
                    }
                }
            }
            dp += __shfl_xor(dp, 32);
            if (valid) {
                if (g == 0) dpk[a] = dp;
                float *dst = dxrow + (size_t)row * kBmDS;
#pragma unroll
                for (int ot = 0; ot < kBmOT; ++ot)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const f32x4 v = {dx[ot][4 * qq], dx[ot][4 * qq + 1], dx[ot][4 * qq + 2], dx[ot][4 * qq + 3]};
                        *(f32x4 *)(dst + ot * 32 + 8 * qq + 4 * g) = v;
                    }
            }
        }
        r = seg_end;
    }
}

// ------------------------------------------------------------------------------------- rows kernel, streamed
// The same computation for experts whose three fragment sets do not fit in LDS together (slice widths 96 and 128,
// or He > 256 at width 64): a block takes tiles of kBmTileWaves x 32 rows of ONE expert and streams the fragments through
// LDS in chunks of hc hidden tiles per row tile, the dL/dx accumulators staying in registers across the chunks.
constexpr int kBmTileWaves = 8;
constexpr int kBmTileRows = kBmTileWaves * 32;
template <int DS>
__global__ __launch_bounds__(kBmTileWaves * 64) void bwd_rows_streamed_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, const char *__restrict__ packed,
    size_t e_stride, size_t off_w2r, size_t off_w1c, size_t off_b1, int He, int hc, int E, int k,
    float *__restrict__ dxrow, float *__restrict__ dpk)
{
    constexpr int KS = DS / 16, OT = DS / 32, THREADS = kBmTileWaves * 64;
    const int HT = He / 32, nchunks = HT / hc;   // hc divides HT
    extern __shared__ __align__(16) char lds[];
    uint4 *w1f = (uint4 *)lds;                          // [hc][KS][64]
    uint4 *w2r = w1f + (size_t)hc * KS * 64;            // [hc][KS][64]
    uint4 *w1c = w2r + (size_t)hc * KS * 64;            // [hc][2][OT][64]
    float *b1s = (float *)(w1c + (size_t)hc * 2 * OT * 64);   // [He]
    int *tile_prefix = (int *)(b1s + He);               // [E + 1]

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            tile_prefix[e] = run;
            run += (offsets[e + 1] - offsets[e] + kBmTileRows - 1) / kBmTileRows;
        }
        tile_prefix[E] = run;
    }
    __syncthreads();
    const int total = tile_prefix[E];
    const int per_block = (total + (int)gridDim.x - 1) / (int)gridDim.x;
    const int t_begin = (int)blockIdx.x * per_block;
    const int t_end = min(total, t_begin + per_block);

    int cur_e = -1, e = 0;
    for (int t = t_begin; t < t_end; ++t) {
        while (tile_prefix[e + 1] <= t) ++e;
        const int row_begin = offsets[e] + (t - tile_prefix[e]) * kBmTileRows;
        const int row_end = offsets[e + 1];
        const char *ew = packed + (size_t)e * e_stride;
        const int row = row_begin + wave * 32 + j;
        const bool valid = row < row_end;
        const int a = perm[valid ? row : row_begin];
        const long long n = a / k;
        const float p = valid ? pk[a] : 0.f;
        const uint4 *xr = (const uint4 *)(x + n * DS), *gr = (const uint4 *)(dout + n * DS);
        bf16x8 xb[KS], gb[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            xb[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);
            gb[ks] = __builtin_bit_cast(bf16x8, gr[2 * ks + g]);
        }
        f32x16 dx[OT];
#pragma unroll
        for (int ot = 0; ot < OT; ++ot)
#pragma unroll
            for (int i = 0; i < 16; ++i) dx[ot][i] = 0.f;
        float dp = 0.f;
        for (int ch = 0; ch < nchunks; ++ch) {
            __syncthreads();   // everyone is done with the previous contents
            stage_bytes(ew + (size_t)ch * hc * KS * 1024, (char *)w1f, (size_t)hc * KS * 1024, tid, THREADS);
            stage_bytes(ew + off_w2r + (size_t)ch * hc * KS * 1024, (char *)w2r, (size_t)hc * KS * 1024, tid, THREADS);
            stage_bytes(ew + off_w1c + (size_t)ch * hc * 2 * OT * 1024, (char *)w1c, (size_t)hc * 2 * OT * 1024, tid, THREADS);
            if (e != cur_e && ch == 0) {
                const float *gb1 = (const float *)(ew + off_b1);
                for (int i = tid; i < He; i += THREADS) b1s[i] = gb1[i];
            }
            __syncthreads();
#pragma unroll 1
            for (int hl = 0; hl < hc; ++hl) {
                const int ht = ch * hc + hl;
                f32x16 u, da;
#pragma unroll
                for (int i = 0; i < 16; ++i) u[i] = da[i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    u = mfma_bf16(__builtin_bit_cast(bf16x8, w1f[(hl * KS + ks) * 64 + lane]), xb[ks], u);
                    da = mfma_bf16(__builtin_bit_cast(bf16x8, w2r[(hl * KS + ks) * 64 + lane]), gb[ks], da);
                }
                uint32_t hb[8], lb[8];
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const f32x4 bb = *(const f32x4 *)(b1s + ht * 32 + 8 * qq + 4 * g);
                    float pdz[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int i = 4 * qq + c;
                        const float z = fmaf(p, u[i], bb[c]);
                        float dens;
                        const float cdf = normal_cdf_pdf(z, &dens);
                        const float dz = da[i] * fmaf(z, dens, cdf);
                        dp = fmaf(dz, u[i], dp);
                        pdz[c] = p * dz;
                    }
                    split_bf16x2(pdz[0], pdz[1], hb[2 * qq], lb[2 * qq]);
                    split_bf16x2(pdz[2], pdz[3], hb[2 * qq + 1], lb[2 * qq + 1]);
                }
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int ot = 0; ot < OT; ++ot) {
                        const bf16x8 wf = __builtin_bit_cast(bf16x8, w1c[((hl * 2 + s) * OT + ot) * 64 + lane]);
                        dx[ot] = mfma_bf16(wf, frag_of(lb, s), dx[ot]);   // small term first
                        dx[ot] = mfma_bf16(wf, frag_of(hb, s), dx[ot]);
                    }
            }
        }
        cur_e = e;
        dp += __shfl_xor(dp, 32);
        if (valid) {
            if (g == 0) dpk[a] = dp;
            float *dst = dxrow + (size_t)row * DS;
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const f32x4 v = {dx[ot][4 * qq], dx[ot][4 * qq + 1], dx[ot][4 * qq + 2], dx[ot][4 * qq + 3]};
                    *(f32x4 *)(dst + ot * 32 + 8 * qq + 4 * g) = v;
                }
        }
    }
}

// --------------------------------------------------------------------------------------------- weights kernel
// grid = chunks (as the vector-ALU expert kernel numbers them, rounded up to eight) x groups of kBmWgWaves hidden tiles, block = one
// wavefront per hidden tile of the group; part: the chunk slots.  Any He % 32 == 0; used at slice width 64.
constexpr int kBmWgWaves = 4;
template <int DS>
__global__ __launch_bounds__(kBmWgWaves * 64, 2) void bwd_weights_mfma_kernel(   // two wavefronts per SIMD
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, const char *__restrict__ packed,
    size_t e_stride, size_t off_w2r, size_t off_b1, int He, int E, int k, int rows_per_chunk, size_t slot_floats,
    float *__restrict__ part)
{
    constexpr int KS = DS / 16, OT = DS / 32;
    const int HT = He / 32;
    extern __shared__ __align__(16) char lds[];
    // this group's fragments only: [wave][KS][64] of w1f, then of w2r, then 32 biases per wavefront
    uint4 *w1f = (uint4 *)lds;
    uint4 *w2r = w1f + kBmWgWaves * KS * 64;
    float *b1s = (float *)(w2r + kBmWgWaves * KS * 64);
    __shared__ int blk[3];

    const int tid = threadIdx.x, lane = tid & 63, jj = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Consecutive blocks go to the eight XCDs in turn, each with its own L2: the groups of a chunk, which read the
    // same rows, take block ids that are equal modulo 8.
    const int groups = (HT + kBmWgWaves - 1) / kBmWgWaves;
    const int ht0 = ((int)(blockIdx.x / 8) % groups) * kBmWgWaves;
    const int chunk = (int)(blockIdx.x / (8 * groups)) * 8 + (int)(blockIdx.x % 8);
    const int ht = ht0 + wave;
    if (tid == 0) {
        int left = chunk, e = 0, begin = 0, end = 0;
        bool found = false;
        for (e = 0; e < E; ++e) {
            const int lo = offsets[e], hi = offsets[e + 1];
            const int nch = (hi - lo + rows_per_chunk - 1) / rows_per_chunk;
            if (left < nch) {
                begin = lo + left * rows_per_chunk;
                end = min(hi, begin + rows_per_chunk);
                found = true;
                break;
            }
            left -= nch;
        }
        blk[0] = found ? e : -1;
        blk[1] = begin;
        blk[2] = end;
    }
    __syncthreads();
    const int e = blk[0], row_begin = blk[1], row_end = blk[2];
    if (e < 0) return;   // uniform over the block
    {   // fragments of the hidden tiles ht0 .. ht0 + 3 that exist (tile-major in the packed block, so one run each)
        const int nt = min(kBmWgWaves, HT - ht0);
        const char *src = packed + (size_t)e * e_stride;
        const size_t run = (size_t)nt * KS * 1024;
        stage_bytes(src + (size_t)ht0 * KS * 1024, (char *)w1f, run, tid, kBmWgWaves * 64);
        stage_bytes(src + off_w2r + (size_t)ht0 * KS * 1024, (char *)w2r, run, tid, kBmWgWaves * 64);
        const float *gb = (const float *)(src + off_b1);
        if (tid < nt * 32) b1s[tid] = gb[ht0 * 32 + tid];
    }
    __syncthreads();
    if (ht >= HT) return;   // a group past the last hidden tile: no more barriers below

    bf16x8 id_even, id_odd;
    identity_fragments(jj, g, id_even, id_odd);
    const float bias = b1s[wave * 32 + jj];

    f32x16 aW1[OT], aW2[OT];
#pragma unroll
    for (int ot = 0; ot < OT; ++ot)
#pragma unroll
        for (int i = 0; i < 16; ++i) aW1[ot][i] = aW2[ot][i] = 0.f;
    float ab1 = 0.f, ab2[OT];
#pragma unroll
    for (int ot = 0; ot < OT; ++ot) ab2[ot] = 0.f;

    for (int r0 = row_begin; r0 < row_end; r0 += 32) {
        const int row = r0 + jj;   // as A operand a lane holds row jj of the unit, contraction slots 8g..8g+7
        const bool valid = row < row_end;
        const int a = perm[valid ? row : row_begin];
        const long long n = a / k;
        const float p_lane = valid ? pk[a] : 0.f;
        const uint4 *xr = (const uint4 *)(x + n * DS), *gr = (const uint4 *)(dout + n * DS);
        bf16x8 xa[KS], ga[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            xa[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);
            const uint4 gv = valid ? gr[2 * ks + g] : make_uint4(0, 0, 0, 0);   // rows past the end add nothing
            ga[ks] = __builtin_bit_cast(bf16x8, gv);
        }
        // transposed results: lane = hidden unit jj of this tile, register i = row acc_feature(i, g) of the unit
        f32x16 u, da;
#pragma unroll
        for (int i = 0; i < 16; ++i) u[i] = da[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u = mfma_bf16(xa[ks], __builtin_bit_cast(bf16x8, w1f[(wave * KS + ks) * 64 + lane]), u);
            da = mfma_bf16(ga[ks], __builtin_bit_cast(bf16x8, w2r[(wave * KS + ks) * 64 + lane]), da);
        }
        uint32_t a1p[8], a1l[8], pdzp[8], pdzl[8];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            float act[2], pdz[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const float p = __shfl(p_lane, acc_feature(i + c, g));   // probability of the register's row
                const float z = fmaf(p, u[i + c], bias);
                float dens;
                const float cdf = normal_cdf_pdf(z, &dens);
                const float dz = da[i + c] * fmaf(z, dens, cdf);
                act[c] = z * cdf;
                pdz[c] = p * dz;
                ab1 += dz;
            }
            split_bf16x2(act[0], act[1], a1p[i / 2], a1l[i / 2]);
            split_bf16x2(pdz[0], pdz[1], pdzp[i / 2], pdzl[i / 2]);
        }
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            // x and dy of the unit with lane = slice feature 32 ot + jj, registers = rows
            f32x16 xt, gt;
#pragma unroll
            for (int i = 0; i < 16; ++i) xt[i] = gt[i] = 0.f;
            xt = mfma_bf16(xa[2 * ot], id_even, xt);
            xt = mfma_bf16(xa[2 * ot + 1], id_odd, xt);
            gt = mfma_bf16(ga[2 * ot], id_even, gt);
            gt = mfma_bf16(ga[2 * ot + 1], id_odd, gt);
            if (ht == 0) {
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += gt[i];
                ab2[ot] += sum;
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 xs = __builtin_bit_cast(bf16x8, make_uint4(pack_exact_bf16x2(xt[8 * s], xt[8 * s + 1]), pack_exact_bf16x2(xt[8 * s + 2], xt[8 * s + 3]),
                                                                         pack_exact_bf16x2(xt[8 * s + 4], xt[8 * s + 5]), pack_exact_bf16x2(xt[8 * s + 6], xt[8 * s + 7])));
                const bf16x8 gs = __builtin_bit_cast(bf16x8, make_uint4(pack_exact_bf16x2(gt[8 * s], gt[8 * s + 1]), pack_exact_bf16x2(gt[8 * s + 2], gt[8 * s + 3]),
                                                                         pack_exact_bf16x2(gt[8 * s + 4], gt[8 * s + 5]), pack_exact_bf16x2(gt[8 * s + 6], gt[8 * s + 7])));
                const bf16x8 ah = __builtin_bit_cast(bf16x8, make_uint4(a1p[4 * s], a1p[4 * s + 1], a1p[4 * s + 2], a1p[4 * s + 3]));
                const bf16x8 al = __builtin_bit_cast(bf16x8, make_uint4(a1l[4 * s], a1l[4 * s + 1], a1l[4 * s + 2], a1l[4 * s + 3]));
                const bf16x8 dh = __builtin_bit_cast(bf16x8, make_uint4(pdzp[4 * s], pdzp[4 * s + 1], pdzp[4 * s + 2], pdzp[4 * s + 3]));
                const bf16x8 dl = __builtin_bit_cast(bf16x8, make_uint4(pdzl[4 * s], pdzl[4 * s + 1], pdzl[4 * s + 2], pdzl[4 * s + 3]));
                // [hidden unit][slice feature]: lane = feature, registers = hidden units; small term first
                aW2[ot] = mfma_bf16(al, gs, aW2[ot]);
                aW2[ot] = mfma_bf16(ah, gs, aW2[ot]);
                // [slice feature][hidden unit]: lane = hidden unit, registers = features
                aW1[ot] = mfma_bf16(xs, dl, aW1[ot]);
                aW1[ot] = mfma_bf16(xs, dh, aW1[ot]);
            }
        }
    }

    // this chunk's slot: dW1 [ds][He] | dW2 [He][ds] | db1 [He] | db2 [ds]
    float *slot = part + (size_t)chunk * slot_floats;
    float *pW1 = slot, *pW2 = pW1 + (size_t)DS * He, *pb1 = pW2 + (size_t)He * DS, *pb2 = pb1 + He;
#pragma unroll
    for (int ot = 0; ot < OT; ++ot)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            pW1[(size_t)(32 * ot + acc_feature(i, g)) * He + 32 * ht + jj] = aW1[ot][i];
            pW2[(size_t)(32 * ht + acc_feature(i, g)) * DS + 32 * ot + jj] = aW2[ot][i];
        }
    ab1 += __shfl_xor(ab1, 32);   // the two lane groups hold different rows of the same hidden unit
    if (g == 0) pb1[32 * ht + jj] = ab1;
    if (ht == 0) {
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            const float t = ab2[ot] + __shfl_xor(ab2[ot], 32);
            if (g == 0) pb2[32 * ot + jj] = t;
        }
    }
}

// ------------------------------------------------------------------------------- weights kernel, wavefront pairs
// The same for slice widths 96 and 128, whose 6 or 8 accumulator tiles plus operands exceed half a SIMD's registers
// (the kernel above then runs one wavefront per SIMD and leaves its latencies uncovered).  Here TWO wavefronts share a
// hidden tile and split the work by operand: wavefront 0 reads the x rows, forms u and accumulates dW1 = x^T (p dz);
// wavefront 1 reads the dy rows, forms da and accumulates dW2 = a1^T dy.  Each evaluates the activation and dL/dz for
// the sixteen rows of one K-step (registers 8 W .. 8 W + 7): they trade the halves of u and da those rows need, then
// the resulting fragments (a1 to wavefront 1, p dz to wavefront 0), through LDS: two barriers per unit, buffers
// alternating with the unit's parity.  Every row piece is read once per pair.
// grid = chunks (rounded up to eight) x hidden tiles, block = the pair.
template <int DS, int W>
__device__ __forceinline__ void bwd_weights_pair_body(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ perm, int He, int k, int row_begin, int row_end, const uint4 *w1f, const uint4 *w2r,
    float *fx, uint4 *xch, const float *b1s, float *red, int ht, int lane, float *__restrict__ slot)
{
    constexpr int KS = DS / 16, OT = DS / 32;
    const int jj = lane & 31, g = lane >> 5;
    bf16x8 id_even, id_odd;
    identity_fragments(jj, g, id_even, id_odd);
    const float bias = b1s[jj];
    const uint4 *wf = W == 0 ? w1f : w2r;            // fragments of this wavefront's first contraction
    const bf16_t *rows = W == 0 ? x : dout;          // and the rows it reads

    f32x16 aW[OT];   // W = 0: dW1 tiles (lane = hidden unit, registers = features); W = 1: dW2 tiles (lane = feature)
    float ab1 = 0.f, ab2[OT];
#pragma unroll
    for (int ot = 0; ot < OT; ++ot) {
        ab2[ot] = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) aW[ot][i] = 0.f;
    }
    int parity = 0;
    for (int r0 = row_begin; r0 < row_end; r0 += 32) {
        const int row = r0 + jj;   // as A operand a lane holds row jj of the unit, contraction slots 8g..8g+7
        const bool valid = row < row_end;
        const int a = perm[valid ? row : row_begin];
        const long long n = a / k;
        const float p_lane = valid ? pk[a] : 0.f;
        const uint4 *rr = (const uint4 *)(rows + n * DS);
        bf16x8 ra[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint4 v = (W == 0 || valid) ? rr[2 * ks + g] : make_uint4(0, 0, 0, 0);   // dy of rows past the end adds nothing
            ra[ks] = __builtin_bit_cast(bf16x8, v);
        }
        // transposed result: lane = hidden unit jj of the tile, register i = row acc_feature(i, g): u (W = 0) or da (W = 1)
        f32x16 v;
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) v = mfma_bf16(ra[ks], __builtin_bit_cast(bf16x8, wf[ks * 64 + lane]), v);
        // the partner evaluates registers 8 (1 - W) ..: it gets those of this result, this wavefront those of the partner's
        float *out = fx + ((parity * 2 + W) * 8) * 64 + lane;
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i * 64] = v[8 * (1 - W) + i];
        __syncthreads();
        const float *in = fx + ((parity * 2 + (1 - W)) * 8) * 64 + lane;
        uint32_t a1p[4], a1l[4], pdzp[4], pdzl[4];
#pragma unroll
        for (int ii = 0; ii < 8; ii += 2) {
            float act[2], pdz[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int i = 8 * W + ii + c;
                const float other = in[(ii + c) * 64];
                const float u = W == 0 ? v[i] : other, da = W == 0 ? other : v[i];
                const float p = __shfl(p_lane, acc_feature(i, g));   // probability of the register's row
                const float z = fmaf(p, u, bias);
                float dens;
                const float cdf = normal_cdf_pdf(z, &dens);
                const float dz = da * fmaf(z, dens, cdf);
                act[c] = z * cdf;
                pdz[c] = p * dz;
                ab1 += dz;
            }
            split_bf16x2(act[0], act[1], a1p[ii / 2], a1l[ii / 2]);
            split_bf16x2(pdz[0], pdz[1], pdzp[ii / 2], pdzl[ii / 2]);
        }
        // wavefront 0 needs p dz of both K-steps, wavefront 1 the activation: each sends what the other lacks
        uint4 *mine = xch + ((parity * 2 + W) * 2) * 64 + lane;
        if (W == 0) {
            mine[0] = make_uint4(a1p[0], a1p[1], a1p[2], a1p[3]);
            mine[64] = make_uint4(a1l[0], a1l[1], a1l[2], a1l[3]);
        } else {
            mine[0] = make_uint4(pdzp[0], pdzp[1], pdzp[2], pdzp[3]);
            mine[64] = make_uint4(pdzl[0], pdzl[1], pdzl[2], pdzl[3]);
        }
        __syncthreads();
        const uint4 *theirs = xch + ((parity * 2 + (1 - W)) * 2) * 64 + lane;
        bf16x8 hi[2], lo[2];   // by K-step (step W is this wavefront's own): p dz for W = 0, the activation for W = 1
        hi[W] = __builtin_bit_cast(bf16x8, W == 0 ? make_uint4(pdzp[0], pdzp[1], pdzp[2], pdzp[3]) : make_uint4(a1p[0], a1p[1], a1p[2], a1p[3]));
        lo[W] = __builtin_bit_cast(bf16x8, W == 0 ? make_uint4(pdzl[0], pdzl[1], pdzl[2], pdzl[3]) : make_uint4(a1l[0], a1l[1], a1l[2], a1l[3]));
        hi[1 - W] = __builtin_bit_cast(bf16x8, theirs[0]);
        lo[1 - W] = __builtin_bit_cast(bf16x8, theirs[64]);
        parity ^= 1;
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            // the rows of the unit with lane = slice feature 32 ot + jj, registers = rows (exact)
            f32x16 t;
#pragma unroll
            for (int i = 0; i < 16; ++i) t[i] = 0.f;
            t = mfma_bf16(ra[2 * ot], id_even, t);
            t = mfma_bf16(ra[2 * ot + 1], id_odd, t);
            if (W == 1 && ht == 0) {
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += t[i];
                ab2[ot] += sum;
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 ts = __builtin_bit_cast(bf16x8, make_uint4(pack_exact_bf16x2(t[8 * s], t[8 * s + 1]), pack_exact_bf16x2(t[8 * s + 2], t[8 * s + 3]),
                                                                         pack_exact_bf16x2(t[8 * s + 4], t[8 * s + 5]), pack_exact_bf16x2(t[8 * s + 6], t[8 * s + 7])));
                if (W == 0) {   // [slice feature][hidden unit]: lane = hidden unit, registers = features; small term first
                    aW[ot] = mfma_bf16(ts, lo[s], aW[ot]);
                    aW[ot] = mfma_bf16(ts, hi[s], aW[ot]);
                } else {        // [hidden unit][slice feature]: lane = feature, registers = hidden units
                    aW[ot] = mfma_bf16(lo[s], ts, aW[ot]);
                    aW[ot] = mfma_bf16(hi[s], ts, aW[ot]);
                }
            }
        }
    }

    // the chunk's slot: dW1 [ds][He] | dW2 [He][ds] | db1 [He] | db2 [ds]
    float *pW1 = slot, *pW2 = pW1 + (size_t)DS * He, *pb1 = pW2 + (size_t)He * DS, *pb2 = pb1 + He;
#pragma unroll
    for (int ot = 0; ot < OT; ++ot) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (W == 0) pW1[(size_t)(32 * ot + acc_feature(i, g)) * He + 32 * ht + jj] = aW[ot][i];
            else pW2[(size_t)(32 * ht + acc_feature(i, g)) * DS + 32 * ot + jj] = aW[ot][i];
        }
        if (W == 1 && ht == 0) {
            const float t = ab2[ot] + __shfl_xor(ab2[ot], 32);
            if (g == 0) pb2[32 * ot + jj] = t;
        }
    }
    // db1: the two lane groups hold different rows of the same hidden unit, the two wavefronts different K-steps
    ab1 += __shfl_xor(ab1, 32);
    if (W == 1 && g == 0) red[jj] = ab1;
    __syncthreads();
    if (W == 0 && g == 0) pb1[32 * ht + jj] = ab1 + red[jj];
}

template <int DS>
__global__ __launch_bounds__(128, 2) void bwd_weights_pair_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, const char *__restrict__ packed,
    size_t e_stride, size_t off_w2r, size_t off_b1, int He, int E, int k, int rows_per_chunk, size_t slot_floats,
    float *__restrict__ part)
{
    constexpr int KS = DS / 16;
    extern __shared__ __align__(16) char lds[];
    uint4 *w1f = (uint4 *)lds;              // [KS][64] fragments of this hidden tile
    uint4 *w2r = w1f + KS * 64;             // [KS][64]
    uint4 *xch = w2r + KS * 64;             // [parity][wavefront][term][64] fragments traded
    float *fx = (float *)(xch + 2 * 2 * 2 * 64);    // [parity][wavefront][8][64] halves of u / da traded
    float *b1s = fx + 2 * 2 * 8 * 64;       // [32]
    float *red = b1s + 32;                  // [32]
    __shared__ int blk[3];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Consecutive blocks go to the eight XCDs in turn, each with its own L2: the HT hidden tiles of a chunk, which
    // read the same rows, take block ids that are equal modulo 8.
    const int HT = He / 32;
    const int ht = (int)(blockIdx.x / 8) % HT;
    const int chunk = (int)(blockIdx.x / (8 * HT)) * 8 + (int)(blockIdx.x % 8);
    if (tid == 0) {
        int left = chunk, e = 0, begin = 0, end = 0;
        bool found = false;
        for (e = 0; e < E; ++e) {
            const int lo = offsets[e], hi = offsets[e + 1];
            const int nch = (hi - lo + rows_per_chunk - 1) / rows_per_chunk;
            if (left < nch) {
                begin = lo + left * rows_per_chunk;
                end = min(hi, begin + rows_per_chunk);
                found = true;
                break;
            }
            left -= nch;
        }
        blk[0] = found ? e : -1;
        blk[1] = begin;
        blk[2] = end;
    }
    __syncthreads();
    const int e = blk[0], row_begin = blk[1], row_end = blk[2];
    if (e < 0) return;   // uniform over the block
    const char *src = packed + (size_t)e * e_stride;
    stage_bytes(src + (size_t)ht * KS * 1024, (char *)w1f, (size_t)KS * 1024, tid, 128);
    stage_bytes(src + off_w2r + (size_t)ht * KS * 1024, (char *)w2r, (size_t)KS * 1024, tid, 128);
    if (tid < 32) b1s[tid] = ((const float *)(src + off_b1))[ht * 32 + tid];
    __syncthreads();
    float *slot = part + (size_t)chunk * slot_floats;
    // the same number of units, hence of barriers, in both wavefronts
    if (wave == 0) bwd_weights_pair_body<DS, 0>(x, dout, pk, perm, He, k, row_begin, row_end, w1f, w2r, fx, xch, b1s, red, ht, lane, slot);
    else bwd_weights_pair_body<DS, 1>(x, dout, pk, perm, He, k, row_begin, row_end, w1f, w2r, fx, xch, b1s, red, ht, lane, slot);
}

// ------------------------------------------------------------------------------------------------------ host
bool backward_mfma_shape(const slicemoe_config &c)
{
    const int ds = c.d / c.S;
    return c.dtype == SLICEMOE_BF16 && (ds == 64 || ds == 96 || ds == 128) && c.He % 32 == 0 &&
           !(c.flags & SLICEMOE_FLAG_FORCE_GENERIC);
}

size_t backward_mfma_packed_bytes(const slicemoe_config &c)
{
    return backward_mfma_shape(c) ? bwd_packed_layout(c.d / c.S, c.He).stride * (size_t)c.E : 0;
}

// Hidden tiles per chunk of the streamed rows kernel: the largest divisor of HT whose fragments fit, and its LDS bytes.
static int streamed_chunk(int ds, int He, int E, size_t *lds)
{
    const int HT = He / 32, KS = ds / 16, OT = ds / 32;
    const size_t per_ht = (size_t)(2 * KS + 2 * OT) * 1024, fixed = (size_t)He * 4 + (size_t)(E + 1) * 4 + 64;
    const size_t want = 140 * 1024, dev = (size_t)max_lds_per_block();
    const size_t budget = dev < want ? dev : want;
    int hc = 1;
    for (int c = HT; c >= 1; --c)
        if (HT % c == 0 && per_ht * c + fixed <= budget) {
            hc = c;
            break;
        }
    *lds = per_ht * hc + fixed;
    return hc;
}

template <int DS>
static hipError_t run_expert_mfma(const slicemoe_config &c, const BwdPacked &L, const void *h, const void *d_out,
                                  const float *pk, const int32_t *offsets, const int32_t *perm, const char *packed,
                                  int rows_per_chunk, long long chunks, size_t slot_floats, float *dxrow, float *dpk,
                                  float *part, hipStream_t s, hipStream_t sw /* stream of the weight-gradient kernel */)
{
    const long long Na = (long long)c.T * c.S * c.k;
    const bf16_t *x = (const bf16_t *)h, *g = (const bf16_t *)d_out;
    hipError_t e;
    if (DS == 64 && (c.He == 64 || c.He == 128 || c.He == 256) && L.stride <= (size_t)max_lds_per_block()) {
        // the whole expert resident in LDS, row units balanced over the blocks across expert boundaries
        long long blocks = (Na + 31) / 32;
        if (blocks > num_compute_units()) blocks = num_compute_units();
        auto rows = c.He == 256 ? bwd_rows_mfma_kernel<8> : c.He == 128 ? bwd_rows_mfma_kernel<4> : bwd_rows_mfma_kernel<2>;
        if ((e = grant_dynamic_lds((const void *)rows, L.stride)) != hipSuccess)
            return e;
        rows<<<(int)blocks, kBmRowThreads, L.stride, s>>>(x, g, pk, offsets, perm, packed, L.stride, L.w2r, L.w1c, L.b1, c.E, c.k,
                                                          dxrow, dpk);
    } else {
        size_t lds = 0;
        const int hc = streamed_chunk(DS, c.He, c.E, &lds);
        long long blocks = (Na + kBmTileRows - 1) / kBmTileRows + c.E;
        if (blocks > num_compute_units()) blocks = num_compute_units();
        auto rows = bwd_rows_streamed_mfma_kernel<DS>;
        if ((e = grant_dynamic_lds((const void *)rows, lds)) != hipSuccess)
            return e;
        rows<<<(int)blocks, kBmTileWaves * 64, lds, s>>>(x, g, pk, offsets, perm, packed, L.stride, L.w2r, L.w1c, L.b1, c.He, hc,
                                                         c.E, c.k, dxrow, dpk);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int HT = c.He / 32;
    if constexpr (DS >= 96) {
        const size_t lds_p = (size_t)2 * (DS / 16) * 1024 + 2 * 2 * 2 * 1024 + 2 * 2 * 8 * 64 * sizeof(float) + 64 * sizeof(float);
        auto pk2 = bwd_weights_pair_mfma_kernel<DS>;
        if ((e = grant_dynamic_lds((const void *)pk2, lds_p)) != hipSuccess) return e;
        pk2<<<(unsigned)((chunks + 7) / 8 * 8 * HT), 128, lds_p, sw>>>(x, g, pk, offsets, perm, packed, L.stride, L.w2r, L.b1, c.He, c.E, c.k,
                                                                   rows_per_chunk, slot_floats, part);
        return hipGetLastError();
    } else {
    const size_t lds_w = (size_t)2 * kBmWgWaves * (DS / 16) * 1024 + kBmWgWaves * 32 * sizeof(float);
    auto wk = bwd_weights_mfma_kernel<DS>;
    if ((e = grant_dynamic_lds((const void *)wk, lds_w)) != hipSuccess) return e;
    wk<<<(unsigned)((chunks + 7) / 8 * 8 * ((HT + kBmWgWaves - 1) / kBmWgWaves)), kBmWgWaves * 64, lds_w, sw>>>(
        x, g, pk, offsets, perm, packed, L.stride, L.w2r, L.b1, c.He, c.E, c.k, rows_per_chunk, slot_floats, part);
    return hipGetLastError();
    }
}

// Packs the backward copies of the expert weights into `packed` (backward_mfma_packed_bytes), then runs the two kernels.
// rows_per_chunk must be a multiple of 32; part holds `chunks` slots of slot_floats floats.
hipError_t launch_backward_expert_mfma(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const void *d_out,
                                       const float *pk, const int32_t *offsets, const int32_t *perm, void *packed,
                                       int rows_per_chunk, long long chunks, size_t slot_floats, float *dxrow, float *dpk,
                                       float *part, hipStream_t s, const SideStream *side)
{
    if (!backward_mfma_shape(c) || rows_per_chunk % 32 != 0) return hipErrorInvalidValue;
    const int He = c.He, E = c.E, ds = c.d / c.S;
    const BwdPacked L = bwd_packed_layout(ds, He);
    char *pb = (char *)packed;
    const size_t wstride = (size_t)ds * He;
    BwdPackJobs jobs;
    jobs.count = 4;
    // w1f: the [ds, He] matrix W1 itself; w2r: the [ds, He] matrix M[c][hidden] = W2[hidden][c]
    jobs.job[0] = bwd_pack_job(kPackLayer1, w.W1, ds, ds, He, He, (size_t)He, 1, wstride, pb + L.w1f, L.stride, E);
    jobs.job[1] = bwd_pack_job(kPackLayer1, w.W2, ds, ds, He, He, 1, (size_t)ds, wstride, pb + L.w2r, L.stride, E);
    // w1c: the [He, ds] matrix M[hidden][c] = W1[c][hidden], contraction over the hidden units in accumulator order
    jobs.job[2] = bwd_pack_job(kPackChain, w.W1, He, He, ds, ds, 1, (size_t)He, wstride, pb + L.w1c, L.stride, E);
    jobs.job[3] = bwd_pack_job(kPackBias, w.b1, He, He, He, He, 0, 0, (size_t)He, pb + L.b1, L.stride, E);
    hipError_t e = bwd_pack_launch(jobs, s);
    if (e != hipSuccess) return e;
    hipStream_t sw = s;
    if (side != nullptr) {   // the weight-gradient kernel starts when the repacked weights are there
        if ((e = hipEventRecord(side->fork, s)) != hipSuccess) return e;
        if ((e = hipStreamWaitEvent(side->stream, side->fork, 0)) != hipSuccess) return e;
        sw = side->stream;
    }
    if (ds == 64) return run_expert_mfma<64>(c, L, h, d_out, pk, offsets, perm, pb, rows_per_chunk, chunks, slot_floats, dxrow, dpk, part, s, sw);
    if (ds == 96) return run_expert_mfma<96>(c, L, h, d_out, pk, offsets, perm, pb, rows_per_chunk, chunks, slot_floats, dxrow, dpk, part, s, sw);
    return run_expert_mfma<128>(c, L, h, d_out, pk, offsets, perm, pb, rows_per_chunk, chunks, slot_floats, dxrow, dpk, part, s, sw);
}

}  // namespace slicemoe
