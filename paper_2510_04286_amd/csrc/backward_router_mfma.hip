// Matrix-core backward of the router and assembly of dL/dh, for slice widths 64 and 96, Hr = 256 and E <= 32 (the
// benchmark shapes with up to 32 experts, and the paper's own).  Same mathematics as bwd_router_kernel in backward.hip; two kernels, both without
// any exchange between wavefronts:
//
//   bwd_route_slices_mfma_kernel   the forward router's layout: a lane owns one slice of a 32-slice tile.  Pass 1
//       recomputes the router exactly as the forward does (hidden layer on bf16 MFMA with the bias preloaded, ReLU,
//       two-term fp16 split, logits on fp16 MFMA; noise; softmax with the temperature) and remembers the ReLU pattern
//       as one bit per hidden unit.  Then, per lane: the selected probabilities, back through the dropout's
//       renormalisation and the softmax to dL/dg (16 of the 32 experts per lane, as the logits).  Pass 2: dL/du =
//       Wr2 dL/dg with dL/dg fed from registers as the B operand (two-term bf16), masked by the ReLU bits, then
//       dL/dx += Wr1 dL/du chained from registers the same way.  Writes dL/dh = that + the k expert-path rows of the
//       slice (one bf16 rounding), and dL/dg as two bf16 tables (hi, lo) for the weight-gradient kernel.
//   bwd_route_weights_mfma_kernel  the transposed layout (see backward_mfma.hip): one wavefront per hidden tile walks
//       the slices of its block.  u^T by operand swap, dL/du^T = dL/dg Wr2^T straight from the dL/dg tables (their rows
//       are A operands as stored), x^T and dL/dg^T by identity-MFMA transposes, then dWr1 += x^T dL/du and
//       dWr2 += u^T dL/dg with two-term operands.  Stores its pieces into the block's slot of partial sums.
#include "bwd_mfma.h"

namespace slicemoe {

typedef _Float16 r_h2 __attribute__((ext_vector_type(2)));
typedef _Float16 r_f16x8 __attribute__((ext_vector_type(8)));

constexpr int kRbHr = 256, kRbHT = 8;
constexpr int kRbThreads = 512;                 // slices kernel: 8 wavefronts
constexpr int kRbWaves = kRbThreads / 64;
constexpr int kRbWgWaves = 4;                   // weights kernel: one wavefront per hidden tile, two groups of four
constexpr int kRbSliceBlock = 512;              // slices per slot of the weights kernel (= kBwdSlices of backward.hip)

// Repacked router (bytes from the start of the buffer); every piece a multiple of 256 bytes.
//   w1f  [8][KS][64]    Wr1 fragments, lane (i, g), slot m: Wr1[16ks + 8g + m][32ht + i]           (bf16)
//   w2f  [8][2][64]     Wr2 for the logits: lane (i, g), slot m: Wr2[32ht + chain(s, g, m)][i]      (fp16, experts >= E zero)
//   w2c  [2][8][64]     Wr2 for dL/du:      lane (i, g), slot m: Wr2[32ht + i][chain(s, g, m)]      (bf16, experts >= E zero)
//   w1c  [8][2][OT][64] Wr1 for dL/dx:      lane (i, g), slot m: Wr1[32ot + i][32ht + chain(s, g, m)] (bf16)
//   w2r  [8][2][64]     rows of Wr2:        lane (i, g), slot m: Wr2[32ht + i][16s + 8g + m]        (bf16, experts >= E zero)
//   b1 [256] fp32, b2 [32] fp32 (zero past E)
struct RouterBwdPacked {
    size_t w1f, w2f, w2c, w1c, w2r, b1, b2, total;
};
static RouterBwdPacked router_bwd_layout(int ds)
{
    RouterBwdPacked L;
    const int KS = ds / 16, OT = ds / 32;
    size_t at = 0;
    L.w1f = at;  at += (size_t)kRbHT * KS * 64 * 16;
    L.w2f = at;  at += (size_t)kRbHT * 2 * 64 * 16;
    L.w2c = at;  at += (size_t)2 * kRbHT * 64 * 16;
    L.w1c = at;  at += (size_t)kRbHT * 2 * OT * 64 * 16;
    L.w2r = at;  at += (size_t)kRbHT * 2 * 64 * 16;
    L.b1 = at;   at += (size_t)kRbHr * 4;
    L.b2 = at;   at += 256;
    L.total = at;
    return L;
}

// ------------------------------------------------------------------------------------------------ slices kernel
template <int DS>
__global__ __launch_bounds__(kRbThreads) void bwd_route_slices_mfma_kernel(
    const bf16_t *__restrict__ x, long long Ns, int E, int k, const char *__restrict__ packed, RouterBwdPacked L,
    const float *__restrict__ noise, float sigma, float inv_tau, const float *__restrict__ drop_u, float rate,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ inv, const float *__restrict__ dpk,
    const float *__restrict__ dxrow, bf16_t *__restrict__ dh, bf16_t *__restrict__ dg_hi, bf16_t *__restrict__ dg_lo)
{
    constexpr int kRbDS = DS, kRbKS = DS / 16, kRbOT = DS / 32;
    extern __shared__ __align__(16) char lds[];
    const uint4 *w1f = (const uint4 *)(lds + L.w1f);
    const uint4 *w2f = (const uint4 *)(lds + L.w2f);
    const uint4 *w2c = (const uint4 *)(lds + L.w2c);
    const uint4 *w1c = (const uint4 *)(lds + L.w1c);
    const float *b1s = (const float *)(lds + L.b1);
    const float *b2s = (const float *)(lds + L.b2);

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    stage_bytes(packed, lds, L.total, tid, kRbThreads);
    __syncthreads();

    const long long ntiles = (Ns + 31) / 32;
    for (long long tile = (long long)wave * gridDim.x + blockIdx.x; tile < ntiles; tile += (long long)gridDim.x * kRbWaves) {
        const long long n = tile * 32 + j;
        const bool valid = n < Ns;
        const long long nn = valid ? n : 0;   // a lane without a slice reads slice 0 and writes nothing
        const uint4 *xr = (const uint4 *)(x + nn * kRbDS);
        bf16x8 xb[kRbKS];
#pragma unroll
        for (int ks = 0; ks < kRbKS; ++ks) xb[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);

        // ---- pass 1: the forward router, remembering which hidden units are active (bit r of half ht & 1 of word ht / 2)
        f32x16 gacc;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 b = *(const f32x4 *)(b2s + 8 * q + 4 * g);
#pragma unroll
            for (int c = 0; c < 4; ++c) gacc[4 * q + c] = b[c];
        }
        uint32_t act0 = 0, act1 = 0, act2 = 0, act3 = 0;
#pragma unroll 1
        for (int ht = 0; ht < kRbHT; ++ht) {
            f32x16 acc;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 b = *(const f32x4 *)(b1s + ht * 32 + 8 * q + 4 * g);
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[4 * q + c] = b[c];
            }
#pragma unroll
            for (int ks = 0; ks < kRbKS; ++ks)
                acc = mfma_bf16(__builtin_bit_cast(bf16x8, w1f[(ht * kRbKS + ks) * 64 + lane]), xb[ks], acc);
            uint32_t t0[8], t1[8], bits = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float u0 = fmaxf(acc[2 * i], 0.f), u1 = fmaxf(acc[2 * i + 1], 0.f);
                bits |= (acc[2 * i] > 0.f ? 1u : 0u) << (2 * i);
                bits |= (acc[2 * i + 1] > 0.f ? 1u : 0u) << (2 * i + 1);
                const r_h2 hi = __builtin_bit_cast(r_h2, __builtin_amdgcn_cvt_pkrtz(u0, u1));
                const float r0 = u0 - (float)hi[0], r1 = u1 - (float)hi[1];   // exact remainders
                t0[i] = __builtin_bit_cast(uint32_t, hi);
                t1[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r0, r1));
            }
            bits <<= (ht & 1) * 16;
            act0 |= (ht >> 1) == 0 ? bits : 0u;
            act1 |= (ht >> 1) == 1 ? bits : 0u;
            act2 |= (ht >> 1) == 2 ? bits : 0u;
            act3 |= (ht >> 1) == 3 ? bits : 0u;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const r_f16x8 u0 = __builtin_bit_cast(r_f16x8, make_uint4(t0[4 * s], t0[4 * s + 1], t0[4 * s + 2], t0[4 * s + 3]));
                const r_f16x8 u1 = __builtin_bit_cast(r_f16x8, make_uint4(t1[4 * s], t1[4 * s + 1], t1[4 * s + 2], t1[4 * s + 3]));
                const r_f16x8 a2 = __builtin_bit_cast(r_f16x8, w2f[(ht * 2 + s) * 64 + lane]);
                gacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, u1, gacc, 0, 0, 0);   // small term first
                gacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, u0, gacc, 0, 0, 0);
            }
        }

        // ---- this lane's 16 logits: expert acc_feature(r, g); noise; softmax of g / tau over the E experts
        float v[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int e = acc_feature(r, g);
            float t = gacc[r];
            if (noise != nullptr && e < E) t = fmaf(sigma, noise[nn * E + e], t);
            v[r] = e < E ? t : -INFINITY;
        }
        float m = v[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) m = fmaxf(m, v[r]);
        m = fmaxf(m, __shfl_xor(m, 32));
        const float sc = 1.4426950408889634f * inv_tau, nm = -m * sc;
        float den = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            v[r] = __builtin_amdgcn_exp2f(fmaf(v[r], sc, nm));
            den += v[r];
        }
        den += __shfl_xor(den, 32);
        const float rden = 1.f / den;
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] *= rden;   // probability of every expert of this lane's half

        // ---- the k selections: probability, upstream gradient, dropout flag (both lanes of a slice do the same)
        float psel[8], dpf[8];
        bool keep[8];
        int ej[8];
        int kept = 0;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            psel[jj] = dpf[jj] = 0.f;
            keep[jj] = false;
            ej[jj] = -1;
            if (jj < k) {
                const long long a = nn * k + jj;
                ej[jj] = idx[a];
                float mine = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) mine = acc_feature(r, g) == ej[jj] ? v[r] : mine;
                psel[jj] = mine + __shfl_xor(mine, 32);   // the expert sits in one of the two halves
                dpf[jj] = inv[a] >= 0 ? dpk[a] : 0.f;     // a capacity-dropped assignment carries no gradient
                keep[jj] = rate > 0.f ? !(drop_u[a] < rate) : true;
                kept += keep[jj] ? 1 : 0;
            }
        }
        if (rate > 0.f) {
            if (kept == 0) keep[0] = true;
            float ssum = 0.f, dot = 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) ssum += keep[jj] ? psel[jj] : 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) dot += keep[jj] ? dpf[jj] * (psel[jj] / ssum) : 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) dpf[jj] = keep[jj] ? (dpf[jj] - dot) / ssum : 0.f;
        }
        // dL/dg_e = (1/tau) (sum_j c_j [e = e_j] - p_e sum_j c_j),  c_j = dL/dp_j p_j
        float csum = 0.f, dg[16];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            dpf[jj] = jj < k ? dpf[jj] * psel[jj] : 0.f;
            csum += dpf[jj];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float t = -v[r] * csum;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) t += acc_feature(r, g) == ej[jj] ? dpf[jj] : 0.f;
            dg[r] = valid ? t * inv_tau : 0.f;
        }
        uint32_t dgh[8], dgl[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) split_bf16x2(dg[2 * i], dg[2 * i + 1], dgh[i], dgl[i]);
        if (valid) {   // experts 8q + 4g .. + 3 of this slice: four bf16 values per table and q
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                *(uint2 *)(dg_hi + n * 32 + 8 * q + 4 * g) = make_uint2(dgh[2 * q], dgh[2 * q + 1]);
                *(uint2 *)(dg_lo + n * 32 + 8 * q + 4 * g) = make_uint2(dgl[2 * q], dgl[2 * q + 1]);
            }
        }

        // ---- pass 2: dL/du = Wr2 dL/dg (ReLU pattern applied), dL/dx += Wr1 dL/du, both chained from registers
        f32x16 dx[kRbOT];
#pragma unroll
        for (int ot = 0; ot < kRbOT; ++ot)
#pragma unroll
            for (int i = 0; i < 16; ++i) dx[ot][i] = 0.f;
#pragma unroll 1
        for (int ht = 0; ht < kRbHT; ++ht) {
            f32x16 du;
#pragma unroll
            for (int i = 0; i < 16; ++i) du[i] = 0.f;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 wf = __builtin_bit_cast(bf16x8, w2c[(s * kRbHT + ht) * 64 + lane]);
                du = mfma_bf16(wf, frag_of(dgl, s), du);
                du = mfma_bf16(wf, frag_of(dgh, s), du);
            }
            const uint32_t word = (ht >> 1) == 0 ? act0 : (ht >> 1) == 1 ? act1 : (ht >> 1) == 2 ? act2 : act3;
            const uint32_t bits = word >> ((ht & 1) * 16);
            uint32_t duh[8], dul[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float d0 = (bits >> (2 * i)) & 1u ? du[2 * i] : 0.f;
                const float d1 = (bits >> (2 * i + 1)) & 1u ? du[2 * i + 1] : 0.f;
                split_bf16x2(d0, d1, duh[i], dul[i]);
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int ot = 0; ot < kRbOT; ++ot) {
                    const bf16x8 wf = __builtin_bit_cast(bf16x8, w1c[((ht * 2 + s) * kRbOT + ot) * 64 + lane]);
                    dx[ot] = mfma_bf16(wf, frag_of(dul, s), dx[ot]);
                    dx[ot] = mfma_bf16(wf, frag_of(duh, s), dx[ot]);
                }
        }

        // ---- dL/dh of the slice: router path plus the expert-path rows of its k assignments, one rounding
        if (valid) {
            int rows[8];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) rows[jj] = jj < k ? inv[n * k + jj] : -1;
#pragma unroll
            for (int ot = 0; ot < kRbOT; ++ot)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int feat = 32 * ot + 8 * q + 4 * g;
                    f32x4 t = {dx[ot][4 * q], dx[ot][4 * q + 1], dx[ot][4 * q + 2], dx[ot][4 * q + 3]};
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj)
                        if (rows[jj] >= 0) t += *(const f32x4 *)(dxrow + (size_t)rows[jj] * kRbDS + feat);
                    *(uint2 *)(dh + n * kRbDS + feat) = make_uint2(pack_bf16x2(t[0], t[1]), pack_bf16x2(t[2], t[3]));
                }
        }
    }
}

// ----------------------------------------------------------------------------------------------- weights kernel
// grid.x = range of kRbSliceBlock slices (its slot of partial sums), grid.y = group of four hidden tiles, block = one
// wavefront per hidden tile of the group.
template <int DS>
__global__ __launch_bounds__(kRbWgWaves * 64, DS <= 64 ? 2 : 1) void bwd_route_weights_mfma_kernel(
    const bf16_t *__restrict__ x, long long Ns, int E, const char *__restrict__ packed, RouterBwdPacked L,
    const bf16_t *__restrict__ dg_hi, const bf16_t *__restrict__ dg_lo, size_t slot_floats, float *__restrict__ part)
{
    constexpr int kRbDS = DS, kRbKS = DS / 16, kRbOT = DS / 32;
    extern __shared__ __align__(16) char lds[];
    // this group's fragments only: [wave][KS][64] of w1f, [wave][2][64] of w2r, 32 biases per wavefront
    uint4 *w1f = (uint4 *)lds;
    uint4 *w2r = w1f + kRbWgWaves * kRbKS * 64;
    float *b1s = (float *)(w2r + kRbWgWaves * 2 * 64);

    const int tid = threadIdx.x, lane = tid & 63, jj = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ht0 = (int)blockIdx.y * kRbWgWaves, ht = ht0 + wave;   // kRbHT is a multiple of the group size
    stage_bytes(packed + L.w1f + (size_t)ht0 * kRbKS * 1024, (char *)w1f, (size_t)kRbWgWaves * kRbKS * 1024, tid, kRbWgWaves * 64);
    stage_bytes(packed + L.w2r + (size_t)ht0 * 2 * 1024, (char *)w2r, (size_t)kRbWgWaves * 2 * 1024, tid, kRbWgWaves * 64);
    if (tid < kRbWgWaves * 32) b1s[tid] = ((const float *)(packed + L.b1))[ht0 * 32 + tid];
    __syncthreads();
    bf16x8 id_even, id_odd;
    identity_fragments(jj, g, id_even, id_odd);
    const float bias = b1s[wave * 32 + jj];

    f32x16 aW1[kRbOT], aW2;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        aW2[i] = 0.f;
#pragma unroll
        for (int ot = 0; ot < kRbOT; ++ot) aW1[ot][i] = 0.f;
    }
    float ab1 = 0.f, ab2 = 0.f;

    const long long n_begin = (long long)blockIdx.x * kRbSliceBlock;
    const long long n_end = min(Ns, n_begin + kRbSliceBlock);
    for (long long n0 = n_begin; n0 < n_end; n0 += 32) {
        const long long n = n0 + jj;   // as A operand a lane holds slice jj of the unit, contraction slots 8g..8g+7
        const bool valid = n < n_end;
        const long long nn = valid ? n : n_begin;
        const uint4 *xr = (const uint4 *)(x + nn * kRbDS);
        bf16x8 xa[kRbKS], gh[2], gl[2];
#pragma unroll
        for (int ks = 0; ks < kRbKS; ++ks) xa[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);
#pragma unroll
        for (int s = 0; s < 2; ++s) {   // experts 16s + 8g .. + 7 of the slice; slices past the end add nothing
            const uint4 z = make_uint4(0, 0, 0, 0);
            gh[s] = __builtin_bit_cast(bf16x8, valid ? *(const uint4 *)(dg_hi + nn * 32 + 16 * s + 8 * g) : z);
            gl[s] = __builtin_bit_cast(bf16x8, valid ? *(const uint4 *)(dg_lo + nn * 32 + 16 * s + 8 * g) : z);
        }
        // transposed: lane = hidden unit jj of this tile, register i = slice acc_feature(i, g) of the unit
        f32x16 u, du;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            u[i] = bias;
            du[i] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < kRbKS; ++ks) u = mfma_bf16(xa[ks], __builtin_bit_cast(bf16x8, w1f[(wave * kRbKS + ks) * 64 + lane]), u);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const bf16x8 wf = __builtin_bit_cast(bf16x8, w2r[(wave * 2 + s) * 64 + lane]);
            du = mfma_bf16(gl[s], wf, du);
            du = mfma_bf16(gh[s], wf, du);
        }
        uint32_t uh[8], ul[8], duh[8], dul[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float u0 = fmaxf(u[2 * i], 0.f), u1 = fmaxf(u[2 * i + 1], 0.f);
            const float d0 = u[2 * i] > 0.f ? du[2 * i] : 0.f, d1 = u[2 * i + 1] > 0.f ? du[2 * i + 1] : 0.f;
            ab1 += d0 + d1;
            split_bf16x2(u0, u1, uh[i], ul[i]);
            split_bf16x2(d0, d1, duh[i], dul[i]);
        }
        // dL/dg of the unit with lane = expert jj, registers = slices (exact: both tables hold bf16 values)
        f32x16 gth, gtl;
#pragma unroll
        for (int i = 0; i < 16; ++i) gth[i] = gtl[i] = 0.f;
        gth = mfma_bf16(gh[0], id_even, gth);
        gth = mfma_bf16(gh[1], id_odd, gth);
        gtl = mfma_bf16(gl[0], id_even, gtl);
        gtl = mfma_bf16(gl[1], id_odd, gtl);
        uint32_t gthp[8], gtlp[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            gthp[i] = pack_exact_bf16x2(gth[2 * i], gth[2 * i + 1]);
            gtlp[i] = pack_exact_bf16x2(gtl[2 * i], gtl[2 * i + 1]);
            if (ht == 0) ab2 += (gth[2 * i] + gtl[2 * i]) + (gth[2 * i + 1] + gtl[2 * i + 1]);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {   // dWr2 [hidden unit][expert]: lane = expert, registers = hidden units
            aW2 = mfma_bf16(frag_of(ul, s), frag_of(gthp, s), aW2);
            aW2 = mfma_bf16(frag_of(uh, s), frag_of(gtlp, s), aW2);
            aW2 = mfma_bf16(frag_of(uh, s), frag_of(gthp, s), aW2);
        }
#pragma unroll
        for (int ot = 0; ot < kRbOT; ++ot) {
            f32x16 xt;
#pragma unroll
            for (int i = 0; i < 16; ++i) xt[i] = 0.f;
            xt = mfma_bf16(xa[2 * ot], id_even, xt);
            xt = mfma_bf16(xa[2 * ot + 1], id_odd, xt);
            uint32_t xtp[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) xtp[i] = pack_exact_bf16x2(xt[2 * i], xt[2 * i + 1]);
#pragma unroll
            for (int s = 0; s < 2; ++s) {   // dWr1 [slice feature][hidden unit]: lane = hidden unit, registers = features
                aW1[ot] = mfma_bf16(frag_of(xtp, s), frag_of(dul, s), aW1[ot]);
                aW1[ot] = mfma_bf16(frag_of(xtp, s), frag_of(duh, s), aW1[ot]);
            }
        }
    }

    // this block's slot: dWr1 [ds][Hr] | dWr2 [Hr][E] | dbr1 [Hr] | dbr2 [E]
    float *slot = part + (size_t)blockIdx.x * slot_floats;
    float *pWr1 = slot, *pWr2 = pWr1 + (size_t)kRbDS * kRbHr, *pbr1 = pWr2 + (size_t)kRbHr * E, *pbr2 = pbr1 + kRbHr;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
        for (int ot = 0; ot < kRbOT; ++ot) pWr1[(size_t)(32 * ot + acc_feature(i, g)) * kRbHr + 32 * ht + jj] = aW1[ot][i];
        if (jj < E) pWr2[(size_t)(32 * ht + acc_feature(i, g)) * E + jj] = aW2[i];
    }
    ab1 += __shfl_xor(ab1, 32);   // the two lane groups hold different slices of the same hidden unit
    if (g == 0) pbr1[32 * ht + jj] = ab1;
    ab2 += __shfl_xor(ab2, 32);
    if (ht == 0 && g == 0 && jj < E) pbr2[jj] = ab2;
}

// ------------------------------------------------------------------------------------------------------ host
bool backward_router_mfma_shape(const slicemoe_config &c)
{
    const int ds = c.d / c.S;
    return c.dtype == SLICEMOE_BF16 && (ds == 64 || ds == 96) && c.Hr == kRbHr && c.E <= 32 &&
           !(c.flags & SLICEMOE_FLAG_FORCE_GENERIC) && router_bwd_layout(ds).total <= (size_t)max_lds_per_block();
}

size_t backward_router_mfma_scratch_bytes(const slicemoe_config &c)
{
    if (!backward_router_mfma_shape(c)) return 0;
    const size_t Ns = (size_t)c.T * c.S;
    return align_up(router_bwd_layout(c.d / c.S).total, 256) + 2 * align_up(Ns * 32 * sizeof(bf16_t), 256);
}

template <int DS>
static hipError_t run_router_mfma(const slicemoe_config &c, const RouterBwdPacked &L, const void *h, const RouteVariant &v,
                                  const float *drop_u, float rate, const int32_t *idx, const int32_t *inv, const float *dpk,
                                  const float *dxrow, void *d_h, const char *pb, bf16_t *dg_hi, bf16_t *dg_lo,
                                  long long slice_blocks, size_t slot_floats, float *part, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    const long long ntiles = (Ns + 31) / 32;
    const long long blocks = ntiles < num_compute_units() ? ntiles : num_compute_units();
    auto sk = bwd_route_slices_mfma_kernel<DS>;
    hipError_t e = hipFuncSetAttribute((const void *)sk, hipFuncAttributeMaxDynamicSharedMemorySize, (int)L.total);
    if (e != hipSuccess) return e;
    sk<<<(int)blocks, kRbThreads, L.total, s>>>((const bf16_t *)h, Ns, c.E, c.k, pb, L, v.sigma > 0.f ? v.noise : nullptr, v.sigma,
                                                v.inv_tau, rate > 0.f ? drop_u : nullptr, rate, idx, inv, dpk, dxrow, (bf16_t *)d_h,
                                                dg_hi, dg_lo);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const size_t lds_w = (size_t)kRbWgWaves * (DS / 16 + 2) * 1024 + kRbWgWaves * 32 * sizeof(float);
    auto wk = bwd_route_weights_mfma_kernel<DS>;
    if ((e = hipFuncSetAttribute((const void *)wk, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_w)) != hipSuccess) return e;
    wk<<<dim3((unsigned)slice_blocks, kRbHT / kRbWgWaves), kRbWgWaves * 64, lds_w, s>>>((const bf16_t *)h, Ns, c.E, pb, L, dg_hi, dg_lo,
                                                                                       slot_floats, part);
    return hipGetLastError();
}

// scratch: backward_router_mfma_scratch_bytes; part: ceil(Ns / 512) slots of slot_floats floats (the slice ranges of
// the vector-ALU router kernel).  dxrow, dpk: the expert stage's row gradients and dL/dp.
hipError_t launch_backward_router_mfma(const slicemoe_config &c, const void *h, const slicemoe_weights &w,
                                       const RouteVariant &v, const float *drop_u, float rate, const int32_t *idx,
                                       const int32_t *inv, const float *dpk, const float *dxrow, void *d_h, void *scratch,
                                       long long slice_blocks, size_t slot_floats, float *part, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    if (!backward_router_mfma_shape(c) || slice_blocks != (Ns + kRbSliceBlock - 1) / kRbSliceBlock) return hipErrorInvalidValue;
    const int E = c.E, Hr = kRbHr, ds = c.d / c.S;
    const RouterBwdPacked L = router_bwd_layout(ds);
    char *pb = (char *)scratch;
    bf16_t *dg_hi = (bf16_t *)(pb + align_up(L.total, 256));
    bf16_t *dg_lo = dg_hi + align_up((size_t)Ns * 32 * sizeof(bf16_t), 256) / sizeof(bf16_t);
    const bf16_t *Wr1 = (const bf16_t *)w.Wr1, *Wr2 = (const bf16_t *)w.Wr2;
    BwdPackJobs jobs;
    jobs.count = 7;
    // w1f: Wr1 [ds, Hr] itself.  w2f: Wr2 [Hr, E] with the hidden units as contraction slots, fp16, experts padded to 32.
    jobs.job[0] = bwd_pack_job(kPackLayer1, Wr1, ds, ds, Hr, Hr, (size_t)Hr, 1, 0, pb + L.w1f, 0, 1);
    jobs.job[1] = bwd_pack_job(kPackChainF16, Wr2, Hr, Hr, 32, E, (size_t)E, 1, 0, pb + L.w2f, 0, 1);
    // w2c: M[e][h] = Wr2[h][e] ([32, Hr], experts as contraction slots).  w1c: M[h][c] = Wr1[c][h] ([Hr, ds]).
    jobs.job[2] = bwd_pack_job(kPackChain, Wr2, 32, E, Hr, Hr, 1, (size_t)E, 0, pb + L.w2c, 0, 1);
    jobs.job[3] = bwd_pack_job(kPackChain, Wr1, Hr, Hr, ds, ds, 1, (size_t)Hr, 0, pb + L.w1c, 0, 1);
    // w2r: M[e][h] = Wr2[h][e] ([32, Hr]) in plain K-steps of 16 experts
    jobs.job[4] = bwd_pack_job(kPackLayer1, Wr2, 32, E, Hr, Hr, 1, (size_t)E, 0, pb + L.w2r, 0, 1);
    jobs.job[5] = bwd_pack_job(kPackBias, w.br1, Hr, Hr, Hr, Hr, 0, 0, 0, pb + L.b1, 0, 1);
    jobs.job[6] = bwd_pack_job(kPackBias, w.br2, E, E, 32, 32, 0, 0, 0, pb + L.b2, 0, 1);
    const hipError_t e = bwd_pack_launch(jobs, s);
    if (e != hipSuccess) return e;
    if (ds == 64)
        return run_router_mfma<64>(c, L, h, v, drop_u, rate, idx, inv, dpk, dxrow, d_h, pb, dg_hi, dg_lo, slice_blocks, slot_floats, part, s);
    return run_router_mfma<96>(c, L, h, v, drop_u, rate, idx, inv, dpk, dxrow, d_h, pb, dg_hi, dg_lo, slice_blocks, slot_floats, part, s);
}

}  // namespace slicemoe
