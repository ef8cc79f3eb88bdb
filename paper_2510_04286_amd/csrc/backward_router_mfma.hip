// Matrix-core backward of the router and assembly of dL/dh, for slice widths 64, 96 and 128, Hr = 256 and up to 64
// experts.  Same mathematics as bwd_router_kernel in backward.hip; three kernels, all without any exchange between
// wavefronts:
//
//   bwd_route_logits_mfma_kernel   the forward router's layout: a lane owns one slice of a 32-slice tile.  Recomputes the
//       router exactly as the forward does (hidden layer on bf16 MFMA with the bias preloaded, ReLU, two-term fp16 split,
//       logits on fp16 MFMA; noise; softmax with the temperature), then per lane: the selected probabilities, back
//       through the dropout's renormalisation and the softmax to dL/dg (16 experts per lane and expert tile, as the
//       logits).  Writes dL/dg as two bf16 tables (hi, lo: a two-term split) and the ReLU pattern, one bit per hidden
//       unit.
//   bwd_route_inputs_mfma_kernel   same layout: dL/du = Wr2 dL/dg with dL/dg read back in accumulator order, i.e. as
//       the B operand, masked by the ReLU bits, then dL/dx += Wr1 dL/du chained from registers (two-term bf16).  Writes
//       dL/dh = that + the k expert-path rows of the slice (one bf16 rounding).  It is a kernel of its own because the
//       fragments of the two halves do not fit in LDS together at width 128 or with 64 experts.
//   bwd_route_weights_mfma_kernel  the transposed layout (see backward_mfma.hip): one wavefront per hidden tile walks
//       the slices of its block.  u^T by operand swap, dL/du^T = dL/dg Wr2^T straight from the dL/dg tables (their rows
//       are A operands as stored), x^T and dL/dg^T by identity-MFMA transposes, then dWr1 += x^T dL/du and
//       dWr2 += u^T dL/dg with two-term operands.  Stores its pieces into the block's slot of partial sums.
#include "bwd_mfma.h"

namespace slicemoe {

typedef _Float16 r_h2 __attribute__((ext_vector_type(2)));
typedef _Float16 r_f16x8 __attribute__((ext_vector_type(8)));

constexpr int kRbHr = 256, kRbHT = 8;
constexpr int kRbThreads = 512;                 // slice kernels: 8 wavefronts
constexpr int kRbWaves = kRbThreads / 64;
constexpr int kRbWgWaves = 4;                   // weights kernel: one wavefront per hidden tile, two groups of four

// Repacked router (bytes from the start of the buffer); KS = ds / 16, OT = ds / 32, ET = expert tiles of 32 (experts
// past E are zero).
//   w1f  [8][KS][64]      Wr1 fragments, lane (i, g), slot m: Wr1[16ks + 8g + m][32ht + i]                   (bf16)
//   w2f  [8][2][ET][64]   Wr2 for the logits: lane (i, g), slot m: Wr2[32ht + chain(s, g, m)][32et + i]       (fp16)
//   w2c  [ET][2][8][64]   Wr2 for dL/du:      lane (i, g), slot m: Wr2[32ht + i][32et + chain(s, g, m)]       (bf16)
//   w1c  [8][2][OT][64]   Wr1 for dL/dx:      lane (i, g), slot m: Wr1[32ot + i][32ht + chain(s, g, m)]       (bf16)
//   w2r  [8][2 ET][64]    rows of Wr2:        lane (i, g), slot m: Wr2[32ht + i][16s + 8g + m]                (bf16)
//   b1 [256] fp32, b2 [32 ET] fp32
struct RouterBwdPacked {
    size_t w1f, w2f, w2c, w1c, w2r, b1, b2, total;
};
static RouterBwdPacked router_bwd_layout(int ds, int ET)
{
    RouterBwdPacked L;
    const int KS = ds / 16, OT = ds / 32;
    size_t at = 0;
    L.w1f = at;  at += (size_t)kRbHT * KS * 1024;
    L.w2f = at;  at += (size_t)ET * kRbHT * 2 * 1024;
    L.w2c = at;  at += (size_t)ET * 2 * kRbHT * 1024;
    L.w1c = at;  at += (size_t)kRbHT * 2 * OT * 1024;
    L.w2r = at;  at += (size_t)kRbHT * 2 * ET * 1024;
    L.b1 = at;   at += (size_t)kRbHr * 4;
    L.b2 = at;   at += 256;
    L.total = at;
    return L;
}

// ------------------------------------------------------------------------------------------------ logits kernel
// LDS: w1f | w2f | b1 | b2 (the first, second, sixth and seventh pieces of the packed buffer).
template <int DS, int ET>
__global__ __launch_bounds__(kRbThreads) void bwd_route_logits_mfma_kernel(
    const bf16_t *__restrict__ x, long long Ns, int E, int k, const char *__restrict__ packed, RouterBwdPacked L,
    const float *__restrict__ noise, float sigma, float inv_tau, const float *__restrict__ drop_u, float rate,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ inv, const float *__restrict__ dpk,
    const float *__restrict__ capg, bf16_t *__restrict__ dg_hi, bf16_t *__restrict__ dg_lo, uint32_t *__restrict__ relu_bits)
{
    constexpr int KS = DS / 16, EP = ET * 32;
    extern __shared__ __align__(16) char lds[];
    uint4 *w1f = (uint4 *)lds;                              // [8][KS][64]
    uint4 *w2f = w1f + kRbHT * KS * 64;                     // [8][2][ET][64]
    float *b1s = (float *)(w2f + ET * kRbHT * 2 * 64);      // [256]
    float *b2s = b1s + kRbHr;                               // [EP]

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    stage_bytes(packed + L.w1f, (char *)w1f, (size_t)kRbHT * KS * 1024, tid, kRbThreads);
    stage_bytes(packed + L.w2f, (char *)w2f, (size_t)ET * kRbHT * 2 * 1024, tid, kRbThreads);
    if (tid < kRbHr) b1s[tid] = ((const float *)(packed + L.b1))[tid];
    if (tid < EP) b2s[tid] = ((const float *)(packed + L.b2))[tid];
    __syncthreads();

    const long long ntiles = (Ns + 31) / 32;
    for (long long tile = (long long)wave * gridDim.x + blockIdx.x; tile < ntiles; tile += (long long)gridDim.x * kRbWaves) {
        const long long n = tile * 32 + j;
        const bool valid = n < Ns;
        const long long nn = valid ? n : 0;   // a lane without a slice reads slice 0 and writes nothing
        const uint4 *xr = (const uint4 *)(x + nn * DS);
        bf16x8 xb[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xb[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);

        // ---- the forward router, remembering which hidden units are active (bit r of half ht & 1 of word ht / 2)
        f32x16 gacc[ET];
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 b = *(const f32x4 *)(b2s + et * 32 + 8 * q + 4 * g);
#pragma unroll
                for (int c = 0; c < 4; ++c) gacc[et][4 * q + c] = b[c];
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
            for (int ks = 0; ks < KS; ++ks)
                acc = mfma_bf16(__builtin_bit_cast(bf16x8, w1f[(ht * KS + ks) * 64 + lane]), xb[ks], acc);
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
#pragma unroll
                for (int et = 0; et < ET; ++et) {
                    const r_f16x8 a2 = __builtin_bit_cast(r_f16x8, w2f[((ht * 2 + s) * ET + et) * 64 + lane]);
                    gacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, u1, gacc[et], 0, 0, 0);   // small term first
                    gacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, u0, gacc[et], 0, 0, 0);
                }
            }
        }

        // ---- this lane's 16 ET logits: expert 32 et + acc_feature(r, g); noise; softmax of g / tau over the E experts
        float v[ET * 16];
#pragma unroll
        for (int i = 0; i < ET * 16; ++i) {
            const int e = (i >> 4) * 32 + acc_feature(i & 15, g);
            float t = gacc[i >> 4][i & 15];
            if (noise != nullptr && e < E) t = fmaf(sigma, noise[nn * E + e], t);
            v[i] = e < E ? t : -INFINITY;
        }
        float m = v[0];
#pragma unroll
        for (int i = 1; i < ET * 16; ++i) m = fmaxf(m, v[i]);
        m = fmaxf(m, __shfl_xor(m, 32));
        const float sc = 1.4426950408889634f * inv_tau, nm = -m * sc;
        float den = 0.f;
#pragma unroll
        for (int i = 0; i < ET * 16; ++i) {
            v[i] = __builtin_amdgcn_exp2f(fmaf(v[i], sc, nm));
            den += v[i];
        }
        den += __shfl_xor(den, 32);
        const float rden = 1.f / den;
#pragma unroll
        for (int i = 0; i < ET * 16; ++i) v[i] *= rden;   // probability of every expert of this lane's half

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
                for (int i = 0; i < ET * 16; ++i) mine = (i >> 4) * 32 + acc_feature(i & 15, g) == ej[jj] ? v[i] : mine;
                psel[jj] = mine + __shfl_xor(mine, 32);   // the expert sits in one of the two halves
                dpf[jj] = inv[a] >= 0 ? dpk[a] : 0.f;     // a capacity-dropped assignment carries no gradient from h'
                if (capg != nullptr) dpf[jj] += capg[min(max(ej[jj], 0), E - 1)];   // but it counts as assigned (capacity loss)
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
        float csum = 0.f;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            dpf[jj] = jj < k ? dpf[jj] * psel[jj] : 0.f;
            csum += dpf[jj];
        }
        if (valid) {
#pragma unroll
            for (int et = 0; et < ET; ++et)
#pragma unroll
                for (int q = 0; q < 4; ++q) {   // experts 32 et + 8q + 4g .. + 3 of this slice: four bf16 values per table
                    float dg[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int i = et * 16 + 4 * q + c, e = et * 32 + 8 * q + 4 * g + c;
                        float t = -v[i] * csum;
#pragma unroll
                        for (int jj = 0; jj < 8; ++jj) t += e == ej[jj] ? dpf[jj] : 0.f;
                        dg[c] = t * inv_tau;
                    }
                    uint32_t h0, l0, h1, l1;
                    split_bf16x2(dg[0], dg[1], h0, l0);
                    split_bf16x2(dg[2], dg[3], h1, l1);
                    *(uint2 *)(dg_hi + n * EP + et * 32 + 8 * q + 4 * g) = make_uint2(h0, h1);
                    *(uint2 *)(dg_lo + n * EP + et * 32 + 8 * q + 4 * g) = make_uint2(l0, l1);
                }
            *(uint4 *)(relu_bits + (n * 2 + g) * 4) = make_uint4(act0, act1, act2, act3);
        }
    }
}

// ------------------------------------------------------------------------------------------------ inputs kernel
// Rows of the per-wavefront staging tile are 36 floats apart: 16-byte reads at a stride of one row then fall into
// distinct banks.
constexpr int kRbStageRow = 36;

// Orders LDS traffic between the lanes of one wavefront (the hardware keeps a wavefront's LDS operations in order; this
// keeps the compiler from moving them across).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// LDS: w2c | w1c (the third and fourth pieces of the packed buffer, adjacent) | staging tiles.
template <int DS, int ET>
__global__ __launch_bounds__(kRbThreads) void bwd_route_inputs_mfma_kernel(
    long long Ns, int k, const char *__restrict__ packed, RouterBwdPacked L, const int32_t *__restrict__ inv,
    const float *__restrict__ dxrow, const bf16_t *__restrict__ dg_hi, const bf16_t *__restrict__ dg_lo,
    const uint32_t *__restrict__ relu_bits, bf16_t *__restrict__ dh)
{
    constexpr int OT = DS / 32, EP = ET * 32;
    extern __shared__ __align__(16) char lds[];
    const uint4 *w2c = (const uint4 *)lds;                       // [ET][2][8][64]
    const uint4 *w1c = w2c + ET * 2 * kRbHT * 64;                // [8][2][OT][64]
    float *stg_all = (float *)(w1c + kRbHT * 2 * OT * 64);       // [8 wavefronts][32][kRbStageRow]

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    stage_bytes(packed + L.w2c, lds, (size_t)(ET * 2 * kRbHT + kRbHT * 2 * OT) * 1024, tid, kRbThreads);
    __syncthreads();
    float *stg = stg_all + wave * 32 * kRbStageRow;

    const long long ntiles = (Ns + 31) / 32;
    for (long long tile = (long long)wave * gridDim.x + blockIdx.x; tile < ntiles; tile += (long long)gridDim.x * kRbWaves) {
        const long long n = tile * 32 + j;
        const bool valid = n < Ns;
        // dL/dg of this lane in accumulator order: register pairs, i.e. B-operand fragments, as they were stored
        uint32_t dgh[ET][8], dgl[ET][8];
        uint4 act = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint2 h = make_uint2(0, 0), l = make_uint2(0, 0);   // a lane without a slice contributes nothing
                if (valid) {
                    h = *(const uint2 *)(dg_hi + n * EP + et * 32 + 8 * q + 4 * g);
                    l = *(const uint2 *)(dg_lo + n * EP + et * 32 + 8 * q + 4 * g);
                }
                dgh[et][2 * q] = h.x;
                dgh[et][2 * q + 1] = h.y;
                dgl[et][2 * q] = l.x;
                dgl[et][2 * q + 1] = l.y;
            }
        if (valid) act = *(const uint4 *)(relu_bits + (n * 2 + g) * 4);

        // dL/du = Wr2 dL/dg (ReLU pattern applied), dL/dx += Wr1 dL/du, both from registers
        f32x16 dx[OT];
#pragma unroll
        for (int ot = 0; ot < OT; ++ot)
#pragma unroll
            for (int i = 0; i < 16; ++i) dx[ot][i] = 0.f;
#pragma unroll 1
        for (int ht = 0; ht < kRbHT; ++ht) {
            f32x16 du;
#pragma unroll
            for (int i = 0; i < 16; ++i) du[i] = 0.f;
#pragma unroll
            for (int et = 0; et < ET; ++et)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const bf16x8 wf = __builtin_bit_cast(bf16x8, w2c[((et * 2 + s) * kRbHT + ht) * 64 + lane]);
                    du = mfma_bf16(wf, frag_of(dgl[et], s), du);
                    du = mfma_bf16(wf, frag_of(dgh[et], s), du);
                }
            const uint32_t word = (ht >> 1) == 0 ? act.x : (ht >> 1) == 1 ? act.y : (ht >> 1) == 2 ? act.z : act.w;
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
                for (int ot = 0; ot < OT; ++ot) {
                    const bf16x8 wf = __builtin_bit_cast(bf16x8, w1c[((ht * 2 + s) * OT + ot) * 64 + lane]);
                    dx[ot] = mfma_bf16(wf, frag_of(dul, s), dx[ot]);
                    dx[ot] = mfma_bf16(wf, frag_of(duh, s), dx[ot]);
                }
        }

        // dL/dh of the slices: router path plus the expert-path rows of their k assignments, one rounding.  The rows are
        // gathered and the result is stored through a tile of LDS private to the wavefront, one 32-feature tile at a
        // time, so that every memory instruction covers whole 128-byte (gather) or 64-byte (store) runs: eight lanes per
        // slice fetch and add the k row pieces, lane (j, g) picks up its accumulator order from the tile, adds the router
        // path, rounds, and puts the packed row back for four lanes per slice to store.
        const long long n0 = tile * 32;
        const int piece = lane & 7, sl = lane >> 3;
        int rws[4][8];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const long long ns = n0 + it * 8 + sl;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) rws[it][jj] = (jj < k && ns < Ns) ? inv[ns * k + jj] : -1;
        }
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 8; ++jj)
                    if (rws[it][jj] >= 0) v += *(const f32x4 *)(dxrow + (size_t)rws[it][jj] * DS + 32 * ot + 4 * piece);
                *(f32x4 *)(stg + (it * 8 + sl) * kRbStageRow + 4 * piece) = v;
            }
            wave_lds_sync();
            uint2 o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 t = *(const f32x4 *)(stg + j * kRbStageRow + 8 * q + 4 * g);
                o[q] = make_uint2(pack_bf16x2(dx[ot][4 * q] + t[0], dx[ot][4 * q + 1] + t[1]),
                                  pack_bf16x2(dx[ot][4 * q + 2] + t[2], dx[ot][4 * q + 3] + t[3]));
            }
            wave_lds_sync();   // every lane has read its sums: the tile now takes the packed rows (64 bytes per slice)
#pragma unroll
            for (int q = 0; q < 4; ++q) *(uint2 *)((char *)(stg + j * kRbStageRow) + (8 * q + 4 * g) * 2) = o[q];
            wave_lds_sync();
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int i = half * 16 + (lane >> 2), pc = lane & 3;
                const long long ns = n0 + i;
                if (ns < Ns) *(uint4 *)(dh + ns * DS + 32 * ot + 8 * pc) = *(const uint4 *)((const char *)(stg + i * kRbStageRow) + pc * 16);
            }
            wave_lds_sync();   // before the next gather overwrites the tile
        }
    }
}

// ----------------------------------------------------------------------------------------------- weights kernel
// grid = ranges of slices_per_block slices (each a slot of partial sums; rounded up to eight) x two groups of four hidden tiles, block = one
// wavefront per hidden tile of the group.
template <int DS, int ET>
__global__ __launch_bounds__(kRbWgWaves * 64, (DS * (ET + 1) <= 256) ? 2 : 1) void bwd_route_weights_mfma_kernel(
    const bf16_t *__restrict__ x, long long Ns, int E, const char *__restrict__ packed, RouterBwdPacked L,
    const bf16_t *__restrict__ dg_hi, const bf16_t *__restrict__ dg_lo, int slices_per_block, size_t slot_floats,
    float *__restrict__ part)
{
    constexpr int KS = DS / 16, OT = DS / 32, EP = ET * 32, GS = 2 * ET;   // GS: K-steps of 16 experts
    extern __shared__ __align__(16) char lds[];
    // this group's fragments only: [wave][KS][64] of w1f, [wave][GS][64] of w2r, 32 biases per wavefront
    uint4 *w1f = (uint4 *)lds;
    uint4 *w2r = w1f + kRbWgWaves * KS * 64;
    float *b1s = (float *)(w2r + kRbWgWaves * GS * 64);

    const int tid = threadIdx.x, lane = tid & 63, jj = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Consecutive blocks go to the eight XCDs in turn, each with its own L2: the two groups of a slice range, which
    // read the same rows, take block ids that are equal modulo 8.
    constexpr int kGroups = kRbHT / kRbWgWaves;   // kRbHT is a multiple of the group size
    const int ht0 = ((int)(blockIdx.x / 8) % kGroups) * kRbWgWaves, ht = ht0 + wave;
    const long long range = (long long)(blockIdx.x / (8 * kGroups)) * 8 + (long long)(blockIdx.x % 8);
    stage_bytes(packed + L.w1f + (size_t)ht0 * KS * 1024, (char *)w1f, (size_t)kRbWgWaves * KS * 1024, tid, kRbWgWaves * 64);
    stage_bytes(packed + L.w2r + (size_t)ht0 * GS * 1024, (char *)w2r, (size_t)kRbWgWaves * GS * 1024, tid, kRbWgWaves * 64);
    if (tid < kRbWgWaves * 32) b1s[tid] = ((const float *)(packed + L.b1))[ht0 * 32 + tid];
    __syncthreads();
    bf16x8 id_even, id_odd;
    identity_fragments(jj, g, id_even, id_odd);
    const float bias = b1s[wave * 32 + jj];

    f32x16 aW1[OT], aW2[ET];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
        for (int et = 0; et < ET; ++et) aW2[et][i] = 0.f;
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) aW1[ot][i] = 0.f;
    }
    float ab1 = 0.f, ab2[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et) ab2[et] = 0.f;

    const long long n_begin = range * slices_per_block;
    if (n_begin >= Ns) return;   // the grid is rounded up to whole groups of eight ranges (no barrier follows)
    const long long n_end = min(Ns, n_begin + slices_per_block);
    for (long long n0 = n_begin; n0 < n_end; n0 += 32) {
        const long long n = n0 + jj;   // as A operand a lane holds slice jj of the unit, contraction slots 8g..8g+7
        const bool valid = n < n_end;
        const long long nn = valid ? n : n_begin;
        const uint4 *xr = (const uint4 *)(x + nn * DS);
        bf16x8 xa[KS], gh[GS], gl[GS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xa[ks] = __builtin_bit_cast(bf16x8, xr[2 * ks + g]);
#pragma unroll
        for (int s = 0; s < GS; ++s) {   // experts 16s + 8g .. + 7 of the slice; slices past the end add nothing
            const uint4 z = make_uint4(0, 0, 0, 0);
            gh[s] = __builtin_bit_cast(bf16x8, valid ? *(const uint4 *)(dg_hi + nn * EP + 16 * s + 8 * g) : z);
            gl[s] = __builtin_bit_cast(bf16x8, valid ? *(const uint4 *)(dg_lo + nn * EP + 16 * s + 8 * g) : z);
        }
        // transposed: lane = hidden unit jj of this tile, register i = slice acc_feature(i, g) of the unit
        f32x16 u, du;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            u[i] = bias;
            du[i] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) u = mfma_bf16(xa[ks], __builtin_bit_cast(bf16x8, w1f[(wave * KS + ks) * 64 + lane]), u);
#pragma unroll
        for (int s = 0; s < GS; ++s) {
            const bf16x8 wf = __builtin_bit_cast(bf16x8, w2r[(wave * GS + s) * 64 + lane]);
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
#pragma unroll
        for (int et = 0; et < ET; ++et) {
            // dL/dg of the unit with lane = expert 32 et + jj, registers = slices (exact: both tables hold bf16 values)
            f32x16 gth, gtl;
#pragma unroll
            for (int i = 0; i < 16; ++i) gth[i] = gtl[i] = 0.f;
            gth = mfma_bf16(gh[2 * et], id_even, gth);
            gth = mfma_bf16(gh[2 * et + 1], id_odd, gth);
            gtl = mfma_bf16(gl[2 * et], id_even, gtl);
            gtl = mfma_bf16(gl[2 * et + 1], id_odd, gtl);
            uint32_t gthp[8], gtlp[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                gthp[i] = pack_exact_bf16x2(gth[2 * i], gth[2 * i + 1]);
                gtlp[i] = pack_exact_bf16x2(gtl[2 * i], gtl[2 * i + 1]);
                if (ht == 0) ab2[et] += (gth[2 * i] + gtl[2 * i]) + (gth[2 * i + 1] + gtl[2 * i + 1]);
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {   // dWr2 [hidden unit][expert]: lane = expert, registers = hidden units
                aW2[et] = mfma_bf16(frag_of(ul, s), frag_of(gthp, s), aW2[et]);
                aW2[et] = mfma_bf16(frag_of(uh, s), frag_of(gtlp, s), aW2[et]);
                aW2[et] = mfma_bf16(frag_of(uh, s), frag_of(gthp, s), aW2[et]);
            }
        }
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
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
    float *slot = part + (size_t)range * slot_floats;
    float *pWr1 = slot, *pWr2 = pWr1 + (size_t)DS * kRbHr, *pbr1 = pWr2 + (size_t)kRbHr * E, *pbr2 = pbr1 + kRbHr;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) pWr1[(size_t)(32 * ot + acc_feature(i, g)) * kRbHr + 32 * ht + jj] = aW1[ot][i];
#pragma unroll
        for (int et = 0; et < ET; ++et)
            if (32 * et + jj < E) pWr2[(size_t)(32 * ht + acc_feature(i, g)) * E + 32 * et + jj] = aW2[et][i];
    }
    ab1 += __shfl_xor(ab1, 32);   // the two lane groups hold different slices of the same hidden unit
    if (g == 0) pbr1[32 * ht + jj] = ab1;
#pragma unroll
    for (int et = 0; et < ET; ++et) {
        const float t = ab2[et] + __shfl_xor(ab2[et], 32);
        if (ht == 0 && g == 0 && 32 * et + jj < E) pbr2[32 * et + jj] = t;
    }
}

// ------------------------------------------------------------------------------------------------------ host
static size_t logits_lds(int ds, int ET) { return (size_t)(kRbHT * (ds / 16) + kRbHT * 2 * ET) * 1024 + (kRbHr + 32 * ET) * sizeof(float); }
static size_t inputs_lds(int ds, int ET)
{
    return (size_t)(ET * 2 * kRbHT + kRbHT * 2 * (ds / 32)) * 1024 + (size_t)kRbWaves * 32 * kRbStageRow * sizeof(float);
}
static size_t weights_lds(int ds, int ET) { return (size_t)kRbWgWaves * (ds / 16 + 2 * ET) * 1024 + kRbWgWaves * 32 * sizeof(float); }

bool backward_router_mfma_shape(const slicemoe_config &c)
{
    const int ds = c.d / c.S, ET = (c.E + 31) / 32;
    return c.dtype == SLICEMOE_BF16 && (ds == 64 || ds == 96 || ds == 128) && c.Hr == kRbHr && c.E <= 64 &&
           !(c.flags & SLICEMOE_FLAG_FORCE_GENERIC) && logits_lds(ds, ET) <= (size_t)max_lds_per_block() &&
           inputs_lds(ds, ET) <= (size_t)max_lds_per_block();
}

// scratch: the repacked router | dL/dg hi [Ns][32 ET] bf16 | dL/dg lo | ReLU bits [Ns][2][4] words
struct RouterBwdScratch {
    size_t dg_hi, dg_lo, bits, total;
};
static RouterBwdScratch router_bwd_scratch(const slicemoe_config &c)
{
    const size_t Ns = (size_t)c.T * c.S, ET = (size_t)(c.E + 31) / 32;
    RouterBwdScratch R;
    size_t at = align_up(router_bwd_layout(c.d / c.S, (int)ET).total, 256);
    R.dg_hi = at;  at += align_up(Ns * 32 * ET * sizeof(bf16_t), 256);
    R.dg_lo = at;  at += align_up(Ns * 32 * ET * sizeof(bf16_t), 256);
    R.bits = at;   at += align_up(Ns * 8 * sizeof(uint32_t), 256);
    R.total = at;
    return R;
}

size_t backward_router_mfma_scratch_bytes(const slicemoe_config &c)
{
    return backward_router_mfma_shape(c) ? router_bwd_scratch(c).total : 0;
}

template <int DS, int ET>
static hipError_t run_router_mfma(const slicemoe_config &c, const RouterBwdPacked &L, const void *h, const RouteVariant &v,
                                  const float *drop_u, float rate, const int32_t *idx, const int32_t *inv, const float *dpk,
                                  const float *dxrow, void *d_h, const char *pb, bf16_t *dg_hi, bf16_t *dg_lo, uint32_t *bits,
                                  int slices_per_block, long long slice_blocks, size_t slot_floats, float *part, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    const long long ntiles = (Ns + 31) / 32, units = (ntiles + kRbWaves - 1) / kRbWaves;
    auto lk = bwd_route_logits_mfma_kernel<DS, ET>;
    hipError_t e = grant_dynamic_lds((const void *)lk, logits_lds(DS, ET));
    if (e != hipSuccess) return e;
    // as many blocks as can be resident at once (registers and LDS allow two per CU for the narrow shapes)
    static int lk_per_cu = 0;   // per instantiation; the same on every device of the machine
    if (lk_per_cu == 0) {
        int n = 1;
        if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void *)lk, kRbThreads, logits_lds(DS, ET))) != hipSuccess) return e;
        lk_per_cu = n < 1 ? 1 : n;
    }
    long long blocks = (long long)num_compute_units() * lk_per_cu;
    if (blocks > units) blocks = units;
    lk<<<(int)blocks, kRbThreads, logits_lds(DS, ET), s>>>((const bf16_t *)h, Ns, c.E, c.k, pb, L, v.sigma > 0.f ? v.noise : nullptr,
                                                           v.sigma, v.inv_tau, rate > 0.f ? drop_u : nullptr, rate, idx, inv, dpk,
                                                           v.capg, dg_hi, dg_lo, bits);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    auto ik = bwd_route_inputs_mfma_kernel<DS, ET>;
    if ((e = grant_dynamic_lds((const void *)ik, inputs_lds(DS, ET))) != hipSuccess) return e;
    // one block per CU: this kernel waits on its row gathers, and a second resident block measured slower (cache misses)
    blocks = num_compute_units() < units ? num_compute_units() : units;
    ik<<<(int)blocks, kRbThreads, inputs_lds(DS, ET), s>>>(Ns, c.k, pb, L, inv, dxrow, dg_hi, dg_lo, bits, (bf16_t *)d_h);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    auto wk = bwd_route_weights_mfma_kernel<DS, ET>;
    if ((e = grant_dynamic_lds((const void *)wk, weights_lds(DS, ET))) != hipSuccess) return e;
    wk<<<(unsigned)((slice_blocks + 7) / 8 * 8 * (kRbHT / kRbWgWaves)), kRbWgWaves * 64, weights_lds(DS, ET), s>>>(
        (const bf16_t *)h, Ns, c.E, pb, L, dg_hi, dg_lo, slices_per_block, slot_floats, part);
    return hipGetLastError();
}

// scratch: backward_router_mfma_scratch_bytes; part: slice_blocks = ceil(Ns / slices_per_block) slots of slot_floats
// floats (the slice ranges of the vector-ALU router kernel; slices_per_block a multiple of 32).  dxrow, dpk: the expert stage's row gradients and dL/dp.
hipError_t launch_backward_router_mfma(const slicemoe_config &c, const void *h, const slicemoe_weights &w,
                                       const RouteVariant &v, const float *drop_u, float rate, const int32_t *idx,
                                       const int32_t *inv, const float *dpk, const float *dxrow, void *d_h, void *scratch,
                                       int slices_per_block, long long slice_blocks, size_t slot_floats, float *part,
                                       hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    if (!backward_router_mfma_shape(c) || slices_per_block < 32 || slices_per_block % 32 != 0 ||
        slice_blocks != (Ns + slices_per_block - 1) / slices_per_block)
        return hipErrorInvalidValue;
    const int E = c.E, Hr = kRbHr, ds = c.d / c.S, ET = (E + 31) / 32, EP = 32 * ET;
    const RouterBwdPacked L = router_bwd_layout(ds, ET);
    const RouterBwdScratch R = router_bwd_scratch(c);
    char *pb = (char *)scratch;
    bf16_t *dg_hi = (bf16_t *)(pb + R.dg_hi), *dg_lo = (bf16_t *)(pb + R.dg_lo);
    uint32_t *bits = (uint32_t *)(pb + R.bits);
    const bf16_t *Wr1 = (const bf16_t *)w.Wr1, *Wr2 = (const bf16_t *)w.Wr2;
    BwdPackJobs jobs;
    jobs.count = 7;
    // w1f: Wr1 [ds, Hr] itself.  w2f: Wr2 [Hr, E] with the hidden units as contraction slots, fp16, experts padded to EP.
    jobs.job[0] = bwd_pack_job(kPackLayer1, Wr1, ds, ds, Hr, Hr, (size_t)Hr, 1, 0, pb + L.w1f, 0, 1);
    jobs.job[1] = bwd_pack_job(kPackChainF16, Wr2, Hr, Hr, EP, E, (size_t)E, 1, 0, pb + L.w2f, 0, 1);
    // w2c: M[e][h] = Wr2[h][e] ([EP, Hr], experts as contraction slots).  w1c: M[h][c] = Wr1[c][h] ([Hr, ds]).
    jobs.job[2] = bwd_pack_job(kPackChain, Wr2, EP, E, Hr, Hr, 1, (size_t)E, 0, pb + L.w2c, 0, 1);
    jobs.job[3] = bwd_pack_job(kPackChain, Wr1, Hr, Hr, ds, ds, 1, (size_t)Hr, 0, pb + L.w1c, 0, 1);
    // w2r: M[e][h] = Wr2[h][e] ([EP, Hr]) in plain K-steps of 16 experts
    jobs.job[4] = bwd_pack_job(kPackLayer1, Wr2, EP, E, Hr, Hr, 1, (size_t)E, 0, pb + L.w2r, 0, 1);
    jobs.job[5] = bwd_pack_job(kPackBias, w.br1, Hr, Hr, Hr, Hr, 0, 0, 0, pb + L.b1, 0, 1);
    jobs.job[6] = bwd_pack_job(kPackBias, w.br2, E, E, EP, EP, 0, 0, 0, pb + L.b2, 0, 1);
    const hipError_t e = bwd_pack_launch(jobs, s);
    if (e != hipSuccess) return e;
#define SLICEMOE_ROUTER_BWD(DSV, ETV)                                                                                            \
    if (ds == DSV && ET == ETV)                                                                                                  \
        return run_router_mfma<DSV, ETV>(c, L, h, v, drop_u, rate, idx, inv, dpk, dxrow, d_h, pb, dg_hi, dg_lo, bits, slices_per_block, slice_blocks, \
                                         slot_floats, part, s);
    SLICEMOE_ROUTER_BWD(64, 1)
    SLICEMOE_ROUTER_BWD(64, 2)
    SLICEMOE_ROUTER_BWD(96, 1)
    SLICEMOE_ROUTER_BWD(96, 2)
    SLICEMOE_ROUTER_BWD(128, 1)
    SLICEMOE_ROUTER_BWD(128, 2)
#undef SLICEMOE_ROUTER_BWD
    return hipErrorInvalidValue;
}

}  // namespace slicemoe
