// Grouped expert FFN on the matrix cores (the "fused batched GEMM" of paper Section 3.4, with
// the expert of Section 3.1 and the input weighting of Eq. 1), bf16 inputs, fp32 accumulation.
//
//   y[r, :] = GELU(p_r * (x_r W1[e]) + b1[e]) W2[e] + b2[e]          (p (x W1) == (p x) W1)
//
// One launch covers all experts; the per-expert row ranges come from offsets[] on the device.
// A wavefront owns a unit of 32*NSUB stacked rows and the whole hidden width.  Per 32-wide
// hidden tile it runs GEMM1 (bf16 MFMA, K = ds), turns its 16 fp32 accumulators per lane into 8
// packed fp16 pairs of activations and feeds them straight into GEMM2 (fp16 MFMA) as the B
// operand (see mfma.h): the [rows, He] hidden activations never exist in memory.  x rows are
// gathered through perm[] by the loads themselves; the rows of the next unit are loaded while
// the current one is computed.  Weights come pre-packed in fragment order and sit in LDS.
// y is written as fp16; the two half-wavefronts exchange registers so that every lane stores
// whole 16-byte pieces of a row.
//
// Activation stage (the part that bounds this kernel: with ds = 64 every hidden element is fed
// by only 16 matrix-core cycles per lane, so the vector ALU work per element decides the speed).
// It runs entirely on packed fp16 instructions, two hidden elements per instruction:
//   A  = cvt_pkrtz(acc0, acc1)                 fp32 accumulators -> fp16 pair
//   s  = A * (kappa p) + kappa b1              s = kappa z, kappa = 1/4           (Eq. 1 scale + bias)
//   v  = s * s - w0
//   Q  = Horner in v, degree kGeluM            s Q(v) ~ Phi(z) - 1/2 on |z| <= zc, and > 1/2 beyond
//   F  = clamp01(s * Q + 1/2)                  ~ Phi(z): the instruction's own [0,1] clamp saturates it
//   g  = s * F                                 = kappa GELU(z)
// W2 is packed pre-multiplied by 1/kappa, so GEMM2 needs no rescaling.  fp16 has three more
// mantissa bits than the bf16 storage type; evaluated this way the activation error is of the
// size of a bf16 rounding: at most 2^-8 (rms below 8e-4) of the larger of |z| and |p a| (the same
// roundings are replayed on the CPU in tests/test_gelu_poly.py).
// Hidden activations beyond +-65504 / kappa would overflow fp16.
//
// Two variants:
//   resident  a whole expert (W1, W2, biases) fits in LDS (ds = 64, He <= 256).  One block of 16
//             wavefronts per CU (four per SIMD, so that one wavefront's matrix work overlaps
//             another's vector work); stacked rows are split evenly over the blocks regardless of
//             expert boundaries; a block re-stages weights only when its range crosses into
//             another expert.  Wavefront priority follows the number of units a wavefront still
//             has to do, which keeps the 16 wavefronts finishing together.
//   streamed  larger experts (ds = 128, He = 512: 256 KiB; ds = 96, He = 384 of the paper's own shape:
//             144 KiB): a block walks tiles of one expert and streams the weights through LDS in chunks
//             of hidden tiles, per row tile.
#include "mfma.h"

namespace slicemoe {

typedef _Float16 half_t;
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Packed fp16 constants of the activation stage, passed by value (uniform: they live in SGPRs).
struct EpiConst {
    uint32_t neg_w0;
    uint32_t q[kGeluM + 1];
    uint32_t half;
};

static uint32_t pack2_f16(float f)
{
    const _Float16 h = (_Float16)f;
    uint16_t u;
    __builtin_memcpy(&u, &h, 2);
    return (uint32_t)u | ((uint32_t)u << 16);
}

static EpiConst make_epi_const()
{
    EpiConst K;
    K.neg_w0 = pack2_f16(-kGeluW0);
    for (int i = 0; i <= kGeluM; ++i) K.q[i] = pack2_f16(kGeluQ[i]);
    K.half = pack2_f16(0.5f);
    return K;
}

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ h2 pk_fma(h2 a, h2 b, h2 c) { return __builtin_elementwise_fma(a, b, c); }
// fused multiply-add with the instruction's output clamp to [0, 1]
__device__ __forceinline__ h2 pk_fma_clamp01(h2 a, h2 b, h2 c)
{
    h2 d;
    asm("v_pk_fma_f16 %0, %1, %2, %3 clamp" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// 16 accumulators of one 32x32 tile -> 8 packed fp16 pairs of kappa * GELU(z); pair i holds the
// accumulator registers 2i and 2i+1, i.e. contraction slots of GEMM2 in register order.
__device__ __forceinline__ void activation_tile(const f32x16 &acc, h2 p2, const h2 (&bias)[8], const EpiConst &K, uint4 (&out)[2])
{
    uint32_t o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const h2 A = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(acc[2 * i], acc[2 * i + 1]));
        const h2 s = pk_fma(A, p2, bias[i]);
        const h2 v = pk_fma(s, s, as_h2(K.neg_w0));
        h2 Q = pk_fma(v, as_h2(K.q[kGeluM]), as_h2(K.q[kGeluM - 1]));
#pragma unroll
        for (int c = kGeluM - 2; c >= 0; --c) Q = pk_fma(Q, v, as_h2(K.q[c]));
        const h2 F = pk_fma_clamp01(s, Q, as_h2(K.half));
        o[i] = __builtin_bit_cast(uint32_t, s * F);
    }
    out[0] = make_uint4(o[0], o[1], o[2], o[3]);
    out[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

template <int DS, int NSUB> struct RowUnit {
    bf16x8 xb[NSUB][SliceTiles<DS>::KS];
    h2 p2[NSUB];   // (kappa p, kappa p), zero for a lane without a row
    int row[NSUB]; // -1: no row
};

// The 16 fp16 biases (already scaled by kappa) of hidden tile ht for lane group g, in accumulator order.
__device__ __forceinline__ void load_bias_tile(const uint4 *__restrict__ b1s, int ht, int g, h2 (&bias)[8])
{
    const uint4 b0 = b1s[(ht * 2 + g) * 2 + 0], b1 = b1s[(ht * 2 + g) * 2 + 1];
    bias[0] = as_h2(b0.x); bias[1] = as_h2(b0.y); bias[2] = as_h2(b0.z); bias[3] = as_h2(b0.w);
    bias[4] = as_h2(b1.x); bias[5] = as_h2(b1.y); bias[6] = as_h2(b1.z); bias[7] = as_h2(b1.w);
}

// AHEAD: the weight fragment of the next K-step is requested from LDS before this step's matrix instructions, so
// that they do not each wait for an LDS round trip (for kernels with few wavefronts per SIMD to cover it).
template <int DS, int NSUB, bool AHEAD = false>
__device__ __forceinline__ void gemm1_tile(const RowUnit<DS, NSUB> &u, const uint4 *__restrict__ w1s, int hl, int lane,
                                           f32x16 (&acc)[NSUB])
{
    constexpr int KS = SliceTiles<DS>::KS;
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[sub][r] = 0.f;
    if constexpr (AHEAD) {
        uint4 nxt = w1s[(hl * KS) * 64 + lane];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a1 = __builtin_bit_cast(bf16x8, nxt);
            if (ks + 1 < KS) nxt = w1s[(hl * KS + ks + 1) * 64 + lane];
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) acc[sub] = mfma_bf16(a1, u.xb[sub][ks], acc[sub]);
        }
    } else {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a1 = __builtin_bit_cast(bf16x8, w1s[(hl * KS + ks) * 64 + lane]);
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) acc[sub] = mfma_bf16(a1, u.xb[sub][ks], acc[sub]);
        }
    }
}

template <int DS, int NSUB, bool AHEAD = false>
__device__ __forceinline__ void gemm2_tile(const uint4 (&hb)[NSUB][2], const uint4 *__restrict__ w2s, int hl, int lane,
                                           f32x16 (&yacc)[NSUB][SliceTiles<DS>::OT])
{
    constexpr int OT = SliceTiles<DS>::OT;
    if constexpr (AHEAD) {
        uint4 nxt = w2s[(hl * 2 * OT) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 2 * OT; ++i) {   // i = s * OT + ot
            const f16x8 a2 = __builtin_bit_cast(f16x8, nxt);
            if (i + 1 < 2 * OT) nxt = w2s[(hl * 2 * OT + i + 1) * 64 + lane];
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                yacc[sub][i % OT] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, __builtin_bit_cast(f16x8, hb[sub][i / OT]), yacc[sub][i % OT], 0, 0, 0);
        }
    } else {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                const f16x8 a2 = __builtin_bit_cast(f16x8, w2s[((hl * 2 + s) * OT + ot) * 64 + lane]);
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub)
                    yacc[sub][ot] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, __builtin_bit_cast(f16x8, hb[sub][s]), yacc[sub][ot], 0, 0, 0);
            }
    }
}

__device__ __forceinline__ uint32_t pack_half2(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}

// y rows as fp16.  Per output tile a lane holds features 8q + 4g + (0..3) of its own row, i.e. half
// of each 16-byte piece; lanes j and j + 32 trade halves (v_permlane32_swap) so that lane (j, g)
// ends up with the whole pieces q = 2*qp + g and stores them with one 16-byte write each.
template <int DS, int NSUB>
__device__ __forceinline__ void store_rows(const RowUnit<DS, NSUB> &u, const f32x16 (&yacc)[NSUB][SliceTiles<DS>::OT],
                                           const float *__restrict__ b2s, half_t *__restrict__ y, int g)
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        half_t *yr = y + (size_t)(u.row[sub] < 0 ? 0 : u.row[sub]) * DS;
#pragma unroll
        for (int ot = 0; ot < SliceTiles<DS>::OT; ++ot)
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) {
                if (ot * 4 + 2 * qp >= SliceTiles<DS>::P) continue;   // padding columns of the last tile
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
                if (u.row[sub] >= 0 && ot * 4 + 2 * qp + g < SliceTiles<DS>::P) {
                    const uint4 v = make_uint4(s0[0], s1[0], s0[1], s1[1]);
                    *(uint4 *)(yr + ot * 32 + 8 * (2 * qp + g)) = v;
                }
            }
    }
}

template <int DS, int NSUB>
__device__ __forceinline__ void zero_acc(f32x16 (&yacc)[NSUB][SliceTiles<DS>::OT])
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int ot = 0; ot < SliceTiles<DS>::OT; ++ot)
#pragma unroll
            for (int r = 0; r < 16; ++r) yacc[sub][ot][r] = 0.f;
}

// Stacked row of lane j in sub-tile `sub` of the unit starting at `base` (or -1 past `end`), and its
// assignment id; a lane without a row reads perm[0], which keeps every later access in bounds.
template <int NSUB>
__device__ __forceinline__ void unit_rows(int base, int end, bool unit_ok, int j, const int32_t *__restrict__ perm,
                                          int (&row)[NSUB], int (&a)[NSUB])
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const int rr = base + sub * 32 + j;
        const bool ok = unit_ok && rr < end;
        row[sub] = ok ? rr : -1;
        a[sub] = perm[ok ? rr : 0];
    }
}

// Issue the gather of one unit: lane (j, g) reads the 16-byte pieces 2*ks + g of its row.
template <int DS, int NSUB>
__device__ __forceinline__ void load_rows(RowUnit<DS, NSUB> &u, const int (&a)[NSUB], const int (&row)[NSUB],
                                          const bf16_t *__restrict__ x, const float *__restrict__ pk, int k, int g,
                                          float (&p)[NSUB])
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        u.row[sub] = row[sub];
        const long long n = a[sub] / k;
        const uint4 *xr = (const uint4 *)(x + n * DS);
#pragma unroll
        for (int ks = 0; ks < SliceTiles<DS>::KS; ++ks) u.xb[sub][ks] = load_row_piece<DS>(xr, ks, g);
        p[sub] = pk[a[sub]];
    }
}

template <int DS, int NSUB>
__device__ __forceinline__ void set_p(RowUnit<DS, NSUB> &u, const float (&p)[NSUB])
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const float pv = u.row[sub] >= 0 ? p[sub] * kGeluKappa : 0.f;
        u.p2[sub] = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(pv, pv));
    }
}

// ------------------------------------------------------------------------------ resident
constexpr int kResU = 32;  // rows per wavefront unit (NSUB = 1)

// One expert block in LDS exactly as it is packed in memory (W1 | W2 | b1 fp16 | b2 fp32, see pack.hip).
// THREADS = 1024 (16 wavefronts of <= 128 registers) for ds = 64; ds = 96 keeps 48 more accumulator and
// row registers per lane and runs 12 wavefronts of <= 168.
template <int DS, int HT, int THREADS>
__global__ __launch_bounds__(THREADS) void ffn_resident_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const char *__restrict__ experts, size_t e_stride, size_t off_w2,
    size_t off_b1, size_t off_b2, int E, int k, EpiConst K, half_t *__restrict__ y)
{
    constexpr int kResWaves = THREADS / 64;
    extern __shared__ __align__(16) char lds[];
    const uint4 *w1s = (const uint4 *)lds;                  // [HT][DS/16][64] fragments
    const uint4 *w2s = (const uint4 *)(lds + off_w2);       // [HT][2][DS/32][64] fragments
    const uint4 *b1s = (const uint4 *)(lds + off_b1);       // [HT][2][16] fp16
    const float *b2s = (const float *)(lds + off_b2);       // [DS]

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // lane e keeps the end of expert e's row range: expert lookups are one ballot, not a chain of loads
    const int off_hi = offsets[min(lane + 1, E)];
    const int n_kept = __builtin_amdgcn_readfirstlane(__shfl(off_hi, E - 1));

    // even split of the kept rows over the blocks, in whole units; blocks that share an XCD (blockIdx % 8)
    // take consecutive row ranges, so an expert's weights are fetched into few L2s
    const int units_total = (n_kept + kResU - 1) / kResU;
    const int units_per_block = (units_total + gridDim.x - 1) / gridDim.x;
    const int vblock = gridDim.x % 8 == 0 ? (int)(blockIdx.x % 8) * (int)(gridDim.x / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    const long long r_begin = (long long)vblock * units_per_block * kResU;
    const int r_end = (int)min((long long)n_kept, r_begin + (long long)units_per_block * kResU);

    int r = (int)min(r_begin, (long long)n_kept);
    while (r < r_end) {
        const int e = __builtin_amdgcn_readfirstlane(__popcll(__ballot(lane < E && off_hi <= r)));
        const int seg_end = min(__builtin_amdgcn_readfirstlane(__shfl(off_hi, e)), r_end);
        const char *ew = experts + (size_t)e * e_stride;
        const int nunits = (seg_end - r + kResU - 1) / kResU;   // this wavefront takes units wave, wave + kResWaves, ...

        __syncthreads();  // everyone is done with the previous expert's weights
        int q_c = wave;
        int row_c[1], a_c[1], row_n[1], a_n[1];
        float p_c[1], p_n[1];
        unit_rows<1>(r + q_c * kResU, seg_end, q_c < nunits, j, perm, row_c, a_c);   // index load rides along with the weights
        // stage the expert block (one linear copy: it is packed exactly as the kernel reads it)
        stage_to_lds<THREADS>(ew, lds, (int)(e_stride / 16), tid);
        RowUnit<DS, 1> cur, nxt;
        load_rows<DS, 1>(cur, a_c, row_c, x, pk, k, g, p_c);
        set_p<DS, 1>(cur, p_c);
        __syncthreads();

        while (q_c < nunits) {
            const int q_n = q_c + kResWaves;
            {   // fewer units left -> lower priority: the wavefronts of a block finish together
                const int left = (nunits - 1 - q_c) / kResWaves;
                if (left >= 3) __builtin_amdgcn_s_setprio(3);
                else if (left == 2) __builtin_amdgcn_s_setprio(2);
                else if (left == 1) __builtin_amdgcn_s_setprio(1);
                else __builtin_amdgcn_s_setprio(0);
            }
            unit_rows<1>(r + q_n * kResU, seg_end, q_n < nunits, j, perm, row_n, a_n);

            f32x16 yacc[1][SliceTiles<DS>::OT];
            zero_acc<DS, 1>(yacc);
            f32x16 acc[2][1];
            uint4 hb[1][2];
            gemm1_tile<DS, 1>(cur, w1s, 0, lane, acc[0]);
#pragma unroll
            for (int hl = 0; hl < HT; ++hl) {
                if (hl + 1 < HT) gemm1_tile<DS, 1>(cur, w1s, hl + 1, lane, acc[(hl + 1) & 1]);
                h2 bias[8];
                load_bias_tile(b1s, hl, g, bias);
                activation_tile(acc[hl & 1][0], cur.p2[0], bias, K, hb[0]);
                gemm2_tile<DS, 1>(hb, w2s, hl, lane, yacc);
                if (hl == (HT - 1) / 2) load_rows<DS, 1>(nxt, a_n, row_n, x, pk, k, g, p_n);   // half a unit of lead time
            }
            store_rows<DS, 1>(cur, yacc, b2s, y, g);
            cur = nxt;
            set_p<DS, 1>(cur, p_n);
            q_c = q_n;
        }
        r = seg_end;
    }
}

// ------------------------------------------------------------------------------ streamed
// THREADS = 512: two wavefronts per SIMD, one's matrix work overlaps the other's vector work.  Slice width 384 needs
// 192 output accumulators and 96 row registers per lane, more than half a SIMD's register file: 256 threads there.

template <int DS, int NSUB, int THREADS>
__global__ __launch_bounds__(THREADS) void ffn_streamed_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const char *__restrict__ experts, size_t e_stride, size_t off_w1,
    size_t off_w2, size_t off_b1, size_t off_b2, int He, int E, int k, int hc, EpiConst K, half_t *__restrict__ y)
{
    constexpr int KS = SliceTiles<DS>::KS;
    constexpr int OT = SliceTiles<DS>::OT;
    constexpr int kFfnWaves = THREADS / 64;
    constexpr int TM = kFfnWaves * NSUB * 32;
    constexpr int kRound = DS <= 64 ? 8 : 4;   // pieces in flight per thread while staging (register budget)
    const int HT = He / 32;
    const int nchunks = HT / hc;

    extern __shared__ __align__(16) char lds[];
    uint4 *w1s = (uint4 *)lds;                                     // [hc][KS][64] fragments
    uint4 *w2s = w1s + (size_t)hc * KS * 64;                       // [hc][2][OT][64] fragments
    uint4 *b1s = w2s + (size_t)hc * 2 * OT * 64;                   // [HT][2][16] fp16 = He * 2 bytes
    float *b2s = (float *)(b1s + He / 8);                          // [OT*32]
    int *tile_prefix = (int *)(b2s + OT * 32);                     // [E+1]

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
        float p[NSUB];
        unit_rows<NSUB>(row_begin + wave * NSUB * 32, row_end, true, j, perm, row, a);
        RowUnit<DS, NSUB> cur;
        load_rows<DS, NSUB>(cur, a, row, x, pk, k, g, p);
        set_p<DS, NSUB>(cur, p);

        f32x16 yacc[NSUB][OT];
        zero_acc<DS, NSUB>(yacc);
        for (int ch = 0; ch < nchunks; ++ch) {
            __syncthreads();  // everyone is done with the previous contents
            stage_to_lds<THREADS, kRound>((const uint4 *)(ew + off_w1) + (size_t)ch * hc * KS * 64, w1s, hc * KS * 64, tid);
            stage_to_lds<THREADS, kRound>((const uint4 *)(ew + off_w2) + (size_t)ch * hc * 2 * OT * 64, w2s, hc * 2 * OT * 64, tid);
            if (new_expert && ch == 0) {
                const uint4 *gb1 = (const uint4 *)(ew + off_b1);
                const float *gb2 = (const float *)(ew + off_b2);
                for (int i = tid; i < He / 8; i += THREADS) b1s[i] = gb1[i];
                for (int i = tid; i < OT * 32; i += THREADS) b2s[i] = gb2[i];   // padded with zeros by the packer
            }
            __syncthreads();
            for (int hl = 0; hl < hc; ++hl) {
                f32x16 acc[NSUB];
                gemm1_tile<DS, NSUB, true>(cur, w1s, hl, lane, acc);
                h2 bias[8];
                load_bias_tile(b1s, ch * hc + hl, g, bias);
                uint4 hb[NSUB][2];
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) activation_tile(acc[sub], cur.p2[sub], bias, K, hb[sub]);
                gemm2_tile<DS, NSUB, true>(hb, w2s, hl, lane, yacc);
            }
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

// Shapes the resident kernel is instantiated for: the benchmark shapes and He = 4 ds of the paper's slice widths.
static bool resident_shape(int ds, int He)
{
    return (ds == 64 && (He == 64 || He == 128 || He == 256)) || (ds == 96 && He == 384) || (ds == 48 && He == 192) ||
           (ds == 24 && He == 96);
}

// Whole expert resident in LDS where an instantiation exists (ds = 96, He = 384 takes 145 KiB), else hidden tiles per
// chunk.
static FfnPlan plan_ffn(const PackedLayout &L)
{
    const int ds = L.ds, He = L.He, E = L.E;
    const int HT = He / 32, KS = L.dsK / 16, OT = L.dsN / 32;
    const size_t frag_per_ht = (size_t)(KS + 2 * OT) * 1024;  // bytes of W1+W2 fragments per hidden tile
    const size_t dev_max = (size_t)max_lds_per_block();
    FfnPlan p;
    if (resident_shape(ds, He) && L.e_stride <= dev_max) {
        p.resident = true;
        p.hc = HT;
        p.lds = L.e_stride;
        return p;
    }
    // a streamed block needs the whole register file of its CU anyway, so chunks may take most of the LDS
    const size_t fixed = (size_t)He * 2 + (size_t)(L.dsN + E + 1) * 4 + 64;
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

template <int DS, int HT, int THREADS>
static hipError_t run_resident(const slicemoe_config &c, const PackedLayout &L, const FfnPlan &pl, const void *h,
                               const float *p, const int32_t *offsets, const int32_t *perm, const char *experts,
                               void *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    const long long max_units = (Na + kResU - 1) / kResU;
    long long blocks = max_units;   // small inputs: spread the units over all CUs rather than fill few blocks
    if (blocks > num_compute_units()) blocks = num_compute_units();
    auto kern = ffn_resident_kernel<DS, HT, THREADS>;
    hipError_t err = grant_dynamic_lds((const void *)kern, pl.lds);
    if (err != hipSuccess) return err;
    kern<<<(int)blocks, THREADS, pl.lds, s>>>((const bf16_t *)h, p, offsets, perm, experts, L.e_stride, L.e_w2, L.e_b1,
                                                  L.e_b2, c.E, c.k, make_epi_const(), (half_t *)y);
    return hipGetLastError();
}

template <int DS, int NSUB, int THREADS = 512>
static hipError_t run_streamed(const slicemoe_config &c, const PackedLayout &L, const FfnPlan &pl, const void *h,
                               const float *p, const int32_t *offsets, const int32_t *perm, const char *experts,
                               void *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    constexpr int TM = THREADS / 64 * NSUB * 32;
    const long long max_tiles = (Na + TM - 1) / TM + c.E;
    long long blocks = (long long)num_compute_units() * (pl.lds <= 78 * 1024 ? 2 : 1);
    if (blocks > max_tiles) blocks = max_tiles;
    auto kern = ffn_streamed_kernel<DS, NSUB, THREADS>;
    hipError_t err = grant_dynamic_lds((const void *)kern, pl.lds);
    if (err != hipSuccess) return err;
    kern<<<(int)blocks, THREADS, pl.lds, s>>>((const bf16_t *)h, p, offsets, perm, experts, L.e_stride, L.e_w1, L.e_w2,
                                                  L.e_b1, L.e_b2, c.He, c.E, c.k, pl.hc, make_epi_const(), (half_t *)y);
    return hipGetLastError();
}

hipError_t launch_ffn_mfma(const slicemoe_config &c, const void *h, const float *p,
                           const int32_t *offsets, const int32_t *perm, const void *packed,
                           void *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    if (Na == 0) return hipSuccess;
    const PackedLayout L = packed_layout(c);
    const FfnPlan pl = plan_ffn(L);
    const char *experts = (const char *)packed + L.experts;
    if (pl.resident) {
        if (L.ds == 24) return run_resident<24, 3, 1024>(c, L, pl, h, p, offsets, perm, experts, y, s);
        if (L.ds == 48) return run_resident<48, 6, 1024>(c, L, pl, h, p, offsets, perm, experts, y, s);
        if (L.ds == 96) return run_resident<96, 12, 768>(c, L, pl, h, p, offsets, perm, experts, y, s);
        if (L.He == 256) return run_resident<64, 8, 1024>(c, L, pl, h, p, offsets, perm, experts, y, s);
        if (L.He == 128) return run_resident<64, 4, 1024>(c, L, pl, h, p, offsets, perm, experts, y, s);
        return run_resident<64, 2, 1024>(c, L, pl, h, p, offsets, perm, experts, y, s);
    }
    if (L.ds == 24) return run_streamed<24, 2>(c, L, pl, h, p, offsets, perm, experts, y, s);
    if (L.ds == 48) return run_streamed<48, 2>(c, L, pl, h, p, offsets, perm, experts, y, s);
    if (L.ds == 64) return run_streamed<64, 2>(c, L, pl, h, p, offsets, perm, experts, y, s);
    if (L.ds == 96) return run_streamed<96, 2>(c, L, pl, h, p, offsets, perm, experts, y, s);
    if (L.ds == 192) return run_streamed<192, 1>(c, L, pl, h, p, offsets, perm, experts, y, s);   // 96 output accumulators per row tile
    if (L.ds == 384) return run_streamed<384, 1, 256>(c, L, pl, h, p, offsets, perm, experts, y, s);
    return run_streamed<128, 2>(c, L, pl, h, p, offsets, perm, experts, y, s);
}

}  // namespace slicemoe
