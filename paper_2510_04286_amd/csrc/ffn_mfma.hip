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
//   A  = cvt_pkrtz(acc0, acc1)                 fp32 accumulators kappa (x W1) -> fp16 pair; kappa = 1/4 sits in the packed W1
//   s  = A * p + kappa b1                      s = kappa z                        (Eq. 1 scale + bias)
//   v  = s * s - w0
//   Q  = Horner in v, degree kGeluM            s Q(v) ~ Phi(z) - 1/2 on |z| <= zc, and > 1/2 beyond
//   F  = clamp01(s * Q + 1/2)                  ~ Phi(z): the instruction's own [0,1] clamp saturates it
//   g  = s * F                                 = kappa GELU(z)
// W2 is packed pre-multiplied by 1/kappa, so GEMM2 needs no rescaling.  fp16 has three more
// mantissa bits than the bf16 storage type; evaluated this way the activation error is of the
// size of a bf16 rounding: at most 2^-8 (rms below 8e-4) of the larger of |z| and |p a| (the same
// roundings are replayed on the CPU in tests/test_gelu_poly.py).
// Range: |x W1| beyond 65504 / kappa saturates the conversion, |z| beyond that overflows fp16.
//
// Three variants:
//   pipelined a whole expert fits in LDS twice over (ds = 64, He <= 256: the benchmark shapes).  One block of
//             eight wavefronts per CU holds the images of up to two experts; stacked rows are split evenly over
//             the blocks regardless of expert boundaries; inside a wavefront the stages of consecutive hidden
//             tiles overlap in time (see the kernel).
//   resident  the same row split with one expert image and a plain tile loop, for the slice widths of the paper's
//             own layer (24, 48, 96), whose tile counts or register needs do not fit the pipelined form: 12 or 16
//             wavefronts, one wavefront's matrix work overlapping another's vector work; a block re-stages
//             weights when its range crosses into another expert; wavefront priority follows the number of units
//             a wavefront still has to do, which keeps them finishing together.
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
    h2 p2[NSUB];   // (p, p), zero for a lane without a row
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
// One call stores the two pieces 2*qp, 2*qp + 1 of output tile ot of the row (row < 0: nothing is written); BIAS: the
// second-layer bias is added here (it is already in the accumulators when they started from it).
template <int DS, bool BIAS>
__device__ __forceinline__ void store_row_pieces(int row, const f32x16 &acc, int ot, int qp, const float *__restrict__ b2s,
                                                 half_t *__restrict__ y, int g)
{
    if (ot * 4 + 2 * qp >= SliceTiles<DS>::P) return;   // padding columns of the last tile
    half_t *yr = y + (size_t)(row < 0 ? 0 : row) * DS;
    uint32_t lo[2], hi[2];  // lo: piece q = 2qp, hi: piece q = 2qp + 1 (this lane's half of each)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int q = 2 * qp + t;
        uint32_t d0, d1;
        if constexpr (BIAS) {
            const f32x4 bb = *(const f32x4 *)(b2s + ot * 32 + 8 * q + 4 * g);
            d0 = pack_half2(acc[4 * q + 0] + bb[0], acc[4 * q + 1] + bb[1]);
            d1 = pack_half2(acc[4 * q + 2] + bb[2], acc[4 * q + 3] + bb[3]);
        } else {   // (an addition of zero would still be an instruction: it can change the sign of a zero)
            d0 = pack_half2(acc[4 * q + 0], acc[4 * q + 1]);
            d1 = pack_half2(acc[4 * q + 2], acc[4 * q + 3]);
        }
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
    if (row >= 0 && ot * 4 + 2 * qp + g < SliceTiles<DS>::P) {
        const uint4 v = make_uint4(s0[0], s1[0], s0[1], s1[1]);
        *(uint4 *)(yr + ot * 32 + 8 * (2 * qp + g)) = v;
    }
}

template <int DS, int NSUB, bool BIAS = true>
__device__ __forceinline__ void store_rows(const RowUnit<DS, NSUB> &u, const f32x16 (&yacc)[NSUB][SliceTiles<DS>::OT],
                                           const float *__restrict__ b2s, half_t *__restrict__ y, int g)
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
        for (int ot = 0; ot < SliceTiles<DS>::OT; ++ot)
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) store_row_pieces<DS, BIAS>(u.row[sub], yacc[sub][ot], ot, qp, b2s, y, g);
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
                                          float (&p)[NSUB], int kshift = -1 /* log2(k) when k is a power of two */)
{
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        u.row[sub] = row[sub];
        const long long n = kshift >= 0 ? (long long)(a[sub] >> kshift) : (long long)(a[sub] / k);
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
        const float pv = u.row[sub] >= 0 ? p[sub] : 0.f;
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

// ------------------------------------------------------------------------------ resident, software-pipelined
// The same row split as the resident kernel, with the three stages of a hidden tile -- GEMM1, activation, GEMM2 --
// taken apart in time inside every wavefront: in one step the wavefront issues GEMM1 of tile t, the activation of tile
// t-1 and GEMM2 of tile t-2, which do not depend on each other, so its matrix instructions and its vector instructions
// interleave one to nine without waiting for one another (in the plain loop the activation waits for the matrix
// instructions just issued, and a wavefront's vector work only overlaps other wavefronts' matrix work).  The steps run
// on across the units of a wavefront: the first two steps of a unit finish the previous unit (its last activation and
// GEMM2s, then its rows are stored), and one more pair of steps after the last unit drains the pipeline.  Weight
// fragments come from LDS through a ring of four register sets, each requested four matrix instructions ahead.
// Every matrix instruction is followed by half of the activation of two pairs of hidden units (nine packed
// instructions from two independent chains); scheduling fences keep that order.  HT even (accumulator and activation
// buffers alternate by tile parity) and a multiple of four matrix instructions per step (the ring position of a
// fragment is then fixed).
// The LDS holds TWO experts: a block whose rows straddle an expert boundary stages both and its wavefronts walk
// the units of both in one pipeline (a unit names its expert's slot), instead of draining, synchronising and
// re-staging at the boundary with a ragged last round of units on either side.  Eight wavefronts, two per SIMD: the
// pipeline needs 160 registers, and eight divide the 64 units of a headline block evenly.
struct PairChains {
    h2 s[2], v[2], Q[2];
};
// The activation of two pairs of hidden units at once, cut in two halves of nine packed instructions: the two
// dependent chains alternate, so no instruction waits for the one just before it.
__device__ __forceinline__ void activation_first_half(PairChains &c, const float (&a)[4], h2 p2, h2 bias0, h2 bias1, const EpiConst &K)
{
    static_assert(kGeluM == 4, "the split below is written for a degree-4 polynomial");
    const h2 A0 = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(a[0], a[1]));
    const h2 A1 = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(a[2], a[3]));
    c.s[0] = pk_fma(A0, p2, bias0);
    c.s[1] = pk_fma(A1, p2, bias1);
    c.v[0] = pk_fma(c.s[0], c.s[0], as_h2(K.neg_w0));
    c.v[1] = pk_fma(c.s[1], c.s[1], as_h2(K.neg_w0));
    c.Q[0] = pk_fma(c.v[0], as_h2(K.q[4]), as_h2(K.q[3]));
    c.Q[1] = pk_fma(c.v[1], as_h2(K.q[4]), as_h2(K.q[3]));
    c.Q[0] = pk_fma(c.Q[0], c.v[0], as_h2(K.q[2]));
}
__device__ __forceinline__ void activation_second_half(PairChains &c, const EpiConst &K, uint32_t &out0, uint32_t &out1)
{
    c.Q[1] = pk_fma(c.Q[1], c.v[1], as_h2(K.q[2]));
    c.Q[0] = pk_fma(c.Q[0], c.v[0], as_h2(K.q[1]));
    c.Q[1] = pk_fma(c.Q[1], c.v[1], as_h2(K.q[1]));
    c.Q[0] = pk_fma(c.Q[0], c.v[0], as_h2(K.q[0]));
    c.Q[1] = pk_fma(c.Q[1], c.v[1], as_h2(K.q[0]));
    const h2 F0 = pk_fma_clamp01(c.s[0], c.Q[0], as_h2(K.half));
    const h2 F1 = pk_fma_clamp01(c.s[1], c.Q[1], as_h2(K.half));
    out0 = __builtin_bit_cast(uint32_t, c.s[0] * F0);
    out1 = __builtin_bit_cast(uint32_t, c.s[1] * F1);
}

template <int DS, int HT>
struct PipeState {
    static constexpr int KS = SliceTiles<DS>::KS, OT = SliceTiles<DS>::OT;
    static constexpr int NM = KS + 2 * OT;   // matrix instructions per step
    static_assert(HT % 2 == 0 && NM % 4 == 0 && NM >= 8 && HT >= 2, "see the kernel's comment");
    bf16x8 xb[KS];          // rows of the unit whose GEMM1 is running
    f32x16 acc[2];          // GEMM1 results, by tile parity
    uint32_t hb[2][8];      // activations as fp16 pairs, by tile parity: [s * 4 + i] is register i of K-step s of GEMM2
    f32x16 yacc[1][OT];
    f32x16 b2acc[OT];       // second-layer bias of the current unit's expert in accumulator layout: GEMM2 starts from it
    uint4 ring[4];          // weight fragments in flight
    uint4 bias[2][2];       // first-layer biases of the tile being activated, by tile parity
};

// The experts' LDS images of three consecutive units of a wavefront, as offsets in 16-byte pieces: the unit whose
// rows are being finished, the one whose GEMM1 runs, and the one after it.
struct PipeSlots {
    int prev, cur, next;
};

// Fragment (offset in 16-byte pieces inside an expert's LDS image) of matrix instruction m of the step whose GEMM1 tile
// is t: m < KS is K-step m of W1's tile t; the rest are W2's fragments (s, ot) of tile t - 2.
template <int DS, int HT>
__device__ __forceinline__ constexpr int pipe_frag(int t, int m, int w2_piece0)
{
    constexpr int KS = SliceTiles<DS>::KS, OT = SliceTiles<DS>::OT;
    if (m < KS) return (t * KS + m) * 64;
    const int t2 = (t + HT - 2) % HT, i = m - KS;
    return w2_piece0 + ((t2 * 2 + i / OT) * OT + i % OT) * 64;
}

// One step: GEMM1 of tile T of the current unit, activation of the tile before (scale p2_act), GEMM2 of the tile before
// that.  Each matrix instruction takes its fragment from the ring and refills the slot with the fragment four matrix
// instructions ahead, from the LDS image of the expert that instruction's unit belongs to.
template <int DS, int HT, int T>
__device__ __forceinline__ void pipe_step(PipeState<DS, HT> &S, const uint4 *__restrict__ lds16, const PipeSlots &E,
                                          int w2_piece0, int b1_piece0, int lane, int g, h2 p2_act, const EpiConst &K)
{
    constexpr int KS = SliceTiles<DS>::KS, OT = SliceTiles<DS>::OT, NM = KS + 2 * OT;
    constexpr int TA = (T + HT - 1) % HT;   // tile being activated
    constexpr int T2 = (T + HT - 2) % HT;   // tile whose GEMM2 runs
    // biases of the tile the NEXT step activates (tile T of the current unit), requested a step ahead
    S.bias[T & 1][0] = lds16[E.cur + b1_piece0 + (T * 2 + g) * 2 + 0];
    S.bias[T & 1][1] = lds16[E.cur + b1_piece0 + (T * 2 + g) * 2 + 1];
    const uint4 bq0 = S.bias[TA & 1][0], bq1 = S.bias[TA & 1][1];
    const uint32_t bw[8] = {bq0.x, bq0.y, bq0.z, bq0.w, bq1.x, bq1.y, bq1.z, bq1.w};
    PairChains chains;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        const uint4 frag = S.ring[m & 3];
        if (m < KS) {
            const bf16x8 a1 = __builtin_bit_cast(bf16x8, frag);
            if (m == 0) {
                f32x16 zero;
#pragma unroll
                for (int r = 0; r < 16; ++r) zero[r] = 0.f;
                S.acc[T & 1] = mfma_bf16(a1, S.xb[m], zero);
            } else {
                S.acc[T & 1] = mfma_bf16(a1, S.xb[m], S.acc[T & 1]);
            }
        } else {
            const int i = m - KS, s = i / OT, ot = i % OT;
            const f16x8 a2 = __builtin_bit_cast(f16x8, frag);
            const f16x8 b2v = __builtin_bit_cast(f16x8, make_uint4(S.hb[T & 1][s * 4 + 0], S.hb[T & 1][s * 4 + 1],
                                                                  S.hb[T & 1][s * 4 + 2], S.hb[T & 1][s * 4 + 3]));
            if (T2 == 0 && s == 0) {
                S.yacc[0][ot] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, b2v, S.b2acc[ot], 0, 0, 0);
            } else {
                S.yacc[0][ot] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, b2v, S.yacc[0][ot], 0, 0, 0);
            }
        }
        // refill the slot: the fragment of matrix instruction m + 4 (of the next step when that runs past this one).
        // A GEMM1 fragment belongs to the unit whose GEMM1 runs then (the next unit after this unit's last step); a
        // GEMM2 fragment to the unit of the tile two steps back (the previous unit during a unit's first two steps).
        {
            const int mn = m + 4;
            int piece;
            if (mn < NM) {
                piece = pipe_frag<DS, HT>(T, mn, w2_piece0) + (mn < KS ? E.cur : (T >= 2 ? E.cur : E.prev));
            } else {
                constexpr int TN = (T + 1) % HT;
                const int mm = mn - NM;
                if (mm < KS) piece = pipe_frag<DS, HT>(TN, mm, w2_piece0) + (T + 1 < HT ? E.cur : E.next);
                else piece = pipe_frag<DS, HT>(TN, mm, w2_piece0) + ((T + 1 >= 2 || T + 1 == HT) ? E.cur : E.prev);
            }
            S.ring[m & 3] = lds16[piece + lane];
        }
        // behind every matrix instruction half of the activation of two pairs of hidden units (eight pairs per tile)
        if (m < 8) {
            const int pp = m & ~1;   // the two pairs pp, pp + 1
            if ((m & 1) == 0) {
                const float a[4] = {S.acc[TA & 1][2 * pp], S.acc[TA & 1][2 * pp + 1], S.acc[TA & 1][2 * pp + 2], S.acc[TA & 1][2 * pp + 3]};
                activation_first_half(chains, a, p2_act, as_h2(bw[pp]), as_h2(bw[pp + 1]), K);
            } else {
                activation_second_half(chains, K, S.hb[TA & 1][pp], S.hb[TA & 1][pp + 1]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Steps T .. HT-1 of a unit.
template <int DS, int HT, int T>
__device__ __forceinline__ void pipe_steps_from(PipeState<DS, HT> &S, const uint4 *__restrict__ lds16, const PipeSlots &E,
                                                int w2_piece0, int b1_piece0, int lane, int g, h2 p2_act, const EpiConst &K)
{
    if constexpr (T < HT) {
        pipe_step<DS, HT, T>(S, lds16, E, w2_piece0, b1_piece0, lane, g, p2_act, K);
        pipe_steps_from<DS, HT, T + 1>(S, lds16, E, w2_piece0, b1_piece0, lane, g, p2_act, K);
    }
}

// The second-layer bias of the expert whose LDS image starts at piece `image`, in accumulator layout.
template <int DS, int HT>
__device__ __forceinline__ void load_b2acc(PipeState<DS, HT> &S, const char *lds, int image, size_t off_b2, int g)
{
    const float *b2s = (const float *)(lds + (size_t)image * 16 + off_b2);
#pragma unroll
    for (int ot = 0; ot < SliceTiles<DS>::OT; ++ot)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 bb = *(const f32x4 *)(b2s + ot * 32 + 8 * q + 4 * g);
#pragma unroll
            for (int c = 0; c < 4; ++c) S.b2acc[ot][4 * q + c] = bb[c];
        }
}

// ---- Which rows a block takes.
// Cutting the stacked rows into equal runs would be simplest, but a run that starts in the middle of an expert's 32-row
// units makes both neighbours pad a partial unit, and a run that holds a whole small expert plus parts of its two
// neighbours needs a second pass over the LDS images.  So the cut is made in UNITS counted from each expert's first
// row, on an axis where an expert is at least as long as one block's share: expert e occupies max(units_e, W) of it, W
// the share itself (the smallest W with  sum_e max(units_e, W) <= W * blocks, found by a few rounds of a fixed-point
// iteration: each round is one wavefront sum).  A block's share of that axis then touches at most two experts; inside
// a stretched (small) expert positions map back to units proportionally.  Lane e holds expert e (E <= 64).
template <int CTRL> __device__ __forceinline__ int lane_move(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }

__device__ __forceinline__ int wavefront_sum(int v)
{
    v += lane_move<0xB1>(v);    // quad_perm [1, 0, 3, 2]
    v += lane_move<0x4E>(v);    // quad_perm [2, 3, 0, 1]
    v += lane_move<0x141>(v);   // row_half_mirror
    v += lane_move<0x140>(v);   // row_mirror: every lane now holds the sum of its row of 16
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

__device__ __forceinline__ int wavefront_exclusive_scan(int v, int lane)
{
    int s = v;
    s += lane_move<0x111>(s);   // row_shr 1, 2, 4, 8 with zero fill: inclusive scan inside a row of 16
    s += lane_move<0x112>(s);
    s += lane_move<0x114>(s);
    s += lane_move<0x118>(s);
    const int r0 = __builtin_amdgcn_readlane(s, 15), r1 = __builtin_amdgcn_readlane(s, 31), r2 = __builtin_amdgcn_readlane(s, 47);
    const int row = lane >> 4;
    return s - v + (row == 0 ? 0 : row == 1 ? r0 : row == 2 ? r0 + r1 : r0 + r1 + r2);
}

__device__ __forceinline__ void block_row_range(int lane, int E, int off_lo, int off_hi, int n_kept, int blocks, int vblock,
                                                int &r_begin, int &r_end)
{
    const int rows = lane < E ? off_hi - off_lo : 0;
    const int units = (rows + kResU - 1) / kResU;
    int W = max(1, (wavefront_sum(units) + blocks - 1) / blocks);
    int C = wavefront_sum(lane < E ? max(units, W) : 0);
    for (int it = 0; it < 3; ++it) {   // uniform: all operands are wavefront sums
        const int Wn = (C + blocks - 1) / blocks;
        if (Wn <= W) break;
        W = Wn;
        C = wavefront_sum(lane < E ? max(units, W) : 0);
    }
    const int cost = lane < E ? max(units, W) : 0;
    const int cb = wavefront_exclusive_scan(cost, lane);
    auto row_at = [&](long long c) {   // stacked row at position c of the axis
        const bool own = lane < E && c >= cb && c < (long long)cb + cost;
        const int u = own ? (int)(((c - cb) * units) / cost) : 0;
        const int rr = off_lo + min(rows, kResU * u);
        const unsigned long long m = __ballot(own);
        return m == 0 ? n_kept : __builtin_amdgcn_readlane(rr, __builtin_ctzll(m));
    };
    r_begin = row_at((long long)vblock * C / blocks);
    r_end = row_at((long long)(vblock + 1) * C / blocks);
}

template <int DS, int HT, int THREADS>
__global__ __launch_bounds__(THREADS) void ffn_pipelined_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, const char *__restrict__ experts, size_t e_stride, size_t off_w2,
    size_t off_b1, size_t off_b2, int E, int k, EpiConst K, half_t *__restrict__ y)
{
    constexpr int kWaves = THREADS / 64;
    constexpr int KS = SliceTiles<DS>::KS;
    extern __shared__ __align__(16) char lds[];             // two expert images of e_stride bytes each
    const uint4 *lds16 = (const uint4 *)lds;                // in an image: W1 fragments [HT][KS][64] from piece 0
    const int w2_piece0 = (int)(off_w2 / 16);               // W2 fragments [HT][2][OT][64]
    const int b1_piece0 = (int)(off_b1 / 16);               // b1 [HT][2][16] fp16
    const int image = (int)(e_stride / 16);                 // pieces per image

    const int tid = threadIdx.x, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kshift = (k & (k - 1)) == 0 ? __ffs(k) - 1 : -1;   // slice of an assignment: a shift when k is a power of two

    // lane e keeps the end of expert e's row range: expert lookups are one ballot, not a chain of loads
    const int off_lo = offsets[min(lane, E)];
    const int off_hi = offsets[min(lane + 1, E)];
    const int n_kept = __builtin_amdgcn_readlane(off_hi, 63);   // lanes past the last expert read offsets[E]
    const int vblock = gridDim.x % 8 == 0 ? (int)(blockIdx.x % 8) * (int)(gridDim.x / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    int r_begin, r_end;
    block_row_range(lane, E, off_lo, off_hi, n_kept, (int)gridDim.x, vblock, r_begin, r_end);

    int r = r_begin;
    while (r < r_end) {
        // up to two experts per pass: rows [r, end0) of expert e0 in image 0, rows [end0, end1) of expert e1 in image 1
        const int e0 = __builtin_amdgcn_readfirstlane(__popcll(__ballot(lane < E && off_hi <= r)));
        const int end0 = min(__builtin_amdgcn_readfirstlane(__shfl(off_hi, e0)), r_end);
        const int e1 = __builtin_amdgcn_readfirstlane(__popcll(__ballot(lane < E && off_hi <= end0)));   // == E past the last row
        const int end1 = end0 < r_end ? min(__builtin_amdgcn_readfirstlane(__shfl(off_hi, min(e1, E - 1))), r_end) : end0;
        const int n0 = (end0 - r + kResU - 1) / kResU, n1 = (end1 - end0 + kResU - 1) / kResU;
        const int mine = wave < n0 + n1 ? (n0 + n1 - wave + kWaves - 1) / kWaves : 0;   // units wave, wave + kWaves, ...
        // unit q of the pass: its rows, and the LDS image of its expert
        auto unit_base = [&](int q) { return q < n0 ? r + q * kResU : end0 + (q - n0) * kResU; };
        auto unit_end = [&](int q) { return q < n0 ? end0 : end1; };
        auto unit_image = [&](int q) { return q < n0 ? 0 : image; };

        __syncthreads();  // everyone is done with the previous pass's weights
        int row_c[1], a_c[1], row_n[1], a_n[1], row_nn[1], a_nn[1];
        float p_c[1], p_n[1];
        unit_rows<1>(unit_base(wave), unit_end(wave), mine > 0, j, perm, row_c, a_c);
        unit_rows<1>(unit_base(wave + kWaves), unit_end(wave + kWaves), mine > 1, j, perm, row_n, a_n);
        stage_to_lds<THREADS>(experts + (size_t)e0 * e_stride, lds, image, tid);
        if (n1 > 0) stage_to_lds<THREADS>(experts + (size_t)e1 * e_stride, lds + e_stride, image, tid);
        RowUnit<DS, 1> cur, nxt;
        load_rows<DS, 1>(cur, a_c, row_c, x, pk, k, g, p_c, kshift);
        set_p<DS, 1>(cur, p_c);
        __syncthreads();

        if (mine > 0) {
            PipeState<DS, HT> S;
            PipeSlots slots;
            slots.prev = slots.cur = unit_image(wave);
            slots.next = unit_image(wave + kWaves);
            load_b2acc<DS, HT>(S, lds, slots.cur, off_b2, g);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) S.xb[ks] = cur.xb[0][ks];
#pragma unroll
            for (int m = 0; m < 4; ++m) S.ring[m] = lds16[slots.cur + pipe_frag<DS, HT>(0, m, w2_piece0) + lane];
            // the stages that lag behind start on nothing: whatever they compute before the first unit's tiles reach
            // them is overwritten (accumulators start from zero at a unit's first tile) and never stored (row -1)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
#pragma unroll
                for (int r16 = 0; r16 < 16; ++r16) S.acc[b][r16] = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) S.hb[b][i] = 0u;
                S.bias[b][0] = S.bias[b][1] = make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int ot = 0; ot < SliceTiles<DS>::OT; ++ot)
#pragma unroll
                for (int r16 = 0; r16 < 16; ++r16) S.yacc[0][ot][r16] = 0.f;
            h2 p2_prev = cur.p2[0];
            RowUnit<DS, 1> done;   // the unit whose rows are stored next (only its row id is used)
            done.row[0] = -1;
            for (int ui = 0; ui <= mine; ++ui) {
                {   // The SIMD serves its oldest wavefront first, which then finishes a third of the kernel earlier than
                    // its partner and leaves it alone on the SIMD, where a lone wavefront overlaps less.  Priority by
                    // units left keeps the two within two units of each other.
                    const int left = mine - ui;
                    if (left >= 6) __builtin_amdgcn_s_setprio(3);
                    else if (left >= 4) __builtin_amdgcn_s_setprio(2);
                    else if (left >= 2) __builtin_amdgcn_s_setprio(1);
                    else __builtin_amdgcn_s_setprio(0);
                }
                // the rows of the next unit are requested now, a whole unit ahead; its row index came a unit earlier
                // still, and the one after next is requested here
                const int q_nn = wave + (ui + 2) * kWaves;
                unit_rows<1>(unit_base(q_nn), unit_end(q_nn), ui + 2 < mine, j, perm, row_nn, a_nn);
                load_rows<DS, 1>(nxt, a_n, row_n, x, pk, k, g, p_n, kshift);
                // steps 0 and 1 finish the previous unit (its accumulators started from the second-layer bias)
                pipe_step<DS, HT, 0>(S, lds16, slots, w2_piece0, b1_piece0, lane, g, p2_prev, K);
                pipe_step<DS, HT, 1>(S, lds16, slots, w2_piece0, b1_piece0, lane, g, cur.p2[0], K);
                store_rows<DS, 1, false>(done, S.yacc, nullptr, y, g);
                if (ui == mine) break;   // that was the drain after the last unit
                pipe_steps_from<DS, HT, 2>(S, lds16, slots, w2_piece0, b1_piece0, lane, g, cur.p2[0], K);
                p2_prev = cur.p2[0];
                done.row[0] = cur.row[0];
                cur.row[0] = nxt.row[0];   // (the rows themselves go straight into the pipeline's operand registers)
                set_p<DS, 1>(cur, p_n);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) S.xb[ks] = nxt.xb[0][ks];
                row_n[0] = row_nn[0];
                a_n[0] = a_nn[0];
                slots.prev = slots.cur;
                slots.cur = slots.next;
                slots.next = unit_image(wave + (ui + 2) * kWaves);
                if (slots.cur != slots.prev) load_b2acc<DS, HT>(S, lds, slots.cur, off_b2, g);   // the next unit is another expert's
            }
        }
        r = end1;
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

constexpr int kPipeThreads = 512;   // eight wavefronts, two per SIMD

template <int DS, int HT, int THREADS>
static hipError_t run_pipelined(const slicemoe_config &c, const PackedLayout &L, const FfnPlan &pl, const void *h,
                                const float *p, const int32_t *offsets, const int32_t *perm, const char *experts,
                                void *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    const long long max_units = (Na + kResU - 1) / kResU;
    long long blocks = max_units;   // small inputs: spread the units over all CUs rather than fill few blocks
    if (blocks > num_compute_units()) blocks = num_compute_units();
    auto kern = ffn_pipelined_kernel<DS, HT, THREADS>;
    const size_t lds = 2 * L.e_stride;   // two expert images
    hipError_t err = grant_dynamic_lds((const void *)kern, lds);
    if (err != hipSuccess) return err;
    kern<<<(int)blocks, THREADS, lds, s>>>((const bf16_t *)h, p, offsets, perm, experts, L.e_stride, L.e_w2, L.e_b1,
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
        if (L.He == 256) return run_pipelined<64, 8, kPipeThreads>(c, L, pl, h, p, offsets, perm, experts, y, s);
        if (L.He == 128) return run_pipelined<64, 4, kPipeThreads>(c, L, pl, h, p, offsets, perm, experts, y, s);
        return run_pipelined<64, 2, kPipeThreads>(c, L, pl, h, p, offsets, perm, experts, y, s);
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
