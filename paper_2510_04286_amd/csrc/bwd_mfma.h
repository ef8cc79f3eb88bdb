// Shared pieces of the matrix-core backward kernels: fragment packing from a strided (possibly transposed) source,
// the normal CDF and density, bf16 pair conversions.  See mfma.h for the operand layouts.
#pragma once
#include "mfma.h"

namespace slicemoe {

// Weight repacking for the backward kernels: a few jobs per launch, one thread per 16-byte fragment (or bias value).
// Generic strided source so that the same code packs a matrix or its transpose: element (kk, col) of the [K, N] matrix
// being packed is src[kk * rs + col * cs] for kk < Kv and col < Nv, and zero in the padding up to K and N (multiples of
// 16 / 32).  nmat matrices, src_stride elements and dst_stride bytes apart.
//   kPackLayer1    [N/32][K/16][64]: lane (i, g), slot m: M[16ks + 8g + m][32nt + i]
//   kPackChain     [K/32][2][N/32][64]: lane (i, g), slot m: M[32ht + chain_feature(s, g, m)][32nt + i], i.e. the
//                  contraction slots follow the accumulator order; kPackChainF16: the same converted to fp16
//   kPackBias      K values per matrix widened to fp32, zero-padded to N
enum { kPackLayer1 = 0, kPackChain = 1, kPackChainF16 = 2, kPackBias = 3 };
struct BwdPackJob {
    int kind, K, Kv, N, Nv;
    const bf16_t *src;
    size_t rs, cs, src_stride;
    char *dst;
    size_t dst_stride;
    long long items;   // threads this job needs
};
struct BwdPackJobs {
    int count;
    BwdPackJob job[8];
};
BwdPackJob bwd_pack_job(int kind, const void *src, int K, int Kv, int N, int Nv, size_t rs, size_t cs, size_t src_stride,
                        char *dst, size_t dst_stride, int nmat);
hipError_t bwd_pack_launch(const BwdPackJobs &jobs, hipStream_t s);

// Phi(z), and phi(z) through *density: the normal CDF by Abramowitz & Stegun 7.1.26 on |z| / sqrt 2 (|error| < 1.5e-7),
// whose exponential exp(-z^2 / 2) is the density's.
__device__ __forceinline__ float normal_cdf_pdf(float z, float *density)
{
    const float ax = fabsf(z) * 0.70710678118654752f;
    const float ex = __builtin_amdgcn_exp2f(-0.72134752044448170f * z * z);   // exp(-z^2 / 2)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.f));
    // half the published coefficients: the factor 1/2 of 1 - Phi = erfc / 2 costs nothing and changes no bit
    float q = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    q = fmaf(q, t, 0.5f * 1.421413741f);
    q = fmaf(q, t, 0.5f * -0.284496736f);
    q = fmaf(q, t, 0.5f * 0.254829592f);
    const float tail = q * t * ex;   // 1 - Phi(|z|)
    *density = 0.39894228040143267794f * ex;
    return z > 0.f ? 1.f - tail : tail;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)   // round to nearest even
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Two-term bf16 split of a pair: hi = bf16(v), lo = bf16(v - hi); hi + lo carries 16 significant bits, so a matrix
// instruction run once per term is as good as an fp32 operand (the other operand being exact bf16 data).
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = pack_bf16x2(a, b);
    lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

// Two fp32 values that are exactly bf16 values (results of an MFMA against an identity): their high halves.
__device__ __forceinline__ uint32_t pack_exact_bf16x2(float a, float b)
{
    return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xffff0000u);
}

__device__ __forceinline__ bf16x8 frag_of(const uint32_t (&p)[8], int s)   // K-step s of eight register pairs
{
    return __builtin_bit_cast(bf16x8, make_uint4(p[4 * s], p[4 * s + 1], p[4 * s + 2], p[4 * s + 3]));
}

// Identity fragments for transposing a row fragment with an MFMA: as B operand of K-step ks against output tile ot,
// slot m of lane (jj, g) is 1 where 16 ks + 8 g + m == 32 ot + jj; only the parity of ks matters.
__device__ __forceinline__ void identity_fragments(int jj, int g, bf16x8 &id_even, bf16x8 &id_odd)
{
    uint32_t ide[4] = {0, 0, 0, 0}, ido[4] = {0, 0, 0, 0};
    const int me = jj - 8 * g, mo = jj - 16 - 8 * g;
#pragma unroll
    for (int t = 0; t < 4; ++t) {   // static indices: the arrays stay in registers
        if (me >= 0 && me < 8 && (me >> 1) == t) ide[t] = (me & 1) ? 0x3f800000u : 0x00003f80u;
        if (mo >= 0 && mo < 8 && (mo >> 1) == t) ido[t] = (mo & 1) ? 0x3f800000u : 0x00003f80u;
    }
    id_even = __builtin_bit_cast(bf16x8, make_uint4(ide[0], ide[1], ide[2], ide[3]));
    id_odd = __builtin_bit_cast(bf16x8, make_uint4(ido[0], ido[1], ido[2], ido[3]));
}

// Block-wide copy of `bytes` (a multiple of 16) from memory to LDS; callers synchronise.
__device__ __forceinline__ void stage_bytes(const char *__restrict__ src, char *lds, size_t bytes, int tid, int nthreads)
{
    const uint4 *g = (const uint4 *)src;
    uint4 *l = (uint4 *)lds;
    const int n = (int)(bytes / 16);
    for (int i = tid; i < n; i += nthreads) l[i] = g[i];
}

}  // namespace slicemoe
