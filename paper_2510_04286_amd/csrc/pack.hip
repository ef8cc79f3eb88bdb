// One-time re-tiling of the bf16 weights into matrix-core fragment order (see mfma.h for the
// operand layout).  A fragment is the 16 bytes one lane feeds to one MFMA: 8 bf16 along the
// contraction dimension.  Biases are widened to fp32.  One thread per fragment / bias element.
//
// Router   W1 frags [Hr/32][ds/16][64 lanes]      lane (i, g), slot m: Wr1[16*ks + 8*g + m][32*ht + i]
//          (ds/16 and ds/32 rounded up: rows and columns past ds are zeros)
//          W2 frags [Epad/32][Hr/32][2][64]       lane (i, g), slot m: Wr2[32*ht + chain_feature(s,g,m)][32*et + i], as fp16
// Expert e W1 frags [He/32][ds/16][64]            kappa * W1[e][16*ks + 8*g + m][32*ht + i]   (kappa = 1/4: exact in bf16)
//          W2 frags [He/32][2][ds/32][64]         W2[e][32*ht + chain_feature(s,g,m)][32*ot + i] / kappa, as fp16
//          b1       [He/32][2 lane groups][16]    kappa * b1[e][32*ht + acc_feature(r, g)], as fp16
//          b2       [ds rounded up to 32] fp32
// The expert kernel evaluates its activation on s = kappa z in packed fp16 (see ffn_mfma.hip), so
// its second GEMM runs on fp16 fragments; bf16 weights convert exactly to fp16 unless they are
// smaller than 2^-14 / 4 (rounded, absolute error below 2^-27) or beyond +-16376 (clamped).
#include "mfma.h"

namespace slicemoe {

__device__ __forceinline__ void store_frag(char *dst, const bf16_t v[8])
{
    uint4 u;
    u.x = v[0] | ((uint32_t)v[1] << 16);
    u.y = v[2] | ((uint32_t)v[3] << 16);
    u.z = v[4] | ((uint32_t)v[5] << 16);
    u.w = v[6] | ((uint32_t)v[7] << 16);
    *(uint4 *)dst = u;
}

// Fragments of a first-layer matrix W[K, N] (row-major), A operand of the transposed GEMM1, times `scale` (a power of
// two: the product is again a bf16 value, exactly, unless it falls into the subnormal range below 2^-126).
__global__ void pack_layer1_kernel(const bf16_t *__restrict__ W, int K, int Kpad, int N, size_t src_stride,
                                   char *__restrict__ dst, size_t dst_stride, int nmat, float scale)
{
    const int KS = Kpad / 16;   // rows K..Kpad-1 are zeros
    const long long per = (long long)(N / 32) * KS * 64;
    const long long f = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= per * nmat) return;
    const int mat = (int)(f / per);
    long long r = f - (long long)mat * per;
    const int lane = (int)(r % 64);
    r /= 64;
    const int ks = (int)(r % KS);
    const int ht = (int)(r / KS);
    const int i = lane & 31, g = lane >> 5;
    const bf16_t *src = W + (size_t)mat * src_stride;
    bf16_t v[8];
    for (int m = 0; m < 8; ++m) {
        const int kk = 16 * ks + 8 * g + m;
        v[m] = kk < K ? f32_to_bf16(bf16_to_f32(src[(size_t)kk * N + 32 * ht + i]) * scale) : (bf16_t)0;
    }
    store_frag(dst + (size_t)mat * dst_stride + (size_t)(f - (long long)mat * per) * 16, v);
}

// Fragments of a second-layer matrix W[K, N] (row-major), A operand of the transposed GEMM2 whose
// contraction slots follow the accumulator layout of GEMM1.  order_outer_first = true lays
// fragments out as [nt][ht][s][lane] (router), false as [ht][s][nt][lane] (experts).
__global__ void pack_layer2_kernel(const bf16_t *__restrict__ W, int K, int N, int Npad, size_t src_stride,
                                   char *__restrict__ dst, size_t dst_stride, int nmat, bool order_outer_first,
                                   bool as_f16, float f16_scale)
{
    const int HT = K / 32, NT = Npad / 32;
    const long long per = (long long)HT * 2 * NT * 64;
    const long long f = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= per * nmat) return;
    const int mat = (int)(f / per);
    long long r = f - (long long)mat * per;
    const int lane = (int)(r % 64);
    r /= 64;
    int ht, s, nt;
    if (order_outer_first) {
        s = (int)(r % 2);
        r /= 2;
        ht = (int)(r % HT);
        nt = (int)(r / HT);
    } else {
        nt = (int)(r % NT);
        r /= NT;
        s = (int)(r % 2);
        ht = (int)(r / 2);
    }
    const int i = lane & 31, g = lane >> 5;
    const int col = 32 * nt + i;
    const bf16_t *src = W + (size_t)mat * src_stride;
    bf16_t v[8];
    for (int m = 0; m < 8; ++m) {
        const bf16_t w = col < N ? src[(size_t)(32 * ht + chain_feature(s, g, m)) * N + col] : (bf16_t)0;
        if (as_f16) {
            const float f = fminf(fmaxf(bf16_to_f32(w) * f16_scale, -65504.f), 65504.f);
            const _Float16 hv = (_Float16)f;
            v[m] = __builtin_bit_cast(bf16_t, hv);
        } else {
            v[m] = w;
        }
    }
    store_frag(dst + (size_t)mat * dst_stride + (size_t)(f - (long long)mat * per) * 16, v);
}

// Expert first-layer biases as fp16, scaled, in the accumulator order of each hidden tile.
__global__ void pack_bias_f16_kernel(const bf16_t *__restrict__ b, int n, size_t src_stride, char *__restrict__ dst,
                                     size_t dst_stride, int nmat, float scale)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (long long)n * nmat) return;
    const int mat = (int)(t / n);
    const int i = (int)(t - (long long)mat * n);
    const int ht = i / 32, g = (i % 32) / 16, r = i % 16;
    const float f = fminf(fmaxf(bf16_to_f32(b[(size_t)mat * src_stride + 32 * ht + acc_feature(r, g)]) * scale, -65504.f), 65504.f);
    ((_Float16 *)(dst + (size_t)mat * dst_stride))[i] = (_Float16)f;
}

__global__ void pack_bias_kernel(const bf16_t *__restrict__ b, int n, int npad, size_t src_stride,
                                 char *__restrict__ dst, size_t dst_stride, int nmat)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (long long)npad * nmat) return;
    const int mat = (int)(t / npad);
    const int i = (int)(t - (long long)mat * npad);
    float *out = (float *)(dst + (size_t)mat * dst_stride);
    out[i] = i < n ? bf16_to_f32(b[(size_t)mat * src_stride + i]) : 0.f;
}

static inline int blocks_for(long long n) { return (int)((n + 255) / 256); }

hipError_t launch_pack(const slicemoe_config &c, const slicemoe_weights &w, void *packed, hipStream_t s)
{
    const PackedLayout L = packed_layout(c);
    char *base = (char *)packed;
    const int ds = L.ds, Hr = L.Hr, He = L.He, E = L.E, Epad = L.Epad;
    // router
    const int dsK = L.dsK, dsN = L.dsN;
    pack_layer1_kernel<<<blocks_for((long long)(Hr / 32) * (dsK / 16) * 64), 256, 0, s>>>(
        (const bf16_t *)w.Wr1, ds, dsK, Hr, 0, base + L.r_w1, 0, 1, 1.f);
    pack_layer2_kernel<<<blocks_for((long long)(Hr / 32) * 2 * (Epad / 32) * 64), 256, 0, s>>>(
        (const bf16_t *)w.Wr2, Hr, E, Epad, 0, base + L.r_w2, 0, 1, true, true, 1.f);
    pack_bias_kernel<<<blocks_for(Hr), 256, 0, s>>>((const bf16_t *)w.br1, Hr, Hr, 0, base + L.r_b1, 0, 1);
    pack_bias_kernel<<<blocks_for(Epad), 256, 0, s>>>((const bf16_t *)w.br2, E, Epad, 0, base + L.r_b2, 0, 1);
    // experts
    char *eb = base + L.experts;
    pack_layer1_kernel<<<blocks_for((long long)E * (He / 32) * (dsK / 16) * 64), 256, 0, s>>>(
        (const bf16_t *)w.W1, ds, dsK, He, (size_t)ds * He, eb + L.e_w1, L.e_stride, E, kGeluKappa);
    pack_layer2_kernel<<<blocks_for((long long)E * (He / 32) * 2 * (dsN / 32) * 64), 256, 0, s>>>(
        (const bf16_t *)w.W2, He, ds, dsN, (size_t)He * ds, eb + L.e_w2, L.e_stride, E, false, true, 1.f / kGeluKappa);
    pack_bias_f16_kernel<<<blocks_for((long long)E * He), 256, 0, s>>>((const bf16_t *)w.b1, He, He, eb + L.e_b1,
                                                                       L.e_stride, E, kGeluKappa);
    pack_bias_kernel<<<blocks_for((long long)E * dsN), 256, 0, s>>>((const bf16_t *)w.b2, ds, dsN, ds, eb + L.e_b2,
                                                                    L.e_stride, E);
    return hipGetLastError();
}

}  // namespace slicemoe
