// Generic (vector-ALU, fp32 arithmetic) router and expert kernels.  They take any shape within
// the library limits and either storage type, and serve the fp32 configuration and every
// shape the matrix-core kernels do not cover.  Straightforward by design: a block stages RB
// slices in LDS, one thread per hidden unit accumulates with fmaf in ascending input order.
#include "common.h"

namespace slicemoe {

constexpr int kRB = 8;          // slices (rows) per block
constexpr int kGenThreads = 256;

// Router of paper Section 3.1: g = ReLU(x Wr1 + br1) Wr2 + br2, softmax over E, top-k on the
// fp32 logits with ties to the lower expert index.
template <typename T>
__global__ __launch_bounds__(kGenThreads) void route_generic_kernel(
    const T *__restrict__ x, long long Ns, int ds, int Hr, int E, int k,
    const T *__restrict__ Wr1, const T *__restrict__ br1, const T *__restrict__ Wr2, const T *__restrict__ br2,
    const float *__restrict__ noise, float sigma, float inv_tau, int32_t *__restrict__ idx, float *__restrict__ pk)
{
    extern __shared__ float smem[];
    float *xs = smem;                 // [kRB][ds]
    float *us = xs + kRB * ds;        // [kRB][Hr]
    float *gs = us + kRB * Hr;        // [kRB][E]
    const int tid = threadIdx.x;
    const long long n0 = (long long)blockIdx.x * kRB;
    const int rows = (int)min((long long)kRB, Ns - n0);

    for (int i = tid; i < kRB * ds; i += kGenThreads) {
        const int r = i / ds;
        xs[i] = r < rows ? Storage<T>::load(x + n0 * ds + i) : 0.f;
    }
    __syncthreads();
    for (int j = tid; j < Hr; j += kGenThreads) {
        float acc[kRB];
        const float b = Storage<T>::load(br1 + j);
#pragma unroll
        for (int r = 0; r < kRB; ++r) acc[r] = b;
        for (int i = 0; i < ds; ++i) {
            const float wv = Storage<T>::load(Wr1 + (size_t)i * Hr + j);
#pragma unroll
            for (int r = 0; r < kRB; ++r) acc[r] = fmaf(xs[r * ds + i], wv, acc[r]);
        }
#pragma unroll
        for (int r = 0; r < kRB; ++r) us[r * Hr + j] = fmaxf(acc[r], 0.f);
    }
    __syncthreads();
    for (int t = tid; t < kRB * E; t += kGenThreads) {
        const int r = t / E, e = t - r * E;
        float acc = Storage<T>::load(br2 + e);
        for (int j = 0; j < Hr; ++j) acc = fmaf(us[r * Hr + j], Storage<T>::load(Wr2 + (size_t)j * E + e), acc);
        // training-time logit noise (Section 5): before the selection and the softmax
        if (noise != nullptr && r < rows) acc = fmaf(sigma, noise[(n0 + r) * E + e], acc);
        gs[t] = acc;
    }
    __syncthreads();
    if (tid < rows) {
        float *g = gs + tid * E;
        float m = g[0];
        for (int e = 1; e < E; ++e) m = fmaxf(m, g[e]);
        float den = 0.f;
        for (int e = 0; e < E; ++e) den += expf((g[e] - m) * inv_tau);   // softmax of g / tau (Appendix B)
        const long long n = n0 + tid;
        for (int j = 0; j < k; ++j) {
            int best = 0;
            float bv = g[0];
            for (int e = 1; e < E; ++e)
                if (g[e] > bv) {
                    bv = g[e];
                    best = e;
                }
            idx[n * k + j] = best;
            pk[n * k + j] = expf((bv - m) * inv_tau) / den;
            g[best] = -INFINITY;
        }
    }
}

// Expert FFN of Section 3.1 on stacked rows with the Eq. 1 input weighting and the gather fused:
// y[r] = GELU((p x) W1[e] + b1[e]) W2[e] + b2[e], exact (erf) GELU.  y is fp32 for fp32 storage and
// fp16 for bf16 storage (same convention as the matrix-core kernel).
template <typename T, typename YT>
__global__ __launch_bounds__(kGenThreads) void ffn_generic_kernel(
    const T *__restrict__ x, const float *__restrict__ pk, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, int ds, int He, int E, int k,
    const T *__restrict__ W1, const T *__restrict__ b1, const T *__restrict__ W2, const T *__restrict__ b2,
    YT *__restrict__ y)
{
    extern __shared__ float smem[];
    float *xs = smem;             // [kRB][ds]  (already multiplied by p)
    float *zs = xs + kRB * ds;    // [kRB][He]
    __shared__ int ex[kRB];
    const int tid = threadIdx.x;
    const long long r0 = (long long)blockIdx.x * kRB;
    const int n_kept = offsets[E];
    if (r0 >= n_kept) return;
    const int rows = (int)min((long long)kRB, n_kept - r0);
    if (tid < kRB) {
        int e = 0;
        if (tid < rows) {
            const int row = (int)r0 + tid;
            while (e + 1 < E && offsets[e + 1] <= row) ++e;
        }
        ex[tid] = e;
    }
    for (int i = tid; i < kRB * ds; i += kGenThreads) {
        const int r = i / ds, c = i - r * ds;
        float v = 0.f;
        if (r < rows) {
            const int a = perm[r0 + r];
            const long long n = a / k;
            v = pk[a] * Storage<T>::load(x + n * ds + c);
        }
        xs[i] = v;
    }
    __syncthreads();
    for (int j = tid; j < He; j += kGenThreads) {
        for (int r = 0; r < rows; ++r) {
            const int e = ex[r];
            const T *w = W1 + (size_t)e * ds * He + j;
            float acc = Storage<T>::load(b1 + (size_t)e * He + j);
            for (int i = 0; i < ds; ++i) acc = fmaf(xs[r * ds + i], Storage<T>::load(w + (size_t)i * He), acc);
            zs[r * He + j] = 0.5f * acc * (1.f + erff(acc * 0.70710678118654752f));
        }
    }
    __syncthreads();
    for (int t = tid; t < rows * ds; t += kGenThreads) {
        const int r = t / ds, c = t - r * ds;
        const int e = ex[r];
        const T *w = W2 + (size_t)e * He * ds + c;
        float acc = Storage<T>::load(b2 + (size_t)e * ds + c);
        for (int j = 0; j < He; ++j) acc = fmaf(zs[r * He + j], Storage<T>::load(w + (size_t)j * ds), acc);
        y[(r0 + r) * ds + c] = (YT)acc;
    }
}

hipError_t launch_route_generic(const slicemoe_config &c, const void *h, const slicemoe_weights &w,
                                int32_t *idx, float *p, hipStream_t s, const RouteVariant &v)
{
    const long long Ns = (long long)c.T * c.S;
    if (Ns == 0) return hipSuccess;
    const int ds = c.d / c.S;
    const int blocks = (int)((Ns + kRB - 1) / kRB);
    const float *noise = v.sigma > 0.f ? v.noise : nullptr;
    const size_t smem = sizeof(float) * (size_t)kRB * (ds + c.Hr + c.E);
    if (c.dtype == SLICEMOE_BF16)
        route_generic_kernel<bf16_t><<<blocks, kGenThreads, smem, s>>>(
            (const bf16_t *)h, Ns, ds, c.Hr, c.E, c.k, (const bf16_t *)w.Wr1, (const bf16_t *)w.br1,
            (const bf16_t *)w.Wr2, (const bf16_t *)w.br2, noise, v.sigma, v.inv_tau, idx, p);
    else
        route_generic_kernel<float><<<blocks, kGenThreads, smem, s>>>(
            (const float *)h, Ns, ds, c.Hr, c.E, c.k, (const float *)w.Wr1, (const float *)w.br1,
            (const float *)w.Wr2, (const float *)w.br2, noise, v.sigma, v.inv_tau, idx, p);
    return hipGetLastError();
}

// Cross-slice dropout (Section 3.3): assignment j of a slice is dropped when its uniform draw is below the rate; the
// remaining probabilities are renormalised to sum to 1, the dropped ones are 0.  A slice whose draws would drop all k
// keeps slot 0.  One thread per slice; k <= 8.
__global__ __launch_bounds__(256) void route_dropout_kernel(float *__restrict__ pk, const float *__restrict__ drop_u,
                                                            long long Ns, int k, float rate)
{
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= Ns) return;
    float p[8];
    bool keep[8];
    int kept = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = 0.f;
        keep[j] = false;
        if (j < k) {
            p[j] = pk[n * k + j];
            keep[j] = !(drop_u[n * k + j] < rate);
            kept += keep[j] ? 1 : 0;
        }
    }
    if (kept == 0) keep[0] = true;
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) sum += keep[j] ? p[j] : 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < k) pk[n * k + j] = keep[j] ? p[j] / sum : 0.f;
}

hipError_t launch_route_dropout(const slicemoe_config &c, float *p, const float *drop_u, float rate, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    if (Ns == 0 || !(rate > 0.f)) return hipSuccess;
    route_dropout_kernel<<<(int)((Ns + 255) / 256), 256, 0, s>>>(p, drop_u, Ns, c.k, rate);
    return hipGetLastError();
}

hipError_t launch_ffn_generic(const slicemoe_config &c, const void *h, const float *p,
                              const int32_t *offsets, const int32_t *perm, const slicemoe_weights &w,
                              void *y, hipStream_t s)
{
    const long long Na = (long long)c.T * c.S * c.k;
    if (Na == 0) return hipSuccess;
    const int ds = c.d / c.S;
    const int blocks = (int)((Na + kRB - 1) / kRB);
    const size_t smem = sizeof(float) * (size_t)kRB * (ds + c.He);
    if (c.dtype == SLICEMOE_BF16)
        ffn_generic_kernel<bf16_t, _Float16><<<blocks, kGenThreads, smem, s>>>(
            (const bf16_t *)h, p, offsets, perm, ds, c.He, c.E, c.k, (const bf16_t *)w.W1,
            (const bf16_t *)w.b1, (const bf16_t *)w.W2, (const bf16_t *)w.b2, (_Float16 *)y);
    else
        ffn_generic_kernel<float, float><<<blocks, kGenThreads, smem, s>>>(
            (const float *)h, p, offsets, perm, ds, c.He, c.E, c.k, (const float *)w.W1,
            (const float *)w.b1, (const float *)w.W2, (const float *)w.b2, (float *)y);
    return hipGetLastError();
}

}  // namespace slicemoe
