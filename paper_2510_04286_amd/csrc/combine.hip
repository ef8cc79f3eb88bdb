// Combine stage (paper Section 3.1): the k expert outputs of a slice are summed and the S
// output slices concatenated.  In the slice view h'[n, :] sits where x[n, :] sat, so the
// output is one contiguous stream: thread g handles V consecutive output elements, reads the
// matching V values of up to k stacked rows (16-byte loads), adds them in fp32 in ascending j
// and writes one rounded vector.  y is fp32 (fp32 storage) or fp16 (bf16 storage).  HBM-bound;
// no reuse, so no LDS.
#include "common.h"

namespace slicemoe {

typedef _Float16 half_t;

template <typename T, int V> struct OutVec;
template <> struct OutVec<float, 4> {
    static __device__ __forceinline__ void store(float *o, const float *v) { *(float4 *)o = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct OutVec<float, 1> {
    static __device__ __forceinline__ void store(float *o, const float *v) { *o = v[0]; }
};
template <> struct OutVec<bf16_t, 1> {
    static __device__ __forceinline__ void store(bf16_t *o, const float *v) { *o = f32_to_bf16(v[0]); }
};
template <> struct OutVec<bf16_t, 8> {
    static __device__ __forceinline__ void store(bf16_t *o, const float *v)
    {
        uint4 u;
        u.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
        u.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
        u.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
        u.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
        *(uint4 *)o = u;
    }
};

// V values of a stacked row added into acc
template <typename YT, int V> struct RowAdd;
template <> struct RowAdd<float, 4> {
    static __device__ __forceinline__ void add(const float *src, float *acc)
    {
        const float4 t = *(const float4 *)src;
        acc[0] += t.x;
        acc[1] += t.y;
        acc[2] += t.z;
        acc[3] += t.w;
    }
};
template <> struct RowAdd<float, 1> {
    static __device__ __forceinline__ void add(const float *src, float *acc) { acc[0] += src[0]; }
};
template <> struct RowAdd<half_t, 1> {
    static __device__ __forceinline__ void add(const half_t *src, float *acc) { acc[0] += (float)src[0]; }
};
template <> struct RowAdd<half_t, 8> {
    static __device__ __forceinline__ void add(const half_t *src, float *acc)
    {
        typedef half_t h8 __attribute__((ext_vector_type(8)));
        const h8 t = *(const h8 *)src;
#pragma unroll
        for (int v = 0; v < 8; ++v) acc[v] += (float)t[v];
    }
};

// K = 2: the common top-2 case with both row indices read by one 8-byte load and both rows requested before either is
// used (a dropped assignment reads row 0 and is not added); K = 0: any k, one row after the other.
template <typename T, typename YT, int V, int K>
__global__ __launch_bounds__(256) void combine_kernel(const YT *__restrict__ y, const int32_t *__restrict__ inv,
                                                      T *__restrict__ out, long long n_vec, int ds, int k)
{
    const int vec_per_slice = ds / V;
    for (long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x; g < n_vec;
         g += (long long)gridDim.x * blockDim.x) {
        const long long n = g / vec_per_slice;
        const int c0 = (int)(g - n * vec_per_slice) * V;
        float acc[V];
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = 0.f;
        if constexpr (K == 2) {
            const int2 r = *(const int2 *)(inv + n * 2);
            float a0[V], a1[V];
#pragma unroll
            for (int v = 0; v < V; ++v) a0[v] = a1[v] = 0.f;
            RowAdd<YT, V>::add(y + (size_t)(r.x < 0 ? 0 : r.x) * ds + c0, a0);
            RowAdd<YT, V>::add(y + (size_t)(r.y < 0 ? 0 : r.y) * ds + c0, a1);
#pragma unroll
            for (int v = 0; v < V; ++v) {   // ascending j, as in the general case
                if (r.x >= 0) acc[v] += a0[v];
                if (r.y >= 0) acc[v] += a1[v];
            }
        } else {
            for (int j = 0; j < k; ++j) {
                const int r = inv[n * k + j];
                if (r < 0) continue;
                RowAdd<YT, V>::add(y + (size_t)r * ds + c0, acc);
            }
        }
        OutVec<T, V>::store(out + (size_t)n * ds + c0, acc);
    }
}

template <typename T, typename YT, int V>
static hipError_t run(const slicemoe_config &c, const void *y, const int32_t *inv, void *h_out, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    const int ds = c.d / c.S;
    const long long n_vec = Ns * (ds / V);
    if (n_vec == 0) return hipSuccess;
    long long blocks = (n_vec + 255) / 256;
    const long long cap = (long long)num_compute_units() * 64;
    if (blocks > cap) blocks = cap;
    if (c.k == 2 && ((uintptr_t)inv & 7) == 0)
        combine_kernel<T, YT, V, 2><<<(int)blocks, 256, 0, s>>>((const YT *)y, inv, (T *)h_out, n_vec, ds, c.k);
    else
        combine_kernel<T, YT, V, 0><<<(int)blocks, 256, 0, s>>>((const YT *)y, inv, (T *)h_out, n_vec, ds, c.k);
    return hipGetLastError();
}

hipError_t launch_combine(const slicemoe_config &c, const void *y, const int32_t *inv, void *h_out,
                          hipStream_t s)
{
    const int ds = c.d / c.S;
    if (c.dtype == SLICEMOE_BF16) {
        if (ds % 8 == 0) return run<bf16_t, half_t, 8>(c, y, inv, h_out, s);
        return run<bf16_t, half_t, 1>(c, y, inv, h_out, s);
    }
    if (ds % 4 == 0) return run<float, float, 4>(c, y, inv, h_out, s);
    return run<float, float, 1>(c, y, inv, h_out, s);
}

}  // namespace slicemoe
