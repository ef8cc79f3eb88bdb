// Combine stage (paper Section 3.1): the k expert outputs of a slice are summed and the S
// output slices concatenated.  In the slice view h'[n, :] sits where x[n, :] sat, so the
// output is one contiguous stream: thread g handles V consecutive output elements, reads the
// matching V floats of up to k stacked rows (fp32, full-line 16-byte loads), adds them in
// ascending j and writes one rounded vector.  HBM-bound; no reuse, so no LDS.
#include "common.h"

namespace slicemoe {

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
template <> struct OutVec<bf16_t, 4> {
    static __device__ __forceinline__ void store(bf16_t *o, const float *v)
    {
        uint2 u;
        u.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
        u.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
        *(uint2 *)o = u;
    }
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

template <typename T, int V>
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ y, const int32_t *__restrict__ inv,
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
        for (int j = 0; j < k; ++j) {
            const int r = inv[n * k + j];
            if (r < 0) continue;
            const float *src = y + (size_t)r * ds + c0;
            if (V >= 4) {
#pragma unroll
                for (int v = 0; v < V; v += 4) {
                    const float4 t = *(const float4 *)(src + v);
                    acc[v] += t.x;
                    acc[v + 1] += t.y;
                    acc[v + 2] += t.z;
                    acc[v + 3] += t.w;
                }
            } else {
                acc[0] += src[0];
            }
        }
        OutVec<T, V>::store(out + (size_t)n * ds + c0, acc);
    }
}

template <typename T, int V>
static hipError_t run(const slicemoe_config &c, const float *y, const int32_t *inv, void *h_out, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S;
    const int ds = c.d / c.S;
    const long long n_vec = Ns * (ds / V);
    if (n_vec == 0) return hipSuccess;
    long long blocks = (n_vec + 255) / 256;
    const long long cap = (long long)num_compute_units() * 64;
    if (blocks > cap) blocks = cap;
    combine_kernel<T, V><<<(int)blocks, 256, 0, s>>>(y, inv, (T *)h_out, n_vec, ds, c.k);
    return hipGetLastError();
}

hipError_t launch_combine(const slicemoe_config &c, const float *y, const int32_t *inv, void *h_out,
                          hipStream_t s)
{
    const int ds = c.d / c.S;
    if (c.dtype == SLICEMOE_BF16) {
        if (ds % 8 == 0) return run<bf16_t, 8>(c, y, inv, h_out, s);
        if (ds % 4 == 0) return run<bf16_t, 4>(c, y, inv, h_out, s);
        return run<bf16_t, 1>(c, y, inv, h_out, s);
    }
    if (ds % 4 == 0) return run<float, 4>(c, y, inv, h_out, s);
    return run<float, 1>(c, y, inv, h_out, s);
}

}  // namespace slicemoe
