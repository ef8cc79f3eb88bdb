// Backward pass of the layer (vector-ALU, fp32 arithmetic): gradients of a loss that depends on h and on the
// weights only through h', by the chain rule through the k-sum, the expert FFN and the Eq. 1 input weighting
// (Section 3.1), and the router (Section 3.1; temperature of Appendix B, logit noise of Section 5 and cross-slice
// dropout of Section 3.3 as in the forward).  The routing decisions -- selected experts, capacity drops, dropout
// zeroes -- are piecewise constant and held fixed; the router receives gradient through the selected probabilities,
// which weight the expert inputs: z = p (x W1) + b1, so dL/dp = sum_hidden dL/dz (x W1).
//
// Two kernels, both straightforward by design (any shape within the library limits, either storage type):
//   bwd_expert_kernel  a block walks up to kBwdRows stacked rows of ONE expert in batches of kRB, one thread per
//                      hidden unit: recomputes u = x W1 and z, forms dz = (dy W2^T) gelu'(z), accumulates its
//                      column of dW1 and its row of dW2 in registers (adds them to memory once, at the end),
//                      reduces dL/dp over the hidden units and writes the row's dL/dx.
//   bwd_router_kernel  a block walks up to kBwdSlices slices in batches of kRB, one thread per router hidden unit:
//                      recomputes the router, goes back through the dropout's renormalisation and the softmax to
//                      dL/dg, accumulates the router's weight gradients the same way, and writes dL/dh = router path
//                      + the k expert-path rows of the slice (the gather that mirrors the combine).
// Wide shapes are cut over the grid: hidden units in groups of 256 (grid.y of the expert kernel; partial dL/dx and
// dL/dp are then added atomically) and slice features in chunks of kBwdCols (grid.z / grid.y; every chunk recomputes
// the shared quantities and owns its slice of the weight gradients and of dL/dx).
// Weight gradients are summed with fp32 atomic adds: their summation order, hence their last bits, vary from run to
// run.
#include "common.h"

namespace slicemoe {

constexpr int kBwdThreads = 256;
constexpr int kBwdRB = 8;         // rows (slices) per batch
constexpr int kBwdRows = 512;     // stacked rows per block of the expert kernel
constexpr int kBwdSlices = 256;   // slices per block of the router kernel
constexpr int kBwdCols = 64;      // slice features per grid chunk (register accumulators per thread)

__global__ void fill_zero_kernel(float *__restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

static hipError_t zero_fill(float *p, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    fill_zero_kernel<<<(int)(want < 4096 ? want : 4096), 256, 0, s>>>(p, n);
    return hipGetLastError();
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// d/dz of the exact GELU z Phi(z): Phi(z) + z phi(z)
__device__ __forceinline__ float gelu_grad(float z, float *act)
{
    const float cdf = 0.5f * (1.f + erff(z * 0.70710678118654752f));
    *act = z * cdf;
    return cdf + z * expf(-0.5f * z * z) * 0.39894228040143267794f;
}

template <typename T>
__global__ __launch_bounds__(kBwdThreads) void bwd_expert_kernel(
    const T *__restrict__ x, const T *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, int ds, int He, int E, int k,
    const T *__restrict__ W1, const T *__restrict__ b1, const T *__restrict__ W2,
    float *__restrict__ dxrow, float *__restrict__ dpk,
    float *__restrict__ dW1, float *__restrict__ db1, float *__restrict__ dW2, float *__restrict__ db2)
{
    extern __shared__ float smem[];
    float *xs = smem;                          // [kBwdRB][ds]   slice rows (not weighted)
    float *gs = xs + kBwdRB * ds;              // [kBwdRB][ds]   dL/dh' of the rows' slices
    float *dzs = gs + kBwdRB * ds;             // [kBwdRB][kBwdThreads] dL/dz of this hidden group
    __shared__ float ps[kBwdRB];               // final probability of each row
    __shared__ float dps[kBwdRB];              // dL/dp of each row (this hidden group's part)
    __shared__ int as[kBwdRB];                 // assignment id of each row
    __shared__ int blk[3];                     // expert, first row, end row of this block

    const int tid = threadIdx.x;
    if (tid == 0) {
        // chunks of kBwdRows rows, never across an expert boundary: find the chunk blockIdx.x names
        int left = (int)blockIdx.x, e = 0, begin = 0, end = 0;
        bool found = false;
        for (e = 0; e < E; ++e) {
            const int lo = offsets[e], hi = offsets[e + 1];
            const int nch = (hi - lo + kBwdRows - 1) / kBwdRows;
            if (left < nch) {
                begin = lo + left * kBwdRows;
                end = min(hi, begin + kBwdRows);
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
    if (e < 0) return;   // grid is sized for the worst case; uniform over the block

    const int j = (int)blockIdx.y * kBwdThreads + tid;        // hidden unit of this thread
    const bool jok = j < He;
    const int c0 = (int)blockIdx.z * kBwdCols;                // first slice feature of this chunk
    const int ncols = min(kBwdCols, ds - c0);
    const bool atomic_rows = gridDim.y > 1;                   // several hidden groups add into dL/dx and dL/dp
    const T *w1 = W1 + (size_t)e * ds * He;
    const T *w2 = W2 + (size_t)e * He * ds;
    const float bias = jok ? Storage<T>::load(b1 + (size_t)e * He + j) : 0.f;

    float aW1[kBwdCols], aW2[kBwdCols];
#pragma unroll
    for (int c = 0; c < kBwdCols; ++c) aW1[c] = aW2[c] = 0.f;
    float ab1 = 0.f, ab2 = 0.f;

    for (int r0 = row_begin; r0 < row_end; r0 += kBwdRB) {
        const int rows = min(kBwdRB, row_end - r0);
        if (tid < kBwdRB) {
            const int a = tid < rows ? perm[r0 + tid] : 0;
            as[tid] = a;
            ps[tid] = tid < rows ? pk[a] : 0.f;
            dps[tid] = 0.f;
        }
        __syncthreads();
        for (int i = tid; i < kBwdRB * ds; i += kBwdThreads) {
            const int r = i / ds, c = i - r * ds;
            float xv = 0.f, gv = 0.f;
            if (r < rows) {
                const long long n = as[r] / k;
                xv = Storage<T>::load(x + n * ds + c);
                gv = Storage<T>::load(dout + n * ds + c);
            }
            xs[i] = xv;
            gs[i] = gv;
        }
        __syncthreads();

        float u[kBwdRB], da[kBwdRB];
#pragma unroll
        for (int r = 0; r < kBwdRB; ++r) u[r] = da[r] = 0.f;
        if (jok) {
            for (int i = 0; i < ds; ++i) {
                const float wv = Storage<T>::load(w1 + (size_t)i * He + j);
                const float vv = Storage<T>::load(w2 + (size_t)j * ds + i);
#pragma unroll
                for (int r = 0; r < kBwdRB; ++r) {
                    u[r] = fmaf(xs[r * ds + i], wv, u[r]);
                    da[r] = fmaf(gs[r * ds + i], vv, da[r]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < kBwdRB; ++r) {
            float dz = 0.f, act = 0.f, pdz = 0.f;
            if (jok && r < rows) {
                const float p = ps[r];
                const float z = fmaf(p, u[r], bias);
                dz = da[r] * gelu_grad(z, &act);
                pdz = p * dz;
                ab1 += dz;
#pragma unroll
                for (int c = 0; c < kBwdCols; ++c)
                    if (c < ncols) {
                        aW2[c] = fmaf(act, gs[r * ds + c0 + c], aW2[c]);
                        aW1[c] = fmaf(xs[r * ds + c0 + c], pdz, aW1[c]);
                    }
            }
            dzs[r * kBwdThreads + tid] = dz;
            const float part = wave_sum(dz * u[r]);   // dL/dp = sum over hidden units of dL/dz (x W1)
            if ((tid & 63) == 0 && r < rows) atomicAdd(&dps[r], part);
        }
        if (blockIdx.y == 0 && tid < ncols)
            for (int r = 0; r < rows; ++r) ab2 += gs[r * ds + c0 + tid];
        __syncthreads();

        // dL/dx of the rows, this chunk's features: p * sum over this hidden group of dL/dz W1[i, j]
        const int jcount = min(kBwdThreads, He - (int)blockIdx.y * kBwdThreads);
        for (int t = tid; t < rows * ncols; t += kBwdThreads) {
            const int r = t / ncols, i = c0 + (t - r * ncols);
            const T *wr = w1 + (size_t)i * He + (size_t)blockIdx.y * kBwdThreads;
            float acc = 0.f;
            for (int jj = 0; jj < jcount; ++jj) acc = fmaf(dzs[r * kBwdThreads + jj], Storage<T>::load(wr + jj), acc);
            float *dst = dxrow + (size_t)(r0 + r) * ds + i;
            if (atomic_rows) atomicAdd(dst, ps[r] * acc);
            else *dst = ps[r] * acc;
        }
        if (blockIdx.z == 0 && tid < rows) {
            if (atomic_rows) atomicAdd(dpk + as[tid], dps[tid]);
            else dpk[as[tid]] = dps[tid];
        }
        __syncthreads();
    }

    if (jok) {
#pragma unroll
        for (int c = 0; c < kBwdCols; ++c)   // constant trip count: the accumulators stay in registers
            if (c < ncols) {
                atomicAdd(dW1 + ((size_t)e * ds + c0 + c) * He + j, aW1[c]);
                atomicAdd(dW2 + ((size_t)e * He + j) * ds + c0 + c, aW2[c]);
            }
        if (blockIdx.z == 0) atomicAdd(db1 + (size_t)e * He + j, ab1);
    }
    if (blockIdx.y == 0 && tid < ncols) atomicAdd(db2 + (size_t)e * ds + c0 + tid, ab2);
}

// Router backward and the assembly of dL/dh.  Hr <= kBwdThreads (one thread per router hidden unit), E <= 64.
template <typename T>
__global__ __launch_bounds__(kBwdThreads) void bwd_router_kernel(
    const T *__restrict__ x, long long Ns, int ds, int Hr, int E, int k,
    const T *__restrict__ Wr1, const T *__restrict__ br1, const T *__restrict__ Wr2, const T *__restrict__ br2,
    const float *__restrict__ noise, float sigma, float inv_tau, const float *__restrict__ drop_u, float rate,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ inv, const float *__restrict__ dpk,
    const float *__restrict__ dxrow, T *__restrict__ dh,
    float *__restrict__ dWr1, float *__restrict__ dbr1, float *__restrict__ dWr2, float *__restrict__ dbr2)
{
    extern __shared__ float smem[];
    float *xs = smem;                      // [kBwdRB][ds]
    float *us = xs + kBwdRB * ds;          // [kBwdRB][Hr]  ReLU output
    float *gs = us + kBwdRB * Hr;          // [kBwdRB][E]   logits, then softmax probabilities
    float *dgs = gs + kBwdRB * E;          // [kBwdRB][E]   dL/dg
    float *dus = dgs + kBwdRB * E;         // [kBwdRB][Hr]  dL/d(pre-activation of the hidden layer)

    const int tid = threadIdx.x;
    const int c0 = (int)blockIdx.y * kBwdCols;
    const int ncols = min(kBwdCols, ds - c0);
    const bool first_chunk = blockIdx.y == 0;
    const long long n_begin = (long long)blockIdx.x * kBwdSlices;
    const long long n_end = min(Ns, n_begin + kBwdSlices);
    const bool hok = tid < Hr;

    float aWr1[kBwdCols], aWr2[64];
#pragma unroll
    for (int c = 0; c < kBwdCols; ++c) aWr1[c] = 0.f;
#pragma unroll
    for (int e = 0; e < 64; ++e) aWr2[e] = 0.f;
    float abr1 = 0.f, abr2 = 0.f;
    const float hbias = hok ? Storage<T>::load(br1 + tid) : 0.f;

    for (long long n0 = n_begin; n0 < n_end; n0 += kBwdRB) {
        const int rows = (int)min((long long)kBwdRB, n_end - n0);
        for (int i = tid; i < kBwdRB * ds; i += kBwdThreads) {
            const int r = i / ds;
            xs[i] = r < rows ? Storage<T>::load(x + n0 * ds + i) : 0.f;
        }
        __syncthreads();
        // forward: hidden layer
        if (hok) {
            float acc[kBwdRB];
#pragma unroll
            for (int r = 0; r < kBwdRB; ++r) acc[r] = hbias;
            for (int i = 0; i < ds; ++i) {
                const float wv = Storage<T>::load(Wr1 + (size_t)i * Hr + tid);
#pragma unroll
                for (int r = 0; r < kBwdRB; ++r) acc[r] = fmaf(xs[r * ds + i], wv, acc[r]);
            }
#pragma unroll
            for (int r = 0; r < kBwdRB; ++r) us[r * Hr + tid] = fmaxf(acc[r], 0.f);
        }
        __syncthreads();
        // forward: logits (with the training-time noise)
        for (int t = tid; t < kBwdRB * E; t += kBwdThreads) {
            const int r = t / E, e = t - r * E;
            float acc = Storage<T>::load(br2 + e);
            for (int jh = 0; jh < Hr; ++jh) acc = fmaf(us[r * Hr + jh], Storage<T>::load(Wr2 + (size_t)jh * E + e), acc);
            if (noise != nullptr && r < rows) acc = fmaf(sigma, noise[(n0 + r) * E + e], acc);
            gs[t] = acc;
        }
        __syncthreads();
        // per slice: softmax, back through the dropout's renormalisation, dL/dg
        if (tid < rows) {
            const long long n = n0 + tid;
            float *g = gs + tid * E, *dg = dgs + tid * E;
            float m = g[0];
            for (int e = 1; e < E; ++e) m = fmaxf(m, g[e]);
            float den = 0.f;
            for (int e = 0; e < E; ++e) {
                g[e] = expf((g[e] - m) * inv_tau);
                den += g[e];
            }
            const float rden = 1.f / den;
            for (int e = 0; e < E; ++e) {
                g[e] *= rden;   // softmax probability of every expert
                dg[e] = 0.f;
            }
            float psel[8], dpf[8];
            bool keep[8];
            int ej[8];
            int kept = 0;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                psel[jj] = dpf[jj] = 0.f;
                keep[jj] = false;
                ej[jj] = 0;
                if (jj < k) {
                    const long long a = n * k + jj;
                    const int ee = idx[a];
                    ej[jj] = ee < 0 ? 0 : (ee >= E ? E - 1 : ee);
                    psel[jj] = g[ej[jj]];
                    dpf[jj] = inv[a] >= 0 ? dpk[a] : 0.f;   // a capacity-dropped assignment carries no gradient
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
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                if (jj < k) {
                    const float c = dpf[jj] * psel[jj] * inv_tau;
                    for (int e = 0; e < E; ++e) dg[e] += c * ((e == ej[jj] ? 1.f : 0.f) - g[e]);
                }
        } else if (tid < kBwdRB) {
            for (int e = 0; e < E; ++e) dgs[tid * E + e] = 0.f;   // rows past the end contribute nothing
        }
        __syncthreads();
        // backward: second layer, ReLU, first layer
        if (hok) {
            for (int r = 0; r < rows; ++r) {
                const float uv = us[r * Hr + tid];
                float acc = 0.f;
                for (int e = 0; e < E; ++e) {
                    const float d = dgs[r * E + e];
                    acc = fmaf(d, Storage<T>::load(Wr2 + (size_t)tid * E + e), acc);
                }
                const float du = uv > 0.f ? acc : 0.f;
                dus[r * Hr + tid] = du;
                if (first_chunk) {
                    abr1 += du;
#pragma unroll
                    for (int e = 0; e < 64; ++e)
                        if (e < E) aWr2[e] = fmaf(uv, dgs[r * E + e], aWr2[e]);
                }
#pragma unroll
                for (int c = 0; c < kBwdCols; ++c)
                    if (c < ncols) aWr1[c] = fmaf(xs[r * ds + c0 + c], du, aWr1[c]);
            }
        }
        if (first_chunk && tid < E)
            for (int r = 0; r < rows; ++r) abr2 += dgs[r * E + tid];
        __syncthreads();
        // dL/dh of the slices, this chunk's features: router path plus the expert-path rows of the k assignments
        for (int t = tid; t < rows * ncols; t += kBwdThreads) {
            const int r = t / ncols, i = c0 + (t - r * ncols);
            const long long n = n0 + r;
            const T *wr = Wr1 + (size_t)i * Hr;
            float acc = 0.f;
            for (int jh = 0; jh < Hr; ++jh) acc = fmaf(dus[r * Hr + jh], Storage<T>::load(wr + jh), acc);
            for (int jj = 0; jj < k; ++jj) {
                const int row = inv[n * k + jj];
                if (row >= 0) acc += dxrow[(size_t)row * ds + i];
            }
            Storage<T>::store(dh + n * ds + i, acc);
        }
        __syncthreads();
    }

    if (hok) {
#pragma unroll
        for (int c = 0; c < kBwdCols; ++c)
            if (c < ncols) atomicAdd(dWr1 + (size_t)(c0 + c) * Hr + tid, aWr1[c]);
        if (first_chunk) {
            atomicAdd(dbr1 + tid, abr1);
#pragma unroll
            for (int e = 0; e < 64; ++e)
                if (e < E) atomicAdd(dWr2 + (size_t)tid * E + e, aWr2[e]);
        }
    }
    if (first_chunk && tid < E) atomicAdd(dbr2 + tid, abr2);
}

size_t backward_lds_bytes(const slicemoe_config &c)
{
    const size_t ds = (size_t)(c.d / c.S);
    const size_t expert = sizeof(float) * (2 * kBwdRB * ds + (size_t)kBwdRB * kBwdThreads);
    const size_t router = sizeof(float) * kBwdRB * (ds + 2 * (size_t)c.Hr + 2 * (size_t)c.E);
    return expert > router ? expert : router;
}

template <typename T>
static hipError_t run_backward(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const RouteVariant &v,
                               const float *drop_u, float rate, const int32_t *idx, const float *pk,
                               const int32_t *offsets, const int32_t *perm, const int32_t *inv, const void *d_out,
                               void *d_h, const slicemoe_weight_grads &g, float *dxrow, float *dpk, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S, Na = Ns * c.k;
    const int ds = c.d / c.S;
    const size_t nW = (size_t)c.E * ds * c.He;
    hipError_t e;
    if ((e = zero_fill(g.Wr1, (size_t)ds * c.Hr, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.br1, (size_t)c.Hr, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.Wr2, (size_t)c.Hr * c.E, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.br2, (size_t)c.E, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.W1, nW, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.b1, (size_t)c.E * c.He, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.W2, nW, s)) != hipSuccess) return e;
    if ((e = zero_fill(g.b2, (size_t)c.E * ds, s)) != hipSuccess) return e;
    if (Ns == 0) return hipSuccess;

    const int hidden_groups = (c.He + kBwdThreads - 1) / kBwdThreads;
    const int col_chunks = (ds + kBwdCols - 1) / kBwdCols;
    if (hidden_groups > 1) {   // partial sums over the hidden groups are added atomically
        if ((e = zero_fill(dxrow, (size_t)Na * ds, s)) != hipSuccess) return e;
        if ((e = zero_fill(dpk, (size_t)Na, s)) != hipSuccess) return e;
    }
    const long long chunks = (Na + kBwdRows - 1) / kBwdRows + c.E;   // worst case: every expert ends on a partial chunk
    const size_t lds_e = sizeof(float) * (2 * (size_t)kBwdRB * ds + (size_t)kBwdRB * kBwdThreads);
    bwd_expert_kernel<T><<<dim3((unsigned)chunks, hidden_groups, col_chunks), kBwdThreads, lds_e, s>>>(
        (const T *)h, (const T *)d_out, pk, offsets, perm, ds, c.He, c.E, c.k, (const T *)w.W1, (const T *)w.b1,
        (const T *)w.W2, dxrow, dpk, g.W1, g.b1, g.W2, g.b2);
    if ((e = hipGetLastError()) != hipSuccess) return e;

    const long long sblocks = (Ns + kBwdSlices - 1) / kBwdSlices;
    const size_t lds_r = sizeof(float) * kBwdRB * ((size_t)ds + 2 * (size_t)c.Hr + 2 * (size_t)c.E);
    bwd_router_kernel<T><<<dim3((unsigned)sblocks, col_chunks), kBwdThreads, lds_r, s>>>(
        (const T *)h, Ns, ds, c.Hr, c.E, c.k, (const T *)w.Wr1, (const T *)w.br1, (const T *)w.Wr2, (const T *)w.br2,
        v.sigma > 0.f ? v.noise : nullptr, v.sigma, v.inv_tau, rate > 0.f ? drop_u : nullptr, rate, idx, inv, dpk, dxrow,
        (T *)d_h, g.Wr1, g.br1, g.Wr2, g.br2);
    return hipGetLastError();
}

hipError_t launch_backward(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const RouteVariant &v,
                           const float *drop_u, float rate, const int32_t *idx, const float *pk, const int32_t *offsets,
                           const int32_t *perm, const int32_t *inv, const void *d_out, void *d_h,
                           const slicemoe_weight_grads &g, float *dxrow, float *dpk, hipStream_t s)
{
    if (c.dtype == SLICEMOE_BF16)
        return run_backward<bf16_t>(c, h, w, v, drop_u, rate, idx, pk, offsets, perm, inv, d_out, d_h, g, dxrow, dpk, s);
    return run_backward<float>(c, h, w, v, drop_u, rate, idx, pk, offsets, perm, inv, d_out, d_h, g, dxrow, dpk, s);
}

}  // namespace slicemoe
