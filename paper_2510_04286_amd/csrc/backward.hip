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
//                      column of dW1 and its row of dW2 in registers (stores them once, at the end),
//                      reduces dL/dp over the hidden units and writes the row's dL/dx.
//   bwd_router_kernel  a block walks up to slices_per_block slices in batches of kRB, one thread per router hidden unit:
//                      recomputes the router, goes back through the dropout's renormalisation and the softmax to
//                      dL/dg, accumulates the router's weight gradients the same way, and writes dL/dh = router path
//                      + the k expert-path rows of the slice (the gather that mirrors the combine).
// Wide shapes: hidden units are taken in groups of 256 that a block of the expert kernel works through in turn (the
// same thread adds each group's part of dL/dx and dL/dp to what it wrote before: no atomics), and slice features are
// cut over the grid in chunks of kBwdCols (grid.z / grid.y; every chunk recomputes the shared quantities and owns its
// slice of the weight gradients and of dL/dx).
// Weight gradients: every block stores its partial sums in its own slot of a scratch buffer, and a second pair of
// kernels adds the slots up in a fixed order (device-wide atomic adds from a thousand blocks cost more than the
// arithmetic, and their order varies from run to run; this way the result is reproducible bit for bit).
#include <mutex>

#include "common.h"

namespace slicemoe {

constexpr int kBwdThreads = 256;
constexpr int kBwdRB = 8;         // rows (slices) per batch
constexpr int kBwdSlices = 512;   // slices per block of the router kernel at least (about a thousand blocks for large batches)
constexpr int kBwdCols = 64;      // slice features per grid chunk (register accumulators per thread)

__host__ __device__ __forceinline__ size_t expert_slot_floats(int ds, int He) { return 2 * (size_t)ds * He + He + ds; }
__host__ __device__ __forceinline__ size_t router_slot_floats(int ds, int Hr, int E) { return (size_t)ds * Hr + (size_t)Hr * E + Hr + E; }

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

// Row stride padding (elements) of the weight slices kept in LDS: an odd number of 32-bit words per row, so that
// threads reading down a column hit different banks.
template <typename T> constexpr int kWPad = sizeof(T) == 2 ? 2 : 1;

// WLDS: this block's slices of W1 (all features x its 256 hidden units) and W2 (its 256 hidden units x all features)
// sit in LDS for the whole block (they fit up to ds = 128 with 16-bit storage); otherwise they are read from memory.
template <typename T, bool WLDS>
__global__ __launch_bounds__(kBwdThreads) void bwd_expert_kernel(
    const T *__restrict__ x, const T *__restrict__ dout, const float *__restrict__ pk,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, int ds, int He, int E, int k,
    const T *__restrict__ W1, const T *__restrict__ b1, const T *__restrict__ W2,
    float *__restrict__ dxrow, float *__restrict__ dpk, int rows_per_chunk, int hidden_groups, float *__restrict__ part)
{
    extern __shared__ float smem[];
    const int dsp = (ds + kBwdCols - 1) / kBwdCols * kBwdCols;   // LDS row stride: whole feature chunks, zero-padded
    float *xs = smem;                          // [kBwdRB][dsp]  slice rows (not weighted)
    float *gs = xs + kBwdRB * dsp;             // [kBwdRB][dsp]  dL/dh' of the rows' slices
    float *dzs = gs + kBwdRB * dsp;            // [kBwdRB][kBwdThreads] dL/dz of this hidden group
    const int w1st = kBwdThreads + kWPad<T>, w2st = ds + kWPad<T>;
    T *w1s = (T *)(dzs + kBwdRB * kBwdThreads);   // [ds][w1st]          (WLDS only)
    T *w2s = w1s + (size_t)ds * w1st;             // [kBwdThreads][w2st] (WLDS only)
    __shared__ float ps[kBwdRB];               // final probability of each row
    __shared__ float dps[kBwdThreads / 64][kBwdRB];   // dL/dp of each row: one partial sum per wavefront
    __shared__ int as[kBwdRB];                 // assignment id of each row
    __shared__ int blk[3];                     // expert, first row, end row of this block

    const int tid = threadIdx.x;
    if (tid == 0) {
        // chunks of rows_per_chunk rows, never across an expert boundary: find the chunk blockIdx.x names
        int left = (int)blockIdx.x, e = 0, begin = 0, end = 0;
        bool found = false;
        for (e = 0; e < E; ++e) {
            const int lo = offsets[e], hi = offsets[e + 1];
            const int nch = (hi - lo + rows_per_chunk - 1) / rows_per_chunk;
            if (left < nch) {
                begin = lo + left * rows_per_chunk;
                end = min(hi, begin + rows_per_chunk);
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

    const int c0 = (int)blockIdx.z * kBwdCols;                // first slice feature of this chunk
    const int ncols = min(kBwdCols, ds - c0);
    const T *w1 = W1 + (size_t)e * ds * He;
    const T *w2 = W2 + (size_t)e * He * ds;
    const int ds4 = (ds + 3) & ~3;
    float *slot = part + (size_t)blockIdx.x * expert_slot_floats(ds, He);
    // The hidden units are taken in groups of one per thread, one group after the other by the same block: the parts of
    // dL/dx and dL/dp that the groups contribute are added by the same thread in the same order on every run.
    for (int grp = 0; grp < hidden_groups; ++grp) {
    const int j = grp * kBwdThreads + tid;                    // hidden unit of this thread
    const bool jok = j < He;
    const float bias = jok ? Storage<T>::load(b1 + (size_t)e * He + j) : 0.f;
    const int jg0 = grp * kBwdThreads;
    if (WLDS) {   // ordered before the first read by the barriers at the top of the row loop (and after the last read of
                  // the previous group by the barrier at its end)
        for (int t = tid; t < ds * kBwdThreads; t += kBwdThreads) {
            const int i = t / kBwdThreads, jj = t - i * kBwdThreads;
            w1s[i * w1st + jj] = jg0 + jj < He ? w1[(size_t)i * He + jg0 + jj] : (T)0;
        }
        for (int t = tid; t < kBwdThreads * ds; t += kBwdThreads) {
            const int jj = t / ds, c = t - jj * ds;
            w2s[jj * w2st + c] = jg0 + jj < He ? w2[(size_t)(jg0 + jj) * ds + c] : (T)0;
        }
    }
    auto w1_at = [&](int i, int jj) -> float {   // W1[e][i][jg0 + jj]
        return WLDS ? Storage<T>::load(w1s + i * w1st + jj) : Storage<T>::load(w1 + (size_t)i * He + jg0 + jj);
    };
    auto w2_at = [&](int jj, int c) -> float {   // W2[e][jg0 + jj][c]
        return WLDS ? Storage<T>::load(w2s + jj * w2st + c) : Storage<T>::load(w2 + (size_t)(jg0 + jj) * ds + c);
    };

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
        }
        __syncthreads();
        for (int i = tid; i < kBwdRB * dsp; i += kBwdThreads) {
            const int r = i / dsp, c = i - r * dsp;
            float xv = 0.f, gv = 0.f;
            if (r < rows && c < ds) {
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
            for (int i = 0; i < ds4; i += 4) {
                float wv[4], vv[4];
                if (i + 4 <= ds) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        wv[q] = w1_at(i + q, tid);
                        vv[q] = w2_at(tid, i + q);
                    }
                } else {   // last, partial group of a width that is not a multiple of 4: the tiles hold zeros there
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        wv[q] = i + q < ds ? w1_at(i + q, tid) : 0.f;
                        vv[q] = i + q < ds ? w2_at(tid, i + q) : 0.f;
                    }
                }
#pragma unroll
                for (int r = 0; r < kBwdRB; ++r) {
                    const float4 xq = *(const float4 *)(xs + r * dsp + i), gq = *(const float4 *)(gs + r * dsp + i);
                    u[r] = fmaf(xq.x, wv[0], fmaf(xq.y, wv[1], fmaf(xq.z, wv[2], fmaf(xq.w, wv[3], u[r]))));
                    da[r] = fmaf(gq.x, vv[0], fmaf(gq.y, vv[1], fmaf(gq.z, vv[2], fmaf(gq.w, vv[3], da[r]))));
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
                // the whole chunk of kBwdCols features: past the slice width the tiles hold zeros
#pragma unroll
                for (int c = 0; c < kBwdCols; c += 4) {
                    const float4 gq = *(const float4 *)(gs + r * dsp + c0 + c), xq = *(const float4 *)(xs + r * dsp + c0 + c);
                    aW2[c] = fmaf(act, gq.x, aW2[c]);
                    aW2[c + 1] = fmaf(act, gq.y, aW2[c + 1]);
                    aW2[c + 2] = fmaf(act, gq.z, aW2[c + 2]);
                    aW2[c + 3] = fmaf(act, gq.w, aW2[c + 3]);
                    aW1[c] = fmaf(xq.x, pdz, aW1[c]);
                    aW1[c + 1] = fmaf(xq.y, pdz, aW1[c + 1]);
                    aW1[c + 2] = fmaf(xq.z, pdz, aW1[c + 2]);
                    aW1[c + 3] = fmaf(xq.w, pdz, aW1[c + 3]);
                }
            }
            dzs[r * kBwdThreads + tid] = dz;
            const float part = wave_sum(dz * u[r]);   // dL/dp = sum over hidden units of dL/dz (x W1)
            if ((tid & 63) == 0) dps[tid >> 6][r] = part;   // added up below in a fixed order
        }
        if (grp == 0 && tid < ncols)
            for (int r = 0; r < rows; ++r) ab2 += gs[r * dsp + c0 + tid];
        __syncthreads();

        // dL/dx of the rows, this chunk's features: p * sum over this hidden group of dL/dz W1[i, j]
        const int jcount = min(kBwdThreads, He - grp * kBwdThreads);
        for (int t = tid; t < rows * ncols; t += kBwdThreads) {
            const int r = t / ncols, i = c0 + (t - r * ncols);
            float acc = 0.f;
#pragma unroll 8
            for (int jj = 0; jj < jcount; ++jj) acc = fmaf(dzs[r * kBwdThreads + jj], w1_at(i, jj), acc);
            float *dst = dxrow + (size_t)(r0 + r) * ds + i;   // the same thread wrote it for the groups before
            *dst = grp > 0 ? *dst + ps[r] * acc : ps[r] * acc;
        }
        if (blockIdx.z == 0 && tid < rows) {
            float dp = 0.f;
#pragma unroll
            for (int wv = 0; wv < kBwdThreads / 64; ++wv) dp += dps[wv][tid];
            dpk[as[tid]] = grp > 0 ? dpk[as[tid]] + dp : dp;
        }
        __syncthreads();
    }

    // this chunk's slot: dW1 [ds][He] | dW2 [He][ds] | db1 [He] | db2 [ds]; the blocks of the chunk (hidden groups x
    // feature chunks) write disjoint parts of it, every element exactly once
    float *pW1 = slot, *pW2 = pW1 + (size_t)ds * He, *pb1 = pW2 + (size_t)He * ds, *pb2 = pb1 + He;
    if (jok) {
#pragma unroll
        for (int c = 0; c < kBwdCols; ++c)   // constant trip count: the accumulators stay in registers
            if (c < ncols) {
                pW1[(size_t)(c0 + c) * He + j] = aW1[c];
                pW2[(size_t)j * ds + c0 + c] = aW2[c];
            }
        if (blockIdx.z == 0) pb1[j] = ab1;
    }
    if (grp == 0 && tid < ncols) pb2[c0 + tid] = ab2;
    }
}

// Sum of the chunk slots of each expert in a fixed order: grid (E, pieces of 64 slot elements); a block is 64 elements
// x 8 interleaved sequences of chunks, whose eight partial sums are added in order at the end.
constexpr int kRedElems = 64, kRedSeqs = 8;
template <int V> struct RedVec;
template <> struct RedVec<1> { typedef float type; };
typedef float red_f32x4 __attribute__((ext_vector_type(4)));
template <> struct RedVec<4> { typedef red_f32x4 type; };
// V = 4: four consecutive entries per thread (16-byte loads and stores) where the tensors' sizes and addresses allow.
template <int V>
__global__ __launch_bounds__(kRedElems * kRedSeqs) void bwd_reduce_expert_kernel(
    const float *__restrict__ part, const int32_t *__restrict__ offsets, int ds, int He, int E, int rows_per_chunk,
    float *__restrict__ dW1, float *__restrict__ db1, float *__restrict__ dW2, float *__restrict__ db2)
{
    typedef typename RedVec<V>::type vec;
    __shared__ vec red[kRedSeqs][kRedElems];
    const int e = blockIdx.x;
    const int ex = threadIdx.x % kRedElems, sq = threadIdx.x / kRedElems;
    const size_t slot = expert_slot_floats(ds, He);
    const size_t t = ((size_t)blockIdx.y * kRedElems + ex) * V;
    // chunks are numbered expert by expert, as the expert kernels find them (E <= 64: one thread per expert)
    __shared__ int nchs[64];
    if (threadIdx.x < 64)
        nchs[threadIdx.x] = (int)threadIdx.x < E ? (offsets[threadIdx.x + 1] - offsets[threadIdx.x] + rows_per_chunk - 1) / rows_per_chunk : 0;
    __syncthreads();
    int first = 0;
    for (int q = 0; q < e; ++q) first += nchs[q];
    const int nch = nchs[e];
    vec acc = {};
    if (t < slot) {
#pragma unroll 4
        for (int c = sq; c < nch; c += kRedSeqs) acc += *(const vec *)(part + (size_t)(first + c) * slot + t);
    }
    red[sq][ex] = acc;
    __syncthreads();
    if (sq != 0 || t >= slot) return;
    acc = vec{};
#pragma unroll
    for (int q = 0; q < kRedSeqs; ++q) acc += red[q][ex];   // fixed order
    const size_t nW = (size_t)ds * He;
    if (t < nW) *(vec *)(dW1 + (size_t)e * nW + t) = acc;
    else if (t < 2 * nW) *(vec *)(dW2 + (size_t)e * nW + (t - nW)) = acc;
    else if (t < 2 * nW + He) *(vec *)(db1 + (size_t)e * He + (t - 2 * nW)) = acc;
    else *(vec *)(db2 + (size_t)e * ds + (t - 2 * nW - He)) = acc;
}

// Router backward and the assembly of dL/dh.  Hr <= kBwdThreads (one thread per router hidden unit), E <= 64.
// WLDS: both router matrices sit in LDS for the whole block (they fit up to ds = 128 with 16-bit storage).
template <typename T, bool WLDS>
__global__ __launch_bounds__(kBwdThreads) void bwd_router_kernel(
    const T *__restrict__ x, long long Ns, int ds, int Hr, int E, int k,
    const T *__restrict__ Wr1, const T *__restrict__ br1, const T *__restrict__ Wr2, const T *__restrict__ br2,
    const float *__restrict__ noise, float sigma, float inv_tau, const float *__restrict__ drop_u, float rate,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ inv, const float *__restrict__ dpk,
    const float *__restrict__ capg, const float *__restrict__ dxrow, T *__restrict__ dh, int slices_per_block,
    float *__restrict__ part)
{
    extern __shared__ float smem[];
    float *xs = smem;                      // [kBwdRB][ds]
    float *us = xs + kBwdRB * ds;          // [kBwdRB][Hr]  ReLU output
    float *gs = us + kBwdRB * Hr;          // [kBwdRB][E]   logits, then softmax probabilities
    float *dgs = gs + kBwdRB * E;          // [kBwdRB][E]   dL/dg
    float *dus = dgs + kBwdRB * E;         // [kBwdRB][Hr]  dL/d(pre-activation of the hidden layer)
    const int w1st = Hr + kWPad<T>, w2st = E + kWPad<T>;
    T *w1s = (T *)(dus + kBwdRB * Hr);     // [ds][w1st]  (WLDS only)
    T *w2s = w1s + (size_t)ds * w1st;      // [Hr][w2st]  (WLDS only)

    const int tid = threadIdx.x;
    const int c0 = (int)blockIdx.y * kBwdCols;
    const int ncols = min(kBwdCols, ds - c0);
    const bool first_chunk = blockIdx.y == 0;
    const long long n_begin = (long long)blockIdx.x * slices_per_block;
    const long long n_end = min(Ns, n_begin + slices_per_block);
    const bool hok = tid < Hr;

    float aWr1[kBwdCols], aWr2[64];
#pragma unroll
    for (int c = 0; c < kBwdCols; ++c) aWr1[c] = 0.f;
#pragma unroll
    for (int e = 0; e < 64; ++e) aWr2[e] = 0.f;
    float abr1 = 0.f, abr2 = 0.f;
    const float hbias = hok ? Storage<T>::load(br1 + tid) : 0.f;
    const bool vec4 = (ds & 3) == 0;
    if (WLDS) {   // ordered before the first read by the barrier after the slice loads
        for (int t = tid; t < ds * Hr; t += kBwdThreads) {
            const int i = t / Hr, jh = t - i * Hr;
            w1s[i * w1st + jh] = Wr1[t];
        }
        for (int t = tid; t < Hr * E; t += kBwdThreads) {
            const int jh = t / E, e = t - jh * E;
            w2s[jh * w2st + e] = Wr2[t];
        }
    }
    auto w1_at = [&](int i, int jh) -> float {   // Wr1[i][jh]
        return WLDS ? Storage<T>::load(w1s + i * w1st + jh) : Storage<T>::load(Wr1 + (size_t)i * Hr + jh);
    };
    auto w2_at = [&](int jh, int e) -> float {   // Wr2[jh][e]
        return WLDS ? Storage<T>::load(w2s + jh * w2st + e) : Storage<T>::load(Wr2 + (size_t)jh * E + e);
    };

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
            if (vec4) {
                for (int i = 0; i < ds; i += 4) {
                    const float w0 = w1_at(i, tid), w1v = w1_at(i + 1, tid), w2v = w1_at(i + 2, tid), w3 = w1_at(i + 3, tid);
#pragma unroll
                    for (int r = 0; r < kBwdRB; ++r) {
                        const float4 xq = *(const float4 *)(xs + r * ds + i);
                        acc[r] = fmaf(xq.x, w0, fmaf(xq.y, w1v, fmaf(xq.z, w2v, fmaf(xq.w, w3, acc[r]))));
                    }
                }
            } else {
                for (int i = 0; i < ds; ++i) {
                    const float wv = w1_at(i, tid);
#pragma unroll
                    for (int r = 0; r < kBwdRB; ++r) acc[r] = fmaf(xs[r * ds + i], wv, acc[r]);
                }
            }
#pragma unroll
            for (int r = 0; r < kBwdRB; ++r) us[r * Hr + tid] = fmaxf(acc[r], 0.f);
        }
        __syncthreads();
        // forward: logits (with the training-time noise)
        for (int t = tid; t < kBwdRB * E; t += kBwdThreads) {
            const int r = t / E, e = t - r * E;
            float acc = Storage<T>::load(br2 + e);
#pragma unroll 8
            for (int jh = 0; jh < Hr; ++jh) acc = fmaf(us[r * Hr + jh], w2_at(jh, e), acc);
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
                    dpf[jj] = inv[a] >= 0 ? dpk[a] : 0.f;   // a capacity-dropped assignment carries no gradient from h'
                    if (capg != nullptr) dpf[jj] += capg[ej[jj]];   // but it counts as assigned (capacity loss)
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
                    acc = fmaf(d, w2_at(tid, e), acc);
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
            float acc = 0.f;
#pragma unroll 8
            for (int jh = 0; jh < Hr; ++jh) acc = fmaf(dus[r * Hr + jh], w1_at(i, jh), acc);
            for (int jj = 0; jj < k; ++jj) {
                const int row = inv[n * k + jj];
                if (row >= 0) acc += dxrow[(size_t)row * ds + i];
            }
            Storage<T>::store(dh + n * ds + i, acc);
        }
        __syncthreads();
    }

    // this block's slot: dWr1 [ds][Hr] | dWr2 [Hr][E] | dbr1 [Hr] | dbr2 [E]; the feature chunks of one range of slices
    // (grid.y) share a slot and write disjoint parts of it
    float *slot = part + (size_t)blockIdx.x * router_slot_floats(ds, Hr, E);
    float *pWr1 = slot, *pWr2 = pWr1 + (size_t)ds * Hr, *pbr1 = pWr2 + (size_t)Hr * E, *pbr2 = pbr1 + Hr;
    if (hok) {
#pragma unroll
        for (int c = 0; c < kBwdCols; ++c)
            if (c < ncols) pWr1[(size_t)(c0 + c) * Hr + tid] = aWr1[c];
        if (first_chunk) {
            pbr1[tid] = abr1;
#pragma unroll
            for (int e = 0; e < 64; ++e)
                if (e < E) pWr2[(size_t)tid * E + e] = aWr2[e];
        }
    }
    if (first_chunk && tid < E) pbr2[tid] = abr2;
}

// Sum of the router slots of all blocks in a fixed order; same scheme as bwd_reduce_expert_kernel.
__global__ __launch_bounds__(kRedElems * kRedSeqs) void bwd_reduce_router_kernel(
    const float *__restrict__ part, int nslots, int ds, int Hr, int E,
    float *__restrict__ dWr1, float *__restrict__ dbr1, float *__restrict__ dWr2, float *__restrict__ dbr2)
{
    __shared__ float red[kRedSeqs][kRedElems];
    const int ex = threadIdx.x % kRedElems, sq = threadIdx.x / kRedElems;
    const size_t slot = router_slot_floats(ds, Hr, E);
    const size_t t = (size_t)blockIdx.x * kRedElems + ex;
    float acc = 0.f;
    if (t < slot) {
#pragma unroll 4
        for (int b = sq; b < nslots; b += kRedSeqs) acc += part[(size_t)b * slot + t];
    }
    red[sq][ex] = acc;
    __syncthreads();
    if (sq != 0 || t >= slot) return;
    acc = 0.f;
#pragma unroll
    for (int q = 0; q < kRedSeqs; ++q) acc += red[q][ex];   // fixed order
    const size_t n1 = (size_t)ds * Hr, n2 = (size_t)Hr * E;
    if (t < n1) dWr1[t] = acc;
    else if (t < n1 + n2) dWr2[t - n1] = acc;
    else if (t < n1 + n2 + Hr) dbr1[t - n1 - n2] = acc;
    else dbr2[t - n1 - n2 - Hr] = acc;
}

size_t backward_lds_bytes(const slicemoe_config &c)
{
    const size_t ds = (size_t)(c.d / c.S);
    const size_t dsp = (ds + kBwdCols - 1) / kBwdCols * kBwdCols;
    const size_t expert = sizeof(float) * (2 * kBwdRB * dsp + (size_t)kBwdRB * kBwdThreads);
    const size_t router = sizeof(float) * kBwdRB * (ds + 2 * (size_t)c.Hr + 2 * (size_t)c.E);
    return expert > router ? expert : router;
}

BackwardPlan backward_plan(const slicemoe_config &c)
{
    BackwardPlan p;
    const size_t Ns = (size_t)c.T * c.S, Na = Ns * c.k;
    const size_t ds = (size_t)(c.d / c.S);
    // about a thousand chunks of stacked rows however large the batch (each has a slot of partial weight gradients),
    // at least 512 rows each, whole batches of rows
    size_t rows = (Na + 1023) / 1024;
    rows = (rows + 31) / 32 * 32;   // whole 32-row units of the matrix-core kernels (and whole batches of kBwdRB)
    p.rows_per_chunk = (int)(rows < 512 ? 512 : rows);
    p.chunks = (long long)((Na + p.rows_per_chunk - 1) / p.rows_per_chunk) + c.E;   // worst case: every expert ends on a partial chunk
    size_t spb = ((Ns + 1023) / 1024 + 31) / 32 * 32;
    p.slices_per_block = (int)(spb < (size_t)kBwdSlices ? (size_t)kBwdSlices : spb);
    p.slice_blocks = (long long)((Ns + p.slices_per_block - 1) / p.slices_per_block);
    size_t at = 0;
    p.dxrow = at;  at = align_up(at + Na * ds * sizeof(float), 256);
    p.dpk = at;    at = align_up(at + Na * sizeof(float), 256);
    p.expert_part = at;  at = align_up(at + (size_t)p.chunks * expert_slot_floats((int)ds, c.He) * sizeof(float), 256);
    p.router_part = at;  at = align_up(at + (size_t)p.slice_blocks * router_slot_floats((int)ds, c.Hr, c.E) * sizeof(float), 256);
    p.packed = at;  at = align_up(at + backward_mfma_packed_bytes(c), 256);
    p.router_scratch = at;  at = align_up(at + backward_router_mfma_scratch_bytes(c), 256);
    p.cap = at;  at = align_up(at + (size_t)c.E * (sizeof(unsigned long long) + sizeof(float)), 256);
    p.total = at + 256;
    return p;
}

// ---- The capacity loss (Section 3.2, Eq. 2) in its differentiable reading.  Eq. 2 is a function of integer counts;
// the router can only be trained with it (Section 3.1) through a stand-in, and the one taken here is the usual one: the
// count of expert e becomes the sum c_e of the final probabilities of the assignments routed to e, the loss
// alpha CV^2(c) with the population variance, and dL_cap/dp_a = alpha (2E / S^2) (c_e(a) - Q / S), S = sum c, Q = sum c^2.
// The sums are exact and the same on every run: each probability, a float in [0, 1], is added as the integer
// p * 2^38 (at most 2^22 * k assignments: no overflow in 64 bits; bits below 2^-38 of a tiny p are rounded off).
constexpr float kCapScale = 274877906944.f;   // 2^38

__global__ __launch_bounds__(256) void bwd_cap_sums_kernel(const int32_t *__restrict__ idx, const float *__restrict__ pk,
                                                           long long Na, int E, unsigned long long *__restrict__ sums)
{
    extern __shared__ unsigned long long cap_s[];
    for (int e = threadIdx.x; e < E; e += blockDim.x) cap_s[e] = 0ull;
    __syncthreads();
    for (long long a = (long long)blockIdx.x * blockDim.x + threadIdx.x; a < Na; a += (long long)gridDim.x * blockDim.x) {
        const int ee = idx[a];
        const int e = ee < 0 ? 0 : (ee >= E ? E - 1 : ee);
        const float p = fminf(fmaxf(pk[a], 0.f), 1.f);
        atomicAdd(&cap_s[e], (unsigned long long)__float2ll_rn(p * kCapScale));
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x)
        if (cap_s[e] != 0ull) atomicAdd(&sums[e], cap_s[e]);
}

// One block.  Every thread adds up all E sums in the same order, then writes its experts' derivatives.
__global__ __launch_bounds__(256) void bwd_cap_coeff_kernel(const unsigned long long *__restrict__ sums, int E, float alpha,
                                                            float *__restrict__ capg)
{
    double S = 0.0, Q = 0.0;
    for (int e = 0; e < E; ++e) {
        const double c = (double)sums[e] / (double)kCapScale;
        S += c;
        Q += c * c;
    }
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const double c = (double)sums[e] / (double)kCapScale;
        capg[e] = S > 0.0 ? (float)((double)alpha * (2.0 * E / (S * S)) * (c - Q / S)) : 0.f;
    }
}

// ---- A stream of the library's own, beside the caller's.  The expert weight gradients (their kernel and the
// reduction after it) depend on nothing that the rest of the backward produces, and nothing but the caller depends on
// them, so they run on this stream while the row gradients and the router's kernels run on the caller's: the two
// chains fill each other's launch gaps and tails.  One stream and two events per device, made at the first backward on
// that device and kept until the process ends; default priority, no implicit synchronisation with the null stream.
// The events are shared by all calls on a device, so the enqueueing of one call (fork .. join) holds a lock.
static std::mutex g_side_mutex;

static hipError_t side_stream(SideStream *out)
{
    static SideStream set[64];
    static bool have[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!have[dev]) {
        SideStream n = {};
        if ((e = hipStreamCreateWithFlags(&n.stream, hipStreamNonBlocking)) != hipSuccess) return e;
        if ((e = hipEventCreateWithFlags(&n.fork, hipEventDisableTiming)) != hipSuccess) return e;
        if ((e = hipEventCreateWithFlags(&n.join, hipEventDisableTiming)) != hipSuccess) return e;
        set[dev] = n;
        have[dev] = true;
    }
    *out = set[dev];
    return hipSuccess;
}

// Joins the side stream back into the caller's stream when the scope ends, on every path out of it.
struct SideJoin {
    const SideStream *side = nullptr;
    hipStream_t s = nullptr;
    hipError_t result = hipSuccess;
    ~SideJoin() { (void)join(); }
    hipError_t join()
    {
        if (side != nullptr) {
            hipError_t e = hipEventRecord(side->join, side->stream);
            if (e == hipSuccess) e = hipStreamWaitEvent(s, side->join, 0);
            if (e != hipSuccess) result = e;
            side = nullptr;
        }
        return result;
    }
};

template <typename T>
static hipError_t run_backward(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const RouteVariant &v_in,
                               const float *drop_u, float rate, const int32_t *idx, const float *pk,
                               const int32_t *offsets, const int32_t *perm, const int32_t *inv, const void *d_out,
                               void *d_h, const slicemoe_weight_grads &g, void *workspace, hipStream_t s)
{
    const long long Ns = (long long)c.T * c.S, Na = Ns * c.k;
    const int ds = c.d / c.S;
    const size_t nW = (size_t)c.E * ds * c.He;
    hipError_t e;
    if (Ns == 0) {   // nothing to sum: the gradients are zero
        if ((e = zero_fill(g.Wr1, (size_t)ds * c.Hr, s)) != hipSuccess) return e;
        if ((e = zero_fill(g.br1, (size_t)c.Hr, s)) != hipSuccess) return e;
        if ((e = zero_fill(g.Wr2, (size_t)c.Hr * c.E, s)) != hipSuccess) return e;
        if ((e = zero_fill(g.br2, (size_t)c.E, s)) != hipSuccess) return e;
        if ((e = zero_fill(g.W1, nW, s)) != hipSuccess) return e;
        if ((e = zero_fill(g.b1, (size_t)c.E * c.He, s)) != hipSuccess) return e;
        if ((e = zero_fill(g.W2, nW, s)) != hipSuccess) return e;
        return zero_fill(g.b2, (size_t)c.E * ds, s);
    }
    const BackwardPlan P = backward_plan(c);
    char *ws = (char *)workspace;
    RouteVariant v = v_in;
    v.capg = nullptr;
    if (v.cap_alpha != 0.f) {
        unsigned long long *sums = (unsigned long long *)(ws + P.cap);
        float *capg = (float *)(sums + c.E);
        if ((e = zero_fill((float *)sums, 2 * (size_t)c.E, s)) != hipSuccess) return e;
        long long blocks = (Na + 256 * 16 - 1) / (256 * 16);
        if (blocks > 1024) blocks = 1024;
        bwd_cap_sums_kernel<<<(unsigned)blocks, 256, (size_t)c.E * sizeof(unsigned long long), s>>>(idx, pk, Na, c.E, sums);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        bwd_cap_coeff_kernel<<<1, 256, 0, s>>>(sums, c.E, v.cap_alpha, capg);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        v.capg = capg;
    }
    float *dxrow = (float *)(ws + P.dxrow), *dpk = (float *)(ws + P.dpk);
    float *epart = (float *)(ws + P.expert_part), *rpart = (float *)(ws + P.router_part);

    const int hidden_groups = (c.He + kBwdThreads - 1) / kBwdThreads;
    const int col_chunks = (ds + kBwdCols - 1) / kBwdCols;
    const size_t eslot = expert_slot_floats(ds, c.He);
    std::unique_lock<std::mutex> side_lock(g_side_mutex, std::defer_lock);
    SideStream side = {};
    SideJoin joiner;
    hipStream_t se = s;   // stream of the expert weight gradients and their reduction
    if (backward_mfma_shape(c) && (c.flags & SLICEMOE_FLAG_SINGLE_STREAM)) {
        e = launch_backward_expert_mfma(c, h, w, d_out, pk, offsets, perm, ws + P.packed, P.rows_per_chunk, P.chunks, eslot,
                                        dxrow, dpk, epart, s);
        if (e != hipSuccess) return e;
    } else if (backward_mfma_shape(c)) {
        side_lock.lock();
        if ((e = side_stream(&side)) != hipSuccess) return e;
        e = launch_backward_expert_mfma(c, h, w, d_out, pk, offsets, perm, ws + P.packed, P.rows_per_chunk, P.chunks, eslot,
                                        dxrow, dpk, epart, s, &side);
        joiner.side = &side;   // from here on the side stream holds work of this call: joined on every way out
        joiner.s = s;
        se = side.stream;
        if (e != hipSuccess) return e;
    } else {
    const size_t dsp = (size_t)(ds + kBwdCols - 1) / kBwdCols * kBwdCols;
    const size_t lds_e = sizeof(float) * (2 * (size_t)kBwdRB * dsp + (size_t)kBwdRB * kBwdThreads);
    const size_t lds_ew = lds_e + sizeof(T) * ((size_t)ds * (kBwdThreads + kWPad<T>) + (size_t)kBwdThreads * (ds + kWPad<T>));
    const dim3 egrid((unsigned)P.chunks, 1, col_chunks);   // the hidden groups are a loop inside the block
    if (lds_ew <= (size_t)max_lds_per_block()) {
        auto kern = bwd_expert_kernel<T, true>;
        if ((e = grant_dynamic_lds((const void *)kern, lds_ew)) != hipSuccess)
            return e;
        kern<<<egrid, kBwdThreads, lds_ew, s>>>((const T *)h, (const T *)d_out, pk, offsets, perm, ds, c.He, c.E, c.k,
                                                 (const T *)w.W1, (const T *)w.b1, (const T *)w.W2, dxrow, dpk,
                                                 P.rows_per_chunk, hidden_groups, epart);
    } else {
        bwd_expert_kernel<T, false><<<egrid, kBwdThreads, lds_e, s>>>(
            (const T *)h, (const T *)d_out, pk, offsets, perm, ds, c.He, c.E, c.k, (const T *)w.W1, (const T *)w.b1,
            (const T *)w.W2, dxrow, dpk, P.rows_per_chunk, hidden_groups, epart);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const bool vec4 = ds % 4 == 0 && c.He % 4 == 0 &&
                      (((uintptr_t)g.W1 | (uintptr_t)g.b1 | (uintptr_t)g.W2 | (uintptr_t)g.b2 | (uintptr_t)epart) & 15) == 0;
    if (vec4)
        bwd_reduce_expert_kernel<4><<<dim3((unsigned)c.E, (unsigned)((eslot / 4 + kRedElems - 1) / kRedElems)), kRedElems * kRedSeqs, 0, se>>>(
            epart, offsets, ds, c.He, c.E, P.rows_per_chunk, g.W1, g.b1, g.W2, g.b2);
    else
        bwd_reduce_expert_kernel<1><<<dim3((unsigned)c.E, (unsigned)((eslot + kRedElems - 1) / kRedElems)), kRedElems * kRedSeqs, 0, se>>>(
            epart, offsets, ds, c.He, c.E, P.rows_per_chunk, g.W1, g.b1, g.W2, g.b2);
    if ((e = hipGetLastError()) != hipSuccess) return e;

    const size_t rslot = router_slot_floats(ds, c.Hr, c.E);
    if (backward_router_mfma_shape(c)) {
        e = launch_backward_router_mfma(c, h, w, v, drop_u, rate, idx, inv, dpk, dxrow, d_h, ws + P.router_scratch,
                                        P.slices_per_block, P.slice_blocks, rslot, rpart, s);
        if (e != hipSuccess) return e;
    } else {
    const size_t lds_r = sizeof(float) * kBwdRB * ((size_t)ds + 2 * (size_t)c.Hr + 2 * (size_t)c.E);
    const size_t lds_rw = lds_r + sizeof(T) * ((size_t)ds * (c.Hr + kWPad<T>) + (size_t)c.Hr * (c.E + kWPad<T>));
    const dim3 rgrid((unsigned)P.slice_blocks, col_chunks);
    const float *nz = v.sigma > 0.f ? v.noise : nullptr, *du = rate > 0.f ? drop_u : nullptr;
    if (lds_rw <= (size_t)max_lds_per_block()) {
        auto kern = bwd_router_kernel<T, true>;
        if ((e = grant_dynamic_lds((const void *)kern, lds_rw)) != hipSuccess)
            return e;
        kern<<<rgrid, kBwdThreads, lds_rw, s>>>((const T *)h, Ns, ds, c.Hr, c.E, c.k, (const T *)w.Wr1, (const T *)w.br1,
                                                 (const T *)w.Wr2, (const T *)w.br2, nz, v.sigma, v.inv_tau, du, rate, idx, inv,
                                                 dpk, v.capg, dxrow, (T *)d_h, P.slices_per_block, rpart);
    } else {
        bwd_router_kernel<T, false><<<rgrid, kBwdThreads, lds_r, s>>>(
            (const T *)h, Ns, ds, c.Hr, c.E, c.k, (const T *)w.Wr1, (const T *)w.br1, (const T *)w.Wr2, (const T *)w.br2,
            nz, v.sigma, v.inv_tau, du, rate, idx, inv, dpk, v.capg, dxrow, (T *)d_h, P.slices_per_block, rpart);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    bwd_reduce_router_kernel<<<(unsigned)((rslot + kRedElems - 1) / kRedElems), kRedElems * kRedSeqs, 0, s>>>(rpart, (int)P.slice_blocks, ds, c.Hr, c.E, g.Wr1,
                                                                           g.br1, g.Wr2, g.br2);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    return joiner.join();
}

hipError_t launch_backward(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const RouteVariant &v,
                           const float *drop_u, float rate, const int32_t *idx, const float *pk, const int32_t *offsets,
                           const int32_t *perm, const int32_t *inv, const void *d_out, void *d_h,
                           const slicemoe_weight_grads &g, void *workspace, hipStream_t s)
{
    if (c.dtype == SLICEMOE_BF16)
        return run_backward<bf16_t>(c, h, w, v, drop_u, rate, idx, pk, offsets, perm, inv, d_out, d_h, g, workspace, s);
    return run_backward<float>(c, h, w, v, drop_u, rate, idx, pk, offsets, perm, inv, d_out, d_h, g, workspace, s);
}

}  // namespace slicemoe
