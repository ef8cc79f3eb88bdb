// How a SIMD of gfx950 issues matrix and vector instructions: the two facts the bounds of the expert and router kernels
// rest on.  Register-only kernels (no memory access inside the timed loops), timed with the shader's cycle counter.
//
//   law          8 x (one 32x32x16 fp16 matrix instruction + n packed fp16 FMAs on other registers), one or two
//                wavefronts per SIMD: cycles of the SIMD per matrix instruction.  Expected max(32, 12 + 4 n): a matrix
//                instruction takes 12 cycles of the SIMD's vector issue, every other vector instruction 4, and the matrix
//                pipe itself 32 cycles per instruction.
//   arbitration  two wavefronts per SIMD issuing matrix instructions only: the wavefront that arrived first runs at 32
//                cycles per instruction as if alone, the other one gets the pipe when the first has finished (its
//                elapsed time per instruction is 64).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
constexpr int kIter = 4000, kGroups = 8, kBlocks = 256;

template <int N>
__global__ __launch_bounds__(512) void issue_kernel(float *out, unsigned long long *cycles, float seed)
{
    f32x16 acc[2];
    for (int i = 0; i < 2; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = seed * (r + i);
    f16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(seed * 1e-3f * (i + 1));
        b[i] = (_Float16)(seed * 1e-3f * (i + (threadIdx.x & 7)));
    }
    h2 x[8];
    const h2 c1 = {(_Float16)0.999f, (_Float16)1.001f}, c2 = {(_Float16)1e-3f, (_Float16)-1e-3f};
    for (int i = 0; i < 8; ++i) x[i] = h2{(_Float16)(seed + i), (_Float16)(seed - i)};
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < kIter; ++it) {
#pragma unroll
        for (int m = 0; m < kGroups; ++m) {
            acc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[m & 1], 0, 0, 0);
#pragma unroll
            for (int v = 0; v < N; ++v) x[(m * N + v) & 7] = __builtin_elementwise_fma(x[(m * N + v) & 7], c1, c2);
            __builtin_amdgcn_sched_barrier(0);   // keep the interleave as written
        }
    }
    const unsigned long long t1 = __builtin_readcyclecounter();
    float s = 0.f;
    for (int i = 0; i < 2; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    for (int i = 0; i < 8; ++i) s += (float)x[i][0] + (float)x[i][1];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0) cycles[(blockIdx.x * blockDim.x + threadIdx.x) >> 6] = t1 - t0;
}

// cycles per matrix instruction: mean over the wavefronts 0..3 of a block, and over the wavefronts 4..7 (two per SIMD)
template <int N>
static void measure(int waves_per_simd, float *out, unsigned long long *cycles, double *first, double *second)
{
    const int threads = 256 * waves_per_simd, wpb = threads / 64;
    for (int rep = 0; rep < 2; ++rep) {   // the second launch is the one read
        issue_kernel<N><<<kBlocks, threads>>>(out, cycles, 0.5f);
        CK(hipGetLastError());
        CK(hipDeviceSynchronize());
    }
    std::vector<unsigned long long> h((size_t)kBlocks * wpb);
    CK(hipMemcpy(h.data(), cycles, h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    double a = 0, b = 0;
    for (int blk = 0; blk < kBlocks; ++blk)
        for (int w = 0; w < wpb; ++w) (w < 4 ? a : b) += (double)h[(size_t)blk * wpb + w];
    *first = a / (kBlocks * 4.0) / ((double)kIter * kGroups);
    *second = wpb > 4 ? b / (kBlocks * 4.0) / ((double)kIter * kGroups) : 0.0;
}

template <int N>
static void law(float *out, unsigned long long *cycles)
{
    for (int w = 1; w <= 2; ++w) {
        double first, second;
        measure<N>(w, out, cycles, &first, &second);
        // two wavefronts: the later one's elapsed time covers both wavefronts' work on the SIMD
        const double per = w == 1 ? first : second / 2.0;
        printf("law n=%d waves_per_simd=%d cycles_per_matrix_instruction=%.2f expected=%d\n", N, w, per, 12 + 4 * N > 32 ? 12 + 4 * N : 32);
    }
}

int main()
{
    float *out;
    unsigned long long *cycles;
    CK(hipMalloc(&out, (size_t)kBlocks * 512 * sizeof(float)));
    CK(hipMalloc(&cycles, (size_t)kBlocks * 8 * sizeof(unsigned long long)));
    law<0>(out, cycles);
    law<4>(out, cycles);
    law<7>(out, cycles);
    law<9>(out, cycles);
    law<12>(out, cycles);
    double first, second;
    measure<0>(2, out, cycles, &first, &second);
    printf("arbitration first_wavefront=%.2f second_wavefront=%.2f cycles elapsed per own matrix instruction\n", first, second);
    CK(hipFree(out));
    CK(hipFree(cycles));
    return 0;
}
