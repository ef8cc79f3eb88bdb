// Fused slice router on the matrix cores (paper Section 3.1): per slice
//   u = ReLU(x Wr1 + br1)  (Hr = 256),  g = u Wr2 + br2,  p = softmax(g),  top-k of g.
// bf16 inputs, fp32 accumulation, logits good to fp32 rounding so that the selected experts
// agree with a reference except on near-ties:
//   GEMM1  bf16 x bf16 products are exact in fp32, accumulated in fp32 (bias preloaded into
//          the accumulators).
//   GEMM2  u stays fp32-grade.  It is split into two fp16 terms u = u0 + u1 + (< 2^-22 u), u0 the
//          round-toward-zero fp16 of u and u1 the fp16 of the exact remainder u - u0 (one mixed-precision
//          multiply-add), and the fp16 MFMA is issued once per term against the fp16 copy of the
//          bf16 weights: 22 significant bits per hidden activation, below the rounding of the fp32
//          accumulation itself, instead of a slow fp32 matrix instruction.  Pairs of activations are
//          converted by one packed instruction, which directly yields the B operand of GEMM2.
//          Range: a hidden activation of 2048 or more keeps u0 and a remainder cut off at 1 (fp16-grade
//          instead of fp32-grade for that unit); beyond 65504 u0 itself saturates.
// Both GEMMs run transposed (see mfma.h): a lane owns one slice and, per 32-expert tile, 16 of
// its logits; the other 16 sit in lane ^ 32.  Softmax and top-k therefore need only registers
// and one cross-lane exchange per step.  A block keeps the whole router (<= 100 KiB packed) in
// LDS and walks slice tiles of 32 per wavefront.
//
// The tiles are handed out in chunks: in round r block b takes chunk c = r * gridDim + b, and its W wavefronts the W
// consecutive tiles of that chunk, i.e. W * 32 * k consecutive assignment ids.  That makes the per-chunk histogram of
// the selected experts -- the first step of the dispatch stage -- a by-product: every wavefront adds its selections to
// a small LDS table of the round, and the wavefront of the chunk that finishes last (an LDS counter tells it; nobody
// waits) writes the chunk's counts to the dispatch table.
#include "mfma.h"

namespace slicemoe {

constexpr int kRouteHr = 256;
constexpr int kRouteHT = kRouteHr / 32;
constexpr int kRouteHistMaxRounds = 32;   // LDS slots for the per-round histograms (65 ints each)

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

// ReLU and the two-term fp16 split of a pair of hidden activations, four instructions: the round-toward-zero conversion
// of the pair; ReLU of both halves as a packed signed-integer max (negative halves are negative integers); and per
// activation one mixed-precision multiply-add a - u0 that rounds to fp16 and clamps to [0, 1].  The clamp is the ReLU of
// the small term (a < 0 has u0 = 0, so a - u0 = a < 0 becomes 0) and leaves a remainder untouched as long as it is
// below 1, i.e. for activations below 2048.
__device__ __forceinline__ void relu_split_pair(float a0, float a1, uint32_t &u0, uint32_t &u1)
{
    const s16x2 raw = __builtin_bit_cast(s16x2, __builtin_amdgcn_cvt_pkrtz(a0, a1));
    const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(raw, s16x2{0, 0}));
    uint32_t lo;
    asm("v_fma_mixlo_f16 %0, %1, -1.0, %2 op_sel_hi:[1,0,0] clamp" : "=v"(lo) : "v"(hi), "v"(a0));
    asm("v_fma_mixhi_f16 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0] clamp" : "+v"(lo) : "v"(hi), "v"(a1));
    u0 = hi;
    u1 = lo;
}

__device__ __forceinline__ f32x16 load_bias_tile(const float *__restrict__ b, int tile, int g)
{
    f32x16 r;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const f32x4 v = *(const f32x4 *)(b + tile * 32 + 8 * q + 4 * g);
#pragma unroll
        for (int c = 0; c < 4; ++c) r[4 * q + c] = v[c];
    }
    return r;
}

// One block per CU shares one LDS copy of the router, with as many wavefronts as the registers allow: a wavefront's
// chain  GEMM1 -> ReLU/split -> GEMM2  is serial, so only other wavefronts fill the matrix pipe while it does vector work or
// waits for the LDS.  THREADS = 1024 (16 wavefronts, <= 128 VGPRs) for the small shapes, 768 (<= 168) where two expert
// tiles or a wide slice need more, 512 where that would spill.  (Measured alternatives that did not pay on the
// T=16384, d=1024, S=16, E=32 workload: eight wavefronts with two tiles each, plain or software-pipelined so that every
// matrix instruction is followed by one pair's vector work of another stage -- 28.4 and 29.0 us against 27.8.)
// W1_LDS = false (slice width 384, whose first layer of 192 KiB exceeds the LDS): the first-layer fragments are read
// from memory as they are used; only the second layer and the biases are staged.
template <int DS, int ET, int THREADS, bool W1_LDS>
__global__ __launch_bounds__(THREADS) void route_mfma_kernel(
    const bf16_t *__restrict__ x, long long Ns, int E, int k, const char *__restrict__ packed,
    size_t off_w1, size_t off_b1, size_t off_b2, const float *__restrict__ noise, float sigma, float exp_scale,
    int32_t *__restrict__ idx, float *__restrict__ pk, void *__restrict__ hist /* may be null */, int hist_stride,
    int hist_rounds, bool hist_narrow)
{
    constexpr int KS = SliceTiles<DS>::KS;
    constexpr int HT = kRouteHT;
    constexpr int kRouteWaves = THREADS / 64;
    constexpr int kChunkTiles = kRouteWaves;   // tiles of a chunk, one per wavefront
    extern __shared__ __align__(16) char lds[];
    const uint4 *w1s = W1_LDS ? (const uint4 *)lds : (const uint4 *)(packed + off_w1);   // [HT][KS][64]
    uint4 *w2s = (uint4 *)lds + (W1_LDS ? HT * KS * 64 : 0);                             // [ET][HT][2][64]
    float *b1s = (float *)(w2s + ET * HT * 2 * 64);    // [Hr]
    float *b2s = b1s + kRouteHr;                       // [ET*32]
    int *hcnt = (int *)(b2s + ET * 32);                // [hist_rounds][64] selections per expert of this block's chunks
    int *hdone = hcnt + hist_rounds * 64;              // [hist_rounds] wavefronts that have added theirs

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31;
    const int g = lane >> 5;

    // first tile's rows are requested before the weights
    const long long ntiles = (Ns + 31) / 32;
    const long long nchunks = (ntiles + kChunkTiles - 1) / kChunkTiles;
    auto load_x = [&](long long tile, bf16x8 (&xb)[KS]) {
        const long long n = tile * 32 + j;
        const bool valid = tile < ntiles && n < Ns;
        const uint4 *xr = (const uint4 *)(x + (valid ? n : 0) * DS);   // a lane without a slice reads slice 0
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xb[ks] = load_row_piece<DS>(xr, ks, g);
    };
    bf16x8 xb[KS];
    load_x((long long)blockIdx.x * kChunkTiles + wave, xb);
    {
        // the whole router (W1 and W2 fragments are adjacent in the packed buffer) goes global -> registers -> LDS
        constexpr int kW1Pieces = HT * KS * 64;
        constexpr int kPieces = (W1_LDS ? kW1Pieces : 0) + ET * HT * 2 * 64;
        const float *gb1 = (const float *)(packed + off_b1);
        const float *gb2 = (const float *)(packed + off_b2);
        const float bv1 = gb1[tid < kRouteHr ? tid : 0];
        const float bv2 = gb2[tid < ET * 32 ? tid : 0];
        stage_to_lds<THREADS>(packed + off_w1 + (W1_LDS ? 0 : (size_t)kW1Pieces * 16), lds, kPieces, tid);
        if (tid < kRouteHr) b1s[tid] = bv1;
        if (tid < ET * 32) b2s[tid] = bv2;
        if (hist != nullptr)
            for (int i = tid; i < hist_rounds * 65; i += THREADS) hcnt[i] = 0;
    }
    __syncthreads();

    int round = 0;
    for (long long chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x, ++round) {
        const long long tile = chunk * kChunkTiles + wave;
        if (tile >= ntiles) break;   // only in the last chunk; this wavefront has no later tile either
        {   // fewer tiles left -> lower priority, so the wavefronts of a block finish together
            const long long left = (nchunks - 1 - chunk) / gridDim.x;
            if (left >= 3) __builtin_amdgcn_s_setprio(3);
            else if (left == 2) __builtin_amdgcn_s_setprio(2);
            else if (left == 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        bf16x8 xn[KS];
        load_x(tile + (long long)gridDim.x * kChunkTiles, xn);   // next tile, consumed after this one
        f32x16 gacc[ET];   // logit accumulators start from the second-layer bias
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 b = *(const f32x4 *)(b2s + et * 32 + 8 * q + 4 * g);
#pragma unroll
                for (int c = 0; c < 4; ++c) gacc[et][4 * q + c] = b[c];
            }

#pragma unroll 1
        for (int ht = 0; ht < HT; ++ht) {
            // GEMM1 with the bias as the first accumulator input
            f32x16 acc = load_bias_tile(b1s, ht, g);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = mfma_bf16(__builtin_bit_cast(bf16x8, w1s[(ht * KS + ks) * 64 + lane]), xb[ks], acc);
            uint32_t t0[8], t1[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) relu_split_pair(acc[2 * i], acc[2 * i + 1], t0[i], t1[i]);
            // GEMM2: two passes per K-step, small term first
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const f16x8 u0 = __builtin_bit_cast(f16x8, make_uint4(t0[4 * s], t0[4 * s + 1], t0[4 * s + 2], t0[4 * s + 3]));
                const f16x8 u1 = __builtin_bit_cast(f16x8, make_uint4(t1[4 * s], t1[4 * s + 1], t1[4 * s + 2], t1[4 * s + 3]));
#pragma unroll
                for (int et = 0; et < ET; ++et) {
                    const f16x8 a2 = __builtin_bit_cast(f16x8, w2s[((et * HT + ht) * 2 + s) * 64 + lane]);
                    gacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, u1, gacc[et], 0, 0, 0);
                    gacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, u0, gacc[et], 0, 0, 0);
                }
            }
        }

        const long long n = tile * 32 + j;
        const bool valid = n < Ns;
        // ---- logits of this lane: expert 32*et + 8*(r/4) + 4*g + r%4, ascending in (et, r)
        float v[ET * 16];
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int r = 0; r < 16; ++r) v[et * 16 + r] = gacc[et][r];
        if (noise != nullptr) {   // training-time logit noise: g += sigma * draw, before the selection and the softmax
            const float *nr = noise + (valid ? n : 0) * E;
            if ((E & 3) == 0) {   // rows of the table are 16-byte aligned: this lane's four consecutive experts at once
#pragma unroll
                for (int et = 0; et < ET; ++et)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int e0 = et * 32 + 8 * q + 4 * g;
                        if (e0 < E) {
                            const f32x4 z = *(const f32x4 *)(nr + e0);
#pragma unroll
                            for (int c = 0; c < 4; ++c) v[et * 16 + 4 * q + c] = fmaf(sigma, z[c], v[et * 16 + 4 * q + c]);
                        }
                    }
            } else {
#pragma unroll
                for (int et = 0; et < ET; ++et)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int e = et * 32 + acc_feature(r, g);
                        if (e < E) v[et * 16 + r] = fmaf(sigma, nr[e], v[et * 16 + r]);
                    }
            }
        }
        if (E != ET * 32) {   // padded experts never win
#pragma unroll
            for (int et = 0; et < ET; ++et)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (et * 32 + acc_feature(r, g) >= E) v[et * 16 + r] = -INFINITY;
        }
        // Largest and second-largest logit of the lane (the median of the running pair and a new value is the new
        // second), then of the slice: lanes j and j + 32 trade values with one swap instruction whose two results are
        // {own, other} in an order that max / min / + do not care about.
        // (the maximum as a median with +infinity: the median instruction takes its operands as they are, while a
        // floating-point maximum would first spend an instruction on quieting each of them)
        float kInf;   // (opaque to the compiler, which would otherwise turn the medians back into maxima)
        asm("v_mov_b32 %0, 0x7f800000" : "=v"(kInf));
        float m = v[0], second = -INFINITY;
#pragma unroll
        for (int i = 1; i < ET * 16; ++i) {
            second = __builtin_amdgcn_fmed3f(m, second, v[i]);
            m = __builtin_amdgcn_fmed3f(m, v[i], kInf);
        }
        {
            const auto sm = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
            const auto ss = __builtin_amdgcn_permlane32_swap(__float_as_uint(second), __float_as_uint(second), false, false);
            const float m0 = __uint_as_float(sm[0]), m1 = __uint_as_float(sm[1]);
            m = __builtin_amdgcn_fmed3f(m0, m1, kInf);
            const float lower = __builtin_amdgcn_fmed3f(m0, m1, -kInf);   // the smaller of the two maxima (the negation is an operand modifier)
            second = __builtin_amdgcn_fmed3f(__builtin_amdgcn_fmed3f(__uint_as_float(ss[0]), __uint_as_float(ss[1]), kInf), lower, kInf);
        }
        // softmax denominator: exp((v - m) / tau) = exp2(v * c - m * c) with c = log2(e) / tau, one multiply-add and
        // one exp2 per logit
        const float kLog2e = exp_scale;
        const float nm = -m * kLog2e;
        float den = 0.f;
#pragma unroll
        for (int i = 0; i < ET * 16; ++i) den += __builtin_amdgcn_exp2f(fmaf(v[i], kLog2e, nm));
        {
            const auto sd = __builtin_amdgcn_permlane32_swap(__float_as_uint(den), __float_as_uint(den), false, false);
            den = __uint_as_float(sd[0]) + __uint_as_float(sd[1]);
        }
        const float rden = __builtin_amdgcn_rcpf(den);   // within one unit in the last place, like the exp2 above

        // k = 2 with distinct top values (wavefront-wide; anything else takes the general selection below): the two
        // experts are where the two values sit, the lowest index among equals of the second value
        bool picked = false;
        if (k == 2 && __builtin_amdgcn_ballot_w64(!(m > second)) == 0) {
            constexpr int kNone = 1 << 20;
            int ia = kNone, ib = kNone;
#pragma unroll
            for (int i = ET * 16 - 1; i >= 0; --i) {
                const int e0 = (i >> 4) * 32 + acc_feature(i & 15, 0);   // + 4 g below: constants here
                ia = v[i] == m ? e0 : ia;
                ib = v[i] == second ? e0 : ib;
            }
            ia += 4 * g;
            ib += 4 * g;
            const auto sa = __builtin_amdgcn_permlane32_swap((uint32_t)ia, (uint32_t)ia, false, false);
            const auto sb = __builtin_amdgcn_permlane32_swap((uint32_t)ib, (uint32_t)ib, false, false);
            ia = min(min((int)sa[0], (int)sa[1]), E - 1);   // the bound only matters for logits that are not numbers
            ib = min(min((int)sb[0], (int)sb[1]), E - 1);
            if (valid && g == 0) {
                idx[n * 2] = ia;
                idx[n * 2 + 1] = ib;
                pk[n * 2] = __builtin_amdgcn_exp2f(fmaf(m, kLog2e, nm)) * rden;
                pk[n * 2 + 1] = __builtin_amdgcn_exp2f(fmaf(second, kLog2e, nm)) * rden;
                if (hist != nullptr) {
                    atomicAdd(&hcnt[round * 64 + ia], 1);
                    atomicAdd(&hcnt[round * 64 + ib], 1);
                }
            }
            picked = true;
        }

        for (int jj = 0; jj < (picked ? 0 : k); ++jj) {
            float bv = v[0];
            int be = acc_feature(0, g);
#pragma unroll
            for (int i = 1; i < ET * 16; ++i) {
                const int e = (i >> 4) * 32 + acc_feature(i & 15, g);
                if (v[i] > bv) {
                    bv = v[i];
                    be = e;
                }
            }
            const float ov = __shfl_xor(bv, 32);
            const int oe = __shfl_xor(be, 32);
            if (ov > bv || (ov == bv && oe < be)) {
                bv = ov;
                be = oe;
            }
#pragma unroll
            for (int i = 0; i < ET * 16; ++i) {
                const int e = (i >> 4) * 32 + acc_feature(i & 15, g);
                if (e == be) v[i] = -INFINITY;
            }
            if (valid && g == 0) {
                idx[n * k + jj] = be;
                pk[n * k + jj] = __builtin_amdgcn_exp2f(fmaf(bv, kLog2e, nm)) * rden;
                if (hist != nullptr) atomicAdd(&hcnt[round * 64 + be], 1);
            }
        }
        if (hist != nullptr) {
            // The LDS executes a wavefront's operations in order, so this wavefront's additions above are in the table
            // before its ticket; the wavefront that draws the last ticket of the chunk therefore sees everybody's.
            int ticket = 0;
            if (lane == 0) ticket = __hip_atomic_fetch_add(&hdone[round], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
            ticket = __builtin_amdgcn_readfirstlane(ticket);
            const long long in_chunk = min((long long)kRouteWaves, ntiles - chunk * kChunkTiles);
            if (ticket == in_chunk - 1 && lane < E) {
                const int cnt = __hip_atomic_load(&hcnt[round * 64 + lane], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (hist_narrow) {
                    uint16_t *row = (uint16_t *)hist + (size_t)lane * hist_stride;
                    row[chunk] = (uint16_t)cnt;
                    if (chunk == nchunks - 1)   // the padding of a row of 16-bit counts reads as zero
                        for (long long c = nchunks; c < hist_stride; ++c) row[c] = 0;
                } else {
                    ((int32_t *)hist)[(size_t)lane * hist_stride + chunk] = cnt;
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xb[ks] = xn[ks];
    }
}

// Threads per block of the instantiation that serves a slice width and a number of 32-expert tiles (see the kernel).
static int route_threads(int ds, int et)
{
    switch (ds) {
        case 24: case 48: case 64: return et == 1 ? 1024 : 512;
        case 96: return et == 1 ? 1024 : 768;
        case 192: return et == 1 ? 768 : 512;
        case 384: return 256;
        default: return 768;   // 128
    }
}

static long long route_blocks(long long Ns, int chunk_tiles)
{
    const long long ntiles = (Ns + 31) / 32;
    const long long nchunks = (ntiles + chunk_tiles - 1) / chunk_tiles;
    const long long cap = (long long)num_compute_units();
    return nchunks < cap ? nchunks : cap;
}

// Assignments per chunk of the histogram this router can leave behind, or 0: the chunk must be worth a dispatch block
// (at least 512 assignments, at most kDispMaxItems rounds of it) and a block's rounds must fit the LDS slots.
int route_mfma_hist_chunk(const slicemoe_config &c)
{
    const long long Ns = (long long)c.T * c.S;
    if (Ns == 0) return 0;
    const int ds = c.d / c.S, et = (c.E + 31) / 32;
    const int chunk_tiles = route_threads(ds, et) / 64;
    const int chunk = chunk_tiles * 32 * c.k;
    if (chunk < 512 || chunk > kDispThreads * kDispMaxItems) return 0;
    const long long ntiles = (Ns + 31) / 32;
    const long long nchunks = (ntiles + chunk_tiles - 1) / chunk_tiles, blocks = route_blocks(Ns, chunk_tiles);
    if ((nchunks + blocks - 1) / blocks > kRouteHistMaxRounds) return 0;
    return chunk;
}

template <int DS, int ET, int THREADS, bool W1_LDS = true>
static hipError_t run_route(const slicemoe_config &c, const void *h, const void *packed, int32_t *idx, float *p,
                            hipStream_t s, const RouteVariant &v, int32_t *hist)
{
    const PackedLayout L = packed_layout(c);
    const long long Ns = (long long)c.T * c.S;
    constexpr int KS = SliceTiles<DS>::KS;
    constexpr int kChunkTiles = THREADS / 64;
    if (route_threads(DS, ET) != THREADS) return hipErrorInvalidValue;
    const long long blocks = route_blocks(Ns, kChunkTiles);
    const long long nchunks = ((Ns + 31) / 32 + kChunkTiles - 1) / kChunkTiles;
    int hist_rounds = 0, hist_stride = 0;
    bool hist_narrow = false;
    if (hist != nullptr) {
        const int chunk = route_mfma_hist_chunk(c);
        if (chunk != kChunkTiles * 32 * c.k) return hipErrorInvalidValue;
        const DispatchGeom g = dispatch_geometry(Ns * c.k, c.E, chunk);
        if (g.nchunks != nchunks) return hipErrorInvalidValue;
        hist_rounds = (int)((nchunks + blocks - 1) / blocks);
        hist_stride = g.stride;
        hist_narrow = g.fused;
    }
    const size_t lds = (size_t)((W1_LDS ? kRouteHT * KS * 64 : 0) + ET * kRouteHT * 2 * 64) * 16 + (kRouteHr + ET * 32) * 4 +
                       (size_t)hist_rounds * 65 * 4;
    auto kern = route_mfma_kernel<DS, ET, THREADS, W1_LDS>;
    hipError_t err = grant_dynamic_lds((const void *)kern, lds);
    if (err != hipSuccess) return err;
    if (L.r_w2 != L.r_w1 + (size_t)kRouteHT * KS * 64 * 16) return hipErrorInvalidValue;   // the kernel copies W1 | W2 as one run
    kern<<<(int)blocks, THREADS, lds, s>>>((const bf16_t *)h, Ns, c.E, c.k, (const char *)packed, L.r_w1, L.r_b1, L.r_b2,
                                           v.sigma > 0.f ? v.noise : nullptr, v.sigma, 1.4426950408889634f * v.inv_tau, idx, p,
                                           hist, hist_stride, hist_rounds, hist_narrow);
    return hipGetLastError();
}

hipError_t launch_route_mfma(const slicemoe_config &c, const void *h, const void *packed, int32_t *idx,
                             float *p, hipStream_t s, const RouteVariant &v, int32_t *hist)
{
    if ((long long)c.T * c.S == 0) return hipSuccess;
    const int ds = c.d / c.S;
    const int et = (c.E + 31) / 32;
    if (ds == 24)   // two K-steps, the second half zeros
        return et == 1 ? run_route<24, 1, 1024>(c, h, packed, idx, p, s, v, hist) : run_route<24, 2, 512>(c, h, packed, idx, p, s, v, hist);
    if (ds == 48)
        return et == 1 ? run_route<48, 1, 1024>(c, h, packed, idx, p, s, v, hist) : run_route<48, 2, 512>(c, h, packed, idx, p, s, v, hist);
    if (ds == 64)
        return et == 1 ? run_route<64, 1, 1024>(c, h, packed, idx, p, s, v, hist) : run_route<64, 2, 512>(c, h, packed, idx, p, s, v, hist);
    if (ds == 96)   // the slice width of the paper's own configuration (d = 768, S = 8): six K-steps
        return et == 1 ? run_route<96, 1, 1024>(c, h, packed, idx, p, s, v, hist) : run_route<96, 2, 768>(c, h, packed, idx, p, s, v, hist);
    if (ds == 192)
        return et == 1 ? run_route<192, 1, 768>(c, h, packed, idx, p, s, v, hist) : run_route<192, 2, 512>(c, h, packed, idx, p, s, v, hist);
    if (ds == 384)
        return et == 1 ? run_route<384, 1, 256, false>(c, h, packed, idx, p, s, v, hist) : run_route<384, 2, 256, false>(c, h, packed, idx, p, s, v, hist);
    return et == 1 ? run_route<128, 1, 768>(c, h, packed, idx, p, s, v, hist) : run_route<128, 2, 768>(c, h, packed, idx, p, s, v, hist);
}

}  // namespace slicemoe
