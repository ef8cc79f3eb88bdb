// Shared declarations of the SliceMoE HIP library: launch prototypes (host side) and small
// device helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/slicemoe.h"

namespace slicemoe {

typedef unsigned short bf16_t;  // storage bit pattern of a bfloat16

// Element size of the stacked expert outputs y: fp32 with fp32 storage, fp16 with bf16 storage.
__host__ __device__ __forceinline__ size_t y_elem_bytes(int dtype) { return dtype == SLICEMOE_BF16 ? 2 : 4; }

// ---- device helpers -------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even conversion (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    __bf16 v = (__bf16)f;
    return __builtin_bit_cast(bf16_t, v);
}

template <typename T> struct Storage;
template <> struct Storage<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Storage<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

__host__ __device__ __forceinline__ size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Block-wide copy of n_pieces 16-byte pieces from global memory to LDS through registers, in rounds of
// ROUND (4 or 8) pieces per thread: the loads of a round are all in flight before its first LDS write, so
// a round costs one memory round trip.  (The direct global->LDS path moves only 16 bytes per cycle and CU.)
// Callers synchronise before reading the copy.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <int THREADS, int ROUND = 4>
__device__ __forceinline__ void stage_to_lds(const void *__restrict__ src, void *dst, int n_pieces, int tid)
{
    static_assert(ROUND == 4 || ROUND == 8, "rounds of 4 or 8 pieces");
    const u32x4 *g = (const u32x4 *)src;
    u32x4 *l = (u32x4 *)dst;
    for (int base = 0; base < n_pieces; base += ROUND * THREADS) {
        u32x4 t[ROUND];
#pragma unroll
        for (int i = 0; i < ROUND; ++i) {
            const int idx = base + tid + i * THREADS;
            t[i] = g[idx < n_pieces ? idx : 0];
        }
        // every piece of the round is requested before any is used
        if constexpr (ROUND == 4) asm volatile("" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]));
        else asm volatile("" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(t[4]), "+v"(t[5]), "+v"(t[6]), "+v"(t[7]));
#pragma unroll
        for (int i = 0; i < ROUND; ++i) {
            const int idx = base + tid + i * THREADS;
            if (idx < n_pieces) l[idx] = t[i];
        }
    }
}

// ---- packed-weight buffer layout (bf16 MFMA path) -------------------------------------
// All offsets in bytes from the start of the packed buffer; every region 256-byte aligned.
struct PackedLayout {
    int ds, Hr, He, E, Epad;     // Epad = E rounded up to a multiple of 32
    int dsK, dsN;                // ds rounded up to whole K-steps (16) and whole output tiles (32); padding is zeros
    size_t r_w1, r_w2, r_b1, r_b2;  // router: Wr1 frags, Wr2 frags, br1 (f32), br2 (f32, Epad)
    size_t experts;                 // start of expert 0
    size_t e_w1, e_w2, e_b1, e_b2;  // offsets inside one expert block: W1 frags (bf16, times kappa), W2 frags (fp16, times 1/kappa),
                                    // b1 (fp16, times kappa, accumulator order per hidden tile), b2 (f32)
    size_t e_stride;                // bytes per expert
    size_t total;
};
PackedLayout packed_layout(const slicemoe_config &cfg);

// ---- dispatch geometry ----------------------------------------------------------------
// The assignment ids are cut into chunks, and the per-chunk histogram is a table of E rows (one per expert, contiguous)
// of `stride` entries (the number of chunks rounded up to a multiple of 8: rows are read in 16-byte pieces).  A small
// table (`fused`) holds 16-bit raw counts and is summed by the scatter blocks themselves; a large one holds int32 and
// is turned into prefixes by a kernel of its own.  A scatter block of kDispThreads threads covers `group` consecutive
// chunks, in rounds of kDispThreads ids, at most kDispMaxItems of them.
constexpr int kDispThreads = 256;
constexpr int kDispMaxItems = 16;
struct DispatchGeom {
    int chunk;     // assignments per chunk of the table
    int nchunks;
    int stride;
    bool fused;
    int group;     // chunks per scatter block
    int blocks;    // scatter blocks
};
// chunk = 0: the dispatch stage's own choice; > 0: a histogram somebody else produces in chunks of that size
DispatchGeom dispatch_geometry(long long Na, int E, int chunk);
size_t dispatch_table_bytes(const DispatchGeom &g, int E);
// Where the matrix-core router can leave the per-chunk histogram of its selections behind: the table it writes
// (layout and entry width as dispatch_geometry(Na, E, chunk) says, chunks of route_mfma_hist_chunk(c) assignments); 0
// when it cannot for this shape.
int route_mfma_hist_chunk(const slicemoe_config &c);

// ---- kernel launchers (each only enqueues; returns hipGetLastError) --------------------
// Training-time variations of the router (softmax temperature: Appendix B; Gaussian logit noise: Section 5); the
// defaults are the inference router.
struct RouteVariant {
    float inv_tau = 1.f;             // softmax of g / tau
    float sigma = 0.f;               // g += sigma * noise[n, e] before the selection and the softmax
    const float *noise = nullptr;    // [Ns, E] standard-normal draws; read only when sigma > 0
    // backward only: weight of the capacity loss's differentiable reading (0: none), and, once the backward has
    // computed it, the device table [E] of its derivatives with respect to each expert's probability sum
    float cap_alpha = 0.f;
    const float *capg = nullptr;
};
hipError_t launch_route_generic(const slicemoe_config &c, const void *h, const slicemoe_weights &w,
                                int32_t *idx, float *p, hipStream_t s, const RouteVariant &v = RouteVariant());
hipError_t launch_route_mfma(const slicemoe_config &c, const void *h, const void *packed,
                             int32_t *idx, float *p, hipStream_t s, const RouteVariant &v = RouteVariant(),
                             int32_t *hist_table = nullptr /* see route_mfma_hist_chunk */);
// Backward pass (backward.hip): weight gradients into g, dL/dh into d_h.  backward_plan: geometry and layout of its
// scratch (row gradients, dL/dp, one slot of partial weight gradients per block); backward_lds_bytes: dynamic LDS its
// kernels ask for at least.
struct BackwardPlan {
    int rows_per_chunk;            // stacked rows per block of the expert kernel
    long long chunks;              // its grid.x (an upper bound on the chunks in use)
    int slices_per_block;          // slices per block of the router kernel (its slot of partial weight gradients)
    long long slice_blocks;        // grid.x of the router kernel
    size_t dxrow, dpk, expert_part, router_part, packed, router_scratch, cap, total;   // byte offsets into the workspace, total size
};
BackwardPlan backward_plan(const slicemoe_config &c);
// Matrix-core expert backward (backward_mfma.hip): shapes it takes, bytes of its repacked weights, and the launch
// (same outputs as the vector-ALU expert kernel: row gradients, dL/dp, one slot of partial weight gradients per chunk).
bool backward_mfma_shape(const slicemoe_config &c);
size_t backward_mfma_packed_bytes(const slicemoe_config &c);
// Matrix-core router backward (backward_router_mfma.hip): shapes it takes, bytes of its scratch (repacked router and
// the dL/dg tables), and the launch (same outputs as the vector-ALU router kernel: dL/dh and one slot of partial
// weight gradients per range of slices_per_block slices).
bool backward_router_mfma_shape(const slicemoe_config &c);
size_t backward_router_mfma_scratch_bytes(const slicemoe_config &c);
hipError_t launch_backward_router_mfma(const slicemoe_config &c, const void *h, const slicemoe_weights &w,
                                       const RouteVariant &v, const float *drop_u, float rate, const int32_t *idx,
                                       const int32_t *inv, const float *dpk, const float *dxrow, void *d_h, void *scratch,
                                       int slices_per_block, long long slice_blocks, size_t slot_floats, float *part,
                                       hipStream_t s);
// side (optional): a second stream with a fork event.  The weight-gradient kernel is then launched on side->stream, ordered
// after the repacking on s by the event; the caller joins the stream back before anything reads `part`.
struct SideStream {
    hipStream_t stream;
    hipEvent_t fork, join;
};
hipError_t launch_backward_expert_mfma(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const void *d_out,
                                       const float *pk, const int32_t *offsets, const int32_t *perm, void *packed,
                                       int rows_per_chunk, long long chunks, size_t slot_floats, float *dxrow, float *dpk,
                                       float *part, hipStream_t s, const SideStream *side = nullptr);
size_t backward_lds_bytes(const slicemoe_config &c);
hipError_t launch_backward(const slicemoe_config &c, const void *h, const slicemoe_weights &w, const RouteVariant &v,
                           const float *drop_u, float rate, const int32_t *idx, const float *pk, const int32_t *offsets,
                           const int32_t *perm, const int32_t *inv, const void *d_out, void *d_h,
                           const slicemoe_weight_grads &g, void *workspace, hipStream_t s);
// Cross-slice dropout (Section 3.3) on the selected probabilities p[Ns, k], in place.
hipError_t launch_route_dropout(const slicemoe_config &c, float *p, const float *drop_u, float rate, hipStream_t s);
hipError_t launch_dispatch(const slicemoe_config &c, const int32_t *idx, int32_t *counts_raw,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                           int32_t *table, float *stats /* nullable */, hipStream_t s,
                           int table_chunk = 0 /* > 0: table already holds the histogram, in chunks of this size */);
// The same dispatch with its table in the library's own fixed device array (for callers that cannot allocate);
// dispatch_static_fits: whether the table of this config fits that array.
bool dispatch_static_fits(const slicemoe_config &c);
hipError_t launch_dispatch_static(const slicemoe_config &c, const int32_t *idx, int32_t *counts_raw, int32_t *counts,
                                  int32_t *offsets, int32_t *perm, int32_t *inv, hipStream_t s);
hipError_t launch_ffn_generic(const slicemoe_config &c, const void *h, const float *p,
                              const int32_t *offsets, const int32_t *perm, const slicemoe_weights &w,
                              void *y, hipStream_t s);
hipError_t launch_ffn_mfma(const slicemoe_config &c, const void *h, const float *p,
                           const int32_t *offsets, const int32_t *perm, const void *packed,
                           void *y, hipStream_t s);
hipError_t launch_combine(const slicemoe_config &c, const void *y, const int32_t *inv, void *h_out,
                          hipStream_t s);
hipError_t launch_load_stats(const slicemoe_config &c, const int32_t *counts_raw, const int32_t *counts,
                             float *stats, hipStream_t s);
hipError_t launch_pack(const slicemoe_config &c, const slicemoe_weights &w, void *packed, hipStream_t s);

int num_compute_units();
// Allows `kern` (a __global__ function) `bytes` of dynamic LDS on the current device.  The attribute sticks to the
// kernel, so the driver is asked only the first time a (kernel, device) pair needs that much; later launches pay a
// table lookup.
hipError_t grant_dynamic_lds(const void *kern, size_t bytes);
int max_lds_per_block();  // bytes of LDS one workgroup may use on the current device

}  // namespace slicemoe
