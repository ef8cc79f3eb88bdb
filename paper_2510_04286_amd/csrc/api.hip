// C ABI of the SliceMoE forward library: argument checks, workspace layout, kernel selection.
// Host code only; every device step lives in the kernel files.
#include <math.h>

#include <mutex>
#include <vector>

#include "common.h"

namespace slicemoe {

int num_compute_units()
{
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

int max_lds_per_block()
{
    static int lds[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 64 * 1024;
    if (lds[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || n <= 0) n = 64 * 1024;
        lds[dev] = n;
    }
    return lds[dev];
}

hipError_t grant_dynamic_lds(const void *kern, size_t bytes)
{
    struct Granted {
        const void *kern;
        int dev;
        size_t bytes;
    };
    static std::mutex mu;
    static std::vector<Granted> table;   // a few dozen kernels: a linear search
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (Granted &g : table)
        if (g.kern == kern && g.dev == dev) {
            if (g.bytes >= bytes) return hipSuccess;
            e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e == hipSuccess) g.bytes = bytes;
            return e;
        }
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) table.push_back({kern, dev, bytes});
    return e;
}

// Shapes the matrix-core kernels are instantiated for: 64 and 128 are the benchmark slice widths; 24, 48, 96 and 192
// are d = 768 cut into 32, 16, 8 and 4 slices (24 and 48 zero-padded to whole K-steps and output tiles), 384 into 2.  The expert
// hidden width is a whole number of 32-wide tiles.
static bool mfma_shape(const slicemoe_config &c)
{
    const int ds = c.d / c.S;
    const bool width = ds == 24 || ds == 48 || ds == 64 || ds == 96 || ds == 128 || ds == 192 || ds == 384;
    return c.dtype == SLICEMOE_BF16 && c.Hr == 256 && width && c.He % 32 == 0;
}

static slicemoe_status validate(const slicemoe_config *c)
{
    if (!c) return SLICEMOE_ERR_INVALID_ARG;
    if (c->T < 0 || c->d < 1 || c->S < 1 || c->k < 1 || c->E < 1 || c->Hr < 1 || c->He < 1) return SLICEMOE_ERR_INVALID_ARG;
    if (c->d % c->S != 0 || c->k > c->E) return SLICEMOE_ERR_INVALID_ARG;
    if (c->dtype != SLICEMOE_F32 && c->dtype != SLICEMOE_BF16) return SLICEMOE_ERR_INVALID_ARG;
    if (isnan(c->capacity_factor)) return SLICEMOE_ERR_INVALID_ARG;
    if (c->E > 64 || c->k > 8) return SLICEMOE_ERR_UNSUPPORTED;
    if ((long long)c->T * c->S * c->k >= (1ll << 31)) return SLICEMOE_ERR_UNSUPPORTED;
    const int ds = c->d / c->S;
    // LDS staging of the generic kernels: 8 rows x (ds + max(Hr + E, He)) floats
    const long long generic_lds = 8ll * 4 * (ds + (c->Hr + c->E > c->He ? c->Hr + c->E : c->He));
    const bool want_mfma = mfma_shape(*c) && !(c->flags & SLICEMOE_FLAG_FORCE_GENERIC);
    if (!want_mfma) {
        if (c->flags & SLICEMOE_FLAG_REQUIRE_MFMA) return SLICEMOE_ERR_UNSUPPORTED;
        if (generic_lds > 60 * 1024) return SLICEMOE_ERR_UNSUPPORTED;
    }
    return SLICEMOE_OK;
}

static bool use_mfma(const slicemoe_config &c)
{
    return mfma_shape(c) && !(c.flags & SLICEMOE_FLAG_FORCE_GENERIC);
}

PackedLayout packed_layout(const slicemoe_config &c)
{
    PackedLayout L;
    L.ds = c.d / c.S;
    L.Hr = c.Hr;
    L.He = c.He;
    L.E = c.E;
    L.Epad = (c.E + 31) / 32 * 32;
    L.dsK = (L.ds + 15) / 16 * 16;
    L.dsN = (L.ds + 31) / 32 * 32;
    size_t at = 0;
    L.r_w1 = at;  at = align_up(at + (size_t)L.dsK * L.Hr * 2, 256);
    L.r_w2 = at;  at = align_up(at + (size_t)L.Hr * L.Epad * 2, 256);
    L.r_b1 = at;  at = align_up(at + (size_t)L.Hr * 4, 256);
    L.r_b2 = at;  at = align_up(at + (size_t)L.Epad * 4, 256);
    L.experts = at;
    size_t e = 0;
    L.e_w1 = e;  e = align_up(e + (size_t)L.dsK * L.He * 2, 256);
    L.e_w2 = e;  e = align_up(e + (size_t)L.He * L.dsN * 2, 256);
    L.e_b1 = e;  e = align_up(e + (size_t)L.He * 2, 256);
    L.e_b2 = e;  e = align_up(e + (size_t)L.dsN * 4, 256);
    L.e_stride = e;
    L.total = L.experts + L.e_stride * (size_t)L.E;
    return L;
}

// Whether slicemoe_forward lets the router write the dispatch histogram, and in chunks of how many assignments.
static int forward_hist_chunk(const slicemoe_config &c) { return use_mfma(c) ? route_mfma_hist_chunk(c) : 0; }

// The per-chunk histogram table of the dispatch: large enough for the stage entry point's chunks and for the router's.
static size_t dispatch_scratch_bytes(const slicemoe_config &c)
{
    const long long Na = (long long)c.T * c.S * c.k;
    size_t bytes = dispatch_table_bytes(dispatch_geometry(Na, c.E, 0), c.E);
    const int rc = forward_hist_chunk(c);
    if (rc > 0) {
        const size_t b = dispatch_table_bytes(dispatch_geometry(Na, c.E, rc), c.E);
        bytes = b > bytes ? b : bytes;
    }
    return bytes;
}

static void make_layout(const slicemoe_config &c, slicemoe_workspace_layout *o)
{
    const size_t Na = (size_t)c.T * c.S * c.k;
    const size_t ds = (size_t)(c.d / c.S);
    size_t at = 0;
    o->topk_idx = at;   at = align_up(at + Na * 4, 256);
    o->topk_p = at;     at = align_up(at + Na * 4, 256);
    o->counts_raw = at; at = align_up(at + (size_t)c.E * 4, 256);
    o->counts = at;     at = align_up(at + (size_t)c.E * 4, 256);
    o->offsets = at;    at = align_up(at + (size_t)(c.E + 1) * 4, 256);
    o->perm = at;       at = align_up(at + Na * 4, 256);
    o->inv = at;        at = align_up(at + Na * 4, 256);
    o->y = at;          at = align_up(at + Na * ds * y_elem_bytes(c.dtype), 256);
    o->stats = at;      at = align_up(at + 4 * 4, 256);
    o->scratch = at;    at += dispatch_scratch_bytes(c);
    o->packed = at;     at = align_up(at + (use_mfma(c) ? packed_layout(c).total : 0), 256);
    o->total = at;
}

static bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

// Packed weights to use for an MFMA call: the caller's, or a fresh pack into the workspace.
static slicemoe_status resolve_packed(const slicemoe_config &c, const slicemoe_weights &w, void *workspace,
                                      size_t workspace_bytes, hipStream_t s, const void **out)
{
    if (w.packed) {
        if (misaligned(w.packed, 256)) return SLICEMOE_ERR_INVALID_ARG;
        *out = w.packed;
        return SLICEMOE_OK;
    }
    slicemoe_workspace_layout L;
    make_layout(c, &L);
    if (!workspace || workspace_bytes < L.total) return SLICEMOE_ERR_WORKSPACE;
    if (misaligned(workspace, 256)) return SLICEMOE_ERR_INVALID_ARG;
    if (!w.Wr1 || !w.br1 || !w.Wr2 || !w.br2 || !w.W1 || !w.b1 || !w.W2 || !w.b2) return SLICEMOE_ERR_INVALID_ARG;
    void *dst = (char *)workspace + L.packed;
    if (launch_pack(c, w, dst, s) != hipSuccess) return SLICEMOE_ERR_HIP;
    *out = dst;
    return SLICEMOE_OK;
}

static bool logical_weights_ok(const slicemoe_weights &w, bool router, bool experts)
{
    if (router && (!w.Wr1 || !w.br1 || !w.Wr2 || !w.br2)) return false;
    if (experts && (!w.W1 || !w.b1 || !w.W2 || !w.b2)) return false;
    return true;
}

}  // namespace slicemoe

using namespace slicemoe;

extern "C" {

const char *slicemoe_status_string(slicemoe_status s)
{
    switch (s) {
        case SLICEMOE_OK: return "ok";
        case SLICEMOE_ERR_INVALID_ARG: return "invalid argument";
        case SLICEMOE_ERR_UNSUPPORTED: return "unsupported configuration";
        case SLICEMOE_ERR_WORKSPACE: return "workspace too small";
        case SLICEMOE_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

int slicemoe_uses_mfma(const slicemoe_config *cfg)
{
    if (validate(cfg) != SLICEMOE_OK) return -1;
    return use_mfma(*cfg) ? 1 : 0;
}

int64_t slicemoe_capacity(const slicemoe_config *cfg)
{
    if (!cfg || !(cfg->capacity_factor > 0.f) || cfg->E < 1) return -1;
    const double na = (double)cfg->T * cfg->S * cfg->k;
    const double c = ceil((double)cfg->capacity_factor * na / cfg->E);
    return c > 9.0e18 ? (int64_t)9e18 : (int64_t)c;
}

size_t slicemoe_workspace_bytes(const slicemoe_config *cfg)
{
    if (validate(cfg) != SLICEMOE_OK) return 0;
    slicemoe_workspace_layout L;
    make_layout(*cfg, &L);
    return L.total;
}

size_t slicemoe_dispatch_workspace_bytes(const slicemoe_config *cfg)
{
    if (validate(cfg) != SLICEMOE_OK) return 0;
    return dispatch_scratch_bytes(*cfg);
}

slicemoe_status slicemoe_get_workspace_layout(const slicemoe_config *cfg, slicemoe_workspace_layout *out)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!out) return SLICEMOE_ERR_INVALID_ARG;
    make_layout(*cfg, out);
    return SLICEMOE_OK;
}

size_t slicemoe_packed_bytes(const slicemoe_config *cfg)
{
    if (validate(cfg) != SLICEMOE_OK || !use_mfma(*cfg)) return 0;
    return packed_layout(*cfg).total;
}

slicemoe_status slicemoe_pack_weights(const slicemoe_config *cfg, const slicemoe_weights *w, void *packed_out,
                                      size_t packed_bytes, slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!use_mfma(*cfg)) return SLICEMOE_OK;
    if (!w || !packed_out || !logical_weights_ok(*w, true, true) || misaligned(packed_out, 256)) return SLICEMOE_ERR_INVALID_ARG;
    if (packed_bytes < packed_layout(*cfg).total) return SLICEMOE_ERR_WORKSPACE;
    return launch_pack(*cfg, *w, packed_out, (hipStream_t)stream) == hipSuccess ? SLICEMOE_OK : SLICEMOE_ERR_HIP;
}

// Router variant from the caller's training parameters; INVALID_ARG when a parameter is out of range or a table of
// draws that the parameters ask for is missing or misaligned.
static slicemoe_status make_route_variant(const slicemoe_route_train_params *tp, const float *noise, const float *drop_u,
                                          RouteVariant *v)
{
    if (!tp) return SLICEMOE_ERR_INVALID_ARG;
    if (!(tp->temperature > 0.f) || isinf(tp->temperature)) return SLICEMOE_ERR_INVALID_ARG;
    if (!(tp->noise_std >= 0.f) || isinf(tp->noise_std)) return SLICEMOE_ERR_INVALID_ARG;
    if (!(tp->dropout_rate >= 0.f) || !(tp->dropout_rate < 1.f)) return SLICEMOE_ERR_INVALID_ARG;
    if (tp->noise_std > 0.f && (!noise || misaligned(noise, 16))) return SLICEMOE_ERR_INVALID_ARG;
    if (tp->dropout_rate > 0.f && !drop_u) return SLICEMOE_ERR_INVALID_ARG;
    if (!(fabsf(tp->capacity_alpha) < INFINITY)) return SLICEMOE_ERR_INVALID_ARG;   // also NaN
    v->inv_tau = 1.f / tp->temperature;
    v->sigma = tp->noise_std;
    v->noise = noise;
    v->cap_alpha = tp->capacity_alpha;
    return SLICEMOE_OK;
}

static slicemoe_status route_common(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                    const RouteVariant &v, const float *drop_u, float rate, int32_t *topk_idx,
                                    float *topk_p, void *workspace, size_t workspace_bytes, hipStream_t s)
{
    if (!w || !topk_idx || !topk_p || (!h && cfg->T > 0)) return SLICEMOE_ERR_INVALID_ARG;
    if (misaligned(h, 16)) return SLICEMOE_ERR_INVALID_ARG;
    hipError_t e;
    if (use_mfma(*cfg)) {
        const void *packed = nullptr;
        const slicemoe_status ps = resolve_packed(*cfg, *w, workspace, workspace_bytes, s, &packed);
        if (ps != SLICEMOE_OK) return ps;
        e = launch_route_mfma(*cfg, h, packed, topk_idx, topk_p, s, v);
    } else {
        if (!logical_weights_ok(*w, true, false)) return SLICEMOE_ERR_INVALID_ARG;
        e = launch_route_generic(*cfg, h, *w, topk_idx, topk_p, s, v);
    }
    if (e == hipSuccess && rate > 0.f) e = launch_route_dropout(*cfg, topk_p, drop_u, rate, s);
    return e == hipSuccess ? SLICEMOE_OK : SLICEMOE_ERR_HIP;
}

slicemoe_status slicemoe_route(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                               int32_t *topk_idx, float *topk_p, void *workspace, size_t workspace_bytes,
                               slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    return route_common(cfg, h, w, RouteVariant(), nullptr, 0.f, topk_idx, topk_p, workspace, workspace_bytes,
                        (hipStream_t)stream);
}

slicemoe_status slicemoe_route_train(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                     const slicemoe_route_train_params *params, const float *noise, const float *drop_u,
                                     int32_t *topk_idx, float *topk_p, void *workspace, size_t workspace_bytes,
                                     slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    RouteVariant v;
    const slicemoe_status vs = make_route_variant(params, noise, drop_u, &v);
    if (vs != SLICEMOE_OK) return vs;
    return route_common(cfg, h, w, v, drop_u, params->dropout_rate, topk_idx, topk_p, workspace, workspace_bytes,
                        (hipStream_t)stream);
}

slicemoe_status slicemoe_dispatch(const slicemoe_config *cfg, const int32_t *topk_idx, int32_t *counts_raw,
                                  int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv, void *workspace,
                                  size_t workspace_bytes, slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!topk_idx || !counts_raw || !counts || !offsets || !perm || !inv) return SLICEMOE_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < dispatch_scratch_bytes(*cfg)) return SLICEMOE_ERR_WORKSPACE;
    if (misaligned(workspace, 256)) return SLICEMOE_ERR_INVALID_ARG;
    return launch_dispatch(*cfg, topk_idx, counts_raw, counts, offsets, perm, inv, (int32_t *)workspace, nullptr,
                           (hipStream_t)stream) == hipSuccess
               ? SLICEMOE_OK
               : SLICEMOE_ERR_HIP;
}

slicemoe_status slicemoe_dispatch_noalloc(const slicemoe_config *cfg, const int32_t *topk_idx, int32_t *counts_raw,
                                          int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                                          slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!topk_idx || !counts_raw || !counts || !offsets || !perm || !inv) return SLICEMOE_ERR_INVALID_ARG;
    if (!dispatch_static_fits(*cfg)) return SLICEMOE_ERR_WORKSPACE;
    return launch_dispatch_static(*cfg, topk_idx, counts_raw, counts, offsets, perm, inv, (hipStream_t)stream) == hipSuccess
               ? SLICEMOE_OK
               : SLICEMOE_ERR_HIP;
}

slicemoe_status slicemoe_expert_ffn(const slicemoe_config *cfg, const void *h, const float *topk_p,
                                    const int32_t *offsets, const int32_t *perm, const slicemoe_weights *w, void *y,
                                    void *workspace, size_t workspace_bytes, slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!w || !topk_p || !offsets || !perm || !y || (!h && cfg->T > 0)) return SLICEMOE_ERR_INVALID_ARG;
    if (misaligned(h, 16) || misaligned(y, 16)) return SLICEMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (use_mfma(*cfg)) {
        const void *packed = nullptr;
        const slicemoe_status ps = resolve_packed(*cfg, *w, workspace, workspace_bytes, s, &packed);
        if (ps != SLICEMOE_OK) return ps;
        return launch_ffn_mfma(*cfg, h, topk_p, offsets, perm, packed, y, s) == hipSuccess ? SLICEMOE_OK
                                                                                            : SLICEMOE_ERR_HIP;
    }
    if (!logical_weights_ok(*w, false, true)) return SLICEMOE_ERR_INVALID_ARG;
    return launch_ffn_generic(*cfg, h, topk_p, offsets, perm, *w, y, s) == hipSuccess ? SLICEMOE_OK : SLICEMOE_ERR_HIP;
}

slicemoe_status slicemoe_combine(const slicemoe_config *cfg, const void *y, const int32_t *inv, void *h_out,
                                 slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!y || !inv || (!h_out && cfg->T > 0)) return SLICEMOE_ERR_INVALID_ARG;
    if (misaligned(y, 16) || misaligned(h_out, 16)) return SLICEMOE_ERR_INVALID_ARG;
    return launch_combine(*cfg, y, inv, h_out, (hipStream_t)stream) == hipSuccess ? SLICEMOE_OK : SLICEMOE_ERR_HIP;
}

slicemoe_status slicemoe_load_stats(const slicemoe_config *cfg, const int32_t *counts_raw, const int32_t *counts,
                                    float *stats, slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (!counts_raw || !counts || !stats) return SLICEMOE_ERR_INVALID_ARG;
    return launch_load_stats(*cfg, counts_raw, counts, stats, (hipStream_t)stream) == hipSuccess ? SLICEMOE_OK
                                                                                                 : SLICEMOE_ERR_HIP;
}

static slicemoe_status forward_common(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                      const RouteVariant &v, const float *drop_u, float rate, void *h_out,
                                      void *workspace, size_t workspace_bytes, slicemoe_stream_t stream)
{
    if (!w || ((!h || !h_out) && cfg->T > 0)) return SLICEMOE_ERR_INVALID_ARG;
    if (misaligned(h, 16) || misaligned(h_out, 16)) return SLICEMOE_ERR_INVALID_ARG;
    slicemoe_workspace_layout L;
    make_layout(*cfg, &L);
    if (!workspace || workspace_bytes < L.total) return SLICEMOE_ERR_WORKSPACE;
    if (misaligned(workspace, 256)) return SLICEMOE_ERR_INVALID_ARG;
    const bool mfma = use_mfma(*cfg);
    if (!logical_weights_ok(*w, !mfma || !w->packed, !mfma || !w->packed)) return SLICEMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    int32_t *idx = (int32_t *)(ws + L.topk_idx);
    float *p = (float *)(ws + L.topk_p);
    int32_t *counts_raw = (int32_t *)(ws + L.counts_raw);
    int32_t *counts = (int32_t *)(ws + L.counts);
    int32_t *offsets = (int32_t *)(ws + L.offsets);
    int32_t *perm = (int32_t *)(ws + L.perm);
    int32_t *inv = (int32_t *)(ws + L.inv);
    void *y = (void *)(ws + L.y);
    float *stats = (float *)(ws + L.stats);

    const void *packed = nullptr;
    if (mfma) {
        const slicemoe_status ps = resolve_packed(*cfg, *w, workspace, workspace_bytes, s, &packed);
        if (ps != SLICEMOE_OK) return ps;
    }
    // the matrix-core router leaves the per-chunk histogram of its selections in the dispatch table
    const int hist_chunk = forward_hist_chunk(*cfg);
    int32_t *table = (int32_t *)(ws + L.scratch);
    hipError_t e = mfma ? launch_route_mfma(*cfg, h, packed, idx, p, s, v, hist_chunk > 0 ? table : nullptr)
                        : launch_route_generic(*cfg, h, *w, idx, p, s, v);
    if (e != hipSuccess) return SLICEMOE_ERR_HIP;
    if (rate > 0.f) {
        e = launch_route_dropout(*cfg, p, drop_u, rate, s);
        if (e != hipSuccess) return SLICEMOE_ERR_HIP;
    }
    // the load statistics ride along in the scan kernel of the dispatch
    e = launch_dispatch(*cfg, idx, counts_raw, counts, offsets, perm, inv, table, stats, s, hist_chunk);
    if (e != hipSuccess) return SLICEMOE_ERR_HIP;
    e = mfma ? launch_ffn_mfma(*cfg, h, p, offsets, perm, packed, y, s)
             : launch_ffn_generic(*cfg, h, p, offsets, perm, *w, y, s);
    if (e != hipSuccess) return SLICEMOE_ERR_HIP;
    e = launch_combine(*cfg, y, inv, h_out, s);
    return e == hipSuccess ? SLICEMOE_OK : SLICEMOE_ERR_HIP;
}

slicemoe_status slicemoe_forward(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w, void *h_out,
                                 void *workspace, size_t workspace_bytes, slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    return forward_common(cfg, h, w, RouteVariant(), nullptr, 0.f, h_out, workspace, workspace_bytes, stream);
}

slicemoe_status slicemoe_forward_train(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                       const slicemoe_route_train_params *params, const float *noise,
                                       const float *drop_u, void *h_out, void *workspace, size_t workspace_bytes,
                                       slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    RouteVariant v;
    const slicemoe_status vs = make_route_variant(params, noise, drop_u, &v);
    if (vs != SLICEMOE_OK) return vs;
    return forward_common(cfg, h, w, v, drop_u, params->dropout_rate, h_out, workspace, workspace_bytes, stream);
}

int slicemoe_backward_uses_mfma(const slicemoe_config *cfg)
{
    if (validate(cfg) != SLICEMOE_OK) return -1;
    return backward_mfma_shape(*cfg) ? 1 : 0;
}

size_t slicemoe_backward_workspace_bytes(const slicemoe_config *cfg)
{
    if (validate(cfg) != SLICEMOE_OK) return 0;
    return backward_plan(*cfg).total;
}

slicemoe_status slicemoe_backward(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                  const slicemoe_route_train_params *params, const float *noise, const float *drop_u,
                                  const void *forward_workspace, size_t forward_workspace_bytes, const void *d_out,
                                  void *d_h, const slicemoe_weight_grads *grads, void *workspace, size_t workspace_bytes,
                                  slicemoe_stream_t stream)
{
    const slicemoe_status st = validate(cfg);
    if (st != SLICEMOE_OK) return st;
    if (cfg->Hr > 256 || backward_lds_bytes(*cfg) > 60 * 1024) return SLICEMOE_ERR_UNSUPPORTED;
    RouteVariant v;
    float rate = 0.f;
    if (params) {
        const slicemoe_status vs = make_route_variant(params, noise, drop_u, &v);
        if (vs != SLICEMOE_OK) return vs;
        rate = params->dropout_rate;
    }
    if (!w || !grads || ((!h || !d_out || !d_h) && cfg->T > 0)) return SLICEMOE_ERR_INVALID_ARG;
    if (misaligned(h, 16) || misaligned(d_out, 16) || misaligned(d_h, 16)) return SLICEMOE_ERR_INVALID_ARG;   // 16-byte row pieces
    if (!logical_weights_ok(*w, true, true)) return SLICEMOE_ERR_INVALID_ARG;
    if (!grads->Wr1 || !grads->br1 || !grads->Wr2 || !grads->br2 || !grads->W1 || !grads->b1 || !grads->W2 || !grads->b2)
        return SLICEMOE_ERR_INVALID_ARG;
    slicemoe_workspace_layout L;
    make_layout(*cfg, &L);
    if (!forward_workspace || forward_workspace_bytes < L.total) return SLICEMOE_ERR_WORKSPACE;
    if (!workspace || workspace_bytes < slicemoe_backward_workspace_bytes(cfg)) return SLICEMOE_ERR_WORKSPACE;
    if (misaligned(forward_workspace, 256) || misaligned(workspace, 256)) return SLICEMOE_ERR_INVALID_ARG;
    const char *fw = (const char *)forward_workspace;
    const hipError_t e = launch_backward(*cfg, h, *w, v, drop_u, rate, (const int32_t *)(fw + L.topk_idx),
                                         (const float *)(fw + L.topk_p), (const int32_t *)(fw + L.offsets),
                                         (const int32_t *)(fw + L.perm), (const int32_t *)(fw + L.inv), d_out, d_h, *grads,
                                         workspace, (hipStream_t)stream);
    return e == hipSuccess ? SLICEMOE_OK : SLICEMOE_ERR_HIP;
}

}  // extern "C"
