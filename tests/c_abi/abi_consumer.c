/*
 * A consumer of the C ABI written against include/slicemoe.h alone: no Python, no PyTorch.  It allocates device memory
 * with the HIP runtime, runs the whole layer through slicemoe_forward on the matrix-core path (bf16 storage, weights
 * packed once), and checks the result against the fp64 C oracle linked next to it (test infrastructure, like every
 * use of the oracle).  Exit code 0 = everything agreed.
 *
 *   abi_consumer            the run on the GPU
 *   abi_consumer --link     no GPU call: the size queries and error codes only (that the library links and answers)
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "slicemoe.h"

/* the oracle (oracle/slicemoe_oracle.c) */
#ifdef __cplusplus
extern "C"
#endif
int oracle_forward(const double *h, int64_t T, int d, int S, int Hr, int E, int k, int He, int64_t capacity,
                   const double *Wr1, const double *br1, const double *Wr2, const double *br2, const double *W1,
                   const double *b1, const double *W2, const double *b2, int act, double *h_out, int32_t *idx_o,
                   double *pk_o, double *margin_o, int32_t *counts_raw_o, int32_t *counts_o, int32_t *offsets_o,
                   int32_t *perm_o, int32_t *inv_o);

#define FAIL(...) do { fprintf(stderr, "abi_consumer: " __VA_ARGS__); fprintf(stderr, "\n"); return 1; } while (0)
#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) FAIL("%s: %s", #x, hipGetErrorString(e_)); } while (0)
#define SM(x) do { slicemoe_status s_ = (x); if (s_ != SLICEMOE_OK) FAIL("%s: %s", #x, slicemoe_status_string(s_)); } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform01(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
/* round to nearest even bf16; returns the bit pattern and leaves the rounded value in *v */
static uint16_t to_bf16(double *v)
{
    float f = (float)*v;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    *v = (double)f;
    return (uint16_t)(u >> 16);
}
/* n values: uniform in [-a, a] (a > 0) or a sum of twelve uniforms (a == 0: about N(0, 1)); rounded to bf16 */
static int fill(size_t n, double a, double **host64, void **dev)
{
    double *v = (double *)malloc(n * sizeof(double));
    uint16_t *b = (uint16_t *)malloc(n * sizeof(uint16_t));
    if (!v || !b) FAIL("out of host memory");
    for (size_t i = 0; i < n; ++i) {
        if (a > 0) v[i] = (2.0 * uniform01() - 1.0) * a;
        else { double s = -6.0; for (int q = 0; q < 12; ++q) s += uniform01(); v[i] = s; }
        b[i] = to_bf16(&v[i]);
    }
    HIP(hipMalloc(dev, n * sizeof(uint16_t)));
    HIP(hipMemcpy(*dev, b, n * sizeof(uint16_t), hipMemcpyHostToDevice));
    free(b);
    *host64 = v;
    return 0;
}

int main(int argc, char **argv)
{
    slicemoe_config c;
    memset(&c, 0, sizeof c);
    c.T = 256; c.d = 512; c.S = 8; c.k = 2; c.E = 16; c.Hr = 256; c.He = 256;
    c.capacity_factor = 0.f; c.dtype = SLICEMOE_BF16; c.flags = SLICEMOE_FLAG_REQUIRE_MFMA;
    const int ds = c.d / c.S;
    const int64_t Ns = (int64_t)c.T * c.S, Na = Ns * c.k;

    /* what needs no GPU */
    if (slicemoe_workspace_bytes(&c) == 0 || slicemoe_packed_bytes(&c) == 0) FAIL("size queries refuse a valid config");
    if (slicemoe_uses_mfma(&c) != 1) FAIL("the matrix-core kernels do not take the shape they are written for");
    slicemoe_workspace_layout L;
    SM(slicemoe_get_workspace_layout(&c, &L));
    if (L.total != slicemoe_workspace_bytes(&c)) FAIL("layout and workspace size disagree");
    slicemoe_config bad = c;
    bad.S = 7;   /* d % S != 0 */
    if (slicemoe_workspace_bytes(&bad) != 0) FAIL("an invalid config got a workspace size");
    if (slicemoe_forward(&bad, NULL, NULL, NULL, NULL, 0, NULL) != SLICEMOE_ERR_INVALID_ARG) FAIL("invalid config accepted");
    if (slicemoe_forward(&c, NULL, NULL, NULL, NULL, 0, NULL) != SLICEMOE_ERR_INVALID_ARG) FAIL("null pointers accepted");
    if (!slicemoe_status_string(SLICEMOE_ERR_WORKSPACE)) FAIL("no text for a status");
    if (argc > 1 && strcmp(argv[1], "--link") == 0) { printf("abi_consumer: linked, queries answered\n"); return 0; }

    /* inputs: the default initialisation of a linear layer, hidden states about N(0, 1), all representable in bf16 */
    double *h, *Wr1, *br1, *Wr2, *br2, *W1, *b1, *W2, *b2;
    void *dh, *dWr1, *dbr1, *dWr2, *dbr2, *dW1, *db1, *dW2, *db2;
    if (fill((size_t)c.T * c.d, 0.0, &h, &dh)) return 1;
    if (fill((size_t)ds * c.Hr, 1.0 / sqrt((double)ds), &Wr1, &dWr1) || fill((size_t)c.Hr, 1.0 / sqrt((double)ds), &br1, &dbr1)) return 1;
    if (fill((size_t)c.Hr * c.E, 1.0 / sqrt((double)c.Hr), &Wr2, &dWr2) || fill((size_t)c.E, 1.0 / sqrt((double)c.Hr), &br2, &dbr2)) return 1;
    if (fill((size_t)c.E * ds * c.He, 1.0 / sqrt((double)ds), &W1, &dW1) || fill((size_t)c.E * c.He, 1.0 / sqrt((double)ds), &b1, &db1)) return 1;
    if (fill((size_t)c.E * c.He * ds, 1.0 / sqrt((double)c.He), &W2, &dW2) || fill((size_t)c.E * ds, 1.0 / sqrt((double)c.He), &b2, &db2)) return 1;

    hipStream_t stream;
    HIP(hipStreamCreate(&stream));
    void *packed, *ws, *dout;
    HIP(hipMalloc(&packed, slicemoe_packed_bytes(&c)));
    HIP(hipMalloc(&ws, L.total));
    HIP(hipMalloc(&dout, (size_t)c.T * c.d * 2));
    slicemoe_weights w = {dWr1, dbr1, dWr2, dbr2, dW1, db1, dW2, db2, NULL};
    SM(slicemoe_pack_weights(&c, &w, packed, slicemoe_packed_bytes(&c), (slicemoe_stream_t)stream));
    w.packed = packed;
    if (slicemoe_forward(&c, dh, &w, dout, ws, L.total - 1, (slicemoe_stream_t)stream) != SLICEMOE_ERR_WORKSPACE)
        FAIL("a workspace one byte short was accepted");

    uint16_t *out[2];
    int32_t *idx = (int32_t *)malloc((size_t)Na * 4), *offsets = (int32_t *)malloc((size_t)(c.E + 1) * 4);
    int32_t *perm = (int32_t *)malloc((size_t)Na * 4), *inv = (int32_t *)malloc((size_t)Na * 4);
    for (int run = 0; run < 2; ++run) {   /* twice: same inputs, same bits */
        out[run] = (uint16_t *)malloc((size_t)c.T * c.d * 2);
        HIP(hipMemsetAsync(dout, 0xFF, (size_t)c.T * c.d * 2, stream));
        SM(slicemoe_forward(&c, dh, &w, dout, ws, L.total, (slicemoe_stream_t)stream));
        HIP(hipStreamSynchronize(stream));
        HIP(hipMemcpy(out[run], dout, (size_t)c.T * c.d * 2, hipMemcpyDeviceToHost));
    }
    if (memcmp(out[0], out[1], (size_t)c.T * c.d * 2) != 0) FAIL("two runs on the same inputs differ");
    HIP(hipMemcpy(idx, (char *)ws + L.topk_idx, (size_t)Na * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(offsets, (char *)ws + L.offsets, (size_t)(c.E + 1) * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(perm, (char *)ws + L.perm, (size_t)Na * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(inv, (char *)ws + L.inv, (size_t)Na * 4, hipMemcpyDeviceToHost));

    /* the oracle on the same values */
    double *ref = (double *)malloc((size_t)c.T * c.d * sizeof(double)), *pk = (double *)malloc((size_t)Na * sizeof(double));
    double *margin = (double *)malloc((size_t)Ns * sizeof(double));
    int32_t *oidx = (int32_t *)malloc((size_t)Na * 4), *ocr = (int32_t *)malloc((size_t)c.E * 4), *oc = (int32_t *)malloc((size_t)c.E * 4);
    int32_t *ooff = (int32_t *)malloc((size_t)(c.E + 1) * 4), *operm = (int32_t *)malloc((size_t)Na * 4), *oinv = (int32_t *)malloc((size_t)Na * 4);
    if (oracle_forward(h, c.T, c.d, c.S, c.Hr, c.E, c.k, c.He, -1, Wr1, br1, Wr2, br2, W1, b1, W2, b2, 0, ref, oidx, pk,
                       margin, ocr, oc, ooff, operm, oinv) != 0)
        FAIL("the oracle refused the inputs");

    /* routing: identical except on near-ties of the oracle's own logits (margin below 1e-6), which are left out */
    int64_t ties = 0;
    char *skip = (char *)calloc((size_t)Ns, 1);
    for (int64_t n = 0; n < Ns; ++n)
        for (int j = 0; j < c.k; ++j)
            if (idx[n * c.k + j] != oidx[n * c.k + j]) {
                if (margin[n] >= 1e-6) FAIL("slice %lld: expert %d selected, the oracle selects %d with margin %.3g", (long long)n,
                                            idx[n * c.k + j], oidx[n * c.k + j], margin[n]);
                if (!skip[n]) ++ties;
                skip[n] = 1;
            }
    if (ties > 4) FAIL("%lld near-tie slices among %lld", (long long)ties, (long long)Ns);
    if (ties == 0) {   /* the grouping is then determined bit for bit */
        if (memcmp(offsets, ooff, (size_t)(c.E + 1) * 4) || memcmp(perm, operm, (size_t)Na * 4) || memcmp(inv, oinv, (size_t)Na * 4))
            FAIL("dispatch tables differ from the oracle's");
    }
    if (offsets[c.E] != Na) FAIL("dropless, yet %d of %lld assignments were kept", offsets[c.E], (long long)Na);

    /* output: max error over the RMS of the oracle's output, bar 2e-2 for bf16 storage */
    double ss = 0.0, worst = 0.0;
    for (size_t i = 0; i < (size_t)c.T * c.d; ++i) ss += ref[i] * ref[i];
    const double rms = sqrt(ss / ((double)c.T * c.d));
    for (int64_t n = 0; n < Ns; ++n) {
        if (skip[n]) continue;
        for (int i = 0; i < ds; ++i) {
            const uint32_t u = (uint32_t)out[0][n * ds + i] << 16;
            float f;
            memcpy(&f, &u, 4);
            if (!(f == f) || isinf(f)) FAIL("output element %lld of slice %lld is not finite", (long long)i, (long long)n);
            const double e = fabs((double)f - ref[n * ds + i]);
            if (e > worst) worst = e;
        }
    }
    printf("abi_consumer: T=%d d=%d S=%d E=%d k=%d He=%d bf16: max|err|/rms = %.3e (bar 2e-2), near-tie slices %lld, "
           "dispatch bit-exact, two runs identical\n", c.T, c.d, c.S, c.E, c.k, c.He, worst / rms, (long long)ties);
    if (!(worst / rms <= 2e-2)) FAIL("output error above the bar");
    return 0;
}
