/*
 * The C boundary used from plain C, without Python or PyTorch: device memory and copies come from
 * the HIP runtime's C API, the step from libgs.so, the expected values from the CPU oracle linked
 * into this test program.  One small layer, device-resident: squared norm accumulated over two
 * ranges, then the fused step over the range split in two at an unaligned point.  With the
 * argument --host-resident it goes on to the host-resident step on pinned memory: in place on a
 * stream confined to a sixteenth of the compute units, then staged through device slots, both
 * with the null stream as the producer stream.  Prints its stages as it goes (unbuffered) and
 * "C ABI OK", and exits 0 when everything matches bit for bit.
 *
 * Built by tests/c_abi/build_demo.py (gcc, C99) and run by a GPU test; the same source is also
 * built against the host-only HIP stand-in (tests/hipmock) and run on the CPU.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "gs.h"

/* oracle (test infrastructure) */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay, max_grad_norm;
    int32_t step;
} gs_oracle_hparams;
double gs_oracle_grad_sqnorm(const uint16_t *const *grads, int k, int64_t begin, int64_t end);
float gs_oracle_clip_coef(double sqnorm_total, float max_norm);
void gs_oracle_accum_adamw(float *p, float *m, float *v, uint16_t *w, const uint16_t *const *grads, int k, int64_t begin,
                           int64_t end, const gs_oracle_hparams *hp, float c);
uint16_t gs_oracle_f32_to_bf16(float f);

#define HIP(x)                                                                            \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define GS(x)                                                                                          \
    do {                                                                                               \
        gs_status s_ = (x);                                                                            \
        if (s_ != GS_OK) {                                                                             \
            printf("%s -> %s (%s) at line %d\n", #x, gs_strerror(s_), gs_last_hip_error(), __LINE__); \
            return 3;                                                                                  \
        }                                                                                              \
    } while (0)

/* small deterministic generator: values only have to be reproducible, not random-looking */
static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }
static float unit(uint32_t *s) { return (float)(lcg(s) >> 8) * (1.0f / 16777216.0f) - 0.5f; }

static int same(const void *a, const void *b, size_t bytes, const char *what)
{
    if (memcmp(a, b, bytes) != 0) {
        printf("MISMATCH: %s\n", what);
        return 0;
    }
    return 1;
}

/* one host-resident pass over pinned copies of the states; returns 1 if it matches the oracle */
static int host_resident_pass(gs_stream_ctx *ctx, const char *what, int64_t n, const float *p, const float *m,
                              const float *v, const float *ep, const float *em, const float *ev, const uint16_t *ew,
                              const uint16_t *const *gt_dev, int k, const gs_adamw_hparams *hp, const double *d_sq,
                              uint16_t *d_w, uint16_t *rw)
{
    const size_t f4 = (size_t)n * 4, b2 = (size_t)n * 2;
    float *hp_ = gs_pinned_alloc(f4), *hm_ = gs_pinned_alloc(f4), *hv_ = gs_pinned_alloc(f4);
    if (!hp_ || !hm_ || !hv_) {
        printf("gs_pinned_alloc failed: %s\n", gs_last_hip_error());
        return 0;
    }
    memcpy(hp_, p, f4); memcpy(hm_, m, f4); memcpy(hv_, v, f4);
    if (hipMemset(d_w, 0, b2) != hipSuccess) return 0;
    printf("stage: %s: enqueue\n", what);
    gs_status st = gs_stream_layer_step(ctx, hp_, hm_, hv_, d_w, gt_dev, k, n, hp, d_sq, NULL);
    if (st != GS_OK) {
        printf("gs_stream_layer_step -> %s (%s)\n", gs_strerror(st), gs_last_hip_error());
        return 0;
    }
    printf("stage: %s: sync\n", what);
    st = gs_stream_ctx_sync(ctx);
    if (st != GS_OK) {
        printf("gs_stream_ctx_sync -> %s (%s)\n", gs_strerror(st), gs_last_hip_error());
        return 0;
    }
    printf("stage: %s: compare\n", what);
    if (hipMemcpy(rw, d_w, b2, hipMemcpyDeviceToHost) != hipSuccess) return 0;
    int ok = same(hp_, ep, f4, what) & same(hm_, em, f4, what) & same(hv_, ev, f4, what) & same(rw, ew, b2, what);
    gs_pinned_free(hp_); gs_pinned_free(hm_); gs_pinned_free(hv_);
    return ok;
}

int main(int argc, char **argv)
{
    enum { K = 3 };
    const int host_resident = argc > 1 && strcmp(argv[1], "--host-resident") == 0;
    setvbuf(stdout, NULL, _IONBF, 0);
    printf("stage: inputs and oracle\n");
    const int64_t n = 512 * 37 + 11, split = 7001;
    const size_t f4 = (size_t)n * 4, b2 = (size_t)n * 2;
    uint32_t seed = 12345u;
    float *p = malloc(f4), *m = malloc(f4), *v = malloc(f4);
    uint16_t *g[K];
    for (int64_t i = 0; i < n; ++i) {
        p[i] = 0.04f * unit(&seed);
        m[i] = 2e-3f * unit(&seed);
        float t = 2e-3f * unit(&seed);
        v[i] = t * t;
    }
    for (int j = 0; j < K; ++j) {
        g[j] = malloc(b2);
        for (int64_t i = 0; i < n; ++i) g[j][i] = gs_oracle_f32_to_bf16(0.02f * unit(&seed));
    }
    const gs_adamw_hparams hp = {1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 0.5f, 4};

    /* expected: the oracle on host copies */
    float *ep = malloc(f4), *em = malloc(f4), *ev = malloc(f4);
    uint16_t *ew = malloc(b2);
    memcpy(ep, p, f4); memcpy(em, m, f4); memcpy(ev, v, f4);
    const uint16_t *gt_host[K] = {g[0], g[1], g[2]};
    const double S_o = gs_oracle_grad_sqnorm(gt_host, K, 0, n);
    const gs_oracle_hparams ohp = {hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.max_grad_norm, hp.step};
    gs_oracle_accum_adamw(ep, em, ev, ew, gt_host, K, 0, n, &ohp, gs_oracle_clip_coef(S_o, hp.max_grad_norm));

    /* device-resident step */
    printf("stage: device memory\n");
    float *d_p, *d_m, *d_v;
    uint16_t *d_w, *d_g[K];
    double *d_sq;
    void *d_ws;
    HIP(hipMalloc((void **)&d_p, f4)); HIP(hipMalloc((void **)&d_m, f4)); HIP(hipMalloc((void **)&d_v, f4));
    HIP(hipMalloc((void **)&d_w, b2)); HIP(hipMalloc((void **)&d_sq, sizeof(double)));
    HIP(hipMalloc(&d_ws, gs_sqnorm_workspace_bytes()));
    HIP(hipMemcpy(d_p, p, f4, hipMemcpyHostToDevice)); HIP(hipMemcpy(d_m, m, f4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(d_v, v, f4, hipMemcpyHostToDevice));
    for (int j = 0; j < K; ++j) {
        HIP(hipMalloc((void **)&d_g[j], b2));
        HIP(hipMemcpy(d_g[j], g[j], b2, hipMemcpyHostToDevice));
    }
    const uint16_t *gt_dev[K] = {d_g[0], d_g[1], d_g[2]};
    printf("stage: norm and step\n");
    GS(gs_grad_sqnorm(gt_dev, K, 0, split, d_sq, 0, d_ws, gs_sqnorm_workspace_bytes(), NULL));
    GS(gs_grad_sqnorm(gt_dev, K, split, n, d_sq, 1, d_ws, gs_sqnorm_workspace_bytes(), NULL));
    GS(gs_accum_adamw(d_p, d_m, d_v, d_w, gt_dev, K, 0, split, &hp, d_sq, NULL));
    GS(gs_accum_adamw(d_p, d_m, d_v, d_w, gt_dev, K, split, n, &hp, d_sq, NULL));
    HIP(hipDeviceSynchronize());
    printf("stage: compare\n");
    double S = 0.0;
    float *rp = malloc(f4), *rm = malloc(f4), *rv = malloc(f4);
    uint16_t *rw = malloc(b2);
    HIP(hipMemcpy(&S, d_sq, sizeof S, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rp, d_p, f4, hipMemcpyDeviceToHost)); HIP(hipMemcpy(rm, d_m, f4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rv, d_v, f4, hipMemcpyDeviceToHost)); HIP(hipMemcpy(rw, d_w, b2, hipMemcpyDeviceToHost));
    int ok = fabs(S - S_o) <= 1e-12 * S_o;
    if (!ok) printf("MISMATCH: norm %.17g vs oracle %.17g\n", S, S_o);
    ok &= same(rp, ep, f4, "p (resident)") & same(rm, em, f4, "m (resident)") & same(rv, ev, f4, "v (resident)") &
          same(rw, ew, b2, "w (resident)");
    if (gs_clip_coefficient(S, hp.max_grad_norm) != gs_oracle_clip_coef(S_o, hp.max_grad_norm)) {
        printf("MISMATCH: clip coefficient\n");
        ok = 0;
    }

    /* a rejected call touches nothing and says why */
    if (gs_accum_adamw(d_p, d_m, d_v, d_w, gt_dev, 0, 0, n, &hp, d_sq, NULL) != GS_ERR_INVALID_ARG) {
        printf("MISMATCH: k = 0 accepted\n");
        ok = 0;
    }
    if (host_resident) {
        /* the norm of the whole layer is in d_sq; the null stream is the producer stream */
        int dev = 0, cus = 0;
        HIP(hipGetDevice(&dev));
        HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        gs_stream_ctx *ctx = NULL;
        printf("stage: in-place context on %d of %d compute units\n", (cus + 15) / 16, cus);
        GS(gs_stream_ctx_create_inplace(&ctx, (cus + 15) / 16));
        ok &= host_resident_pass(ctx, "host-resident in place", n, p, m, v, ep, em, ev, ew, gt_dev, K, &hp, d_sq, d_w, rw);
        GS(gs_stream_ctx_destroy(ctx));
        printf("stage: staged context\n");
        GS(gs_stream_ctx_create(&ctx, 4099, 3));
        ok &= host_resident_pass(ctx, "host-resident staged", n, p, m, v, ep, em, ev, ew, gt_dev, K, &hp, d_sq, d_w, rw);
        GS(gs_stream_ctx_destroy(ctx));
    }
    printf(ok ? "C ABI OK: n=%lld k=%d S=%.9e\n" : "C ABI FAILED: n=%lld k=%d S=%.9e\n", (long long)n, K, S);
    return ok ? 0 : 1;
}
