// gs_api.hip -- the C ABI: argument validation, per-step constants, launch plumbing.
// Every check runs before the first HIP call, so the error paths need no GPU.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>

#include "gs_internal.h"

namespace gs {

static thread_local char g_hip_err[256] = "";

gs_status hip_fail(hipError_t e, const char *what)
{
    snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", what, hipGetErrorString(e));
    return GS_ERR_HIP;
}

static bool finite_f(float x) { return std::isfinite(x); }

gs_status validate_hparams(const gs_adamw_hparams *hp)
{
    if (!hp) return GS_ERR_INVALID_ARG;
    if (!finite_f(hp->lr) || hp->lr < 0.0f) return GS_ERR_INVALID_ARG;
    if (!finite_f(hp->beta1) || hp->beta1 < 0.0f || hp->beta1 >= 1.0f) return GS_ERR_INVALID_ARG;
    if (!finite_f(hp->beta2) || hp->beta2 < 0.0f || hp->beta2 >= 1.0f) return GS_ERR_INVALID_ARG;
    if (!finite_f(hp->eps) || hp->eps < 0.0f) return GS_ERR_INVALID_ARG;
    if (!finite_f(hp->weight_decay) || hp->weight_decay < 0.0f) return GS_ERR_INVALID_ARG;
    if (std::isnan(hp->max_grad_norm)) return GS_ERR_INVALID_ARG;
    if (hp->step < 1) return GS_ERR_INVALID_ARG;
    return GS_OK;
}

gs_status validate_grads(const uint16_t *const *grads, int k)
{
    if (!grads || k < 1 || k > GS_MAX_K) return GS_ERR_INVALID_ARG;
    for (int j = 0; j < k; ++j) {
        if (!grads[j] || (reinterpret_cast<uintptr_t>(grads[j]) & 15u)) return GS_ERR_INVALID_ARG;
    }
    return GS_OK;
}

// Bias corrections 1-beta^t and the derived factors: double on the host, one rounding to float.
StepConsts make_consts(const gs_adamw_hparams &hp)
{
    StepConsts s;
    const double b1 = hp.beta1, b2 = hp.beta2, t = (double)hp.step;
    const double bc1 = 1.0 - std::pow(b1, t);
    const double bc2 = 1.0 - std::pow(b2, t);
    s.beta1 = hp.beta1;
    s.beta2 = hp.beta2;
    s.omb1 = (float)(1.0 - b1);
    s.omb2 = (float)(1.0 - b2);
    s.eps = hp.eps;
    s.step_size = (float)((double)hp.lr / bc1);
    s.rsbc2 = (float)std::sqrt(bc2);
    s.decay = (float)(1.0 - (double)hp.lr * (double)hp.weight_decay);
    return s;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace gs

using namespace gs;

extern "C" {

size_t gs_sqnorm_workspace_bytes(void) { return (size_t)(GS_SQNORM_MAX_BLOCKS + GS_FINAL_SLICES) * sizeof(double); }

size_t gs_sqnorm_workspace_bytes_for(int64_t range_elems)
{
    const size_t base = gs_sqnorm_workspace_bytes();
    if (range_elems <= 0) return base;
    // one partial per 256-element tile (+2 for ragged ends) and the folding slices
    const size_t want = ((size_t)(range_elems / (GS_WAVE_BLOCK * 4)) + 2 + GS_FINAL_SLICES) * sizeof(double);
    return want > base ? want : base;
}

static gs_status sqnorm_impl(const uint16_t *const *grads, int k, int64_t begin, int64_t end, float *acc,
                             double *d_sqnorm, int accumulate, void *d_workspace, size_t workspace_bytes,
                             void *stream)
{
    gs_status st = validate_grads(grads, k);
    if (st != GS_OK) return st;
    if (begin < 0 || end < begin) return GS_ERR_INVALID_ARG;
    if (!d_sqnorm || (reinterpret_cast<uintptr_t>(d_sqnorm) & 7u)) return GS_ERR_INVALID_ARG;
    if (!d_workspace || workspace_bytes < gs_sqnorm_workspace_bytes()) return GS_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 7u) return GS_ERR_WORKSPACE;
    if (begin == end && accumulate) return GS_OK;

    SqnormArgs A;
    memset(&A, 0, sizeof A);
    for (int j = 0; j < k; ++j) A.gt.g[j] = grads[j];
    A.k = k;
    A.begin = begin;
    A.end = end;
    A.partials = static_cast<double *>(d_workspace);
    A.acc = acc;
    hipError_t e = launch_grad_sqnorm(A, workspace_bytes, d_sqnorm, accumulate, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "gs_grad_sqnorm launch");
    return GS_OK;
}

gs_status gs_grad_sqnorm(const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                         double *d_sqnorm, int accumulate,
                         void *d_workspace, size_t workspace_bytes, void *stream)
{
    return sqnorm_impl(grads, k, begin, end, nullptr, d_sqnorm, accumulate, d_workspace, workspace_bytes, stream);
}

gs_status gs_grad_accum_sqnorm(const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                               float *acc_f32, double *d_sqnorm, int accumulate,
                               void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!acc_f32 || !aligned16(acc_f32)) return GS_ERR_INVALID_ARG;
    return sqnorm_impl(grads, k, begin, end, acc_f32, d_sqnorm, accumulate, d_workspace, workspace_bytes, stream);
}

gs_status gs_accum_add(float *acc_f32, const uint16_t *grad_bf16, int first, int64_t begin, int64_t end,
                       double *d_sqnorm, int accumulate,
                       void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!acc_f32 || !grad_bf16 || !aligned16(acc_f32) || !aligned16(grad_bf16)) return GS_ERR_INVALID_ARG;
    if (begin < 0 || end < begin) return GS_ERR_INVALID_ARG;
    if (d_sqnorm) {
        if (reinterpret_cast<uintptr_t>(d_sqnorm) & 7u) return GS_ERR_INVALID_ARG;
        if (!d_workspace || workspace_bytes < gs_sqnorm_workspace_bytes()) return GS_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(d_workspace) & 7u) return GS_ERR_WORKSPACE;
    }
    if (begin == end && (!d_sqnorm || accumulate)) return GS_OK;

    AccumAddArgs A;
    memset(&A, 0, sizeof A);
    A.acc = acc_f32;
    A.g = grad_bf16;
    A.begin = begin;
    A.end = end;
    A.partials = d_sqnorm ? static_cast<double *>(d_workspace) : nullptr;
    hipError_t e = launch_accum_add(A, first != 0, workspace_bytes, d_sqnorm, accumulate, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "gs_accum_add launch");
    return GS_OK;
}

gs_status gs_acc_sqnorm(const float *acc_f32, int64_t begin, int64_t end, double *d_sqnorm, int accumulate,
                        void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!acc_f32 || !aligned16(acc_f32)) return GS_ERR_INVALID_ARG;
    if (begin < 0 || end < begin) return GS_ERR_INVALID_ARG;
    if (!d_sqnorm || (reinterpret_cast<uintptr_t>(d_sqnorm) & 7u)) return GS_ERR_INVALID_ARG;
    if (!d_workspace || workspace_bytes < gs_sqnorm_workspace_bytes()) return GS_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 7u) return GS_ERR_WORKSPACE;
    if (begin == end && accumulate) return GS_OK;
    hipError_t e = launch_acc_sqnorm(acc_f32, begin, end, static_cast<double *>(d_workspace), workspace_bytes, d_sqnorm,
                                     accumulate, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "gs_acc_sqnorm launch");
    return GS_OK;
}

// host mirror of the kernels' clip coefficient
static float clip_coefficient_host(double sqnorm_total, float max_norm)
{
    if (!(max_norm > 0.0f)) return 1.0f;
    const float norm = (float)std::sqrt(sqnorm_total);
    const float c = max_norm / (norm + 1e-6f);
    return c < 1.0f ? c : 1.0f;
}

// Byte range of elements [begin,end) of an array.
struct ByteRange {
    uintptr_t lo, hi;
};
static ByteRange range_of(const void *base, int64_t begin, int64_t end, size_t elem)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(base);
    return {a + (uintptr_t)begin * elem, a + (uintptr_t)end * elem};
}
static bool overlap(const ByteRange &x, const ByteRange &y) { return x.lo < y.hi && y.lo < x.hi; }

// Every output (p_out, m_out, v_out, w) against every input and every other output: an output may
// be exactly its own input (the in-place entry points), anything else that overlaps is rejected --
// a wave would read elements another wave has already overwritten.
static bool aliasing_ok(const float *p, const float *m, const float *v, const float *po, const float *mo,
                        const float *vo, const uint16_t *w, const uint16_t *const *grads, int k, const float *acc,
                        int64_t begin, int64_t end)
{
    const ByteRange out[4] = {range_of(po, begin, end, 4), range_of(mo, begin, end, 4), range_of(vo, begin, end, 4),
                              range_of(w, begin, end, 2)};
    const void *own_in[4] = {p, m, v, nullptr};
    const void *out_ptr[4] = {po, mo, vo, w};
    for (int a = 0; a < 4; ++a)
        for (int b = a + 1; b < 4; ++b)
            if (overlap(out[a], out[b])) return false;
    const void *in_ptr[3] = {p, m, v};
    for (int o = 0; o < 4; ++o) {
        for (int i = 0; i < 3; ++i) {
            if (in_ptr[i] == out_ptr[o] && own_in[o] == in_ptr[i]) continue;      // in place
            if (overlap(out[o], range_of(in_ptr[i], begin, end, 4))) return false;
        }
        if (acc && overlap(out[o], range_of(acc, begin, end, 4))) return false;
        if (!acc)
            for (int j = 0; j < k; ++j)
                if (overlap(out[o], range_of(grads[j], begin, end, 2))) return false;
    }
    return true;
}

// spec_norm_out != nullptr: speculative pass (c = 1, squared norm reduced into *spec_norm_out)
static gs_status adamw_impl(const float *p, const float *m, const float *v, float *po, float *mo, float *vo,
                            uint16_t *w_bf16, const uint16_t *const *grads, int k, const float *acc,
                            int64_t begin, int64_t end, const gs_adamw_hparams *hp,
                            const double *d_sqnorm, double *spec_norm_out, int accumulate,
                            void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!p || !m || !v || !po || !mo || !vo || !w_bf16) return GS_ERR_INVALID_ARG;
    if (!aligned16(p) || !aligned16(m) || !aligned16(v) || !aligned16(w_bf16)) return GS_ERR_INVALID_ARG;
    if (!aligned16(po) || !aligned16(mo) || !aligned16(vo)) return GS_ERR_INVALID_ARG;
    if (acc) {
        if (!aligned16(acc)) return GS_ERR_INVALID_ARG;
    } else {
        gs_status sg = validate_grads(grads, k);
        if (sg != GS_OK) return sg;
    }
    if (begin < 0 || end < begin) return GS_ERR_INVALID_ARG;
    if (!aliasing_ok(p, m, v, po, mo, vo, w_bf16, grads, k, acc, begin, end)) return GS_ERR_INVALID_ARG;
    gs_status st = validate_hparams(hp);
    if (st != GS_OK) return st;
    if (d_sqnorm && (reinterpret_cast<uintptr_t>(d_sqnorm) & 7u)) return GS_ERR_INVALID_ARG;
    if (spec_norm_out) {
        if (reinterpret_cast<uintptr_t>(spec_norm_out) & 7u) return GS_ERR_INVALID_ARG;
        if (!d_workspace || workspace_bytes < gs_sqnorm_workspace_bytes()) return GS_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(d_workspace) & 7u) return GS_ERR_WORKSPACE;
    }
    if (begin == end && !(spec_norm_out && !accumulate)) return GS_OK;

    StepArgs A;
    memset(&A, 0, sizeof A);
    A.p = p;
    A.m = m;
    A.v = v;
    A.po = po;
    A.mo = mo;
    A.vo = vo;
    A.w = w_bf16;
    if (!acc)
        for (int j = 0; j < k; ++j) A.gt.g[j] = grads[j];
    A.k = acc ? 0 : k;
    A.acc = acc;
    A.begin = begin;
    A.end = end;
    A.c = make_consts(*hp);
    A.max_norm = hp->max_grad_norm;
    A.d_sqnorm = d_sqnorm;
    hipError_t e;
    if (spec_norm_out)
        e = launch_accum_adamw_spec(A, static_cast<double *>(d_workspace), workspace_bytes, spec_norm_out, accumulate,
                                    static_cast<hipStream_t>(stream));
    else
        e = launch_accum_adamw(A, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "gs_accum_adamw launch");
    return GS_OK;
}

gs_status gs_accum_adamw(float *p, float *m, float *v, uint16_t *w_bf16,
                         const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                         const gs_adamw_hparams *hp, const double *d_sqnorm, void *stream)
{
    return adamw_impl(p, m, v, p, m, v, w_bf16, grads, k, nullptr, begin, end, hp, d_sqnorm, nullptr, 0, nullptr, 0,
                      stream);
}

gs_status gs_accum_adamw_oop(const float *p, const float *m, const float *v,
                             float *p_out, float *m_out, float *v_out, uint16_t *w_bf16,
                             const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *stream)
{
    return adamw_impl(p, m, v, p_out, m_out, v_out, w_bf16, grads, k, nullptr, begin, end, hp, d_sqnorm, nullptr, 0,
                      nullptr, 0, stream);
}

gs_status gs_accum_adamw_spec(const float *p, const float *m, const float *v,
                              float *p_out, float *m_out, float *v_out, uint16_t *w_bf16,
                              const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                              const gs_adamw_hparams *hp, double *d_sqnorm, int accumulate,
                              void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_sqnorm) return GS_ERR_INVALID_ARG;
    return adamw_impl(p, m, v, p_out, m_out, v_out, w_bf16, grads, k, nullptr, begin, end, hp, nullptr, d_sqnorm,
                      accumulate, d_workspace, workspace_bytes, stream);
}

float gs_clip_coefficient(double sqnorm_total, float max_grad_norm)
{
    return clip_coefficient_host(sqnorm_total, max_grad_norm);
}

gs_status gs_adamw_from_acc(float *p, float *m, float *v, uint16_t *w_bf16, const float *acc_f32,
                            int64_t begin, int64_t end, const gs_adamw_hparams *hp,
                            const double *d_sqnorm, void *stream)
{
    if (!acc_f32) return GS_ERR_INVALID_ARG;
    return adamw_impl(p, m, v, p, m, v, w_bf16, nullptr, 0, acc_f32, begin, end, hp, d_sqnorm, nullptr, 0, nullptr, 0,
                      stream);
}

gs_status gs_cu_stream_create(void **stream, int num_cus)
{
    if (!stream) return GS_ERR_INVALID_ARG;
    *stream = nullptr;
    if (num_cus < 1) return GS_ERR_INVALID_ARG;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(e, "hipDeviceGetAttribute");
    if (num_cus > cus) return GS_ERR_INVALID_ARG;
    // the driver spreads the mask over the dies; fewer than two CUs per die is not a validated shape
    if (num_cus < (cus + 15) / 16) return GS_ERR_INVALID_ARG;
    // one bit per CU, lowest-numbered CUs enabled (the driver rejects scattered masks)
    const uint32_t words = (uint32_t)((cus + 31) / 32);
    uint32_t mask[64] = {0};
    if (words > 64) return GS_ERR_INVALID_ARG;
    for (int cu = 0; cu < num_cus; ++cu) mask[cu / 32] |= (1u << (cu % 32));
    hipStream_t s = nullptr;
    e = hipExtStreamCreateWithCUMask(&s, words, mask);
    if (e != hipSuccess) {
        gs_status r = hip_fail(e, "hipExtStreamCreateWithCUMask");
        (void)hipGetLastError();
        return r;
    }
    *stream = s;
    return GS_OK;
}

gs_status gs_cu_stream_destroy(void *stream)
{
    if (!stream) return GS_ERR_INVALID_ARG;
    hipError_t e = hipStreamDestroy(static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "hipStreamDestroy");
    return GS_OK;
}

void *gs_pinned_alloc(size_t bytes)
{
    if (bytes == 0) return nullptr;
    void *ptr = nullptr;
    hipError_t e = hipHostMalloc(&ptr, bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        hip_fail(e, "hipHostMalloc");
        (void)hipGetLastError();   // do not leave a sticky error for the caller's next HIP call
        return nullptr;
    }
    return ptr;
}

void gs_pinned_free(void *ptr)
{
    if (ptr) (void)hipHostFree(ptr);
}

const char *gs_strerror(gs_status s)
{
    switch (s) {
    case GS_OK: return "ok";
    case GS_ERR_INVALID_ARG: return "invalid argument";
    case GS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GS_ERR_HIP: return "HIP runtime error";
    case GS_ERR_NOMEM: return "out of memory";
    case GS_ERR_IO: return "file read or write failed";
    case GS_ERR_TOO_LARGE: return "range longer than the no-allocation entry point's fixed scratch array covers";
    }
    return "unknown status";
}

const char *gs_last_hip_error(void) { return g_hip_err; }

}  // extern "C"
