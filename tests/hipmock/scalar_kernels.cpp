// Host stand-ins for the library's kernel launchers, for running the plain-C ABI program
// (tests/c_abi/step_demo.c) against the HIP stand-in without a GPU.  Each launcher enqueues a
// scalar loop on the mock stream.  The loops do the step's arithmetic with the per-step constants
// the library's host code prepared (one rounding per operation, built with -ffp-contract=off), so
// the program's bit-for-bit comparison with the oracle also checks that every element went through
// the plumbing exactly once.  Test infrastructure only.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>

#include "gs_internal.h"

namespace gs {

static float widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t narrow(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

static float sum_of(const GradTable &gt, int k, int64_t i)
{
    float a = 0.0f;
    for (int j = 0; j < k; ++j) a += widen(gt.g[j][i]);
    return a;
}

hipError_t launch_accum_adamw(const StepArgs &A, hipStream_t stream)
{
    StepArgs a = A;
    hipmock_enqueue(stream, [a] {
        float c = 1.0f;
        if (a.d_sqnorm && a.max_norm > 0.0f) {
            const float norm = (float)std::sqrt(*a.d_sqnorm);
            const float q = a.max_norm / (norm + 1e-6f);
            c = q < 1.0f ? q : 1.0f;
        }
        for (int64_t i = a.begin; i < a.end; ++i) {
            const float g = c * (a.acc ? a.acc[i] : sum_of(a.gt, a.k, i));
            const float m = a.c.beta1 * a.m[i] + a.c.omb1 * g;
            const float v = a.c.beta2 * a.v[i] + a.c.omb2 * (g * g);
            const float d = std::sqrt(v) / a.c.rsbc2 + a.c.eps;
            const float p = a.p[i] * a.c.decay - a.c.step_size * (m / d);
            a.po[i] = p;
            a.mo[i] = m;
            a.vo[i] = v;
            a.w[i] = narrow(p);
        }
    });
    return hipSuccess;
}

hipError_t launch_grad_sqnorm(const SqnormArgs &A, size_t, double *d_out, int accumulate, hipStream_t stream)
{
    SqnormArgs a = A;
    hipmock_enqueue(stream, [a, d_out, accumulate] {
        double s = 0.0;
        for (int64_t i = a.begin; i < a.end; ++i) {
            const float x = sum_of(a.gt, a.k, i);
            if (a.acc) a.acc[i] = x;
            s += (double)x * (double)x;
        }
        *d_out = accumulate ? *d_out + s : s;
    });
    return hipSuccess;
}

hipError_t launch_accum_adamw_spec(const StepArgs &, double *, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_accum_add(const AccumAddArgs &, int, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_acc_sqnorm(const float *, int64_t, int64_t, double *, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }

}  // namespace gs
