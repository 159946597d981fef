// gs_internal.h -- types shared by the library's own translation units (not installed).
#ifndef GS_INTERNAL_H
#define GS_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "gs.h"

#define GS_STEP_BLOCK 128             // threads per workgroup of the step kernel for many gradient streams, and of the
                                      // staged norm kernel (2 wave64)
#define GS_WAVE_BLOCK 64              // single-wave workgroups: the step kernel otherwise, and the fast shapes of the
                                      // kernels that step or add and leave a norm partial per workgroup
#define GS_STEP_WIDE_MIN_K 15         // gradient streams from which the step kernel takes GS_STEP_BLOCK lanes
#define GS_STATE_WAIT_MAX_K 7         // up to this many gradient streams each state load is waited for on its own
#define GS_BLOCK 256                  // threads per workgroup of the norm kernel (4 wave64)
#define GS_TILE (GS_BLOCK * 4)        // elements per norm tile: one group of 4 per lane
#define GS_FINAL_BLOCK 1024           // threads of the partial-folding kernels
#define GS_FINAL_SLICES 128           // workgroups of the first folding stage for large partial counts
#define GS_FINAL_DIRECT_MAX 8192      // up to this many partials are folded by one workgroup directly
#define GS_STAGE_BLOCK 1024           // threads per workgroup of the staged norm kernel
#define GS_SQNORM_MAX_BLOCKS 262144   // upper bound on block partials => workspace size (2 MB)
#define GS_NORM_SPAN 8                // consecutive tiles per norm workgroup (grows for huge ranges)

namespace gs {

// Per-step constants, formed on the host in double and rounded to float once.
struct StepConsts {
    float beta1, beta2, omb1, omb2, eps, step_size, rsbc2, decay;
};

struct GradTable {
    const uint16_t *g[GS_MAX_K];
};

struct StepArgs {
    const float *p, *m, *v;   // states in
    float *po, *mo, *vo;      // states out (the same arrays for the in-place entry points)
    uint16_t *w;
    GradTable gt;
    int k;
    int64_t begin, end;
    StepConsts c;
    float max_norm;
    const double *d_sqnorm;
    const float *acc;   // non-null: staged fp32 gradient sum replaces the k bf16 streams
};

struct SqnormArgs {
    GradTable gt;
    int k;
    int64_t begin, end;
    double *partials;
    float *acc;         // non-null: also write the fp32 gradient sum here
};

struct AccumAddArgs {
    float *acc;
    const uint16_t *g;
    int64_t begin, end;
    double *partials;   // used only when a norm is asked for
};

hipError_t launch_accum_adamw(const StepArgs &A, hipStream_t stream);
hipError_t launch_accum_adamw_spec(const StepArgs &A, double *partials, size_t workspace_bytes, double *d_out,
                                   int accumulate, hipStream_t stream);
hipError_t launch_grad_sqnorm(const SqnormArgs &A, size_t workspace_bytes, double *d_out, int accumulate,
                              hipStream_t stream);

// d_out == nullptr: no norm (then the workspace is not touched)
hipError_t launch_accum_add(const AccumAddArgs &A, int first, size_t workspace_bytes, double *d_out, int accumulate,
                            hipStream_t stream);

// squared norm of a finished fp32 buffer over [begin,end)
hipError_t launch_acc_sqnorm(const float *acc, int64_t begin, int64_t end, double *partials, size_t workspace_bytes,
                             double *d_out, int accumulate, hipStream_t stream);

// host side (gs_api.hip)
gs_status validate_hparams(const gs_adamw_hparams *hp);
gs_status validate_grads(const uint16_t *const *grads, int k);
StepConsts make_consts(const gs_adamw_hparams &hp);
gs_status hip_fail(hipError_t e, const char *what);

}  // namespace gs
#endif
