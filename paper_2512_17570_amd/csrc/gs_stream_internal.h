// gs_stream_internal.h -- the streaming context, shared by the host-resident step and the file
// tier built on top of it (not installed).
#ifndef GS_STREAM_INTERNAL_H
#define GS_STREAM_INTERNAL_H

#include <hip/hip_runtime_api.h>

#include <vector>

#include "gs_internal.h"

struct gs_stream_ctx {
    int device = 0;
    bool staged = false;                    // false: kernel in place on host memory; true: copy-engine pipeline
    int num_cus = 0;                        // in-place mode; 0: the compute stream may use every CU
    hipStream_t s_comp = nullptr;           // the step kernels
    hipStream_t s_note = nullptr;           // carries only host-function notifications (file tier)
    hipEvent_t ev_producer = nullptr;

    // staged mode only
    int64_t chunk = 0;
    int slots = 0;
    int64_t slot_elems = 0;                 // chunk + 8 (room for the (b mod 8) offset), rounded up
    hipStream_t s_h2d = nullptr, s_d2h = nullptr;
    float *pool = nullptr;                  // slots * 3 * slot_elems floats of device memory
    std::vector<hipEvent_t> ev_h2d, ev_comp, ev_d2h;
    std::vector<char> used;                 // ev_d2h[slot] has been recorded at least once
    int64_t next_chunk = 0;                 // running chunk counter across calls -> slot rotation
    int copies_overlap = -1;                // creation-time check: 1 the three streams ran side by side, 0 a pair
                                            // still took turns after every retry, -1 not checked (tiny slots)
};

namespace gs {

// Checks shared by the entry points that step a layer in host memory (everything except the
// state pointers).
gs_status stream_validate(const gs_stream_ctx *c, const uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                          int64_t n, const gs_adamw_hparams *hp, const double *d_sqnorm);

// GS_OK if h[0] and h[n-1] (n >= 1) are page-locked host memory that the device addresses at the same
// pointer; GS_ERR_INVALID_ARG otherwise (pageable memory under a kernel would fault the GPU).
gs_status stream_check_mapped(const float *h, int64_t n);

// Makes the compute stream wait for what `producer_stream` holds now and fills the parts of A
// that are the same for every launch of a layer.
gs_status stream_begin_layer(gs_stream_ctx *c, StepArgs &A, uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream);

// Enqueues the step over elements [b,e) of the layer, in place on states that start at
// host_p/host_m/host_v (the addresses of element b) in pinned, device-accessible host memory.
// The addresses must satisfy (address - 4*b) % 16 == 0, i.e. element 0 of the (virtual) array is
// 16-byte aligned.
gs_status stream_range(gs_stream_ctx *c, StepArgs &A, float *host_p, float *host_m, float *host_v, int64_t b, int64_t e);

}  // namespace gs
#endif
