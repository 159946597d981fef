// gs_stream_internal.h -- the streaming context, shared by the host<->HBM pipeline and the
// file tier built on top of it (not installed).
#ifndef GS_STREAM_INTERNAL_H
#define GS_STREAM_INTERNAL_H

#include <hip/hip_runtime_api.h>

#include <vector>

#include "gs_internal.h"

struct gs_stream_ctx {
    int device = 0;
    int64_t chunk = 0;
    int slots = 0;
    int64_t slot_elems = 0;                 // chunk + 8 (room for the (b mod 8) offset)
    hipStream_t s_h2d = nullptr, s_comp = nullptr, s_d2h = nullptr;
    float *pool = nullptr;                  // slots * 3 * slot_elems floats
    std::vector<hipEvent_t> ev_h2d, ev_comp, ev_d2h;
    std::vector<char> used;                 // slot has a pending/finished download recorded
    hipEvent_t ev_producer = nullptr;
    int64_t next_chunk = 0;                 // running chunk counter across calls -> slot rotation
};

namespace gs {

// Checks shared by the entry points that stream a layer (everything except the state pointers).
gs_status stream_validate(const gs_stream_ctx *c, const uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                          int64_t n, const gs_adamw_hparams *hp, const double *d_sqnorm);

// Makes the compute stream wait for what `producer_stream` holds now and fills the parts of A
// that are the same for every chunk of a layer.
gs_status stream_begin_layer(gs_stream_ctx *c, StepArgs &A, uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream);

// Enqueues one chunk: elements [b,e) of the layer, whose states start at src_p/src_m/src_v in
// pinned host memory, go up into the next slot, through the step kernel and back to the same
// host addresses.  *slot_out (if given) receives the slot whose ev_d2h marks the download's end.
gs_status stream_chunk(gs_stream_ctx *c, StepArgs &A, float *src_p, float *src_m, float *src_v, int64_t b, int64_t e,
                       int *slot_out);

}  // namespace gs
#endif
