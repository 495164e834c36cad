// Internal layout of a layer object (shared by layer.hip and net.hip).
#pragma once

#include <utility>
#include <vector>

#include "common.h"

struct dcnn_layer {
    dcnn_ctx* ctx;
    dcnn_layer_desc d;
    int oh, ow, oc;
    int64_t in_pixels, out_pixels;
    bool inited;
    bool alias_mask;            // output mask / index list are those of input 0
    bool has_bias;
    bool has_bias2 = false;     // bias of the fused projection
    size_t state_bytes;
    // pieces of the caller-provided state memory
    void* buf0; size_t buf0_bytes;      // x^A | stored input frame | dense output
    void* buf1; size_t buf1_bytes;      // x^T
    void* buf2; size_t buf2_bytes;      // dense accumulated output of a layer with fuse_accum
    void* out_data;
    uint8_t* out_mask;
    int32_t* out_idx;
    int32_t* out_count;
    uint8_t* out_mask_alt;              // second output mask of a layer that alternates between two (see dcnn_layer_step)
    int mask_phase;                     // which of the two the NEXT step writes
    int32_t* list;                      // work list when the layer builds its own
    int32_t* list_count;
    uint32_t* taps;                     // per work-list entry: flagged window taps (dense convolutions, 1x1 / 3x3)
    uint8_t* xt_flags;                  // per output pixel: 0 = its x^T row is all zero and need not be read (layers whose
                                        // sparse steps run on the wave-specialised kernel); nullptr: none
    bool counting = false, counted = false;   // statistics mode (dcnn_layer_set_counting); the last step was counted
    mutable bool xt_flags_stale = false;  // the state memory was handed out: the flags are rebuilt from x^T before the next step
    void* wpacked;
    void* bias;
    void* wpacked2;                     // fused projection: weights in the main plan's column grouping (sparse steps)
    void* wpacked2_dense;               // ... and packed as a convolution of its own (dense first frame)
    void* bias2;
    int32_t* counters;
    // bookkeeping of the last step
    dcnn_delta view;
    const int32_t* last_in_count;
    const int32_t* last_work_count;
    const int32_t* last_in2_count;
    const uint8_t* last_in_mask;        // for statistics of inputs that come without a count
    const uint8_t* last_in2_mask;
    // optional kernel timing
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
    size_t events_used = 0;
};

namespace dcnn {
// dcnn_layer_create with the weights and bias of a fused projection passed on their own.
dcnn_status layer_create(dcnn_ctx* ctx, const dcnn_layer_desc* desc, const void* weights_dev, const void* bias_dev,
                         const void* proj_weights_dev, const void* proj_bias_dev, void* state_dev, size_t state_bytes,
                         dcnn_layer** out);
}  // namespace dcnn
