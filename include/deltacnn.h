/*
 * deltacnn.h -- C ABI of the MI355X (gfx950) sparse frame-difference CNN inference library.
 *
 * The library implements the per-frame hot path of DeltaCNN (arXiv 2203.03996): after one
 * dense first frame has initialised every layer's buffers, each later frame travels through
 * the network as a sparse update (delta feature map + per-pixel update mask).
 *
 * Conventions that hold for every call
 * ------------------------------------
 *  - Pointers named *_dev are DEVICE pointers, *_host are HOST pointers.  The library never
 *    allocates device memory: every buffer (tensors, layer state, workspace, the network arena)
 *    is allocated by the caller with the sizes the *_query calls report, and must stay valid
 *    until the object that uses it is destroyed.  All device buffers must be 256-byte aligned.
 *  - Feature maps are NHWC, element type dcnn_dtype.  Masks are uint8 [n,h,w] holding 0 or 1.
 *    Index lists are int32, the ascending linear pixel indices (n*H + y)*W + x of the flagged
 *    pixels; `count` is one int32 in device memory.  Active counts never travel to the host.
 *  - A delta feature map is defined only where its mask is 1.  Everywhere else its memory is
 *    undefined, is never read by the library, and may hold anything (supplementary Section 1.3).
 *  - Every call returns a dcnn_status; nothing throws.  Arguments are validated before anything
 *    is launched.  dcnn_last_error() gives a text for the last failure of a context.
 *  - All work is enqueued on the context's HIP stream; no call synchronises except
 *    dcnn_layer_stats, dcnn_net_stats and dcnn_ctx_sync.  Calls on one context must not overlap.
 *  - Results are deterministic run to run: no floating-point atomics, ordered compaction.
 *  - fp16 tensors are stored as IEEE binary16 and all arithmetic is done in fp32 with one
 *    round-to-nearest-even at each store; thresholds are fp32.
 */
#ifndef DELTACNN_H
#define DELTACNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DCNN_OK = 0,
    DCNN_EINVAL = 1,        /* null pointer, bad enum, bad size */
    DCNN_ESHAPE = 2,        /* shapes of inputs / descriptor do not fit together */
    DCNN_EDTYPE = 3,
    DCNN_ESTATE = 4,        /* step before init, object not bound, ... */
    DCNN_ENOMEM = 5,        /* a caller-provided buffer is too small */
    DCNN_EHIP = 6,          /* a HIP call failed; text in dcnn_last_error */
    DCNN_EUNSUPPORTED = 7
} dcnn_status;

typedef enum { DCNN_F32 = 0, DCNN_F16 = 1 } dcnn_dtype;

typedef enum {
    DCNN_DELTAGEN = 0,      /* input layer: dense frame -> (delta, mask)            Fig. 2; Section 4   */
    DCNN_CONV = 1,          /* k x k dense-weight convolution on deltas              Section 3.1, Eq. 1  */
    DCNN_DWCONV = 2,        /* k x k depthwise convolution on deltas                 suppl. Section 1.2  */
    DCNN_ACT = 3,           /* activation + truncation, optionally of a sum of two   Section 3.1 Eqs 4-6 */
    DCNN_MAXPOOL = 4,       /* max pooling with accumulated-input buffer             Section 3.1, Eq. 3  */
    DCNN_UPSAMPLE = 5,      /* nearest-neighbour upsampling                          Section 3.4         */
    DCNN_ACCUM = 6,         /* output layer: deltas accumulated into a dense map     Fig. 2              */
    DCNN_CONCAT = 7,        /* channel concatenation of two updates (linear)         Section 3.4         */
    DCNN_UPSAMPLE_BILINEAR = 8, /* bilinear upsampling, half-pixel centres (linear)  Section 3.4         */
    DCNN_GAVGPOOL = 9       /* global average pooling to a 1x1 map (linear)          Section 3.4         */
} dcnn_kind;

typedef enum { DCNN_ACT_NONE = 0, DCNN_ACT_RELU = 1, DCNN_ACT_RELU6 = 2 } dcnn_act;

/* A sparse update.  All pointers are device pointers owned by the caller (or, for a layer's
 * output, carved by the library out of the layer's caller-provided state memory).
 * idx has room for n*h*w entries.  For DCNN_DELTAGEN the single input is a dense frame:
 * only `data` and the shape are used. */
typedef struct {
    void*    data;          /* [n,h,w,c] NHWC                                      */
    uint8_t* mask;          /* [n,h,w], 0/1                                         */
    int32_t* idx;           /* ascending flagged pixel indices, first *count valid  */
    int32_t* count;         /* number of flagged pixels; NULL where it is not produced (see want_idx) */
    int32_t  n, h, w, c;
    int32_t  dtype;         /* dcnn_dtype                                           */
} dcnn_delta;

/* One layer.  n,h,w,c is the shape of the (first) input.
 *  CONV / DWCONV : kh = kw in 1..7 (odd windows for CONV in the networks here; DWCONV also serves 2x2 average
 *                  pooling), stride in {1,2}, pad < k; cout (DWCONV: cout == c).
 *                  act != NONE fuses activation + truncation (threshold eps) behind the
 *                  convolution; n_in == 2 adds a second delta stream of the OUTPUT shape
 *                  (residual) before the activation.
 *  ACT           : n_in in {1,2}: activation + truncation of the input / of the sum of both.
 *                  act == NONE with n_in == 2 is a plain, stateless add.
 *  DELTAGEN      : eps is the input threshold, dilate_r the radius of the square mask dilation.
 *  MAXPOOL       : kh, stride, pad.     UPSAMPLE : factor.     ACCUM : nothing else.
 *  UPSAMPLE_BILINEAR : factor (2..16); an output pixel is flagged iff a source pixel that carries
 *                  weight is flagged.   GAVGPOOL : nothing else; output [n, 1, 1, c].
 *  CONCAT        : n_in == 2; c = channels of input 0, cout = c + channels of input 1.  The output
 *                  mask is the OR of both; a stream that is not flagged at a pixel contributes zeros.
 * The update rule is "update iff max_c |dy_c| >= eps": eps < 0 updates every visited pixel,
 * eps = +infinity none. */
typedef struct {
    int32_t kind;           /* dcnn_kind  */
    int32_t dtype;          /* dcnn_dtype */
    int32_t n, h, w, c;
    int32_t kh, kw, stride, pad, cout;
    int32_t act;            /* dcnn_act   */
    float   eps;
    int32_t n_in;
    int32_t dilate_r;
    int32_t factor;
    int32_t want_idx;       /* 0: the output's idx/count need not be produced (no consumer reads them): a layer with
                             * an activation then hands out count = NULL, and dcnn_layer_stats counts its mask */
    /* Optional fused projection shortcut (CONV with activation and n_in == 2 only; 0 = none): input 1 is
     * then not a residual of the output shape but the [n, proj_h, proj_w, proj_c] input of a 1x1
     * convolution (stride proj_stride, no padding, proj_c -> cout) whose result is added before the
     * activation -- conv_a(x) + conv_b(z) is linear in both deltas (Section 3.1, Eq. 1).  Each of the two
     * results is rounded to the storage type before the addition, as if it had been stored. */
    int32_t proj_c, proj_h, proj_w, proj_stride;
    /* 1: the layer also is the network's output layer (Fig. 2): it keeps the dense accumulated output O
     * (state buffer 2, dcnn_layer_output's data) and adds every delta it emits to it instead of storing
     * the delta.  CONV with activation and without a residual input only. */
    int32_t fuse_accum;
    /* 1: a layer with an activation keeps no buffer of truncated values x^T (Section 6: the buffer can be
     * left out to save memory): a truncated update is dropped, an update is x^A <- x^A + dx.  Small changes
     * below the threshold are then lost instead of accumulated (Eq. 6 does not hold). */
    int32_t no_xT;
    /* 1: on an update the layer keeps in x^T what the stored x^A lost to rounding, x^T <- s - round(s), instead
     * of 0 (s = x^A + x^T + dx in fp32; Eq. 6 then holds to the precision of the arithmetic rather than of the
     * storage type, which removes the slow error growth of long runs in fp16 -- supplementary Section 1.4).
     * The emitted delta and the threshold test are unchanged.  Layers with an activation and an x^T buffer
     * only; with fp32 storage the residue is zero and the option changes nothing.  x^T rows are then read and
     * written at every visited pixel. */
    int32_t xT_residue;
} dcnn_layer_desc;

typedef struct {
    size_t  state_bytes;    /* persistent per-layer device memory (buffers + outputs + packed weights) */
    int32_t on, oh, ow, oc; /* output shape */
} dcnn_layer_sizes;

/* Counters of the last step of a layer (Section 5 reports the same quantities per network). */
typedef struct {
    int64_t pixels_in;      /* flagged pixels of input 0                       */
    int64_t pixels_in2;     /* flagged pixels of input 1 (0 if there is none)  */
    int64_t pixels_work;    /* pixels the layer visited (its work list)        */
    int64_t pixels_out;     /* flagged pixels of the output                    */
    int64_t pixels_total;   /* n*h*w of the output                             */
    int64_t pixels_in_total;/* n*h*w of input 0                                */
    int64_t pixels_in2_total;/* n*h*w of input 1 (0 if there is none)           */
    int32_t kind;           /* dcnn_kind of the layer                          */
    int32_t act;            /* fused activation (dcnn_act)                     */
    int32_t n_in;
    int32_t c_in, c_out;    /* channels                                        */
    int32_t k, stride;      /* window (convolutions, pooling), else 1          */
    int32_t proj_c;         /* channels of the fused projection's input (input 1), 0 if none */
    int32_t fuse_accum;     /* 1: the layer also accumulates the dense output             */
    int32_t reserved;
    /* Bytes of the truncated-values buffer x^T the last step read / wrote, in whole pixel rows.  Only counted
     * while dcnn_layer_set_counting is on, and only by convolutions whose sparse steps skip x^T rows that are
     * all zero (an update leaves zeros); otherwise both are -1: x^T is read and written at every visited pixel. */
    int64_t xT_bytes_read;
    int64_t xT_bytes_written;
} dcnn_stats;

typedef struct dcnn_ctx dcnn_ctx;
typedef struct dcnn_layer dcnn_layer;
typedef struct dcnn_net dcnn_net;

/* ---- context ------------------------------------------------------------------------------- */
/* hip_stream: a hipStream_t (may be NULL = default stream), borrowed.  workspace_dev: scratch
 * shared by all layers of the context (partial counts, survivor bits); dcnn_workspace_bytes(p)
 * is enough for any layer whose output has at most p = n*h*w pixels.  All work of one context is
 * issued to its one stream; the workspace must not be used by anything else meanwhile. */
size_t      dcnn_workspace_bytes(int64_t max_pixels);
dcnn_status dcnn_ctx_create(void* hip_stream, void* workspace_dev, size_t workspace_bytes, dcnn_ctx** out);
void        dcnn_ctx_destroy(dcnn_ctx* ctx);
dcnn_status dcnn_ctx_sync(dcnn_ctx* ctx);
const char* dcnn_status_str(dcnn_status s);
const char* dcnn_last_error(const dcnn_ctx* ctx);

/* ---- mask propagation + ordered compaction (Section 3.2 "Update mask"; Section 3.3) ---------- */
/* mask_out[o] = OR of mask_in over the in-bounds taps of the k x k window of output pixel o
 * (k = 1, stride 1, pad 0: a copy), optionally OR-ed with mask_b (a second mask of the OUTPUT
 * shape, may be NULL); then idx_out = ascending indices of the flagged output pixels and
 * *count_out their number.  mask_out may be NULL (only the list is wanted).  Output shape:
 * oh = (h + 2*pad - k)/stride + 1, same for ow. */
dcnn_status dcnn_mask_compact(dcnn_ctx* ctx, const uint8_t* mask_in_dev, int32_t n, int32_t h, int32_t w,
                              int32_t k, int32_t stride, int32_t pad, const uint8_t* mask_b_dev,
                              uint8_t* mask_out_dev, int32_t* idx_out_dev, int32_t* count_out_dev);

/* The same operation for callers that cannot allocate device memory or provide a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The chunk counts (and, when
 * mask_out_dev is NULL, the output mask) live in a static device array inside the library instead of the
 * context's workspace: 8 KiB + 4 MiB per GPU, held until the process ends; its device address is resolved
 * once per device by dcnn_ctx_create.  The context may have been created without a workspace.  Limit: at
 * most 4 Mi (4 * 2^20) OUTPUT pixels n*oh*ow per call, beyond which DCNN_ENOMEM is returned and nothing is
 * launched.  The call allocates and frees nothing and does not synchronise; every entry of the scratch that
 * is read has been written by the same call, so nothing is cleared between calls.  All calls on one GPU
 * share that GPU's array: calls that overlap on one GPU (different streams, different contexts) race.
 * Arguments, results and error behaviour are otherwise those of dcnn_mask_compact. */
dcnn_status dcnn_mask_compact_static(dcnn_ctx* ctx, const uint8_t* mask_in_dev, int32_t n, int32_t h, int32_t w,
                                     int32_t k, int32_t stride, int32_t pad, const uint8_t* mask_b_dev,
                                     uint8_t* mask_out_dev, int32_t* idx_out_dev, int32_t* count_out_dev);

/* ---- layers -------------------------------------------------------------------------------- */
dcnn_status dcnn_layer_query(const dcnn_layer_desc* desc, dcnn_layer_sizes* out);
/* weights_dev: CONV [kh][kw][cin][cout], DWCONV [kh][kw][c]; bias_dev [cout] or NULL; with a fused
 * projection the [proj_c][cout] weights follow the main ones and bias_dev is [2][cout].  Both of the
 * layer's dtype, read once here (packed into state memory) -- they may be freed after
 * dcnn_ctx_sync.  state_dev: at least state_bytes from dcnn_layer_query, zero-filled or not. */
dcnn_status dcnn_layer_create(dcnn_ctx* ctx, const dcnn_layer_desc* desc, const void* weights_dev,
                              const void* bias_dev, void* state_dev, size_t state_bytes, dcnn_layer** out);
void        dcnn_layer_destroy(dcnn_layer* layer);
/* Frame 1 (Fig. 2): dense inputs -> dense output (the layer's ordinary definition, with bias),
 * and the layer's buffers are initialised (x^A <- dense input of the non-linearity, x^T <- 0,
 * input layer: stored frame, output layer: dense output).  dense_out_dev has the output shape.
 * Afterwards the layer's sparse output is empty (mask 0, count 0). */
dcnn_status dcnn_layer_init(dcnn_layer* layer, const void* const* dense_in_dev, int32_t n_in, void* dense_out_dev);
/* Frames >= 2: consume sparse inputs, update the buffers, produce the sparse output, which
 * lives in the layer's state memory and is described by dcnn_layer_output.  For DCNN_ACCUM the
 * output's data is the dense accumulated map (all pixels valid).  The view is that of the LAST step: ask
 * again after every step (a layer may alternate between two mask arrays), and read it before the next. */
dcnn_status dcnn_layer_step(dcnn_layer* layer, const dcnn_delta* const* in, int32_t n_in);
dcnn_status dcnn_layer_output(const dcnn_layer* layer, dcnn_delta* out_view);
/* Forget the buffers: the next call must be dcnn_layer_init (supplementary Section 1.4). */
dcnn_status dcnn_layer_reset(dcnn_layer* layer);
/* Replace the truncation threshold of a layer that has one (DCNN_DELTAGEN, or any layer with an
 * activation): thresholds are per layer and tuned front to back (Section 4).  Takes effect at the next
 * step; the buffers are kept.  DCNN_EINVAL for NaN or for a layer without a threshold. */
dcnn_status dcnn_layer_set_eps(dcnn_layer* layer, float eps);
/* which: 0 = x^A (ACT/CONV+act/MAXPOOL), stored frame (DELTAGEN), dense output (ACCUM); 1 = x^T;
 * 2 = dense output of a layer with fuse_accum.
 * Returns the device pointer and byte size of that buffer inside the state memory.
 * Writing through the pointer (restoring a checkpoint, teacher forcing) is allowed between steps, with one
 * rule for x^T: the library keeps, per pixel, whether the x^T row is all zero and skips such rows; it rebuilds
 * that knowledge from x^T before the next step ONLY IF dcnn_layer_state(which = 1) has been called since the
 * last step.  So call dcnn_layer_state(layer, 1, ...) again before EVERY external write of x^T -- a pointer
 * kept from an earlier call must not be written through after a step has run in between. */
dcnn_status dcnn_layer_state(const dcnn_layer* layer, int32_t which, void** ptr_dev, size_t* bytes);
/* Counters of the last step; synchronises the stream. */
dcnn_status dcnn_layer_stats(dcnn_layer* layer, dcnn_stats* stats_host);
/* Kernel timing for measurements: with max_steps > 0 the layer brackets its main compute kernel
 * (not its mask passes; for the delta generation layer: the generation pass together with the
 * list emission that belongs to it) with HIP events on the context's stream for up to max_steps
 * steps; 0 switches it off.  dcnn_layer_timing synchronises, reports the summed kernel time and the
 * number of timed launches since the last call, and starts over. */
dcnn_status dcnn_layer_set_timing(dcnn_layer* layer, int32_t max_steps);
/* Statistics for measurements: with on = 1 every step of the layer also counts the x^T rows its kernel reads and
 * writes (two small extra launches around the main kernel -- keep it off in timed runs); see dcnn_stats. */
dcnn_status dcnn_layer_set_counting(dcnn_layer* layer, int32_t on);
dcnn_status dcnn_layer_timing(dcnn_layer* layer, float* total_ms_host, int32_t* launches_host);

/* ---- networks ------------------------------------------------------------------------------ */
/* A network is a DAG of plain nodes (kinds above with act/n_in unfused: CONV has no activation,
 * ACT has one input, adds are ACT nodes with act NONE and two inputs).  dcnn_net_finalize fuses
 * conv -> (add) -> act chains into single layers and plans the buffers. */
dcnn_status dcnn_net_create(dcnn_ctx* ctx, int32_t dtype, int32_t n, int32_t h, int32_t w, int32_t c, dcnn_net** out);
void        dcnn_net_destroy(dcnn_net* net);
/* inputs: node ids returned by earlier calls (none for DELTAGEN).  weights/bias as in
 * dcnn_layer_create, DEVICE pointers that must stay valid until dcnn_net_bind has returned and
 * the context has been synchronised.  Returns the node id in *node_id. */
dcnn_status dcnn_net_add(dcnn_net* net, const dcnn_layer_desc* desc, const int32_t* inputs, int32_t n_inputs,
                         const void* weights_dev, const void* bias_dev, int32_t* node_id);
/* flags: bit 0 fuses conv -> (add) -> activation chains into one layer (otherwise every node is a
 * layer of its own); bit 1 makes every layer produce its output index list even when no consumer
 * reads it; bit 2 runs independent branches of the graph on up to three HIP streams (the context's own
 * plus streams the network creates at dcnn_net_bind, all at the default priority; each gets a workspace
 * of its own inside the arena; every dcnn_net_init / dcnn_net_step starts behind the work already on the
 * context's stream and the context's stream continues behind all of them, so callers see one stream).
 * Results do not depend on the flags.  Reports the arena size. */
dcnn_status dcnn_net_finalize(dcnn_net* net, int32_t flags, size_t* arena_bytes);
dcnn_status dcnn_net_bind(dcnn_net* net, void* arena_dev, size_t arena_bytes);
/* First frame / later frames.  frame_dev: dense [n,h,w,c].  out_dev: dense output of the last
 * node, or NULL (the dense output also lives in the arena: dcnn_net_output). */
dcnn_status dcnn_net_init(dcnn_net* net, const void* frame_dev, void* out_dev);
dcnn_status dcnn_net_step(dcnn_net* net, const void* frame_dev, void* out_dev);
dcnn_status dcnn_net_reset(dcnn_net* net);
dcnn_status dcnn_net_output(const dcnn_net* net, dcnn_delta* out_view);
int32_t     dcnn_net_num_layers(const dcnn_net* net);
/* Layer i of the fused plan, and the node id whose output it produces. */
dcnn_status dcnn_net_layer(const dcnn_net* net, int32_t i, dcnn_layer** layer, int32_t* node_id);
/* Per-layer counters of the last step, stats_host[dcnn_net_num_layers]; synchronises. */
dcnn_status dcnn_net_stats(dcnn_net* net, dcnn_stats* stats_host);

#ifdef __cplusplus
}
#endif
#endif /* DELTACNN_H */
