// Layer objects: validation, carve-up of the caller-provided state memory, and the launch
// sequence of one layer for the first (dense) frame and for later (sparse) frames.
#include <new>

#include "layer.h"

using namespace dcnn;

namespace dcnn {

static bool has_act(const dcnn_layer_desc& d) { return d.act != DCNN_ACT_NONE; }
static bool has_proj(const dcnn_layer_desc& d) { return d.proj_c > 0; }

// Does the layer build a work list of its own (window dilation / union of two masks), or does
// it walk the index list of its first input as it is?
static bool own_list(const dcnn_layer_desc& d) {
    switch (d.kind) {
        case DCNN_CONV:
        case DCNN_DWCONV: return !(d.kh == 1 && d.stride == 1 && d.n_in == 1);
        case DCNN_ACT: return d.n_in == 2;
        case DCNN_MAXPOOL:
        case DCNN_UPSAMPLE:
        case DCNN_UPSAMPLE_BILINEAR:
        case DCNN_GAVGPOOL:
        case DCNN_CONCAT: return true;
        default: return false;
    }
}

static dcnn_status out_shape(const dcnn_layer_desc& d, int* oh, int* ow, int* oc) {
    *oh = d.h; *ow = d.w; *oc = d.c;
    switch (d.kind) {
        case DCNN_CONV:
        case DCNN_DWCONV:
        case DCNN_MAXPOOL:
            if (d.kh < 1 || d.kh > 7 || d.kw != d.kh || d.stride < 1 || d.stride > 2 || d.pad < 0 || d.pad >= d.kh)
                return DCNN_EINVAL;
            if (d.h + 2 * d.pad < d.kh || d.w + 2 * d.pad < d.kh) return DCNN_ESHAPE;
            *oh = (d.h + 2 * d.pad - d.kh) / d.stride + 1;
            *ow = (d.w + 2 * d.pad - d.kh) / d.stride + 1;
            if (d.kind != DCNN_MAXPOOL) {
                if (d.cout < 1) return DCNN_EINVAL;
                if (d.kind == DCNN_DWCONV && d.cout != d.c) return DCNN_ESHAPE;
                *oc = d.cout;
            }
            return DCNN_OK;
        case DCNN_CONCAT:
            if (d.cout <= d.c) return DCNN_EINVAL;
            *oc = d.cout;
            return DCNN_OK;
        case DCNN_UPSAMPLE:
        case DCNN_UPSAMPLE_BILINEAR:
            if (d.factor < (d.kind == DCNN_UPSAMPLE ? 1 : 2) || d.factor > 16) return DCNN_EINVAL;
            *oh = d.h * d.factor; *ow = d.w * d.factor;
            return DCNN_OK;
        case DCNN_GAVGPOOL:
            if (d.n > 65535) return DCNN_ESHAPE;
            *oh = 1; *ow = 1;
            return DCNN_OK;
        default: return DCNN_OK;
    }
}

static dcnn_status validate_desc(const dcnn_layer_desc& d) {
    if (d.kind < DCNN_DELTAGEN || d.kind > DCNN_GAVGPOOL) return DCNN_EINVAL;
    if (d.dtype != DCNN_F32 && d.dtype != DCNN_F16) return DCNN_EDTYPE;
    if (d.n < 1 || d.h < 1 || d.w < 1 || d.c < 1) return DCNN_ESHAPE;
    if ((int64_t)d.n * d.h * d.w > INT32_MAX / 4) return DCNN_ESHAPE;
    if (d.act < DCNN_ACT_NONE || d.act > DCNN_ACT_RELU6) return DCNN_EINVAL;
    if (d.eps != d.eps) return DCNN_EINVAL;                               // NaN threshold
    switch (d.kind) {
        case DCNN_DELTAGEN: if (d.n_in != 0 && d.n_in != 1) return DCNN_EINVAL; break;
        case DCNN_CONV:
        case DCNN_DWCONV: if (d.n_in != 1 && d.n_in != 2) return DCNN_EINVAL; break;
        case DCNN_ACT:
            if (d.n_in != 1 && d.n_in != 2) return DCNN_EINVAL;
            if (d.n_in == 1 && d.act == DCNN_ACT_NONE) return DCNN_EINVAL;  // would be the identity
            break;
        case DCNN_CONCAT: if (d.n_in != 2 || d.act != DCNN_ACT_NONE) return DCNN_EINVAL; break;
        default: if (d.n_in != 1) return DCNN_EINVAL;
    }
    int oh, ow, oc;
    const dcnn_status st = out_shape(d, &oh, &ow, &oc);
    if (st != DCNN_OK) return st;
    if (d.proj_c < 0) return DCNN_EINVAL;
    if (has_proj(d)) {
        if (d.kind != DCNN_CONV || d.n_in != 2 || d.act == DCNN_ACT_NONE) return DCNN_EINVAL;
        if (d.proj_stride < 1 || d.proj_stride > 2 || d.proj_h < 1 || d.proj_w < 1) return DCNN_EINVAL;
        if ((d.proj_h - 1) / d.proj_stride + 1 != oh || (d.proj_w - 1) / d.proj_stride + 1 != ow) return DCNN_ESHAPE;
    }
    if (d.fuse_accum != 0 && d.fuse_accum != 1) return DCNN_EINVAL;
    if (d.no_xT != 0 && d.no_xT != 1) return DCNN_EINVAL;
    if (d.no_xT && (d.act == DCNN_ACT_NONE || d.kind == DCNN_DELTAGEN)) return DCNN_EINVAL;
    if (d.xT_residue != 0 && d.xT_residue != 1) return DCNN_EINVAL;
    if (d.xT_residue && (d.act == DCNN_ACT_NONE || d.kind == DCNN_DELTAGEN || d.no_xT)) return DCNN_EINVAL;
    if (d.fuse_accum && (d.kind != DCNN_CONV || d.act == DCNN_ACT_NONE || (d.n_in == 2 && !has_proj(d)))) return DCNN_EINVAL;
    return DCNN_OK;
}

// Walks the state memory and hands out aligned pieces; with base == nullptr it only measures.
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* b) : base(static_cast<char*>(b)) {}
    void* take(size_t bytes) {
        void* p = base ? base + off : nullptr;
        off += align_up(bytes);
        return p;
    }
};

// Do the sparse steps of this convolution run on the wave-specialised kernel?  (The same conditions the launcher
// tests; they depend on the description only.)
static bool ws_steps(const dcnn_layer_desc& d, int64_t in_pixels, int64_t out_pixels, int oc) {
    if (has_proj(d))
        return conv_proj_supported(nullptr, d.dtype, d.kh, d.c, d.proj_c, oc, in_pixels * d.c,
                                   (int64_t)d.n * d.proj_h * d.proj_w * d.proj_c, out_pixels * oc);
    return conv_ws_supported(nullptr, d.dtype, d.kh, d.c, oc, in_pixels * d.c, out_pixels * oc);
}

static void carve(dcnn_layer* L, void* state) {
    const dcnn_layer_desc& d = L->d;
    const size_t es = dtype_size(d.dtype);
    Carver cv(state);
    const size_t in_map = (size_t)L->in_pixels * d.c * es;
    const size_t out_map = (size_t)L->out_pixels * L->oc * es;
    const bool act = has_act(d), own = own_list(d);
    L->buf0 = L->buf1 = L->buf2 = nullptr; L->buf0_bytes = L->buf1_bytes = L->buf2_bytes = 0;
    L->out_data = nullptr; L->out_mask = nullptr; L->out_idx = nullptr; L->out_count = nullptr;
    L->out_mask_alt = nullptr; L->mask_phase = 0;
    L->list = nullptr; L->list_count = nullptr; L->taps = nullptr; L->wpacked = nullptr; L->bias = nullptr;
    L->wpacked2 = nullptr; L->wpacked2_dense = nullptr; L->bias2 = nullptr; L->xt_flags = nullptr;
    L->counters = static_cast<int32_t*>(cv.take(kAlign));      // stays all zero: doubles as the zero page of the gathers
    switch (d.kind) {
        case DCNN_DELTAGEN:
            L->buf0 = cv.take(in_map); L->buf0_bytes = in_map;
            break;
        case DCNN_CONV:
        case DCNN_DWCONV:
        case DCNN_ACT:
            if (act) {
                L->buf0 = cv.take(out_map); L->buf0_bytes = out_map;
                if (!d.no_xT) { L->buf1 = cv.take(out_map); L->buf1_bytes = out_map; }
            }
            if (d.fuse_accum) { L->buf2 = cv.take(out_map); L->buf2_bytes = out_map; }
            if (act && !d.no_xT && d.kind == DCNN_CONV && ws_steps(d, L->in_pixels, L->out_pixels, L->oc))
                L->xt_flags = static_cast<uint8_t*>(cv.take((size_t)L->out_pixels));
            break;
        case DCNN_MAXPOOL:
            L->buf0 = cv.take(in_map); L->buf0_bytes = in_map;
            break;
        case DCNN_ACCUM:
            L->buf0 = cv.take(out_map); L->buf0_bytes = out_map;
            break;
        default: break;
    }
    if (d.kind != DCNN_ACCUM) {
        L->out_data = cv.take(out_map);
        // a stateless, mask-preserving layer (1x1 s1 conv without activation) forwards its input's
        // mask and index list; every other layer owns them
        L->alias_mask = !act && !own && (d.kind == DCNN_CONV || d.kind == DCNN_DWCONV);
        if (!L->alias_mask) {
            L->out_mask = static_cast<uint8_t*>(cv.take((size_t)L->out_pixels));
            L->out_idx = static_cast<int32_t*>(cv.take((size_t)L->out_pixels * sizeof(int32_t)));
            L->out_count = static_cast<int32_t*>(cv.take(kAlign));
            // A convolution or activation that walks its input's own list and truncates needs an output mask that is 0
            // wherever it does not write.  Instead of a mask pass per step it alternates between two masks, and
            // its kernel clears the one of the next step while it runs (clear_ahead).
            if (act && !own && (d.kind == DCNN_CONV || d.kind == DCNN_ACT))
                L->out_mask_alt = static_cast<uint8_t*>(cv.take((size_t)L->out_pixels));
        }
        if (own) {
            if (act) {                                            // work list distinct from the output list
                L->list = static_cast<int32_t*>(cv.take((size_t)L->out_pixels * sizeof(int32_t)));
                L->list_count = static_cast<int32_t*>(cv.take(kAlign));
            } else {
                L->list = L->out_idx;
                L->list_count = L->out_count;
            }
            if (d.kind == DCNN_CONV && (d.kh == 1 || d.kh == 3))
                L->taps = static_cast<uint32_t*>(cv.take((size_t)L->out_pixels * sizeof(uint32_t)));
        }
    } else {
        L->alias_mask = true;
    }
    if (d.kind == DCNN_CONV || d.kind == DCNN_DWCONV) {
        L->wpacked = cv.take(conv_packed_weight_bytes(d.dtype, d.kh, d.c, L->oc, d.kind == DCNN_DWCONV, act));
        L->bias = cv.take((size_t)L->oc * es);
        if (has_proj(d)) {
            L->wpacked2 = cv.take(conv_proj_weight_bytes(d.dtype, d.kh, d.c, d.proj_c, L->oc));
            L->wpacked2_dense = cv.take(conv_packed_weight_bytes(d.dtype, 1, d.proj_c, L->oc, 0, false));
            L->bias2 = cv.take((size_t)L->oc * es);
        }
    }
    L->state_bytes = cv.off;
}

// the block that holds a layer's output count also holds, 64 bytes in, two 64-bit counters of x^T vectors read / written
constexpr int kXtIoOffset = 16;                                  // in int32 units
constexpr int kStatsScratchOffset = 8;                           // where dcnn_layer_stats counts a mask that came without a count

static dcnn_status clear_sparse_output(dcnn_layer* L) {
    if (L->alias_mask) return DCNN_OK;
    dcnn_status st = launch_fill_u8(L->ctx, L->out_mask, 0, (int64_t)align_up((size_t)L->out_pixels, 4));
    if (st == DCNN_OK && L->out_mask_alt) st = launch_fill_u8(L->ctx, L->out_mask_alt, 0, (int64_t)align_up((size_t)L->out_pixels, 4));
    L->mask_phase = 0;
    if (st != DCNN_OK) return st;
    st = launch_fill_i32(L->ctx, L->out_count, 0, kXtIoOffset + 4);     // the count, the statistics scratch and the x^T row counters behind it
    if (st != DCNN_OK) return st;
    if (L->list_count && L->list_count != L->out_count) st = launch_fill_i32(L->ctx, L->list_count, 0, 1);
    return st;
}

static ListArgs full_list(int64_t pixels) {
    ListArgs l{};
    l.list = nullptr; l.count = nullptr; l.count_host = pixels; l.max_count = pixels;
    return l;
}

static dcnn_status check_input(dcnn_layer* L, const dcnn_delta* in, int which, int h, int w, int c, bool need_idx) {
    dcnn_ctx* ctx = L->ctx;
    if (!in) return fail(ctx, DCNN_EINVAL, "step: input %d is null", which);
    if (in->dtype != L->d.dtype) return fail(ctx, DCNN_EDTYPE, "step: input %d has dtype %d, layer %d", which, in->dtype, L->d.dtype);
    if (in->n != L->d.n || in->h != h || in->w != w || in->c != c)
        return fail(ctx, DCNN_ESHAPE, "step: input %d is [%d,%d,%d,%d], expected [%d,%d,%d,%d]", which, in->n, in->h,
                    in->w, in->c, L->d.n, h, w, c);
    if (!in->data) return fail(ctx, DCNN_EINVAL, "step: input %d has no data", which);
    if (L->d.kind != DCNN_DELTAGEN) {
        if (!in->mask) return fail(ctx, DCNN_EINVAL, "step: input %d has no mask", which);
        if (need_idx && (!in->idx || !in->count)) return fail(ctx, DCNN_EINVAL, "step: input %d has no index list", which);
    }
    return DCNN_OK;
}

}  // namespace dcnn

extern "C" {

dcnn_status dcnn_layer_query(const dcnn_layer_desc* desc, dcnn_layer_sizes* out) {
    if (!desc || !out) return DCNN_EINVAL;
    dcnn_status st = validate_desc(*desc);
    if (st != DCNN_OK) return st;
    dcnn_layer tmp{};
    tmp.d = *desc;
    out_shape(*desc, &tmp.oh, &tmp.ow, &tmp.oc);
    tmp.in_pixels = (int64_t)desc->n * desc->h * desc->w;
    tmp.out_pixels = (int64_t)desc->n * tmp.oh * tmp.ow;
    carve(&tmp, nullptr);
    out->state_bytes = tmp.state_bytes;
    out->on = desc->n; out->oh = tmp.oh; out->ow = tmp.ow; out->oc = tmp.oc;
    return DCNN_OK;
}

dcnn_status dcnn_layer_create(dcnn_ctx* ctx, const dcnn_layer_desc* desc, const void* weights_dev, const void* bias_dev,
                              void* state_dev, size_t state_bytes, dcnn_layer** out) {
    if (!ctx) return DCNN_EINVAL;
    if (!desc || !out) return fail(ctx, DCNN_EINVAL, "layer_create: null argument");
    // a fused projection's weights and bias follow the main ones
    const void* w2 = nullptr;
    const void* b2 = nullptr;
    if (desc->proj_c > 0 && desc->kind == DCNN_CONV && desc->cout > 0 && desc->kh > 0 && desc->c > 0 && weights_dev) {
        const size_t es = dtype_size(desc->dtype);
        w2 = static_cast<const char*>(weights_dev) + (size_t)desc->kh * desc->kh * desc->c * desc->cout * es;
        if (bias_dev) b2 = static_cast<const char*>(bias_dev) + (size_t)desc->cout * es;
    }
    return dcnn::layer_create(ctx, desc, weights_dev, bias_dev, w2, b2, state_dev, state_bytes, out);
}

}  // extern "C"

namespace dcnn {

dcnn_status layer_create(dcnn_ctx* ctx, const dcnn_layer_desc* desc, const void* weights_dev, const void* bias_dev,
                         const void* proj_weights_dev, const void* proj_bias_dev, void* state_dev, size_t state_bytes,
                         dcnn_layer** out) {
    *out = nullptr;
    dcnn_status st = validate_desc(*desc);
    if (st != DCNN_OK) return fail(ctx, st, "layer_create: invalid descriptor (kind %d)", desc->kind);
    if (!state_dev || (reinterpret_cast<uintptr_t>(state_dev) % kAlign) != 0)
        return fail(ctx, DCNN_EINVAL, "layer_create: state memory missing or not 256-byte aligned");
    dcnn_layer* L = new (std::nothrow) dcnn_layer();
    if (!L) return fail(ctx, DCNN_ENOMEM, "layer_create: host allocation failed");
    L->ctx = ctx;
    L->d = *desc;
    out_shape(*desc, &L->oh, &L->ow, &L->oc);
    L->in_pixels = (int64_t)desc->n * desc->h * desc->w;
    L->out_pixels = (int64_t)desc->n * L->oh * L->ow;
    L->inited = false;
    carve(L, state_dev);
    if (L->state_bytes > state_bytes) {
        st = fail(ctx, DCNN_ENOMEM, "layer_create: state memory of %zu bytes, need %zu", state_bytes, L->state_bytes);
        delete L;
        return st;
    }
    const bool conv = desc->kind == DCNN_CONV || desc->kind == DCNN_DWCONV;
    if (conv) {
        if (!weights_dev) { delete L; return fail(ctx, DCNN_EINVAL, "layer_create: convolution without weights"); }
        char why[256];
        if (!conv_supported(ctx, desc->dtype, desc->kh, desc->c, L->oc, desc->kind == DCNN_DWCONV, has_act(*desc), why,
                            sizeof(why))) {
            delete L;
            return fail(ctx, DCNN_EUNSUPPORTED, "layer_create: %s", why);
        }
        st = launch_pack_weights(ctx, desc->dtype, weights_dev, L->wpacked, desc->kh, desc->c, L->oc,
                                 desc->kind == DCNN_DWCONV, has_act(*desc));
        if (st == DCNN_OK && bias_dev) st = launch_copy(ctx, L->bias, bias_dev, (size_t)L->oc * dtype_size(desc->dtype));
        if (st == DCNN_OK && has_proj(*desc)) {
            const size_t es = dtype_size(desc->dtype);
            if (!conv_proj_supported(ctx, desc->dtype, desc->kh, desc->c, desc->proj_c, L->oc, L->in_pixels * desc->c,
                                     (int64_t)desc->n * desc->proj_h * desc->proj_w * desc->proj_c, L->out_pixels * L->oc) ||
                !conv_supported(ctx, desc->dtype, 1, desc->proj_c, L->oc, 0, false, why, sizeof(why))) {
                delete L;
                return fail(ctx, DCNN_EUNSUPPORTED, "layer_create: conv %dx%d %d->%d with a fused projection of %d channels is not covered",
                            desc->kh, desc->kh, desc->c, L->oc, desc->proj_c);
            }
            if (!proj_weights_dev) { delete L; return fail(ctx, DCNN_EINVAL, "layer_create: fused projection without weights"); }
            const void* w2 = proj_weights_dev;
            st = launch_pack_weights_proj(ctx, desc->dtype, w2, L->wpacked2, desc->kh, desc->c, desc->proj_c, L->oc);
            if (st == DCNN_OK) st = launch_pack_weights(ctx, desc->dtype, w2, L->wpacked2_dense, 1, desc->proj_c, L->oc, 0, false);
            if (st == DCNN_OK && proj_bias_dev) st = launch_copy(ctx, L->bias2, proj_bias_dev, (size_t)L->oc * es);
            L->has_bias2 = proj_bias_dev != nullptr;
        }
        if (st == DCNN_OK && desc->fuse_accum &&
            !conv_ws_supported(ctx, desc->dtype, desc->kh, desc->c, L->oc, L->in_pixels * desc->c, L->out_pixels * L->oc)) {
            delete L;
            return fail(ctx, DCNN_EUNSUPPORTED, "layer_create: conv %dx%d %d->%d with a fused final accumulation is not covered",
                        desc->kh, desc->kh, desc->c, L->oc);
        }
        if (st != DCNN_OK) { delete L; return st; }
        L->has_bias = bias_dev != nullptr;
    }
    if (desc->kind == DCNN_DELTAGEN && (desc->dilate_r < 0 || desc->dilate_r > 15)) {
        delete L;
        return fail(ctx, DCNN_EINVAL, "layer_create: input-mask dilation radius %d out of range (0..15)", desc->dilate_r);
    }
    st = clear_sparse_output(L);
    if (st == DCNN_OK) st = launch_fill_i32(ctx, L->counters, 0, kAlign / sizeof(int32_t));
    if (st != DCNN_OK) { delete L; return st; }
    *out = L;
    return DCNN_OK;
}

}  // namespace dcnn

extern "C" {

static void drop_events(dcnn_layer* L) {
    for (auto& e : L->events) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
    L->events.clear();
    L->events_used = 0;
}

void dcnn_layer_destroy(dcnn_layer* layer) {
    if (!layer) return;
    drop_events(layer);
    delete layer;
}

dcnn_status dcnn_layer_set_eps(dcnn_layer* L, float eps) {
    if (!L) return DCNN_EINVAL;
    if (eps != eps) return fail(L->ctx, DCNN_EINVAL, "set_eps: the threshold is NaN");
    if (L->d.kind != DCNN_DELTAGEN && L->d.act == DCNN_ACT_NONE)
        return fail(L->ctx, DCNN_EINVAL, "set_eps: the layer has no truncation threshold");
    L->d.eps = eps;
    return DCNN_OK;
}

dcnn_status dcnn_layer_set_timing(dcnn_layer* L, int32_t max_steps) {
    if (!L) return DCNN_EINVAL;
    if (max_steps < 0 || max_steps > 65536) return fail(L->ctx, DCNN_EINVAL, "set_timing: max_steps out of range");
    drop_events(L);
    for (int i = 0; i < max_steps; ++i) {
        hipEvent_t a, b;
        dcnn_status st = check_hip(L->ctx, hipEventCreate(&a), "hipEventCreate");
        if (st != DCNN_OK) return st;
        st = check_hip(L->ctx, hipEventCreate(&b), "hipEventCreate");
        if (st != DCNN_OK) { (void)hipEventDestroy(a); return st; }
        L->events.emplace_back(a, b);
    }
    return DCNN_OK;
}

dcnn_status dcnn_layer_set_counting(dcnn_layer* L, int32_t on) {
    if (!L) return DCNN_EINVAL;
    if (on != 0 && on != 1) return fail(L->ctx, DCNN_EINVAL, "set_counting: on must be 0 or 1");
    L->counting = on != 0;
    if (!on) L->counted = false;
    return DCNN_OK;
}

dcnn_status dcnn_layer_timing(dcnn_layer* L, float* total_ms, int32_t* launches) {
    if (!L || !total_ms || !launches) return DCNN_EINVAL;
    dcnn_status st = check_hip(L->ctx, hipStreamSynchronize(L->ctx->stream), "hipStreamSynchronize");
    if (st != DCNN_OK) return st;
    float sum = 0.0f;
    for (size_t i = 0; i < L->events_used; ++i) {
        float ms = 0.0f;
        st = check_hip(L->ctx, hipEventElapsedTime(&ms, L->events[i].first, L->events[i].second), "hipEventElapsedTime");
        if (st != DCNN_OK) return st;
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int32_t)L->events_used;
    L->events_used = 0;
    return DCNN_OK;
}

dcnn_status dcnn_layer_reset(dcnn_layer* layer) {
    if (!layer) return DCNN_EINVAL;
    layer->inited = false;
    return clear_sparse_output(layer);
}

dcnn_status dcnn_layer_init(dcnn_layer* L, const void* const* dense_in, int32_t n_in, void* dense_out) {
    if (!L) return DCNN_EINVAL;
    dcnn_ctx* ctx = L->ctx;
    const dcnn_layer_desc& d = L->d;
    const int want_in = d.kind == DCNN_DELTAGEN ? 1 : d.n_in;
    if (!dense_in || n_in != want_in) return fail(ctx, DCNN_EINVAL, "init: expected %d dense inputs, got %d", want_in, n_in);
    for (int i = 0; i < n_in; ++i)
        if (!dense_in[i]) return fail(ctx, DCNN_EINVAL, "init: dense input %d is null", i);
    if (!dense_out && d.kind != DCNN_ACCUM) return fail(ctx, DCNN_EINVAL, "init: dense output is null");
    const size_t es = dtype_size(d.dtype);
    dcnn_status st = DCNN_OK;
    switch (d.kind) {
        case DCNN_DELTAGEN:
            st = launch_copy(ctx, L->buf0, dense_in[0], L->buf0_bytes);
            if (st == DCNN_OK && dense_out != dense_in[0]) st = launch_copy(ctx, dense_out, dense_in[0], L->buf0_bytes);
            break;
        case DCNN_CONV:
        case DCNN_DWCONV: {
            if (has_proj(d)) {
                // the projection runs as a dense convolution of its own into the output buffer, which the
                // main convolution then reads as its residual (each pixel is read before it is rewritten)
                ConvArgs c2{};
                c2.in_data = dense_in[1]; c2.in_mask = nullptr; c2.wpacked = L->wpacked2_dense; c2.zero_page = L->counters;
                c2.n = d.n; c2.h = d.proj_h; c2.w = d.proj_w; c2.cin = d.proj_c; c2.oh = L->oh; c2.ow = L->ow; c2.cout = L->oc;
                c2.k = 1; c2.stride = d.proj_stride; c2.pad = 0; c2.depthwise = 0;
                EpilogueArgs e2{};
                e2.c = L->oc; e2.act = DCNN_ACT_NONE; e2.eps = 0.0f; e2.bias = L->has_bias2 ? L->bias2 : nullptr;
                e2.out_data = dense_out;
                st = launch_conv(ctx, d.dtype, true, full_list(L->out_pixels), c2, e2);
                if (st != DCNN_OK) break;
            }
            ConvArgs c{};
            c.in_data = dense_in[0]; c.in_mask = nullptr; c.wpacked = L->wpacked; c.zero_page = L->counters;
            c.n = d.n; c.h = d.h; c.w = d.w; c.cin = d.c; c.oh = L->oh; c.ow = L->ow; c.cout = L->oc;
            c.k = d.kh; c.stride = d.stride; c.pad = d.pad; c.depthwise = d.kind == DCNN_DWCONV;
            EpilogueArgs e{};
            e.c = L->oc; e.act = d.act; e.eps = d.eps; e.bias = L->has_bias ? L->bias : nullptr;
            e.res_data = d.n_in == 2 ? (has_proj(d) ? dense_out : dense_in[1]) : nullptr; e.res_mask = nullptr;
            e.xA = L->buf0; e.xT = L->buf1; e.out_data = dense_out; e.out_mask = nullptr; e.surv = nullptr;
            st = launch_conv(ctx, d.dtype, true, full_list(L->out_pixels), c, e);
            if (st == DCNN_OK && d.fuse_accum) st = launch_copy(ctx, L->buf2, dense_out, L->buf2_bytes);
            break;
        }
        case DCNN_ACT: {
            ActArgs a{dense_in[0], nullptr};
            EpilogueArgs e{};
            e.c = L->oc; e.act = d.act; e.eps = d.eps; e.bias = nullptr;
            e.res_data = d.n_in == 2 ? dense_in[1] : nullptr; e.res_mask = nullptr;
            e.xA = L->buf0; e.xT = L->buf1; e.out_data = dense_out;
            st = launch_act(ctx, d.dtype, true, full_list(L->out_pixels), a, e);
            break;
        }
        case DCNN_MAXPOOL: {
            st = launch_copy(ctx, L->buf0, dense_in[0], L->buf0_bytes);
            if (st != DCNN_OK) break;
            PoolArgs a{};
            a.in_data = nullptr; a.in_mask = nullptr; a.xA = L->buf0; a.out_data = dense_out;
            a.n = d.n; a.h = d.h; a.w = d.w; a.c = d.c; a.oh = L->oh; a.ow = L->ow; a.k = d.kh; a.stride = d.stride; a.pad = d.pad;
            st = launch_maxpool_out(ctx, d.dtype, true, full_list(L->out_pixels), a);
            break;
        }
        case DCNN_UPSAMPLE:
        case DCNN_UPSAMPLE_BILINEAR: {
            UpsampleArgs a{dense_in[0], dense_out, d.n, d.h, d.w, d.c, d.factor, d.kind == DCNN_UPSAMPLE_BILINEAR ? 1 : 0, nullptr};
            st = launch_upsample(ctx, d.dtype, full_list(L->out_pixels), a);
            break;
        }
        case DCNN_GAVGPOOL: {
            GapArgs a{dense_in[0], nullptr, dense_out, d.h * d.w, d.c};
            st = launch_gavgpool(ctx, d.dtype, full_list(L->out_pixels), a);
            break;
        }
        case DCNN_CONCAT: {
            ConcatArgs a{dense_in[0], dense_in[1], nullptr, nullptr, dense_out, d.c, d.cout - d.c};
            st = launch_concat(ctx, d.dtype, full_list(L->out_pixels), a);
            break;
        }
        case DCNN_ACCUM:
            st = launch_copy(ctx, L->buf0, dense_in[0], L->buf0_bytes);
            if (st == DCNN_OK && dense_out) st = launch_copy(ctx, dense_out, dense_in[0], L->buf0_bytes);
            break;
    }
    (void)es;
    if (st != DCNN_OK) return st;
    st = clear_sparse_output(L);
    if (st != DCNN_OK) return st;
    if (L->xt_flags) {                                        // the first frame leaves x^T all zero
        st = launch_fill_u8(ctx, L->xt_flags, 0, L->out_pixels);
        if (st != DCNN_OK) return st;
        L->xt_flags_stale = false;
    }
    L->inited = true;
    L->last_in_count = nullptr;
    L->last_in2_count = nullptr;
    L->last_in_mask = nullptr;
    L->last_in2_mask = nullptr;
    L->last_work_count = nullptr;
    L->view = dcnn_delta{};
    return DCNN_OK;
}

dcnn_status dcnn_layer_step(dcnn_layer* L, const dcnn_delta* const* in, int32_t n_in) {
    if (!L) return DCNN_EINVAL;
    dcnn_ctx* ctx = L->ctx;
    const dcnn_layer_desc& d = L->d;
    if (!L->inited) return fail(ctx, DCNN_ESTATE, "step: the layer has not seen a first frame (call init)");
    const int want_in = d.kind == DCNN_DELTAGEN ? 1 : d.n_in;
    if (!in || n_in != want_in) return fail(ctx, DCNN_EINVAL, "step: expected %d inputs, got %d", want_in, n_in);
    const bool act = has_act(d), own = own_list(d);
    dcnn_status st = check_input(L, in[0], 0, d.h, d.w, d.c, !own || d.kind == DCNN_MAXPOOL);
    if (st != DCNN_OK) return st;
    if (n_in == 2) {
        st = has_proj(d) ? check_input(L, in[1], 1, d.proj_h, d.proj_w, d.proj_c, false)
             : d.kind == DCNN_CONCAT ? check_input(L, in[1], 1, L->oh, L->ow, d.cout - d.c, false)
                                     : check_input(L, in[1], 1, L->oh, L->ow, L->oc, false);
        if (st != DCNN_OK) return st;
    }
    Workspace ws;
    st = workspace_view(ctx, L->out_pixels > L->in_pixels ? L->out_pixels : L->in_pixels, &ws);
    if (st != DCNN_OK) return st;

    // the output view (aliases are refreshed every step)
    dcnn_delta& v = L->view;
    v.n = d.n; v.h = L->oh; v.w = L->ow; v.c = L->oc; v.dtype = d.dtype;
    v.data = d.fuse_accum ? L->buf2 : L->out_data;
    // (a layer with two output masks: this step writes one, which is all zero, and clears the other for the next step)
    uint8_t* const mask_cur = (L->out_mask_alt && L->mask_phase) ? L->out_mask_alt : L->out_mask;
    uint8_t* const mask_next = L->out_mask_alt ? (L->mask_phase ? L->out_mask : L->out_mask_alt) : nullptr;
    v.mask = L->alias_mask ? in[0]->mask : mask_cur;
    v.idx = L->alias_mask ? in[0]->idx : L->out_idx;
    // A layer with an activation whose output list nobody walks (want_idx == 0) does not count its flagged outputs:
    // atomics on one counter are served one after the other (~2.4 ns each; a few thousand waves adding their share at
    // the end of a kernel cost 10-20 us), and nothing on a step's path needs the number.  Statistics count the mask.
    v.count = L->alias_mask ? in[0]->count : ((act && !d.want_idx) ? nullptr : L->out_count);
    L->last_in_count = in[0]->count;
    L->last_in2_count = n_in == 2 ? in[1]->count : nullptr;
    L->last_in_mask = in[0]->mask;
    L->last_in2_mask = n_in == 2 ? in[1]->mask : nullptr;

    if (d.kind == DCNN_DELTAGEN) {
        DeltaGenArgs a{};
        a.frame = in[0]->data; a.P = L->buf0; a.out_data = L->out_data; a.out_mask = L->out_mask;
        a.out_idx = L->out_idx; a.out_count = L->out_count; a.pixels = L->in_pixels;
        a.n = d.n; a.h = d.h; a.w = d.w; a.c = d.c; a.eps = d.eps; a.dilate_r = d.dilate_r;
        L->last_in_count = nullptr;
        L->last_work_count = L->out_count;
        // optional timing: the generation pass together with the list emission that belongs to it
        const bool timed_gen = L->events_used < L->events.size();
        if (timed_gen) {
            st = check_hip(ctx, hipEventRecord(L->events[L->events_used].first, ctx->stream), "hipEventRecord");
            if (st != DCNN_OK) return st;
        }
        st = launch_deltagen(ctx, d.dtype, a);
        if (st == DCNN_OK && timed_gen) {
            st = check_hip(ctx, hipEventRecord(L->events[L->events_used].second, ctx->stream), "hipEventRecord");
            if (st == DCNN_OK) ++L->events_used;
        }
        return st;
    }

    // ---- work list -----------------------------------------------------------------------------
    ListArgs l{};
    l.max_count = L->out_pixels;
    if (own) {
        MaskPassArgs m{};
        m.mask_in = in[0]->mask; m.mask_b = n_in == 2 ? in[1]->mask : nullptr;
        m.mask_out = L->out_mask; m.idx_out = L->list; m.count_out = L->list_count;
        m.n = d.n; m.h = d.h; m.w = d.w; m.oh = L->oh; m.ow = L->ow;
        m.k = 1; m.stride = 1; m.pad = 0; m.up = 1; m.emit_only = 0;
        m.zero_count = nullptr;
        if (d.kind == DCNN_CONV || d.kind == DCNN_DWCONV || d.kind == DCNN_MAXPOOL) { m.k = d.kh; m.stride = d.stride; m.pad = d.pad; }
        if (d.kind == DCNN_UPSAMPLE || d.kind == DCNN_UPSAMPLE_BILINEAR) { m.up = d.factor; m.bilinear = d.kind == DCNN_UPSAMPLE_BILINEAR; }
        if (d.kind == DCNN_GAVGPOOL) { m.k = d.h; m.kw = d.w; m.pad_w = 0; }   // one window over the whole map
        m.taps_out = L->taps;
        if (has_proj(d) && !(d.proj_stride == 1 && d.proj_h == L->oh && d.proj_w == L->ow)) {
            m.b_stride = d.proj_stride; m.b_h = d.proj_h; m.b_w = d.proj_w;
        }
        st = launch_mask_compact(ctx, m);
        if (st != DCNN_OK) return st;
        l.list = L->list; l.count = L->list_count; l.taps = L->taps;
    } else {
        l.list = in[0]->idx; l.count = in[0]->count;
        if (act && !mask_next) {
            // the truncation below rewrites the mask at the visited pixels only: start from a copy
            MaskPassArgs m{};
            m.mask_in = in[0]->mask; m.mask_out = L->out_mask; m.idx_out = nullptr;
            m.n = d.n; m.h = d.h; m.w = d.w; m.oh = L->oh; m.ow = L->ow; m.k = 1; m.stride = 1; m.pad = 0; m.up = 1;
            m.zero_count = nullptr;
            st = launch_mask_compact(ctx, m);
            if (st != DCNN_OK) return st;
        }
    }
    L->last_work_count = l.count;

    // ---- compute -------------------------------------------------------------------------------
    const bool timed = L->events_used < L->events.size();
    if (timed) {
        st = check_hip(ctx, hipEventRecord(L->events[L->events_used].first, ctx->stream), "hipEventRecord");
        if (st != DCNN_OK) return st;
    }
    switch (d.kind) {
        case DCNN_CONV:
        case DCNN_DWCONV: {
            ConvArgs c{};
            c.in_data = in[0]->data; c.in_mask = in[0]->mask; c.wpacked = L->wpacked; c.zero_page = L->counters;
            c.in_count = in[0]->count;
            c.n = d.n; c.h = d.h; c.w = d.w; c.cin = d.c; c.oh = L->oh; c.ow = L->ow; c.cout = L->oc;
            c.k = d.kh; c.stride = d.stride; c.pad = d.pad; c.depthwise = d.kind == DCNN_DWCONV;
            EpilogueArgs e{};
            e.c = L->oc; e.act = d.act; e.eps = d.eps; e.bias = nullptr;
            e.res_data = n_in == 2 ? in[1]->data : nullptr; e.res_mask = n_in == 2 ? in[1]->mask : nullptr;
            if (has_proj(d)) {
                c.in2_data = in[1]->data; c.wpacked2 = L->wpacked2;
                c.h2 = d.proj_h; c.w2 = d.proj_w; c.cin2 = d.proj_c; c.stride2 = d.proj_stride;
                e.res_data = nullptr; e.res_mask = nullptr;
            }
            e.xA = L->buf0; e.xT = L->buf1; e.out_data = L->out_data;
            e.accum_O = d.fuse_accum ? L->buf2 : nullptr;
            e.carry = d.xT_residue;
            if (L->xt_flags) {
                if (L->xt_flags_stale) {                          // the caller may have written x^T: look at it once
                    st = launch_row_flags(ctx, d.dtype, L->buf1, L->xt_flags, L->out_pixels, L->oc);
                    if (st != DCNN_OK) return st;
                    L->xt_flags_stale = false;
                }
                e.xt_flags = L->xt_flags;
            }
            e.out_mask = act ? mask_cur : nullptr;
            e.clear_mask = mask_next; e.clear_bytes = mask_next ? L->out_pixels : 0;
            e.surv = (act && d.want_idx) ? ws.surv : nullptr;
            e.out_count = nullptr;                                 // (see the output view above)
            // statistics mode: which x^T rows the kernel will read, and afterwards which it wrote
            const bool counting = L->counting && L->xt_flags && L->out_count && !timed;
            unsigned long long* io = counting ? reinterpret_cast<unsigned long long*>(L->out_count + kXtIoOffset) : nullptr;
            if (counting) {
                st = launch_fill_i32(ctx, L->out_count + kXtIoOffset, 0, 4);
                if (st == DCNN_OK) st = launch_xt_row_count(ctx, 0, l, L->xt_flags, ws.scratch_mask2, io);
                if (st != DCNN_OK) break;
            }
            st = launch_conv(ctx, d.dtype, false, l, c, e);
            if (st == DCNN_OK && counting) st = launch_xt_row_count(ctx, 1, l, L->xt_flags, ws.scratch_mask2, io);
            L->counted = counting;
            break;
        }
        case DCNN_ACT: {
            ActArgs a{in[0]->data, n_in == 2 ? in[0]->mask : nullptr};
            EpilogueArgs e{};
            e.c = L->oc; e.act = d.act; e.eps = d.eps;
            e.res_data = n_in == 2 ? in[1]->data : nullptr; e.res_mask = n_in == 2 ? in[1]->mask : nullptr;
            e.xA = L->buf0; e.xT = L->buf1; e.out_data = L->out_data;
            e.carry = d.xT_residue;
            e.out_mask = act ? mask_cur : nullptr;
            e.clear_mask = mask_next; e.clear_bytes = mask_next ? L->out_pixels : 0;
            e.surv = (act && d.want_idx) ? ws.surv : nullptr;
            e.out_count = nullptr;                                 // (see the output view above)
            st = launch_act(ctx, d.dtype, false, l, a, e);
            break;
        }
        case DCNN_MAXPOOL: {
            PoolArgs a{};
            a.in_data = in[0]->data; a.in_mask = in[0]->mask; a.xA = L->buf0; a.out_data = L->out_data;
            a.n = d.n; a.h = d.h; a.w = d.w; a.c = d.c; a.oh = L->oh; a.ow = L->ow; a.k = d.kh; a.stride = d.stride; a.pad = d.pad;
            st = launch_maxpool_out(ctx, d.dtype, false, l, a);
            if (st != DCNN_OK) break;
            ListArgs li{};
            li.list = in[0]->idx; li.count = in[0]->count; li.max_count = L->in_pixels;
            st = launch_maxpool_commit(ctx, d.dtype, li, a);
            break;
        }
        case DCNN_UPSAMPLE:
        case DCNN_UPSAMPLE_BILINEAR: {
            UpsampleArgs a{in[0]->data, L->out_data, d.n, d.h, d.w, d.c, d.factor, d.kind == DCNN_UPSAMPLE_BILINEAR ? 1 : 0, in[0]->mask};
            st = launch_upsample(ctx, d.dtype, l, a);
            break;
        }
        case DCNN_GAVGPOOL: {
            GapArgs a{in[0]->data, in[0]->mask, L->out_data, d.h * d.w, d.c};
            st = launch_gavgpool(ctx, d.dtype, l, a);
            break;
        }
        case DCNN_CONCAT: {
            ConcatArgs a{in[0]->data, in[1]->data, in[0]->mask, in[1]->mask, L->out_data, d.c, d.cout - d.c};
            st = launch_concat(ctx, d.dtype, l, a);
            break;
        }
        case DCNN_ACCUM: {
            AccumArgs a{in[0]->data, L->buf0, d.c};
            v.data = L->buf0;
            st = launch_accum(ctx, d.dtype, l, a);
            break;
        }
        default: return fail(ctx, DCNN_EINVAL, "step: bad layer kind");
    }
    if (st != DCNN_OK) return st;
    if (mask_next) L->mask_phase ^= 1;
    if (timed) {
        st = check_hip(ctx, hipEventRecord(L->events[L->events_used].second, ctx->stream), "hipEventRecord");
        if (st != DCNN_OK) return st;
        ++L->events_used;
    }
    // ---- ordered list of the pixels that stayed flagged ------------------------------------------
    if (act && d.want_idx && (d.kind == DCNN_CONV || d.kind == DCNN_DWCONV || d.kind == DCNN_ACT))
        st = launch_emit_sublist(ctx, l.list, l.count, L->out_pixels, ws.surv, L->out_idx, L->out_count);
    return st;
}

dcnn_status dcnn_layer_output(const dcnn_layer* L, dcnn_delta* out_view) {
    if (!L || !out_view) return DCNN_EINVAL;
    if (L->view.data == nullptr) {
        // before the first step: an empty update
        dcnn_delta v{};
        v.n = L->d.n; v.h = L->oh; v.w = L->ow; v.c = L->oc; v.dtype = L->d.dtype;
        v.data = L->d.kind == DCNN_ACCUM ? L->buf0 : (L->d.fuse_accum ? L->buf2 : L->out_data);
        v.mask = L->out_mask; v.idx = L->out_idx;
        v.count = (has_act(L->d) && !L->d.want_idx) ? nullptr : L->out_count;
        *out_view = v;
        return DCNN_OK;
    }
    *out_view = L->view;
    return DCNN_OK;
}

dcnn_status dcnn_layer_state(const dcnn_layer* L, int32_t which, void** ptr_dev, size_t* bytes) {
    if (!L || !ptr_dev || !bytes) return DCNN_EINVAL;
    if (which == 0 && L->buf0) { *ptr_dev = L->buf0; *bytes = L->buf0_bytes; return DCNN_OK; }
    if (which == 1 && L->buf1) { L->xt_flags_stale = true; *ptr_dev = L->buf1; *bytes = L->buf1_bytes; return DCNN_OK; }
    if (which == 2 && L->buf2) { *ptr_dev = L->buf2; *bytes = L->buf2_bytes; return DCNN_OK; }
    return fail(L->ctx, DCNN_EINVAL, "layer_state: the layer has no buffer %d", which);
}

dcnn_status dcnn_layer_stats(dcnn_layer* L, dcnn_stats* s) {
    if (!L || !s) return DCNN_EINVAL;
    dcnn_ctx* ctx = L->ctx;
    dcnn_status st = check_hip(ctx, hipStreamSynchronize(ctx->stream), "hipStreamSynchronize");
    if (st != DCNN_OK) return st;
    auto read = [&](const int32_t* p, int64_t* dst) -> dcnn_status {
        *dst = 0;
        if (!p) return DCNN_OK;
        int32_t v = 0;
        dcnn_status r = check_hip(ctx, hipMemcpy(&v, p, sizeof(v), hipMemcpyDeviceToHost), "hipMemcpy(count)");
        *dst = v;
        return r;
    };
    s->pixels_total = L->out_pixels;
    s->pixels_in_total = L->in_pixels;
    s->pixels_in2_total = L->d.n_in == 2 ? (L->d.proj_c > 0 ? (int64_t)L->d.n * L->d.proj_h * L->d.proj_w : L->out_pixels) : 0;
    // an update that comes without a count (see dcnn_layer_step): its mask is counted here, off every step's path
    int32_t* scratch = L->out_count ? L->out_count + kStatsScratchOffset : nullptr;
    auto read_or_count = [&](const int32_t* p, const uint8_t* mask, int64_t pixels, int64_t* dst) -> dcnn_status {
        if (p || !mask || !scratch) return read(p, dst);
        dcnn_status r = launch_mask_sum(ctx, mask, pixels, scratch);
        if (r == DCNN_OK) r = check_hip(ctx, hipStreamSynchronize(ctx->stream), "hipStreamSynchronize");
        return r == DCNN_OK ? read(scratch, dst) : r;
    };
    st = read_or_count(L->last_in_count, L->last_in_mask, s->pixels_in_total, &s->pixels_in);
    if (st == DCNN_OK) st = read_or_count(L->last_in2_count, L->last_in2_mask, s->pixels_in2_total, &s->pixels_in2);
    if (st == DCNN_OK) st = read(L->last_work_count, &s->pixels_work);
    if (st == DCNN_OK) st = read_or_count(L->view.count, L->view.mask, L->out_pixels, &s->pixels_out);
    s->kind = L->d.kind; s->act = L->d.act; s->n_in = L->d.n_in;
    s->c_in = L->d.c; s->c_out = L->oc;
    const bool window = L->d.kind == DCNN_CONV || L->d.kind == DCNN_DWCONV || L->d.kind == DCNN_MAXPOOL;
    s->k = window ? L->d.kh : 1; s->stride = window ? L->d.stride : 1; s->proj_c = L->d.proj_c; s->fuse_accum = L->d.fuse_accum; s->reserved = 0;
    s->xT_bytes_read = s->xT_bytes_written = -1;
    if (st == DCNN_OK && L->counted) {
        unsigned long long io[2] = {0, 0};
        st = check_hip(ctx, hipMemcpy(io, L->out_count + kXtIoOffset, sizeof(io), hipMemcpyDeviceToHost), "hipMemcpy(x^T counters)");
        const int64_t row = (int64_t)L->oc * (int64_t)dtype_size(L->d.dtype);
        s->xT_bytes_read = (int64_t)io[0] * row;
        s->xT_bytes_written = (int64_t)io[1] * row;
    }
    return st;
}

}  // extern "C"
