// Context, error reporting and workspace carve-up (host code).
#include <new>

#include "common.h"

namespace dcnn {

dcnn_status fail(dcnn_ctx* ctx, dcnn_status s, const char* fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

dcnn_status check_hip(dcnn_ctx* ctx, hipError_t e, const char* what) {
    if (e == hipSuccess) return DCNN_OK;
    return fail(ctx, DCNN_EHIP, "%s: %s", what, hipGetErrorString(e));
}

size_t workspace_bytes(int64_t max_pixels) {
    if (max_pixels < 1) max_pixels = 1;
    return align_up((size_t)cdiv(max_pixels, kChunk) * sizeof(int32_t)) +
           align_up((size_t)cdiv(max_pixels, kTile) * sizeof(uint32_t)) + 2 * align_up((size_t)max_pixels) + kAlign;
}

dcnn_status workspace_view(dcnn_ctx* ctx, int64_t pixels, Workspace* out) {
    if (!ctx->ws || workspace_bytes(pixels) > ctx->ws_bytes)
        return fail(ctx, DCNN_ENOMEM, "workspace of %zu bytes is too small for %lld pixels (need %zu)", ctx->ws_bytes,
                    (long long)pixels, workspace_bytes(pixels));
    // carve for the largest pixel count the workspace can hold, so every layer sees the same offsets
    char* p = ctx->ws;
    const size_t a = align_up((size_t)cdiv(pixels, kChunk) * sizeof(int32_t));
    const size_t b = align_up((size_t)cdiv(pixels, kTile) * sizeof(uint32_t));
    out->chunk_counts = reinterpret_cast<int32_t*>(p);
    out->surv = reinterpret_cast<uint32_t*>(p + a);
    out->scratch_mask = reinterpret_cast<uint8_t*>(p + a + b);
    out->scratch_mask2 = out->scratch_mask + align_up((size_t)pixels);
    out->max_pixels = pixels;
    return DCNN_OK;
}

}  // namespace dcnn

using namespace dcnn;

extern "C" {

size_t dcnn_workspace_bytes(int64_t max_pixels) { return workspace_bytes(max_pixels); }

dcnn_status dcnn_ctx_create(void* hip_stream, void* workspace_dev, size_t workspace_bytes, dcnn_ctx** out) {
    if (!out) return DCNN_EINVAL;
    *out = nullptr;
    if (workspace_dev && (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign) != 0) return DCNN_EINVAL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DCNN_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return DCNN_EHIP;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return DCNN_EUNSUPPORTED;   // kernels are built for CDNA4 only
    if (prop.sharedMemPerBlock < 160 * 1024) return DCNN_EUNSUPPORTED;           // the conv plans assume 160 KB of LDS
    // set-up of the entry point that allocates nothing: the address of this device's copy of the static scratch array
    if (static_scratch_setup(dev) != hipSuccess) return DCNN_EHIP;
    dcnn_ctx* c = new (std::nothrow) dcnn_ctx();
    if (!c) return DCNN_ENOMEM;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->device = dev;
    c->ws = static_cast<char*>(workspace_dev);
    c->ws_bytes = workspace_bytes;
    c->num_cu = prop.multiProcessorCount;
    c->max_lds = prop.sharedMemPerBlock;                // 160 KB on gfx950; the conv plans rely on it
    c->err[0] = 0;
    *out = c;
    return DCNN_OK;
}

void dcnn_ctx_destroy(dcnn_ctx* ctx) { delete ctx; }

dcnn_status dcnn_ctx_sync(dcnn_ctx* ctx) {
    if (!ctx) return DCNN_EINVAL;
    return check_hip(ctx, hipStreamSynchronize(ctx->stream), "hipStreamSynchronize");
}

const char* dcnn_status_str(dcnn_status s) {
    switch (s) {
        case DCNN_OK: return "ok";
        case DCNN_EINVAL: return "invalid argument";
        case DCNN_ESHAPE: return "shape mismatch";
        case DCNN_EDTYPE: return "dtype mismatch";
        case DCNN_ESTATE: return "wrong state (init before step, bind before run)";
        case DCNN_ENOMEM: return "caller-provided buffer too small";
        case DCNN_EHIP: return "HIP error";
        case DCNN_EUNSUPPORTED: return "unsupported configuration";
    }
    return "unknown status";
}

const char* dcnn_last_error(const dcnn_ctx* ctx) { return ctx ? ctx->err : "no context"; }

}  // extern "C"
