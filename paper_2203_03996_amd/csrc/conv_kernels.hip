// Host side of the convolution: plan queries, weight packing and dispatch to the per-variant
// translation units (conv_inst.hip).
#include "conv_ws_impl.h"

namespace dcnn {

size_t conv_packed_weight_bytes(int dtype, int k, int cin, int cout, int depthwise, bool fused) {
    if (depthwise) return align_up((size_t)k * k * cout * dtype_size(dtype));
    const ConvPlan p = conv_plan(dtype, k, cin, cout, fused);
    // an unsupported shape is refused when the layer is created; size it for the widest padding
    return align_up(p.ok ? p.w_bytes : (size_t)k * k * cdiv(cin, 8) * 2 * cdiv(cout, 512) * 512 * 16);
}

bool conv_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cout, int depthwise, bool fused, char* why,
                    size_t why_len) {
    if (depthwise) return true;
    if (k * k > 64) { snprintf(why, why_len, "kernel size %d too large", k); return false; }
    const ConvPlan p = conv_plan(dtype, k, cin, cout, fused);
    if (!p.ok || ctx->max_lds < kLdsBytes) {
        snprintf(why, why_len, "conv %dx%d %d->%d%s: no tiling of the output channels fits the %zu bytes of LDS", k, k, cin,
                 cout, fused ? " with fused activation" : "", ctx->max_lds);
        return false;
    }
    return true;
}

// Packed layout: [pass][tap][kc][g][col][KPACK]; channel = (2*kc + g)*KPACK + e, cout = (pass*nb*32) + col.
template <typename T>
__global__ void pack_weights_kernel(const T* w, T* packed, int k, int cin, int cout, int nb, int npass, int kch) {
    constexpr int KP = Mma<T>::KPACK;
    const int cols = nb * 32;
    const int64_t total = (int64_t)npass * k * k * kch * 2 * cols * KP;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = i;
        const int e = (int)(r % KP); r /= KP;
        const int col = (int)(r % cols); r /= cols;
        const int g = (int)(r % 2); r /= 2;
        const int kc = (int)(r % kch); r /= kch;
        const int tap = (int)(r % (k * k)); r /= (k * k);
        const int pass = (int)r;
        const int ch = (2 * kc + g) * KP + e;
        const int co = pass * cols + col;
        T v = (T)0.0f;
        if (ch < cin && co < cout) v = w[((int64_t)tap * cin + ch) * cout + co];
        packed[i] = v;
    }
}

dcnn_status launch_pack_weights(dcnn_ctx* ctx, int dtype, const void* w, void* wpacked, int k, int cin, int cout,
                                int depthwise, bool fused) {
    if (depthwise)
        return launch_copy(ctx, wpacked, w, (size_t)k * k * cout * dtype_size(dtype));
    const ConvPlan p = conv_plan(dtype, k, cin, cout, fused);
    if (!p.ok) return fail(ctx, DCNN_EUNSUPPORTED, "pack_weights: unsupported convolution shape");
    const int64_t total = (int64_t)p.w_bytes / (int64_t)dtype_size(dtype);
    const int grid = (int)(cdiv(total, 256) < 4096 ? cdiv(total, 256) : 4096);
    if (p.flat) { cin = k * k * cin; k = 1; }                 // [k][k][cin][cout] read as [k*k*cin][cout]
    if (dtype == DCNN_F16)
        hipLaunchKernelGGL((pack_weights_kernel<f16>), dim3(grid), dim3(256), 0, ctx->stream, static_cast<const f16*>(w),
                           static_cast<f16*>(wpacked), k, cin, cout, p.nb, p.npass * p.cs, p.kch);
    else
        hipLaunchKernelGGL((pack_weights_kernel<float>), dim3(grid), dim3(256), 0, ctx->stream,
                           static_cast<const float*>(w), static_cast<float*>(wpacked), k, cin, cout, p.nb, p.npass * p.cs, p.kch);
    return check_hip(ctx, hipGetLastError(), "pack_weights_kernel launch");
}

bool conv_ws_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cout, int64_t in_elems, int64_t out_elems) {
    const size_t es = dtype_size(dtype);
    // (ctx may be null: every context that exists has the LDS the plans assume)
    if ((ctx && ctx->max_lds < kLdsBytes) || (k != 1 && k != 3) || ((size_t)cin * es) % 16 != 0) return false;
    const ConvPlan p = conv_plan(dtype, k, cin, cout, true);
    if (!p.ok || conv_ws_lds_bytes(p, dtype, k, cout, 0) == 0) return false;
    const uint64_t lim = kWsMaxBytes / es;
    return (uint64_t)in_elems <= lim && (uint64_t)out_elems <= lim;
}

bool conv_proj_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cin2, int cout, int64_t in_elems,
                         int64_t in2_elems, int64_t out_elems) {
    const size_t es = dtype_size(dtype);
    if ((ctx && ctx->max_lds < kLdsBytes) || (k != 1 && k != 3)) return false;
    if (((size_t)cin * es) % 16 != 0 || ((size_t)cin2 * es) % 16 != 0) return false;
    const ConvPlan p = conv_plan(dtype, k, cin, cout, true);
    if (!p.ok || conv_ws_lds_bytes(p, dtype, k, cout, cin2) == 0) return false;
    const uint64_t lim = kWsMaxBytes / es;
    return (uint64_t)in_elems <= lim && (uint64_t)in2_elems <= lim && (uint64_t)out_elems <= lim;
}

size_t conv_proj_weight_bytes(int dtype, int k, int cin, int cin2, int cout) {
    const ConvPlan p = conv_plan(dtype, k, cin, cout, true);
    const int kch2 = (int)cdiv(cin2, dtype == DCNN_F16 ? 16 : 8);
    return align_up((size_t)kch2 * 2 * (p.ok ? p.cout_pad : (int)cdiv(cout, 512) * 512) * 16);
}

dcnn_status launch_pack_weights_proj(dcnn_ctx* ctx, int dtype, const void* w2, void* wpacked2, int k, int cin, int cin2,
                                     int cout) {
    const ConvPlan p = conv_plan(dtype, k, cin, cout, true);
    if (!p.ok) return fail(ctx, DCNN_EUNSUPPORTED, "pack_weights: unsupported convolution shape");
    const int kch2 = (int)cdiv(cin2, dtype == DCNN_F16 ? 16 : 8);
    const int64_t total = (int64_t)kch2 * 2 * p.cout_pad * 16 / (int64_t)dtype_size(dtype);
    const int grid = (int)(cdiv(total, 256) < 4096 ? cdiv(total, 256) : 4096);
    if (dtype == DCNN_F16)
        hipLaunchKernelGGL((pack_weights_kernel<f16>), dim3(grid), dim3(256), 0, ctx->stream, static_cast<const f16*>(w2),
                           static_cast<f16*>(wpacked2), 1, cin2, cout, p.nb, p.npass * p.cs, kch2);
    else
        hipLaunchKernelGGL((pack_weights_kernel<float>), dim3(grid), dim3(256), 0, ctx->stream,
                           static_cast<const float*>(w2), static_cast<float*>(wpacked2), 1, cin2, cout, p.nb, p.npass * p.cs, kch2);
    return check_hip(ctx, hipGetLastError(), "pack_weights_kernel launch");
}

#define DCNN_DECL(TN, NB) dcnn_status launch_conv_##TN##_nb##NB(dcnn_ctx*, bool, const ListArgs&, const ConvArgs&, const EpilogueArgs&, const ConvPlan&);
#define DCNN_DECL_ALL(TN) DCNN_DECL(TN, 1) DCNN_DECL(TN, 2) DCNN_DECL(TN, 3) DCNN_DECL(TN, 4)
DCNN_DECL_ALL(f16)
DCNN_DECL_ALL(f32)
#undef DCNN_DECL_ALL
#undef DCNN_DECL

dcnn_status launch_conv(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ConvArgs& c_in,
                        const EpilogueArgs& e) {
    if (c_in.depthwise) return launch_dwconv(ctx, dtype, init, l, c_in, e);
    ConvArgs c = c_in;
    const bool fused = e.act != DCNN_ACT_NONE;
    char why[256];
    if (!conv_supported(ctx, dtype, c.k, c.cin, c.cout, 0, fused, why, sizeof(why)))
        return fail(ctx, DCNN_EUNSUPPORTED, "%s", why);
    const ConvPlan p = conv_plan(dtype, c.k, c.cin, c.cout, fused);
    c.cout_pad = p.cout_pad;
    c.kch = p.kch;
    c.flat = p.flat ? 1 : 0;
    c.kch2 = c.in2_data ? (int)cdiv(c.cin2, dtype == DCNN_F16 ? 16 : 8) : 0;
    c.div_ow = make_fastdiv((uint32_t)c.ow);
    c.div_oh = make_fastdiv((uint32_t)c.oh);
#define DCNN_CASE(NB) case NB: return dtype == DCNN_F16 ? launch_conv_f16_nb##NB(ctx, init, l, c, e, p) : launch_conv_f32_nb##NB(ctx, init, l, c, e, p);
    switch (p.nb) {
        DCNN_CASE(1) DCNN_CASE(2) DCNN_CASE(3) DCNN_CASE(4)
    }
#undef DCNN_CASE
    return fail(ctx, DCNN_EUNSUPPORTED, "conv: no kernel for %d column blocks", p.nb);
}

}  // namespace dcnn
