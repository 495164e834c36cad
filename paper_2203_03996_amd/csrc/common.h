// Internal declarations shared by the translation units of libdeltacnn (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/deltacnn.h"

namespace dcnn {

constexpr int kWave = 64;            // gfx950 wavefront
constexpr int kTile = 32;            // list entries one wave processes at a time (= MFMA N)
constexpr int kChunk = 2048;         // pixels per workgroup in the pixel-space mask passes
constexpr int kXcd = 8;              // accelerator complex dies, each with its own L2
constexpr size_t kAlign = 256;

inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t dtype_size(int dt) { return dt == DCNN_F16 ? 2 : 4; }

// Division of a 31-bit unsigned number by a constant known on the host: q = (mulhi(n, m) + n) >> s
// with s = ceil(log2 d), m = ceil(2^(32+s) / d) - 2^32.  Exact for 0 <= n < 2^31.
struct FastDiv {
    uint32_t m, s, d;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    f.s = 0;
    while ((1ull << f.s) < d) ++f.s;
    f.m = (uint32_t)((((1ull << (32 + f.s)) + d - 1) / d) - (1ull << 32));
    return f;
}

}  // namespace dcnn

struct dcnn_ctx {
    hipStream_t stream;
    int device;              // HIP device that was current when the context was created
    char* ws;
    size_t ws_bytes;
    int num_cu;
    size_t max_lds;
    char err[512];
};

namespace dcnn {

dcnn_status fail(dcnn_ctx* ctx, dcnn_status s, const char* fmt, ...);
dcnn_status check_hip(dcnn_ctx* ctx, hipError_t e, const char* what);

// Workspace carve-up (all offsets 256-byte aligned).
struct Workspace {
    int32_t* chunk_counts;   // one per kChunk pixels
    uint32_t* surv;          // one survivor word per kTile list entries
    uint8_t* scratch_mask;   // mask of a pass whose caller only wants the list
    uint8_t* scratch_mask2;  // second intermediate mask (separable dilation of the input mask)
    int64_t max_pixels;
};
size_t workspace_bytes(int64_t max_pixels);
dcnn_status workspace_view(dcnn_ctx* ctx, int64_t pixels, Workspace* out);

// ---- kernel launchers (defined in the *.hip files) -------------------------------------------
struct MaskPassArgs {
    const uint8_t* mask_in;      // [n,h,w] or nullptr (treated as all zero)
    const uint8_t* mask_b;       // [n,oh,ow] or nullptr
    uint8_t* mask_out;           // [n,oh,ow] or nullptr
    int32_t* idx_out;            // may be nullptr (then only mask_out is written)
    int32_t* count_out;
    int n, h, w, oh, ow, k, stride, pad;
    int up;                      // > 1: nearest upsampling of the input mask by this factor (k = 1)
    int bilinear;                // with up > 1: bilinear upsampling instead (sources that carry weight)
    int32_t* zero_count;         // optional counter the pass resets to 0 (survivor count of the layer)
    int emit_only;               // 1: mask_in is final and its chunk counts are in the workspace already
    uint32_t* taps_out;          // optional [n*oh*ow]: per list entry, which window taps are flagged (k*k <= 25 bits);
                                 // bit 30: the entry's pixel is flagged in mask_b
    int b_stride, b_h, b_w;      // b_stride > 0: mask_b is [n,b_h,b_w] and output pixel (y,x) looks at (y,x)*b_stride
    int kw, pad_w;               // kw > 0: the window is k rows x kw columns with padding pad / pad_w (stride 1)
};
dcnn_status launch_mask_compact(dcnn_ctx* ctx, const MaskPassArgs& a);
// Resolves the device address of the library's static scratch array for HIP device `dev`, which must be the
// current device (set-up step of dcnn_mask_compact_static; called by dcnn_ctx_create).
hipError_t static_scratch_setup(int dev);

// Ordered compaction of the entries of a work list that survived (bit set in surv).
dcnn_status launch_emit_sublist(dcnn_ctx* ctx, const int32_t* list, const int32_t* count, int64_t max_count,
                                const uint32_t* surv, int32_t* idx_out, int32_t* count_out);
dcnn_status launch_fill_i32(dcnn_ctx* ctx, int32_t* p, int32_t v, int64_t n);
// Statistics (never on a timed path): *out = number of non-zero bytes among mask[0 .. pixels).
dcnn_status launch_mask_sum(dcnn_ctx* ctx, const uint8_t* mask, int64_t pixels, int32_t* out);
// flags[p] = 1 iff row p of `data` ([pixels, c] elements) has a non-zero bit.
dcnn_status launch_row_flags(dcnn_ctx* ctx, int dtype, const void* data, uint8_t* flags, int64_t pixels, int c);
dcnn_status launch_fill_u8(dcnn_ctx* ctx, uint8_t* p, uint8_t v, int64_t n);

// Element-wise tail shared by CONV / ACT: (+bias) (+residual) activation, truncation, state.
struct EpilogueArgs {
    int c;                       // channels of the output pixel
    int act;                     // dcnn_act
    float eps;
    const void* bias;            // [c] or nullptr (first frame only)
    const void* res_data;        // second delta stream (output shape) or nullptr
    const uint8_t* res_mask;     // nullptr in the first frame (dense residual)
    void* xA;                    // nullptr when act == NONE
    void* xT;
    void* out_data;
    uint8_t* out_mask;           // written at every visited pixel (0 or 1); nullptr: not written
    uint32_t* surv;              // survivor word per tile; nullptr: not written
    int32_t* out_count;          // when surv is null: survivors are added here, one atomic per wave.  The layer code
                                 // passes nullptr: atomics on one address are served one after the other, and a
                                 // few thousand of them at the end of a kernel cost 10-20 us (see dcnn_layer_step)
    uint8_t* xt_flags;           // optional, per output pixel: 0 = the pixel's x^T row is all zero bits in memory and is
                                 // not read; 1 = it may hold values.  Kept up to date by the wave-specialised kernel only.
    void* accum_O;               // fused final accumulation: dense output O (output shape); the emitted delta is
                                 // added to it and not stored (sparse steps of layers with an activation only)
    int carry;                   // 1: an update leaves the rounding residue of x^A in x^T (s - round(s)) instead of 0
    uint8_t* clear_mask;         // optional: a byte array every workgroup of the grid zeroes a share of before anything else
    int64_t clear_bytes;         // (the output mask of the layer's NEXT step, see dcnn_layer_step)
};

struct ListArgs {
    const int32_t* list;         // nullptr: identity (entry j is pixel j)
    const int32_t* count;        // nullptr: use count_host
    int64_t count_host;
    int64_t max_count;           // upper bound used to size the grid
    const uint32_t* taps;        // optional, per entry: bit t set iff window tap t of the entry's pixel is in
                                 // bounds and flagged in the input mask (written with the list by the mask pass)
};

// Statistics (never on a timed path): x^T rows a convolution that keeps row flags reads and writes in one step.
// phase 0, before the step's kernel: before[j] = flag of list entry j's pixel, io[0] = their number (rows read);
// phase 1, after it: io[1] = entries whose row held values before or holds values now (rows written).
dcnn_status launch_xt_row_count(dcnn_ctx* ctx, int phase, const ListArgs& l, const uint8_t* flags, uint8_t* before,
                                unsigned long long* io);

struct ConvArgs {
    const void* in_data;
    const uint8_t* in_mask;      // nullptr: every in-bounds pixel is flagged (first frame)
    const int32_t* in_count;     // optional, device: number of flagged input pixels (how dense the window taps are)
    const void* wpacked;
    const void* zero_page;       // >= 16 bytes of zeros: what lanes read instead of an unflagged / padded input
    int n, h, w, cin, oh, ow, cout, cout_pad, k, stride, pad, kch;
    int depthwise;
    int flat;                    // filled by launch_conv: kch counts K-steps over the flat (tap, channel) dimension
    FastDiv div_ow, div_oh;      // filled by launch_conv
    // optional projection: a 1x1 convolution (stride2, no padding) of a second input [n,h2,w2,cin2] whose
    // result is added to this one's before the epilogue; its update flag is bit 30 of the list's tap words
    const void* in2_data;        // nullptr: none
    const void* wpacked2;
    int h2, w2, cin2, stride2, kch2;
};
dcnn_status launch_conv(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ConvArgs& c,
                        const EpilogueArgs& e);
size_t conv_packed_weight_bytes(int dtype, int k, int cin, int cout, int depthwise, bool fused);
dcnn_status launch_pack_weights(dcnn_ctx* ctx, int dtype, const void* w, void* wpacked, int k, int cin, int cout,
                                int depthwise, bool fused);
bool conv_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cout, int depthwise, bool fused,
                    char* why, size_t why_len);
// Convolution + activation with a fused 1x1 projection of a second input (cin2 channels): supported when the
// sparse step can run on the wave-specialised kernel with both weight tensors resident in LDS.
// Convolution + activation whose sparse step runs on the wave-specialised kernel (needed for a fused final
// accumulation).
bool conv_ws_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cout, int64_t in_elems, int64_t out_elems);
bool conv_proj_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cin2, int cout, int64_t in_elems,
                         int64_t in2_elems, int64_t out_elems);
size_t conv_proj_weight_bytes(int dtype, int k, int cin, int cin2, int cout);
// Packs the projection's [cin2][cout] weights in the column grouping of the main convolution's plan.
dcnn_status launch_pack_weights_proj(dcnn_ctx* ctx, int dtype, const void* w2, void* wpacked2, int k, int cin, int cin2,
                                     int cout);

struct ActArgs {
    const void* in_data;         // first delta stream
    const uint8_t* in_mask;      // nullptr: always valid (single input: the list is its mask)
};
dcnn_status launch_act(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ActArgs& a,
                       const EpilogueArgs& e);
dcnn_status launch_dwconv(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ConvArgs& c,
                          const EpilogueArgs& e);

struct DeltaGenArgs {
    const void* frame;
    void* P;
    void* out_data;
    uint8_t* out_mask;
    int32_t* out_idx;
    int32_t* out_count;
    int64_t pixels;
    int n, h, w, c;
    float eps;
    int dilate_r;
};
dcnn_status launch_deltagen(dcnn_ctx* ctx, int dtype, const DeltaGenArgs& a);
dcnn_status launch_copy(dcnn_ctx* ctx, void* dst, const void* src, size_t bytes);

struct AccumArgs {
    const void* in_data;
    void* O;
    int c;
};
dcnn_status launch_accum(dcnn_ctx* ctx, int dtype, const ListArgs& l, const AccumArgs& a);

struct PoolArgs {
    const void* in_data;         // delta at flagged input pixels
    const uint8_t* in_mask;
    void* xA;                    // accumulated dense input [n,h,w,c]
    void* out_data;              // [n,oh,ow,c]
    int n, h, w, c, oh, ow, k, stride, pad;
};
// work list = flagged OUTPUT pixels; a second pass over the flagged INPUT pixels folds the delta into xA
dcnn_status launch_maxpool_out(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const PoolArgs& a);
dcnn_status launch_maxpool_commit(dcnn_ctx* ctx, int dtype, const ListArgs& l_in, const PoolArgs& a);

struct ConcatArgs {
    const void* a_data;          // [pixels, ca]
    const void* b_data;          // [pixels, cb]
    const uint8_t* a_mask;       // nullptr: dense (first frame)
    const uint8_t* b_mask;
    void* out_data;              // [pixels, ca + cb]
    int ca, cb;
};
dcnn_status launch_concat(dcnn_ctx* ctx, int dtype, const ListArgs& l, const ConcatArgs& a);

struct UpsampleArgs {
    const void* in_data;
    void* out_data;
    int n, h, w, c, factor;
    int bilinear;                // 0: nearest neighbour; 1: bilinear, half-pixel centres
    const uint8_t* in_mask;      // bilinear: unflagged sources count as zero (nullptr: all flagged)
};

// Global average pooling: one list entry per stream with an update; out[n, c] = sum over the stream's flagged
// pixels / (h * w).
struct GapArgs {
    const void* in_data;         // [n, h*w, c]
    const uint8_t* in_mask;      // nullptr: every pixel counts (first frame)
    void* out_data;              // [n, c]
    int hw, c;
};
dcnn_status launch_gavgpool(dcnn_ctx* ctx, int dtype, const ListArgs& l_out, const GapArgs& a);
dcnn_status launch_upsample(dcnn_ctx* ctx, int dtype, const ListArgs& l_out, const UpsampleArgs& a);

}  // namespace dcnn
