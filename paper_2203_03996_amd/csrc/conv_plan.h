// Shared by the convolution translation units: launch constants, MFMA traits and the plan that
// packing, sizing and launching agree on.
#pragma once

#include "device_utils.h"

namespace dcnn {

constexpr int kStagePad = 16;                       // bytes added to a staging row against bank conflicts
constexpr int kGroup = 4;                           // K-steps per streamed weight slice
constexpr size_t kLdsBytes = 160 * 1024;            // LDS of one gfx950 compute unit; the context refuses less

template <typename T> struct Mma;
template <> struct Mma<f16> {
    typedef f16x8 Vec;
    static constexpr int KPACK = 8;
    static __device__ __forceinline__ void run(f32x16& acc, const Vec& w, const Vec& x) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(w, x, acc, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    typedef f32x4 Vec;
    static constexpr int KPACK = 4;
    static __device__ __forceinline__ void run(f32x16& acc, const Vec& w, const Vec& x) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w[j], x[j], acc, 0, 0, 0);
    }
};

// accumulators -> staging tile [pixel][nb*32 channels] in the storage type.  Lane (col, g) holds,
// for pixel `col`, the output channels 8*q + 4*g + {0..3} of every 32-channel block.  With ADD the
// rounded accumulators are added to what the tile holds (and the sum is rounded again).
template <typename T, int NB, bool ADD = false>
__device__ __forceinline__ void stage_accumulators(const f32x16 (&acc)[NB], unsigned char* row, int g) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            T* dst = reinterpret_cast<T*>(row) + b * 32 + 8 * q + 4 * g;
            if constexpr (sizeof(T) == 2) {
                f16x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (f16)acc[b][4 * q + i];
                if constexpr (ADD) {
                    const f16x4 old = *reinterpret_cast<const f16x4*>(dst);
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (f16)((float)old[i] + (float)v[i]);
                }
                *reinterpret_cast<f16x4*>(dst) = v;
            } else {
                f32x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = acc[b][4 * q + i];
                if constexpr (ADD) {
                    const f32x4 old = *reinterpret_cast<const f32x4*>(dst);
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = old[i] + v[i];
                }
                *reinterpret_cast<f32x4*>(dst) = v;
            }
        }
    }
}

// How the output channels of a layer are spread: every wave holds `nb` MFMA column blocks (32
// output channels each) in its accumulators, `cs` waves share one tile of 32 pixels and split its
// channels between them, and `npass` passes cover layers wider than nb*cs*32 channels.
struct ConvPlan {
    int nb, cs, npass;
    int waves;         // wavefronts per workgroup
    int cout_pad;      // npass * cs * nb * 32
    int kch;           // K-steps per tap, each covering 2 * KPACK input channels
    size_t w_bytes;    // packed weights
    bool stream;       // weights do not fit LDS: stream them in slices
    bool flat;         // the window's (tap, channel) pairs form one flat K dimension (stems with very few channels)
    bool full_tail;    // one pass: the activation tail sees the whole pixel
    size_t lds_bytes;
    bool ok;
};

inline size_t conv_stage_bytes(int waves, int nb, int dtype) { return (size_t)waves * kTile * (nb * 32 * dtype_size(dtype) + kStagePad); }
inline size_t conv_xchg_bytes(int waves) { return (size_t)2 * waves * kTile * sizeof(float); }

// A k x k window over fewer channels than one 16-byte vector holds (network stems: 3 channels) would spend one
// K-step per tap on mostly padding.  Its k*k*cin values are one flat K dimension instead: the weights
// [k][k][cin][cout] already are [k*k*cin][cout], and the gather decodes (tap, channel) per element.
constexpr int kFlatMaxK = 256;                       // flat K values (the decode table sits in LDS)
inline bool conv_flat_k(int dtype, int k, int cin) {
    return k > 1 && (size_t)cin * dtype_size(dtype) < 16 && k * k * cin <= kFlatMaxK;
}
inline size_t conv_flat_lut_bytes() { return (size_t)kFlatMaxK * 8; }

inline ConvPlan conv_plan_window(int dtype, int k, int cin, int cout, bool need_full_tail);

// The plan depends only on the layer's description, so packing, sizing and launching agree on it.
inline ConvPlan conv_plan(int dtype, int k, int cin, int cout, bool need_full_tail) {
    if (conv_flat_k(dtype, k, cin)) {
        ConvPlan p = conv_plan_window(dtype, 1, k * k * cin, cout, need_full_tail);
        if (p.ok && !p.stream && p.lds_bytes + conv_flat_lut_bytes() <= kLdsBytes) {
            p.flat = true;
            p.lds_bytes += conv_flat_lut_bytes();
            return p;
        }
    }
    return conv_plan_window(dtype, k, cin, cout, need_full_tail);
}

inline ConvPlan conv_plan_window(int dtype, int k, int cin, int cout, bool need_full_tail) {
    const int kpack = dtype == DCNN_F16 ? 8 : 4;
    const int vec = dtype == DCNN_F16 ? 8 : 4;
    const bool vec_out = cout % vec == 0;
    const int nbt = (int)cdiv(cout, 32);
    ConvPlan best{};
    best.ok = false;
    long best_score = -1;
    // preference among equally padded layouts: two blocks per wave first (small accumulators, one
    // cache line per pixel and array in the tail), then three, four, one
    static const int nb_pref[] = {2, 3, 4, 1};
    static const int cs_list[] = {1, 2, 4};
    for (int pi = 0; pi < 4; ++pi) {
        const int nb = nb_pref[pi];
        for (int cs : cs_list) {
            if (!vec_out && (nb > 2 || cs > 1)) continue;          // element-wise tail: one wave, <= 64 channels
            const int cap = nb * cs;
            const int npass = (int)cdiv(nbt, cap);
            if (need_full_tail && npass > 1) continue;
            if (!vec_out && npass > 1) continue;
            ConvPlan p{};
            p.nb = nb; p.cs = cs; p.npass = npass;
            p.cout_pad = npass * cap * 32;
            p.kch = (int)cdiv(cin, 2 * kpack);
            p.w_bytes = (size_t)k * k * p.kch * 2 * p.cout_pad * 16;
            p.full_tail = npass == 1;
            // 8 waves per workgroup (up to 256 registers each) share the weights in LDS
            bool placed = false;
            {
                const int waves = 8;
                const size_t fixed = conv_stage_bytes(waves, nb, dtype) + conv_xchg_bytes(waves);
                const size_t slice = (size_t)2 * cs * kGroup * 2 * nb * 32 * 16;   // double-buffered weight slice
                if (p.w_bytes + fixed <= kLdsBytes) { p.stream = false; p.lds_bytes = p.w_bytes + fixed; placed = true; }
                else if (slice + fixed <= kLdsBytes) { p.stream = true; p.lds_bytes = slice + fixed; placed = true; }
                p.waves = waves;
            }
            if (!placed) continue;
            p.ok = true;
            // fewer padded blocks first, then fewer passes, then fewer waves per tile, then preference
            const long score = (long)npass * cap * 100000L + (long)npass * 1000L + (nb > 2 ? 500L : 0L) + cs * 10L + pi;
            if (best_score < 0 || score < best_score) { best = p; best_score = score; }
        }
    }
    return best;
}

}  // namespace dcnn
