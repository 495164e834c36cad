// Sparse delta convolution with dense weights as a gather-GEMM on the matrix cores.
//
// The work list holds the flagged OUTPUT pixels in ascending order.  One wavefront owns a tile
// of 32 consecutive list entries and all output channels:
//     D[cout][pixel] += W_tap[cout][cin] * X_tap[cin][pixel]        for every window tap
// with MFMA 32x32 blocks (A operand = weights from LDS, B operand = the pixel's channels gathered
// straight from the NHWC delta map into registers, 16 bytes per lane).  A tap contributes only
// where the input pixel is in bounds AND flagged: unflagged memory is never read (it is invalid
// by contract), and a tap no lane of the wave needs is skipped altogether.
// When the packed weight tensor of the layer fits, it stays resident in LDS (160 KB per CU on
// gfx950) for the lifetime of the persistent workgroup.  Larger layers stream it: the four waves of
// a workgroup walk the K dimension in lockstep and a double-buffered 4-K-step slice of the weights
// is copied global -> registers -> LDS while the matrix cores consume the previous slice.
// The fp32 result tile is rounded to the storage type, staged through LDS and handed to the
// activation + truncation tail with coalesced accesses (once per pixel when all output channels
// fit the staging tile, else per pass of output channels for layers without activation).
#include "device_utils.h"

namespace dcnn {

constexpr int kConvWaves = 4;
constexpr int kConvThreads = kConvWaves * kWave;
constexpr int kStagePad = 16;                       // bytes added to a staging row against bank conflicts
constexpr int kGroup = 4;                           // K-steps whose gathers are issued together

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

struct ConvPlan {
    int nb;            // 32-column blocks of output channels held in accumulators per pass
    int npass;
    int cout_pad;      // npass * nb * 32
    int kch;           // K-steps per tap, each covering 2 * KPACK input channels
    size_t w_bytes;    // packed weights
    bool stream;       // weights do not fit LDS: stream them in slices
    bool full_tail;    // the staging tile holds all output channels (needed for a fused activation)
    size_t lds_bytes;
    bool ok;
};

static size_t stage_bytes(int cols, int dtype) { return (size_t)kConvWaves * kTile * (cols * dtype_size(dtype) + kStagePad); }

static ConvPlan conv_plan(int dtype, int k, int cin, int cout, size_t max_lds, bool need_full_tail) {
    const int kpack = dtype == DCNN_F16 ? 8 : 4;
    const int vec = dtype == DCNN_F16 ? 8 : 4;
    ConvPlan p{};
    const int nbt = (int)cdiv(cout, 32);
    static const int cand[] = {8, 6, 5, 4, 3, 2, 1};
    p.nb = 1;
    for (int nb : cand) {                                   // largest block count wasting <= 15 % on padding
        if (cdiv(nbt, nb) * nb * 100 <= (int64_t)nbt * 115) { p.nb = nb; break; }
    }
    p.npass = (int)cdiv(nbt, p.nb);
    p.cout_pad = p.npass * p.nb * 32;
    p.kch = (int)cdiv(cin, 2 * kpack);
    p.w_bytes = (size_t)k * k * p.kch * 2 * p.cout_pad * 16;
    const size_t slice = (size_t)2 * kGroup * 2 * p.nb * 32 * 16;          // double-buffered weight slice
    const int nvec = cout % vec == 0 ? cout / vec : cout;                  // vectors per pixel in the tail
    const bool tail_fits_wave = nvec <= kWave;
    const size_t full = stage_bytes(p.cout_pad, dtype), part = stage_bytes(p.nb * 32, dtype);
    p.ok = true;
    if (tail_fits_wave && p.w_bytes + full <= max_lds) { p.stream = false; p.full_tail = true; p.lds_bytes = p.w_bytes + full; }
    else if (tail_fits_wave && slice + full <= max_lds) { p.stream = true; p.full_tail = true; p.lds_bytes = slice + full; }
    else if (!need_full_tail && cout % vec == 0 && slice + part <= max_lds) { p.stream = true; p.full_tail = false; p.lds_bytes = slice + part; }
    else p.ok = false;
    return p;
}

size_t conv_packed_weight_bytes(int dtype, int k, int cin, int cout, int depthwise) {
    if (depthwise) return align_up((size_t)k * k * cout * dtype_size(dtype));
    return align_up(conv_plan(dtype, k, cin, cout, 0, false).w_bytes);
}

bool conv_supported(const dcnn_ctx* ctx, int dtype, int k, int cin, int cout, int depthwise, bool fused, char* why,
                    size_t why_len) {
    if (depthwise) return true;
    if (k * k > 64) { snprintf(why, why_len, "kernel size %d too large", k); return false; }
    const ConvPlan p = conv_plan(dtype, k, cin, cout, ctx->max_lds, fused);
    if (!p.ok) {
        snprintf(why, why_len, "conv %dx%d %d->%d%s: the output tile does not fit the %zu bytes of LDS", k, k, cin, cout,
                 fused ? " with fused activation" : "", ctx->max_lds);
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
                                int depthwise) {
    if (depthwise)
        return launch_copy(ctx, wpacked, w, (size_t)k * k * cout * dtype_size(dtype));
    const ConvPlan p = conv_plan(dtype, k, cin, cout, 0, false);
    const int64_t total = (int64_t)p.w_bytes / (int64_t)dtype_size(dtype);
    const int grid = (int)(cdiv(total, 256) < 4096 ? cdiv(total, 256) : 4096);
    if (dtype == DCNN_F16)
        hipLaunchKernelGGL((pack_weights_kernel<f16>), dim3(grid), dim3(256), 0, ctx->stream, static_cast<const f16*>(w),
                           static_cast<f16*>(wpacked), k, cin, cout, p.nb, p.npass, p.kch);
    else
        hipLaunchKernelGGL((pack_weights_kernel<float>), dim3(grid), dim3(256), 0, ctx->stream,
                           static_cast<const float*>(w), static_cast<float*>(wpacked), k, cin, cout, p.nb, p.npass, p.kch);
    return check_hip(ctx, hipGetLastError(), "pack_weights_kernel launch");
}

// accumulators -> staging tile [pixel][cout] in the storage type.  Lane (col, g) holds, for pixel
// `col`, the output channels 8*q + 4*g + {0..3} of every 32-channel block.
template <typename T, int NB>
__device__ __forceinline__ void stage_accumulators(const f32x16 (&acc)[NB], unsigned char* row, int first_col, int g) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            T* dst = reinterpret_cast<T*>(row) + first_col + b * 32 + 8 * q + 4 * g;
            if constexpr (sizeof(T) == 2) {
                f16x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (f16)acc[b][4 * q + i];
                *reinterpret_cast<f16x4*>(dst) = v;
            } else {
                f32x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = acc[b][4 * q + i];
                *reinterpret_cast<f32x4*>(dst) = v;
            }
        }
    }
}

__device__ __forceinline__ void wave_lds_fence() {
    // the staging tile is private to one wave: order its LDS writes and reads without a block barrier
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T, int NB, int V, bool ALIGNED, bool STREAM>
__global__ __launch_bounds__(kConvThreads) void conv_mfma_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, int init,
                                                                 int npass, int full_tail) {
    typedef typename Mma<T>::Vec Vec;
    constexpr int KP = Mma<T>::KPACK;
    constexpr int COLS = NB * 32;
    constexpr int SLICE = kGroup * 2 * COLS;                   // 16-byte vectors of one weight slice
    extern __shared__ __align__(16) unsigned char smem[];

    const int64_t count = list_count(l);
    const WgTileRange r = wg_tile_range((count + kConvWaves * kTile - 1) / (kConvWaves * kTile));
    if (r.begin >= r.end) return;                              // nothing for this workgroup: skip the weight load

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int col = lane % 32, g = lane / 32;
    const int taps = c.k * c.k, kch = c.kch;
    const int ksteps = taps * kch;
    const int groups = (kch + kGroup - 1) / kGroup;            // slices per tap
    const int w_vecs = STREAM ? 2 * SLICE : npass * ksteps * 2 * COLS;
    Vec* w_lds = reinterpret_cast<Vec*>(smem);
    const int stage_cols = full_tail ? c.cout_pad : COLS;
    const int stage_stride = stage_cols * (int)sizeof(T) + kStagePad;
    unsigned char* stage = smem + (size_t)w_vecs * 16 + (size_t)wave * kTile * stage_stride;
    const Vec* wglob = static_cast<const Vec*>(c.wpacked);

    if constexpr (!STREAM) {
        for (int i = threadIdx.x; i < w_vecs; i += kConvThreads) w_lds[i] = wglob[i];
        __syncthreads();
    }

    const T* in = static_cast<const T*>(c.in_data);
    for (int64_t wt = r.begin; wt < r.end; wt += r.step) {
        const int64_t tile = wt * kConvWaves + wave;
        const int64_t base = tile * kTile;
        const bool tile_on = base < count;
        if constexpr (!STREAM) {
            if (!tile_on) continue;                            // streaming waves stay in step for the barriers
        }
        const int64_t j = base + col;
        const bool valid = j < count;
        const int64_t p = valid ? (l.list ? (int64_t)l.list[j] : j) : 0;
        const int ox = (int)(p % c.ow);
        const int64_t t1 = p / c.ow;
        const int oy = (int)(t1 % c.oh);
        const int64_t n = t1 / c.oh;
        const int iy0 = oy * c.stride - c.pad, ix0 = ox * c.stride - c.pad;

        // which taps does this lane's pixel need, and which does any lane of the wave need
        uint64_t tapbits = 0, tapany = 0;
        for (int t = 0; t < taps; ++t) {
            const int iy = iy0 + t / c.k, ix = ix0 + t % c.k;
            bool ok = valid && iy >= 0 && iy < c.h && ix >= 0 && ix < c.w;
            if (ok && c.in_mask) ok = c.in_mask[(n * c.h + iy) * c.w + ix] != 0;
            if (ok) tapbits |= 1ull << t;
            if (__ballot(ok)) tapany |= 1ull << t;
        }

        auto gather = [&](int t, int kc0, Vec (&x)[kGroup]) {
            const bool ok = (tapbits >> t) & 1;
            const int iy = iy0 + t / c.k, ix = ix0 + t % c.k;
            const T* src = in + ((n * c.h + iy) * c.w + ix) * c.cin;
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                Vec v;
#pragma unroll
                for (int i = 0; i < KP; ++i) v[i] = (T)0.0f;
                const int ch = (2 * (kc0 + u) + g) * KP;
                if (ok && kc0 + u < kch) {
                    if constexpr (ALIGNED) {
                        if (ch < c.cin) v = *reinterpret_cast<const Vec*>(src + ch);
                    } else {
#pragma unroll
                        for (int i = 0; i < KP; ++i)
                            if (ch + i < c.cin) v[i] = src[ch + i];
                    }
                }
                x[u] = v;
            }
        };

        for (int pass = 0; pass < npass; ++pass) {
            f32x16 acc[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

            if constexpr (!STREAM) {
                // software pipeline over (tap, group of K-steps): the gathers of the next group are in
                // flight while the matrix cores work on the current one; taps no lane needs are skipped
                int t = 0, kc0 = 0;
                while (t < taps && !((tapany >> t) & 1)) ++t;
                Vec xa[kGroup];
                if (t < taps) gather(t, 0, xa);
                while (t < taps) {
                    int tn = t, kn = kc0 + kGroup;
                    if (kn >= kch) {
                        kn = 0;
                        ++tn;
                        while (tn < taps && !((tapany >> tn) & 1)) ++tn;
                    }
                    Vec xb[kGroup];
                    if (tn < taps) gather(tn, kn, xb);
                    const Vec* wrow = w_lds + ((size_t)(pass * ksteps + t * kch + kc0) * 2 + g) * COLS + col;
#pragma unroll
                    for (int u = 0; u < kGroup; ++u) {
                        if (kc0 + u < kch) {
#pragma unroll
                            for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wrow[(size_t)u * 2 * COLS + b * 32], xa[u]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kGroup; ++u) xa[u] = xb[u];
                    t = tn;
                    kc0 = kn;
                }
            } else {
                // all waves of the workgroup walk the slices (tap, group) in lockstep; slice s+1 travels
                // global -> registers while slice s is multiplied, then registers -> LDS, one barrier
                const int nslices = taps * groups;
                auto slice_src = [&](int s, int* nvec) {
                    const int t = s / groups, kc0 = (s % groups) * kGroup;
                    const int steps = kch - kc0 < kGroup ? kch - kc0 : kGroup;
                    *nvec = steps * 2 * COLS;
                    return wglob + ((size_t)(pass * ksteps + t * kch + kc0) * 2) * COLS;
                };
                Vec wreg[NB];                                   // SLICE / kConvThreads == NB vectors per thread
                auto slice_load = [&](int s) {
                    int nv;
                    const Vec* src = slice_src(s, &nv);
#pragma unroll
                    for (int i = 0; i < NB; ++i) {
                        const int vi = threadIdx.x + i * kConvThreads;
                        if (vi < nv) wreg[i] = src[vi];
                    }
                };
                auto slice_store = [&](int s) {
                    int nv;
                    slice_src(s, &nv);
                    Vec* dst = w_lds + (size_t)(s & 1) * SLICE;
#pragma unroll
                    for (int i = 0; i < NB; ++i) {
                        const int vi = threadIdx.x + i * kConvThreads;
                        if (vi < nv) dst[vi] = wreg[i];
                    }
                };
                Vec xa[kGroup];
                slice_load(0);
                gather(0, 0, xa);
                slice_store(0);
                __syncthreads();
                for (int s = 0; s < nslices; ++s) {
                    const int t = s / groups, kc0 = (s % groups) * kGroup;
                    Vec xb[kGroup];
                    if (s + 1 < nslices) {
                        slice_load(s + 1);
                        gather((s + 1) / groups, ((s + 1) % groups) * kGroup, xb);
                    }
                    if ((tapany >> t) & 1) {
                        const Vec* wrow = w_lds + (size_t)(s & 1) * SLICE + (size_t)g * COLS + col;
#pragma unroll
                        for (int u = 0; u < kGroup; ++u) {
                            if (kc0 + u < kch) {
#pragma unroll
                                for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wrow[(size_t)u * 2 * COLS + b * 32], xa[u]);
                            }
                        }
                    }
                    if (s + 1 < nslices) slice_store(s + 1);
                    __syncthreads();
#pragma unroll
                    for (int u = 0; u < kGroup; ++u) xa[u] = xb[u];
                }
            }

            stage_accumulators<T, NB>(acc, stage + (size_t)col * stage_stride, full_tail ? pass * COLS : 0, g);
            if (!full_tail) {
                // pass-through layers too wide for one staging tile: write this pass's channels now
                wave_lds_fence();
                const int ch0 = pass * COLS;
                const int nch = e.c - ch0 < COLS ? e.c - ch0 : COLS;
                if (tile_on && nch > 0) {
                    auto dxp = [&](int ent, int64_t, int c0, float (&o)[V]) {
                        load_vec<T, V>(reinterpret_cast<const T*>(stage + (size_t)ent * stage_stride) + (c0 - ch0), o);
                    };
                    act_trunc_tile<T, V, 1>(e, init != 0, l.list, base, count, lane, dxp, ch0, nch);
                }
                wave_lds_fence();
            }
        }
        if (full_tail) {
            wave_lds_fence();
            if (tile_on) {
                auto dx = [&](int ent, int64_t, int c0, float (&o)[V]) {
                    load_vec<T, V>(reinterpret_cast<const T*>(stage + (size_t)ent * stage_stride) + c0, o);
                };
                const uint32_t bits = act_trunc_tile<T, V, 1>(e, init != 0, l.list, base, count, lane, dx);
                if (e.surv && lane == 0) e.surv[tile] = bits;
            }
            wave_lds_fence();
        }
    }
}

template <typename T, int NB>
static dcnn_status launch_conv_nb(dcnn_ctx* ctx, bool init, const ListArgs& l, const ConvArgs& c, const EpilogueArgs& e,
                                  const ConvPlan& p) {
    constexpr int VEC = Elem<T>::VEC;
    const bool vec_out = (e.c % VEC) == 0;
    const bool aligned = ((size_t)c.cin * sizeof(T)) % 16 == 0;
    int64_t want = cdiv(l.max_count > 0 ? l.max_count : 1, kConvWaves * kTile);
    int64_t per_cu = (int64_t)(ctx->max_lds / p.lds_bytes);
    per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
    int64_t cap = (int64_t)ctx->num_cu * per_cu;
    const int grid = (int)(cdiv(want < cap ? want : cap, kXcd) * kXcd);
    const int ini = init ? 1 : 0, full = p.full_tail ? 1 : 0;
    hipError_t err = hipSuccess;
#define DCNN_CONV_LAUNCH(V, AL, ST)                                                                              \
    do {                                                                                                         \
        auto kern = conv_mfma_kernel<T, NB, V, AL, ST>;                                                          \
        static bool attr_set = false;                                                                            \
        if (!attr_set) {                                                                                         \
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                      (int)ctx->max_lds);                                                        \
            attr_set = (err == hipSuccess);                                                                      \
        }                                                                                                        \
        if (err == hipSuccess)                                                                                   \
            hipLaunchKernelGGL(kern, dim3(grid), dim3(kConvThreads), p.lds_bytes, ctx->stream, l, c, e, ini, p.npass, full); \
    } while (0)
#define DCNN_CONV_PICK(V)                                                                                        \
    do {                                                                                                         \
        if (p.stream) { if (aligned) DCNN_CONV_LAUNCH(V, true, true); else DCNN_CONV_LAUNCH(V, false, true); }   \
        else { if (aligned) DCNN_CONV_LAUNCH(V, true, false); else DCNN_CONV_LAUNCH(V, false, false); }          \
    } while (0)
    if (vec_out) DCNN_CONV_PICK(VEC); else DCNN_CONV_PICK(1);
#undef DCNN_CONV_PICK
#undef DCNN_CONV_LAUNCH
    if (err != hipSuccess) return check_hip(ctx, err, "hipFuncSetAttribute(conv_mfma_kernel)");
    return check_hip(ctx, hipGetLastError(), "conv_mfma_kernel launch");
}

template <typename T>
static dcnn_status launch_conv_t(dcnn_ctx* ctx, bool init, const ListArgs& l, ConvArgs c, const EpilogueArgs& e) {
    const int dtype = sizeof(T) == 2 ? DCNN_F16 : DCNN_F32;
    const bool fused = e.act != DCNN_ACT_NONE;
    char why[256];
    if (!conv_supported(ctx, dtype, c.k, c.cin, c.cout, 0, fused, why, sizeof(why)))
        return fail(ctx, DCNN_EUNSUPPORTED, "%s", why);
    const ConvPlan p = conv_plan(dtype, c.k, c.cin, c.cout, ctx->max_lds, fused);
    c.cout_pad = p.cout_pad;
    c.kch = p.kch;
    switch (p.nb) {
        case 1: return launch_conv_nb<T, 1>(ctx, init, l, c, e, p);
        case 2: return launch_conv_nb<T, 2>(ctx, init, l, c, e, p);
        case 3: return launch_conv_nb<T, 3>(ctx, init, l, c, e, p);
        case 4: return launch_conv_nb<T, 4>(ctx, init, l, c, e, p);
        case 5: return launch_conv_nb<T, 5>(ctx, init, l, c, e, p);
        case 6: return launch_conv_nb<T, 6>(ctx, init, l, c, e, p);
        case 8: return launch_conv_nb<T, 8>(ctx, init, l, c, e, p);
    }
    return fail(ctx, DCNN_EUNSUPPORTED, "conv: no kernel for %d column blocks", p.nb);
}

dcnn_status launch_conv(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ConvArgs& c,
                        const EpilogueArgs& e) {
    if (c.depthwise) return launch_dwconv(ctx, dtype, init, l, c, e);
    return dtype == DCNN_F16 ? launch_conv_t<f16>(ctx, init, l, c, e) : launch_conv_t<float>(ctx, init, l, c, e);
}

}  // namespace dcnn
