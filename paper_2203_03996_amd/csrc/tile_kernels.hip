// Memory-bound kernels of the sparse path: input delta generation, activation + truncation
// (optionally of a sum of two streams), depthwise convolution, max pooling, upsampling and the
// final accumulation.  All of them walk a compacted work list of flagged pixels; LP lanes share
// one pixel so every access is a coalesced 16-byte vector of channels (NHWC).
#include "device_utils.h"

namespace dcnn {

constexpr int kTileWaves = 4;                       // waves (tiles) per workgroup
constexpr int kTileThreads = kTileWaves * kWave;

static int list_grid(const dcnn_ctx* ctx, int64_t max_count, int entries_per_wg, int wg_per_cu) {
    int64_t want = cdiv(max_count > 0 ? max_count : 1, entries_per_wg);
    int64_t cap = (int64_t)ctx->num_cu * wg_per_cu;
    int64_t g = want < cap ? want : cap;
    return (int)(cdiv(g, kXcd) * kXcd);
}

// A wave serves the pixels of its tile one iteration after the other; when one pixel's channels fill the whole
// wave (or half of it) that is 32 (16) dependent round trips to memory.  Such tiles are shared by 4 (2) waves:
// each keeps a run of 8 (16) consecutive entries (the others look empty to it) and stores its byte (half) of
// the tile's survivor word.
constexpr int kSplitMaxVpl = 4;
static int tile_parts(int nvec, int vpl) {
    int lp = 1;
    while (lp < (int)cdiv(nvec, vpl)) lp <<= 1;
    lp = lp < 2 ? 2 : (lp > kWave ? kWave : lp);
    const int iters = kTile / (kWave / lp);
    return iters >= 32 ? 4 : (iters >= 16 ? 2 : 1);
}

__device__ __forceinline__ void store_survivors(uint32_t* surv, int64_t tile, int part, int parts, uint32_t bits) {
    if (parts == 1) surv[tile] = bits;
    else if (parts == 2) reinterpret_cast<uint16_t*>(surv)[tile * 2 + part] = (uint16_t)(bits >> (16 * part));
    else reinterpret_cast<uint8_t*>(surv)[tile * 4 + part] = (uint8_t)(bits >> (8 * part));
}

// ---- activation + truncation (+ add) ----------------------------------------------------------
template <typename T, int V, int VPL, bool SPLIT>
__global__ __launch_bounds__(kTileThreads) void act_kernel(ListArgs l, ActArgs a, EpilogueArgs e, int init, int parts) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr int UB = (V * VPL >= 16) ? 2 : 4;
    const int64_t count = list_count(l);
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int C = e.c;
    const T* in = static_cast<const T*>(a.in_data);
    const uint8_t* in_mask = a.in_mask;
    auto dx = [&](int, int64_t p, int c0) -> Raw {
        if (in_mask == nullptr || in_mask[p] != 0) return raw_load<T, V>(in + p * C + c0);
        return raw_zero<T, V>();
    };
    int survivors = 0;
    if constexpr (SPLIT) {
        const int64_t ntiles = (count + kTile - 1) / kTile;
        const int run = kTile / parts;                          // tile entries per wave
        const WgTileRange r = wg_tile_range((ntiles * parts + kTileWaves - 1) / kTileWaves);
        for (int64_t wt = r.begin; wt < r.end; wt += r.step) {
            const int64_t unit = wt * kTileWaves + wave;
            const int64_t tile = unit / parts;
            const int part = (int)(unit - tile * parts);
            const int64_t base = tile * kTile;
            if (base >= count) continue;
            const int j = lane % kTile;
            const int p_mine = (j / run == part) ? list_pixel(l.list, base + j, count) : -1;
            const uint32_t bits = act_trunc_tile<T, V, VPL, UB, false>(e, init != 0, p_mine, lane, dx, 0, e.c, e.c, MaxExchange{nullptr, 1, 0});
            if (e.surv) { if (lane == 0) store_survivors(e.surv, tile, part, parts, bits); }
            else survivors += __popc(bits);
        }
    } else {
        const WgTileRange r = wg_tile_range((count + kTileWaves * kTile - 1) / (kTileWaves * kTile));
        for (int64_t wt = r.begin; wt < r.end; wt += r.step) {
            const int64_t tile = wt * kTileWaves + wave;
            const int64_t base = tile * kTile;
            if (base >= count) continue;
            const int p_mine = list_pixel(l.list, base + lane % kTile, count);
            const uint32_t bits = act_trunc_tile<T, V, VPL, UB, false>(e, init != 0, p_mine, lane, dx, 0, e.c, e.c, MaxExchange{nullptr, 1, 0});
            if (e.surv) { if (lane == 0) e.surv[tile] = bits; }
            else survivors += __popc(bits);
        }
    }
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

template <typename T>
static dcnn_status launch_act_t(dcnn_ctx* ctx, bool init, const ListArgs& l, const ActArgs& a, const EpilogueArgs& e) {
    constexpr int VEC = Elem<T>::VEC;
    const bool vec = (e.c % VEC) == 0;
    const int nvec = vec ? e.c / VEC : e.c;
    const int vpl = (int)cdiv(nvec, kWave);
    const int vpl_used = vpl <= 1 ? 1 : (vpl <= 2 ? 2 : (vpl <= 4 ? 4 : 8));
    // pixels of 8 vectors per lane keep one wave per tile (that form holds its whole batch in registers)
    const int parts = vpl_used <= kSplitMaxVpl ? tile_parts(nvec, vpl_used) : 1;
    const int grid = list_grid(ctx, l.max_count, kTileWaves * kTile / parts, 8);
    dim3 g(grid), b(kTileThreads);
    const int ini = init ? 1 : 0;
#define DCNN_ACT_LAUNCH(V, VPL)                                                                                      \
    do {                                                                                                             \
        if (parts > 1) hipLaunchKernelGGL((act_kernel<T, V, VPL, (VPL <= kSplitMaxVpl)>), g, b, 0, ctx->stream, l, a, e, ini, parts); \
        else hipLaunchKernelGGL((act_kernel<T, V, VPL, false>), g, b, 0, ctx->stream, l, a, e, ini, 1);              \
    } while (0)
    if (vec) {
        if (vpl <= 1) DCNN_ACT_LAUNCH(VEC, 1);
        else if (vpl <= 2) DCNN_ACT_LAUNCH(VEC, 2);
        else if (vpl <= 4) DCNN_ACT_LAUNCH(VEC, 4);
        else if (vpl <= 8 && sizeof(T) == 4) DCNN_ACT_LAUNCH(VEC, 8);
        else return fail(ctx, DCNN_EUNSUPPORTED, "activation: %d channels exceed the supported 8 KB per pixel", e.c);
    } else {
        if (vpl <= 1) DCNN_ACT_LAUNCH(1, 1);
        else if (vpl <= 2) DCNN_ACT_LAUNCH(1, 2);
        else if (vpl <= 4) DCNN_ACT_LAUNCH(1, 4);
        else return fail(ctx, DCNN_EUNSUPPORTED, "activation: %d unaligned channels exceed 256 per pixel", e.c);
    }
#undef DCNN_ACT_LAUNCH
    return check_hip(ctx, hipGetLastError(), "act_kernel launch");
}

dcnn_status launch_act(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ActArgs& a, const EpilogueArgs& e) {
    return dtype == DCNN_F16 ? launch_act_t<f16>(ctx, init, l, a, e) : launch_act_t<float>(ctx, init, l, a, e);
}

// ---- depthwise convolution: the first delta stream is formed on the fly ------------------------
// Work list = flagged OUTPUT pixels.  Every tap's update flag is checked before its values are
// read (unflagged memory is invalid).  KS = 1, 2, 3: the flags of the whole tile are fetched first (entry
// lane%32 per lane, one round trip) and packed into a tap word; the taps of a pixel are then loaded
// back to back, an unflagged or padded tap reading the zero page instead, so no load waits for a flag.
// KS = 0: any window, flag and values per tap.
template <typename T, int V, int VPL, int KS>
__global__ __launch_bounds__(kTileThreads) void dwconv_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, int init, int parts) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr int UB = 2;
    const int64_t count = list_count(l);
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int C = e.c;
    const T* in = static_cast<const T*>(c.in_data);
    const T* wgt = static_cast<const T*>(c.wpacked);           // [k][k][C], unpacked
    const T* zeros = static_cast<const T*>(c.zero_page);
    // KS > 0: per tile entry the tap word and the input pixel under tap (0,0) (which may lie outside the map);
    // handed from the lane that computed them to the lanes that serve the entry through LDS (a lane shuffle
    // inside the divergent per-vector code would read disabled lanes)
    __shared__ int2 s_taps[kTileWaves][kTile];
    auto dx_any = [&](int, int64_t p, int c0) -> Raw {
        const int ox = (int)(p % c.ow);
        const int64_t t = p / c.ow;
        const int oy = (int)(t % c.oh);
        const int64_t n = t / c.oh;
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;
        for (int ky = 0; ky < c.k; ++ky) {
            const int iy = oy * c.stride - c.pad + ky;
            if (iy < 0 || iy >= c.h) continue;
            for (int kx = 0; kx < c.k; ++kx) {
                const int ix = ox * c.stride - c.pad + kx;
                if (ix < 0 || ix >= c.w) continue;
                const int64_t q = (n * c.h + iy) * c.w + ix;
                if (c.in_mask && c.in_mask[q] == 0) continue;
                const Raw xv = raw_load<T, V>(in + q * C + c0);
                const Raw wv = raw_load<T, V>(wgt + (int64_t)(ky * c.k + kx) * C + c0);
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = fmaf(raw_get<T, V>(xv, i), raw_get<T, V>(wv, i), acc[i]);
            }
        }
        Raw o;
#pragma unroll
        for (int i = 0; i < V; ++i) raw_set<T, V>(o, i, acc[i]);
        return o;
    };
    auto dx_taps = [&](int ent, int64_t, int c0) -> Raw {
        constexpr int KK = KS > 0 ? KS * KS : 1;
        const int2 tq = s_taps[wave][ent & (kTile - 1)];
        const uint32_t word = (uint32_t)tq.x;
        const int q0 = tq.y;
        Raw xv[KK], wv[KK];
#pragma unroll
        for (int t = 0; t < KK; ++t) {
            const int64_t q = (int64_t)q0 + (t / (KS > 0 ? KS : 1)) * c.w + (t % (KS > 0 ? KS : 1));
            const T* src = ((word >> t) & 1u) ? in + q * C + c0 : zeros;
            xv[t] = raw_load<T, V>(src);
        }
#pragma unroll
        for (int t = 0; t < KK; ++t) wv[t] = raw_load<T, V>(wgt + (int64_t)t * C + c0);
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;
#pragma unroll
        for (int t = 0; t < KK; ++t)
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = fmaf(raw_get<T, V>(xv[t], i), raw_get<T, V>(wv[t], i), acc[i]);
        Raw o;
#pragma unroll
        for (int i = 0; i < V; ++i) raw_set<T, V>(o, i, acc[i]);
        return o;
    };
    int survivors = 0;
    const int64_t ntiles = (count + kTile - 1) / kTile;
    const WgTileRange r = wg_tile_range((ntiles * parts + kTileWaves - 1) / kTileWaves);
    for (int64_t wt = r.begin; wt < r.end; wt += r.step) {
        const int64_t unit = wt * kTileWaves + wave;
        const int64_t tile = unit / parts;
        const int part = (int)(unit - tile * parts);
        const int64_t base = tile * kTile;
        if (base >= count) continue;
        const int j = lane % kTile;
        const int p_mine = (j / (kTile / parts) == part) ? list_pixel(l.list, base + j, count) : -1;   // the others look empty
        uint32_t bits;
        if constexpr (KS > 0) {
            uint32_t tap_word = 0;
            int q_first = 0;
            if (p_mine >= 0) {
                const int ox = p_mine % c.ow;
                const int t = p_mine / c.ow;
                const int oy = t % c.oh, n = t / c.oh;
                const int iy0 = oy * c.stride - c.pad, ix0 = ox * c.stride - c.pad;
                q_first = (n * c.h + iy0) * c.w + ix0;
                uint32_t inb = 0;
                int qq[KS * KS];
#pragma unroll
                for (int t2 = 0; t2 < KS * KS; ++t2) {
                    const int iy = iy0 + t2 / KS, ix = ix0 + t2 % KS;
                    const bool ok = iy >= 0 && iy < c.h && ix >= 0 && ix < c.w;
                    inb |= ok ? (1u << t2) : 0u;
                    qq[t2] = ok ? q_first + (t2 / KS) * c.w + t2 % KS : 0;       // a tap outside the map re-reads flag 0 (ignored)
                }
                tap_word = inb;
                if (c.in_mask) {
                    uint32_t f[KS * KS];
#pragma unroll
                    for (int t2 = 0; t2 < KS * KS; ++t2) f[t2] = c.in_mask[qq[t2]];
                    tap_word = 0;
#pragma unroll
                    for (int t2 = 0; t2 < KS * KS; ++t2) tap_word |= f[t2] ? (1u << t2) : 0u;
                }
                tap_word &= inb;
            }
            s_taps[wave][lane % kTile] = make_int2((int)tap_word, q_first);     // both wave halves store the same pair
            bits = act_trunc_tile<T, V, VPL, UB, false>(e, init != 0, p_mine, lane, dx_taps, 0, e.c, e.c, MaxExchange{nullptr, 1, 0});
        } else {
            bits = act_trunc_tile<T, V, VPL, UB, false>(e, init != 0, p_mine, lane, dx_any, 0, e.c, e.c, MaxExchange{nullptr, 1, 0});
        }
        if (e.surv) { if (lane == 0) store_survivors(e.surv, tile, part, parts, bits); }
        else survivors += __popc(bits);
    }
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

template <typename T>
static dcnn_status launch_dwconv_t(dcnn_ctx* ctx, bool init, const ListArgs& l, const ConvArgs& c, const EpilogueArgs& e) {
    constexpr int VEC = Elem<T>::VEC;
    const bool vec = (e.c % VEC) == 0;
    const int nvec = vec ? e.c / VEC : e.c;
    const int vpl = (int)cdiv(nvec, kWave);
    if (vpl > 4) return fail(ctx, DCNN_EUNSUPPORTED, "depthwise conv: %d channels not supported", e.c);
    const int vpl_used = vpl <= 1 ? 1 : (vpl <= 2 ? 2 : 4);
    const int parts = tile_parts(nvec, vpl_used);
    const int grid = list_grid(ctx, l.max_count, kTileWaves * kTile / parts, 8);
    dim3 g(grid), b(kTileThreads);
    const int ini = init ? 1 : 0;
    // the tap-word forms address input pixels with 32-bit indices
    const bool small = (int64_t)c.n * c.h * c.w < ((int64_t)1 << 31) - 4 * (int64_t)c.w;
    const int ks = (small && c.k >= 1 && c.k <= 3) ? c.k : 0;
#define DCNN_DW_LAUNCH(V, VPL, KS) hipLaunchKernelGGL((dwconv_kernel<T, V, VPL, KS>), g, b, 0, ctx->stream, l, c, e, ini, parts)
#define DCNN_DW_KS(V, VPL)                                                                                         \
    do {                                                                                                           \
        if (ks == 3) DCNN_DW_LAUNCH(V, VPL, 3);                                                                    \
        else if (ks == 2) DCNN_DW_LAUNCH(V, VPL, 2);                                                               \
        else if (ks == 1) DCNN_DW_LAUNCH(V, VPL, 1);                                                               \
        else DCNN_DW_LAUNCH(V, VPL, 0);                                                                            \
    } while (0)
    if (vec) {
        if (vpl_used == 1) DCNN_DW_KS(VEC, 1);
        else if (vpl_used == 2) DCNN_DW_KS(VEC, 2);
        else DCNN_DW_KS(VEC, 4);
    } else {
        if (vpl_used == 1) DCNN_DW_KS(1, 1);
        else if (vpl_used == 2) DCNN_DW_KS(1, 2);
        else DCNN_DW_KS(1, 4);
    }
#undef DCNN_DW_KS
#undef DCNN_DW_LAUNCH
    return check_hip(ctx, hipGetLastError(), "dwconv_kernel launch");
}

dcnn_status launch_dwconv(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const ConvArgs& c,
                          const EpilogueArgs& e) {
    return dtype == DCNN_F16 ? launch_dwconv_t<f16>(ctx, init, l, c, e) : launch_dwconv_t<float>(ctx, init, l, c, e);
}

// ---- input delta generation (dense pass over the frame) ---------------------------------------
// Per pixel: d = frame - P (P = value last propagated); flagged iff max_c |d_c| >= eps;
// flagged: delta <- d, P <- frame.  Writes the whole mask and one count per chunk of pixels.
// With out_data == nullptr only the mask is written (the flags are dilated before anything is
// propagated, Section 4; deltagen_apply_kernel then serves the dilated list).
constexpr int kDeltaGenThreads = 1024;                       // 16 waves per chunk of pixels: enough loads in flight per compute unit
template <typename T, int V, int VPL>
__global__ __launch_bounds__(kDeltaGenThreads) void deltagen_kernel(DeltaGenArgs a, int32_t* chunk_counts) {
    __shared__ int s_count;
    if (threadIdx.x == 0) s_count = 0;
    __syncthreads();
    const int C = a.c;
    const int nvec = (C + V - 1) / V;
    int LP = pow2_ceil((nvec + VPL - 1) / VPL);
    LP = LP > kWave ? kWave : LP;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int sub = lane % LP, grp = lane / LP, PPI = kWave / LP;
    const T* frame = static_cast<const T*>(a.frame);
    T* P = static_cast<T*>(a.P);
    T* out = static_cast<T*>(a.out_data);
    const int64_t chunk_begin = (int64_t)blockIdx.x * kChunk;
    const int64_t chunk_end = min(chunk_begin + kChunk, a.pixels);
    int mine = 0;
    constexpr int NW = kDeltaGenThreads / kWave;
    typedef typename RawOf<T, V>::type Raw;
    constexpr int UB = VPL == 1 ? 4 : (VPL == 2 ? 2 : 1);      // pixel groups whose loads are in flight together
    // The pass is bound by memory latency: the loads of UB pixel groups (frame and P) are issued back
    // to back before any of them is consumed.
    for (int64_t p0 = chunk_begin + (int64_t)wave * PPI; p0 < chunk_end; p0 += (int64_t)UB * NW * PPI) {
        Raw rf[UB][VPL], rq[UB][VPL];
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            const int64_t p = p0 + (int64_t)ub * NW * PPI + grp;
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const int vi = sub + v * LP;
                rf[ub][v] = raw_zero<T, V>(); rq[ub][v] = raw_zero<T, V>();
                if (p < chunk_end && vi < nvec) {
                    rf[ub][v] = raw_load<T, V>(frame + p * C + vi * V);
                    rq[ub][v] = raw_load<T, V>(P + p * C + vi * V);
                }
            }
        }
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            const int64_t p = p0 + (int64_t)ub * NW * PPI + grp;
            const bool valid = p < chunk_end;
            Raw rd[VPL];
            float u = 0.0f;
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const float d = raw_get<T, V>(rf[ub][v], i) - raw_get<T, V>(rq[ub][v], i);
                    u = fmaxf(u, fabsf(d));
                    raw_set<T, V>(rd[v], i, d);
                }
            }
            for (int m = LP >> 1; m >= 1; m >>= 1) u = fmaxf(u, __shfl_xor(u, m, kWave));
            const bool flag = valid && (u >= a.eps);
            if (flag && out != nullptr) {
#pragma unroll
                for (int v = 0; v < VPL; ++v) {
                    const int vi = sub + v * LP;
                    if (vi < nvec) {
                        raw_store<T, V>(out + p * C + vi * V, rd[v]);
                        raw_store<T, V>(P + p * C + vi * V, rf[ub][v]);
                    }
                }
            }
            if (valid && sub == 0) {
                a.out_mask[p] = flag ? 1 : 0;
                mine += flag ? 1 : 0;
            }
        }
    }
    if (mine) atomicAdd(&s_count, mine);
    __syncthreads();
    if (threadIdx.x == 0) chunk_counts[blockIdx.x] = s_count;
}

// Delta generation for a given list of pixels (the dilated input mask): delta <- frame - P, P <- frame.
template <typename T, int V>
__global__ __launch_bounds__(256) void deltagen_apply_kernel(ListArgs l, DeltaGenArgs a) {
    const int64_t count = list_count(l);
    const int C = a.c;
    const int nvec = (C + V - 1) / V;
    const T* frame = static_cast<const T*>(a.frame);
    T* P = static_cast<T*>(a.P);
    T* out = static_cast<T*>(a.out_data);
    const int64_t total = count * nvec;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / nvec;
        const int vi = (int)(i - j * nvec);
        const int64_t p = l.list ? (int64_t)l.list[j] : j;
        float f[V], q[V], d[V];
        load_vec<T, V>(frame + p * C + vi * V, f);
        load_vec<T, V>(P + p * C + vi * V, q);
#pragma unroll
        for (int k = 0; k < V; ++k) d[k] = f[k] - q[k];
        store_vec<T, V>(out + p * C + vi * V, d);
        store_vec<T, V>(P + p * C + vi * V, f);
    }
}

// ---- final accumulation, max pooling, upsampling ----------------------------------------------
template <typename T, int V>
__global__ __launch_bounds__(256) void accum_kernel(ListArgs l, AccumArgs a) {
    const int64_t count = list_count(l);
    const int C = a.c;
    const int nvec = (C + V - 1) / V;
    const T* in = static_cast<const T*>(a.in_data);
    T* O = static_cast<T*>(a.O);
    const int64_t total = count * nvec;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / nvec;
        const int vi = (int)(i - j * nvec);
        const int64_t p = l.list ? (int64_t)l.list[j] : j;
        float d[V], o[V];
        load_vec<T, V>(in + p * C + vi * V, d);
        load_vec<T, V>(O + p * C + vi * V, o);
#pragma unroll
        for (int k = 0; k < V; ++k) o[k] = o[k] + d[k];
        store_vec<T, V>(O + p * C + vi * V, o);
    }
}

// Pooling output pass over the flagged OUTPUT pixels: dy = max_w(x^A (+ delta at flagged inputs)) - max_w(x^A).
// x^A itself is brought up to date by the commit pass afterwards.
template <typename T, int V>
__global__ __launch_bounds__(256) void maxpool_out_kernel(ListArgs l, PoolArgs a, int init) {
    const int64_t count = list_count(l);
    const int C = a.c;
    const int nvec = (C + V - 1) / V;
    const T* in = static_cast<const T*>(a.in_data);
    const T* xA = static_cast<const T*>(a.xA);
    T* out = static_cast<T*>(a.out_data);
    const int64_t total = count * nvec;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / nvec;
        const int vi = (int)(i - j * nvec);
        const int64_t p = l.list ? (int64_t)l.list[j] : j;
        const int ox = (int)(p % a.ow);
        const int64_t t = p / a.ow;
        const int oy = (int)(t % a.oh);
        const int64_t n = t / a.oh;
        float mo[V], mn[V];
#pragma unroll
        for (int k = 0; k < V; ++k) { mo[k] = -INFINITY; mn[k] = -INFINITY; }
        for (int ky = 0; ky < a.k; ++ky) {
            const int iy = oy * a.stride - a.pad + ky;
            if (iy < 0 || iy >= a.h) continue;
            for (int kx = 0; kx < a.k; ++kx) {
                const int ix = ox * a.stride - a.pad + kx;
                if (ix < 0 || ix >= a.w) continue;
                const int64_t q = (n * a.h + iy) * a.w + ix;
                float x[V];
                load_vec<T, V>(xA + q * C + vi * V, x);
#pragma unroll
                for (int k = 0; k < V; ++k) mo[k] = fmaxf(mo[k], x[k]);
                if (!init && a.in_mask[q] != 0) {
                    float d[V];
                    load_vec<T, V>(in + q * C + vi * V, d);
#pragma unroll
                    for (int k = 0; k < V; ++k) x[k] = round_store<T>(x[k] + d[k]);
                }
#pragma unroll
                for (int k = 0; k < V; ++k) mn[k] = fmaxf(mn[k], x[k]);
            }
        }
        float r[V];
#pragma unroll
        for (int k = 0; k < V; ++k) r[k] = init ? mo[k] : mn[k] - mo[k];
        store_vec<T, V>(out + p * C + vi * V, r);
    }
}

template <typename T, int V>
__global__ __launch_bounds__(256) void maxpool_commit_kernel(ListArgs l, PoolArgs a) {
    const int64_t count = list_count(l);
    const int C = a.c;
    const int nvec = (C + V - 1) / V;
    const T* in = static_cast<const T*>(a.in_data);
    T* xA = static_cast<T*>(a.xA);
    const int64_t total = count * nvec;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / nvec;
        const int vi = (int)(i - j * nvec);
        const int64_t p = l.list ? (int64_t)l.list[j] : j;
        float d[V], x[V];
        load_vec<T, V>(in + p * C + vi * V, d);
        load_vec<T, V>(xA + p * C + vi * V, x);
#pragma unroll
        for (int k = 0; k < V; ++k) x[k] = x[k] + d[k];
        store_vec<T, V>(xA + p * C + vi * V, x);
    }
}

template <typename T, int V>
__global__ __launch_bounds__(256) void upsample_kernel(ListArgs l, UpsampleArgs a) {
    const int64_t count = list_count(l);
    const int C = a.c;
    const int nvec = (C + V - 1) / V;
    const T* in = static_cast<const T*>(a.in_data);
    T* out = static_cast<T*>(a.out_data);
    const int ow = a.w * a.factor, oh = a.h * a.factor;
    const int64_t total = count * nvec;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / nvec;
        const int vi = (int)(i - j * nvec);
        const int64_t p = l.list ? (int64_t)l.list[j] : j;
        const int ox = (int)(p % ow);
        const int64_t t = p / ow;
        const int oy = (int)(t % oh);
        const int64_t n = t / oh;
        const int64_t q = (n * a.h + oy / a.factor) * a.w + ox / a.factor;
        float x[V];
        load_vec<T, V>(in + q * C + vi * V, x);
        store_vec<T, V>(out + p * C + vi * V, x);
    }
}

// Channel concatenation over the listed pixels: out[p] = [a[p] or zeros, b[p] or zeros] (a stream that is
// not flagged at p contributes zeros; its memory there is not read).  One element per thread: the channel
// counts of the two inputs need not be multiples of the vector width.
template <typename T>
__global__ __launch_bounds__(256) void concat_kernel(ListArgs l, ConcatArgs a) {
    const int64_t count = list_count(l);
    const int C = a.ca + a.cb;
    const T* xa = static_cast<const T*>(a.a_data);
    const T* xb = static_cast<const T*>(a.b_data);
    T* out = static_cast<T*>(a.out_data);
    const int64_t total = count * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / C;
        const int ch = (int)(i - j * C);
        const int64_t p = l.list ? (int64_t)l.list[j] : j;
        T v = (T)0.0f;
        if (ch < a.ca) {
            if (a.a_mask == nullptr || a.a_mask[p]) v = xa[p * a.ca + ch];
        } else {
            if (a.b_mask == nullptr || a.b_mask[p]) v = xb[p * a.cb + (ch - a.ca)];
        }
        out[p * C + ch] = v;
    }
}

static int flat_grid(const dcnn_ctx* ctx, int64_t max_count, int c, int vec) {
    int64_t total = (max_count > 0 ? max_count : 1) * cdiv(c, vec);
    int64_t want = cdiv(total, 256);
    int64_t cap = (int64_t)ctx->num_cu * 8;
    return (int)(want < cap ? want : cap);
}

#define DCNN_FLAT_DISPATCH(KERNEL, CHANNELS, MAXCOUNT, ...)                                               \
    do {                                                                                                  \
        if (dtype == DCNN_F16) {                                                                          \
            if ((CHANNELS) % 8 == 0)                                                                      \
                hipLaunchKernelGGL((KERNEL<f16, 8>), dim3(flat_grid(ctx, MAXCOUNT, CHANNELS, 8)), dim3(256), 0, \
                                   ctx->stream, __VA_ARGS__);                                             \
            else                                                                                          \
                hipLaunchKernelGGL((KERNEL<f16, 1>), dim3(flat_grid(ctx, MAXCOUNT, CHANNELS, 1)), dim3(256), 0, \
                                   ctx->stream, __VA_ARGS__);                                             \
        } else {                                                                                          \
            if ((CHANNELS) % 4 == 0)                                                                      \
                hipLaunchKernelGGL((KERNEL<float, 4>), dim3(flat_grid(ctx, MAXCOUNT, CHANNELS, 4)), dim3(256), 0, \
                                   ctx->stream, __VA_ARGS__);                                             \
            else                                                                                          \
                hipLaunchKernelGGL((KERNEL<float, 1>), dim3(flat_grid(ctx, MAXCOUNT, CHANNELS, 1)), dim3(256), 0, \
                                   ctx->stream, __VA_ARGS__);                                             \
        }                                                                                                 \
    } while (0)

dcnn_status launch_accum(dcnn_ctx* ctx, int dtype, const ListArgs& l, const AccumArgs& a) {
    DCNN_FLAT_DISPATCH(accum_kernel, a.c, l.max_count, l, a);
    return check_hip(ctx, hipGetLastError(), "accum_kernel launch");
}

dcnn_status launch_maxpool_out(dcnn_ctx* ctx, int dtype, bool init, const ListArgs& l, const PoolArgs& a) {
    const int ini = init ? 1 : 0;
    DCNN_FLAT_DISPATCH(maxpool_out_kernel, a.c, l.max_count, l, a, ini);
    return check_hip(ctx, hipGetLastError(), "maxpool_out_kernel launch");
}

dcnn_status launch_maxpool_commit(dcnn_ctx* ctx, int dtype, const ListArgs& l, const PoolArgs& a) {
    DCNN_FLAT_DISPATCH(maxpool_commit_kernel, a.c, l.max_count, l, a);
    return check_hip(ctx, hipGetLastError(), "maxpool_commit_kernel launch");
}

dcnn_status launch_upsample(dcnn_ctx* ctx, int dtype, const ListArgs& l, const UpsampleArgs& a) {
    DCNN_FLAT_DISPATCH(upsample_kernel, a.c, l.max_count, l, a);
    return check_hip(ctx, hipGetLastError(), "upsample_kernel launch");
}

dcnn_status launch_concat(dcnn_ctx* ctx, int dtype, const ListArgs& l, const ConcatArgs& a) {
    const int grid = flat_grid(ctx, l.max_count, a.ca + a.cb, 1);
    if (dtype == DCNN_F16) hipLaunchKernelGGL((concat_kernel<f16>), dim3(grid), dim3(256), 0, ctx->stream, l, a);
    else hipLaunchKernelGGL((concat_kernel<float>), dim3(grid), dim3(256), 0, ctx->stream, l, a);
    return check_hip(ctx, hipGetLastError(), "concat_kernel launch");
}

dcnn_status launch_deltagen(dcnn_ctx* ctx, int dtype, const DeltaGenArgs& a_in) {
    if (a_in.dilate_r < 0 || a_in.dilate_r > 15) return fail(ctx, DCNN_EINVAL, "input-mask dilation radius %d out of range", a_in.dilate_r);
    Workspace ws;
    dcnn_status st = workspace_view(ctx, a_in.pixels, &ws);
    if (st != DCNN_OK) return st;
    // With a dilation the first pass only flags (into scratch), nothing is propagated yet.
    DeltaGenArgs a = a_in;
    if (a.dilate_r > 0) { a.out_data = nullptr; a.out_mask = ws.scratch_mask; }
    const int nchunks = (int)cdiv(a.pixels, kChunk);
    dim3 g(nchunks), b(kDeltaGenThreads);
#define DCNN_DG_LAUNCH(T, V, VPL) hipLaunchKernelGGL((deltagen_kernel<T, V, VPL>), g, b, 0, ctx->stream, a, ws.chunk_counts)
#define DCNN_DG_PICK(T, V)                                                                       \
    do {                                                                                         \
        const int64_t vpl = cdiv(cdiv(a.c, V), kWave);                                           \
        if (vpl <= 1) DCNN_DG_LAUNCH(T, V, 1);                                                   \
        else if (vpl <= 2) DCNN_DG_LAUNCH(T, V, 2);                                              \
        else if (vpl <= 4) DCNN_DG_LAUNCH(T, V, 4);                                              \
        else return fail(ctx, DCNN_EUNSUPPORTED, "delta generation: %d channels not supported", a.c); \
    } while (0)
    if (dtype == DCNN_F16) {
        if (a.c % 8 == 0) DCNN_DG_PICK(f16, 8); else DCNN_DG_PICK(f16, 1);
    } else {
        if (a.c % 4 == 0) DCNN_DG_PICK(float, 4); else DCNN_DG_PICK(float, 1);
    }
#undef DCNN_DG_PICK
#undef DCNN_DG_LAUNCH
    st = check_hip(ctx, hipGetLastError(), "deltagen_kernel launch");
    if (st != DCNN_OK) return st;
    if (a.dilate_r > 0) {
        // square dilation as a row pass and a column pass (Section 4: the input mask is dilated so that
        // small changes next to changed pixels are propagated with them), then the list-driven update
        const int k = 2 * a.dilate_r + 1;
        MaskPassArgs h{};
        h.mask_in = ws.scratch_mask; h.mask_out = ws.scratch_mask2; h.idx_out = nullptr;
        h.n = a.n; h.h = a.h; h.w = a.w; h.oh = a.h; h.ow = a.w; h.stride = 1; h.up = 1;
        h.k = 1; h.pad = 0; h.kw = k; h.pad_w = a.dilate_r;
        st = launch_mask_compact(ctx, h);
        if (st != DCNN_OK) return st;
        MaskPassArgs v = h;
        v.mask_in = ws.scratch_mask2; v.mask_out = a_in.out_mask; v.idx_out = a_in.out_idx; v.count_out = a_in.out_count;
        v.k = k; v.pad = a.dilate_r; v.kw = 1; v.pad_w = 0;
        st = launch_mask_compact(ctx, v);
        if (st != DCNN_OK) return st;
        ListArgs l{};
        l.list = a_in.out_idx; l.count = a_in.out_count; l.max_count = a_in.pixels;
        DCNN_FLAT_DISPATCH(deltagen_apply_kernel, a_in.c, l.max_count, l, a_in);
        return check_hip(ctx, hipGetLastError(), "deltagen_apply_kernel launch");
    }
    // ordered emission of the flagged pixels from the mask just written and the chunk counts
    MaskPassArgs m{};
    m.mask_in = a.out_mask;
    m.mask_out = nullptr;
    m.idx_out = a.out_idx;
    m.count_out = a.out_count;
    m.n = a.n; m.h = a.h; m.w = a.w; m.oh = a.h; m.ow = a.w; m.k = 1;
    m.stride = 1; m.pad = 0; m.up = 1; m.emit_only = 1;
    return launch_mask_compact(ctx, m);
}

// ---- small utilities ------------------------------------------------------------------------
template <typename T> __global__ void fill_kernel(T* p, T v, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

dcnn_status launch_fill_i32(dcnn_ctx* ctx, int32_t* p, int32_t v, int64_t n) {
    int grid = (int)(cdiv(n, 256) < 2048 ? cdiv(n, 256) : 2048);
    hipLaunchKernelGGL((fill_kernel<int32_t>), dim3(grid > 0 ? grid : 1), dim3(256), 0, ctx->stream, p, v, n);
    return check_hip(ctx, hipGetLastError(), "fill_kernel launch");
}

dcnn_status launch_fill_u8(dcnn_ctx* ctx, uint8_t* p, uint8_t v, int64_t n) {
    // fill 4 bytes at a time where the length allows (buffers are 256-byte aligned)
    if (n % 4 == 0) {
        const int32_t w = (int32_t)(0x01010101u * v);
        return launch_fill_i32(ctx, reinterpret_cast<int32_t*>(p), w, n / 4);
    }
    int grid = (int)(cdiv(n, 256) < 2048 ? cdiv(n, 256) : 2048);
    hipLaunchKernelGGL((fill_kernel<uint8_t>), dim3(grid > 0 ? grid : 1), dim3(256), 0, ctx->stream, p, v, n);
    return check_hip(ctx, hipGetLastError(), "fill_kernel launch");
}

dcnn_status launch_copy(dcnn_ctx* ctx, void* dst, const void* src, size_t bytes) {
    return check_hip(ctx, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, ctx->stream), "hipMemcpyAsync");
}

}  // namespace dcnn
