// Sparse delta convolution with dense weights as a gather-GEMM on the matrix cores: the plain kernel
// (every wave does gather, MFMA and tail of its tile in turn).  It serves the dense first frame, layers
// whose weights are streamed, windows other than 1x1 / 3x3 and channel counts that do not fill 16-byte
// vectors; the sparse steps of everything else run on the wave-specialised kernel (conv_ws_impl.h) or, with
// weights too large for LDS and a long list, on the register-blocked kernel (conv_direct_impl.h), which
// launch_conv_nb below dispatches to.
//
// The work list holds the flagged OUTPUT pixels in ascending order.  A tile of 32 consecutive list
// entries is owned by `cs` wavefronts, each computing nb*32 of the output channels:
//     D[cout][pixel] += W_tap[cout][cin] * X_tap[cin][pixel]        for every window tap
// with MFMA 32x32 blocks (A operand = weights from LDS, B operand = the pixel's channels gathered
// straight from the NHWC delta map into registers, 16 bytes per lane).  A tap contributes only
// where the input pixel is in bounds AND flagged; every other lane reads a page of zeros instead,
// so the inner loop has no branches and unflagged memory (invalid by contract) is never touched.
// When the packed weight tensor of the layer fits, it stays resident in LDS (160 KB per CU on
// gfx950) for the lifetime of the persistent workgroup.  Larger layers stream it: the waves of a
// workgroup walk the K dimension in lockstep and a double-buffered 4-K-step slice of the weights
// is copied global -> registers -> LDS while the matrix cores consume the previous slice.
// The fp32 result tile is rounded to the storage type, staged through LDS (private to the wave)
// and handed to the activation + truncation tail with coalesced accesses; waves that share a tile
// agree on the per-pixel maximum through LDS.
#pragma once

#include "conv_plan.h"
#include "conv_ws_impl.h"
#include "conv_direct_impl.h"

namespace dcnn {

#ifndef DCNN_CONV_BOUNDS
#define DCNN_CONV_BOUNDS 512
#endif
// WMODE: where the weight operands come from -- 0 resident in LDS, 1 streamed through LDS in slices (8 waves in
// lockstep), 2 loaded straight from global memory / L2 by each wave together with its gathers, several K-steps in
// flight (short work lists on layers whose weights do not fit LDS; 4 waves of up to 512 registers).
template <typename T, int NB, int V, bool ALIGNED, int WMODE, int KS>
__global__ __launch_bounds__(WMODE == 2 ? 256 : DCNN_CONV_BOUNDS) void conv_mfma_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, int init,
                                                                 int npass, int cs, int pass_split) {
    typedef typename Mma<T>::Vec Vec;
    typedef typename RawOf<T, V>::type Raw;
    constexpr int KP = Mma<T>::KPACK;
    constexpr int COLS = NB * 32;
    constexpr int GK = 4;                                      // K-steps whose gathers are in flight together
    constexpr bool STREAM = WMODE == 1;
    extern __shared__ __align__(16) unsigned char smem[];
    clear_ahead(e);

    const int nwaves = blockDim.x / kWave, nthreads = blockDim.x;
    const int tiles_per_iter = nwaves / cs;
    const int64_t count = list_count(l);
    const WgTileRange r = wg_tile_range((count + tiles_per_iter * kTile - 1) / (tiles_per_iter * kTile));
    if (r.begin >= r.end) return;                              // nothing for this workgroup: skip the weight load

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int col = lane % 32, g = lane / 32;
    const int slot = wave / cs, part = wave % cs;              // which tile of the iteration, which channel slice
    const int ksz = KS ? KS : c.k;
    const int taps = ksz * ksz, kch = c.kch;
    // flat K (stems with very few channels, unaligned kernels only): the K loop sees ONE tap of kch K-steps whose
    // elements are (tap, channel) pairs; which window tap an element belongs to is looked up per element
    const bool flat = !ALIGNED && c.flat != 0;
    const int ktaps = flat ? 1 : taps;
    const int ksteps = ktaps * kch;
    const bool full_tail = npass == 1;
    const int slice_vecs = cs * kGroup * 2 * COLS;             // one streamed slice (all channel slices)
    const int w_vecs = WMODE == 2 ? 0 : (STREAM ? 2 * slice_vecs : npass * cs * ksteps * 2 * COLS);
    Vec* w_lds = reinterpret_cast<Vec*>(smem);
    constexpr int stage_stride = COLS * (int)sizeof(T) + kStagePad;
    unsigned char* stage = smem + (size_t)w_vecs * 16 + (size_t)wave * kTile * stage_stride;
    float* xchg = reinterpret_cast<float*>(smem + (size_t)w_vecs * 16 + (size_t)nwaves * kTile * stage_stride) +
                  (size_t)slot * 2 * cs * kTile;
    const Vec* wglob = static_cast<const Vec*>(c.wpacked);
    const T* in = static_cast<const T*>(c.in_data);
    const T* zeros = static_cast<const T*>(c.zero_page);

    // flat K: element j of the K dimension -> (offset of its value from the window's first input element, tap)
    int2* flat_lut = reinterpret_cast<int2*>(smem + (size_t)w_vecs * 16 + (size_t)nwaves * kTile * stage_stride +
                                             (size_t)2 * nwaves * kTile * sizeof(float));
    if constexpr (WMODE == 0) {
        for (int i = threadIdx.x; i < w_vecs; i += nthreads) w_lds[i] = wglob[i];
        if constexpr (!ALIGNED) {
            if (flat) {
                for (int j = threadIdx.x; j < taps * c.cin; j += nthreads) {
                    const int tap = j / c.cin, ch = j - tap * c.cin;
                    const int dy = tap / ksz, dx = tap - dy * ksz;
                    flat_lut[j] = make_int2((dy * c.w + dx) * c.cin + ch, tap);
                }
            }
        }
        lds_block_sync();
    }

    // First frame: the bias joins the fp32 sum BEFORE its one rounding to the storage type (a convolution with
    // bias is one operation); the tail sees a finished result.
    const T* bias_f = (init != 0) ? static_cast<const T*>(e.bias) : nullptr;
    int survivors = 0;                                         // per-wave count, added to the layer's counter once
    // tail loads are prefetched when a tile takes at most 4 lane-iterations (narrow channel slices)
    constexpr int TAIL_LP = (COLS / V) <= 2 ? 2 : ((COLS / V) <= 4 ? 4 : ((COLS / V) <= 8 ? 8 : ((COLS / V) <= 16 ? 16 : ((COLS / V) <= 32 ? 32 : 64))));
    constexpr int NIT = kTile / (kWave / TAIL_LP);
    constexpr bool PREFETCH_TAIL = NIT <= 4 && WMODE == 0;
    // Software pipeline over tiles: the list entry of tile n+2 and the update flags of tile n+1 are
    // requested while tile n is processed, so neither round trip sits on a tile's critical path.
    struct TileGeom { int p32; bool valid; int iy0, ix0, q00; };
    auto geometry = [&](int p32) {
        TileGeom gm;
        gm.p32 = p32;
        gm.valid = p32 >= 0;
        const uint32_t pu = gm.valid ? (uint32_t)p32 : 0u;
        const uint32_t t1 = fast_div(pu, c.div_ow);
        const int ox = (int)(pu - t1 * (uint32_t)c.ow);
        const uint32_t n = fast_div(t1, c.div_oh);
        const int oy = (int)(t1 - n * (uint32_t)c.oh);
        gm.iy0 = oy * c.stride - c.pad;
        gm.ix0 = ox * c.stride - c.pad;
        gm.q00 = ((int)n * c.h + gm.iy0) * c.w + gm.ix0;       // pixel index of tap (0,0); only used when in bounds
        return gm;
    };
    constexpr int NFLAG = KS ? KS * KS : 1;
    auto request_flags = [&](const TileGeom& gm, uint8_t (&flag)[NFLAG]) {
        // fixed window: all update flags of the window are requested at once (tested one tile later)
        if constexpr (KS != 0) {
#pragma unroll
            for (int t = 0; t < KS * KS; ++t) {
                const int dy = t / KS, dx = t % KS;
                const bool inb = gm.valid && (unsigned)(gm.iy0 + dy) < (unsigned)c.h && (unsigned)(gm.ix0 + dx) < (unsigned)c.w;
                const int q = inb ? gm.q00 + dy * c.w + dx : 0;
                flag[t] = c.in_mask ? c.in_mask[q] : (uint8_t)1;
                if (!inb) flag[t] = 0;
            }
        }
    };
    auto entry = [&](int64_t wt_) {
        return wt_ < r.end ? list_pixel(l.list, (wt_ * tiles_per_iter + slot) * kTile + col, count) : -1;
    };
    TileGeom g_next = geometry(entry(r.begin));
    int p32_next2 = entry(r.begin + r.step);
    uint8_t flag_next[NFLAG];
    request_flags(g_next, flag_next);
    for (int64_t wt = r.begin; wt < r.end; wt += r.step) {
        // ---- the tile: pixel of this lane's column, window origin, which taps are needed ---------
        // (pixel indices fit 31 bits; only the final element offset is 64-bit)
        const int64_t tile = wt * tiles_per_iter + slot;
        const int64_t base = tile * kTile;
        const TileGeom gm = g_next;
        const int p32 = gm.p32;
        const bool valid = gm.valid;
        const int iy0 = gm.iy0, ix0 = gm.ix0, q00 = gm.q00;
        uint64_t tapbits = 0;
        if constexpr (KS != 0) {
#pragma unroll
            for (int t = 0; t < KS * KS; ++t)
                if (flag_next[t]) tapbits |= 1ull << t;
        } else {
            for (int t = 0, dy = 0, dx = 0; t < taps; ++t) {
                bool ok = valid && (unsigned)(iy0 + dy) < (unsigned)c.h && (unsigned)(ix0 + dx) < (unsigned)c.w;
                if (ok && c.in_mask) ok = c.in_mask[q00 + dy * c.w + dx] != 0;
                if (ok) tapbits |= 1ull << t;
                if (++dx == ksz) { dx = 0; ++dy; }
            }
        }
        // requests for the tiles to come
        g_next = geometry(p32_next2);
        p32_next2 = entry(wt + 2 * r.step);
        request_flags(g_next, flag_next);

        // Wave-uniform cursor over groups of GK K-steps: tap t = (dy, dx), first K-step kc0 of the group.
        struct Cursor { int t, dy, dx, kc0; };
        auto advance = [&](Cursor& cu) {
            cu.kc0 += GK;
            if (cu.kc0 >= kch) {
                cu.kc0 = 0; ++cu.t;
                if (++cu.dx == ksz) { cu.dx = 0; ++cu.dy; }
            }
            // (flat K: t counts to ktaps = 1, dy / dx are not used)
        };
        // 16 bytes of input channels per K-step for this lane's pixel; lanes that do not need the tap
        // (or whose channels are padding) read the zero page instead: no branches, no invalid reads
        auto gather_group = [&](const Cursor& cu, Vec (&x)[GK]) {
            if constexpr (!ALIGNED) {
                if (flat) {
                    const T* first = in + (int64_t)q00 * c.cin;   // element of tap (0,0), channel 0; only used with a flagged tap
                    const int nflat = taps * c.cin;
#pragma unroll
                    for (int u = 0; u < GK; ++u) {
                        Vec v;
#pragma unroll
                        for (int i = 0; i < KP; ++i) {
                            const int j = (2 * (cu.kc0 + u) + g) * KP + i;
                            const bool inside = cu.t < ktaps && cu.kc0 + u < kch && j < nflat;
                            const int2 lt = flat_lut[inside ? j : 0];
                            const bool ok = inside && ((tapbits >> lt.y) & 1);
                            v[i] = ok ? first[lt.x] : (T)0.0f;
                        }
                        x[u] = v;
                    }
                    return;
                }
            }
            const bool tap_ok = cu.t < taps && ((tapbits >> cu.t) & 1);
            const T* src = in + (int64_t)(q00 + cu.dy * c.w + cu.dx) * c.cin;
#pragma unroll
            for (int u = 0; u < GK; ++u) {
                const int ch = (2 * (cu.kc0 + u) + g) * KP;
                const bool ok = tap_ok && cu.kc0 + u < kch && ch < c.cin;
                const T* ptr = ok ? src + ch : zeros;
                if constexpr (ALIGNED) {
                    x[u] = *reinterpret_cast<const Vec*>(ptr);
                } else {
                    Vec v;
#pragma unroll
                    for (int i = 0; i < KP; ++i) v[i] = (ok && ch + i < c.cin) ? ptr[i] : (T)0.0f;
                    x[u] = v;
                }
            }
        };

        // passes are independent (each writes its own output channels): short work lists spread them over
        // blockIdx.y so that more compute units stream weights
        const int pass_first = blockIdx.y * pass_split;
        const int pass_last = pass_first + pass_split < npass ? pass_first + pass_split : npass;
        for (int pass = pass_first; pass < pass_last; ++pass) {
            const int cgroup = pass * cs + part;               // which group of COLS output channels
            const int ch0 = cgroup * COLS;
            int nch = e.c - ch0;
            nch = nch < 0 ? 0 : (nch > COLS ? COLS : nch);
            TailRegs<T, V, PREFETCH_TAIL ? NIT : 1> tl;
            if constexpr (PREFETCH_TAIL) tail_prefetch<T, V, NIT>(e, init != 0, p32, lane, ch0, nch, tl);
            f32x16 acc[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

            if constexpr (WMODE == 2) {
                // weights from global memory: every K-step's operands (one gathered input vector, NB weight vectors)
                // are requested RH K-steps at a time, two such sets in flight; no LDS, no barrier in the loop.
                // K-steps are walked linearly over (tap, channel group); past the end a step gathers zeros.
                constexpr int RH = 8;
                const Vec* wbase = wglob + ((size_t)cgroup * ksteps * 2 + g) * COLS + col;
                struct Lin { int ks, t, kc, dy, dx; };
                auto issue = [&](Lin& li, Vec (&x)[RH], Vec (&wv)[RH][NB]) {
#pragma unroll
                    for (int u = 0; u < RH; ++u) {
                        const bool live = li.ks < ksteps;
                        const bool tap_ok = live && ((tapbits >> (li.t & 63)) & 1);
                        const int ch = (2 * li.kc + g) * KP;
                        const bool ok = tap_ok && ch < c.cin;
                        const T* ptr = ok ? in + (int64_t)(q00 + li.dy * c.w + li.dx) * c.cin + ch : zeros;
                        x[u] = *reinterpret_cast<const Vec*>(ptr);
                        const Vec* wrow = wbase + (size_t)(live ? li.ks : 0) * 2 * COLS;
#pragma unroll
                        for (int b = 0; b < NB; ++b) wv[u][b] = wrow[b * 32];
                        ++li.ks;
                        if (++li.kc == kch) {
                            li.kc = 0; ++li.t;
                            if (++li.dx == ksz) { li.dx = 0; ++li.dy; }
                        }
                    }
                };
                auto mma = [&](const Vec (&x)[RH], const Vec (&wv)[RH][NB]) {
#pragma unroll
                    for (int u = 0; u < RH; ++u)
#pragma unroll
                        for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wv[u][b], x[u]);
                };
                Vec xa[RH], xb[RH], wa[RH][NB], wb[RH][NB];
                Lin li{0, 0, 0, 0, 0};
                issue(li, xa, wa);
                for (int ks0 = 0; ks0 < ksteps; ks0 += 2 * RH) {
                    issue(li, xb, wb);
                    mma(xa, wa);
                    issue(li, xa, wa);
                    mma(xb, wb);
                }
            } else if constexpr (!STREAM) {
                // weights resident: waves run independently; the gathers of the next group of K-steps
                // are in flight while the matrix cores work on the current group (two register sets)
                const Vec* wbase = w_lds + ((size_t)cgroup * ksteps * 2 + g) * COLS + col;
                auto mma_group = [&](const Cursor& cu, const Vec (&x)[GK]) {
                    // all weight operands of the group are requested from LDS before the first MFMA issues,
                    // so their latency is paid once per group instead of once per instruction
                    const Vec* wrow = wbase + (size_t)(cu.t * kch + cu.kc0) * 2 * COLS;
                    Vec wv[GK][NB];
#pragma unroll
                    for (int u = 0; u < GK; ++u)
#pragma unroll
                        for (int b = 0; b < NB; ++b)
                            wv[u][b] = (cu.kc0 + u < kch) ? wrow[(size_t)u * 2 * COLS + b * 32] : wrow[b * 32];
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int u = 0; u < GK; ++u) {
                        if (cu.kc0 + u < kch) {
#pragma unroll
                            for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wv[u][b], x[u]);
                        }
                    }
                };
                Vec xa[GK], xb[GK];
                Cursor ca{0, 0, 0, 0}, cb;
                gather_group(ca, xa);
                while (ca.t < ktaps) {
                    cb = ca; advance(cb);
                    if (cb.t < ktaps) gather_group(cb, xb);
                    mma_group(ca, xa);
                    if (cb.t >= ktaps) break;
                    ca = cb; advance(ca);
                    if (ca.t < ktaps) gather_group(ca, xa);
                    mma_group(cb, xb);
                }
            } else {
                // weights streamed: all waves walk the slices (tap, group of 4 K-steps) in lockstep;
                // slice i+1 travels global -> registers while slice i is multiplied, then registers ->
                // LDS, one barrier per slice.  A slice holds the weights of all `cs` channel slices.
                const int groups = (kch + kGroup - 1) / kGroup;
                const int nslices = taps * groups;
                constexpr int kConvThreads = 8 * kWave;         // streaming workgroups always have 8 waves
                constexpr int WREG = 4 * NB / 2;               // >= cs * kGroup * 2 * COLS / kConvThreads for cs <= 4
                Vec wreg[WREG];
                auto slice_load = [&](int si) {
                    const int t = si / groups, kc0 = (si % groups) * kGroup;
                    const int steps = kch - kc0 < kGroup ? kch - kc0 : kGroup;
                    const int per_part = steps * 2 * COLS;
#pragma unroll
                    for (int i = 0; i < WREG; ++i) {
                        const int vi = threadIdx.x + i * kConvThreads;
                        const int q = vi / (kGroup * 2 * COLS), o = vi - q * (kGroup * 2 * COLS);
                        if (q < cs && o < per_part)
                            wreg[i] = wglob[((size_t)((pass * cs + q) * ksteps + t * kch + kc0) * 2) * COLS + o];
                    }
                };
                auto slice_store = [&](int si) {
                    const int kc0 = (si % groups) * kGroup;
                    const int steps = kch - kc0 < kGroup ? kch - kc0 : kGroup;
                    const int per_part = steps * 2 * COLS;
                    Vec* dst = w_lds + (size_t)(si & 1) * slice_vecs;
#pragma unroll
                    for (int i = 0; i < WREG; ++i) {
                        const int vi = threadIdx.x + i * kConvThreads;
                        const int q = vi / (kGroup * 2 * COLS), o = vi - q * (kGroup * 2 * COLS);
                        if (q < cs && o < per_part) dst[vi] = wreg[i];
                    }
                };
                static_assert(GK == kGroup, "the streamed slice is one group of K-steps");
                auto gather_slice = [&](int si, Vec (&x)[kGroup]) {
                    const int t = si / groups;
                    Cursor cu{t, t / ksz, t % ksz, (si % groups) * kGroup};
                    gather_group(cu, x);
                };
                Vec xa[kGroup], xb[kGroup];
                slice_load(0);
                gather_slice(0, xa);
                slice_store(0);
                lds_block_sync();
                for (int si = 0; si < nslices; ++si) {
                    const int kc0 = (si % groups) * kGroup;
                    if (si + 1 < nslices) {
                        slice_load(si + 1);
                        gather_slice(si + 1, xb);
                    }
                    const Vec* wrow = w_lds + (size_t)(si & 1) * slice_vecs + (size_t)part * (kGroup * 2 * COLS) +
                                      (size_t)g * COLS + col;
#pragma unroll
                    for (int u = 0; u < kGroup; ++u) {
                        if (kc0 + u < kch) {
#pragma unroll
                            for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wrow[(size_t)u * 2 * COLS + b * 32], xa[u]);
                        }
                    }
                    if (si + 1 < nslices) slice_store(si + 1);
                    lds_block_sync();
#pragma unroll
                    for (int u = 0; u < kGroup; ++u) xa[u] = xb[u];
                }
            }

            // ---- tail: this wave's channel slice of the tile ------------------------------------
            if (bias_f) {
                // accumulator i of block b, quad q belongs to output channel b*32 + 8*q + 4*g + i
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int ch = ch0 + b * 32 + 8 * q + 4 * g + i;
                            if (ch < e.c) acc[b][4 * q + i] += (float)bias_f[ch];
                        }
            }
            stage_accumulators<T, NB>(acc, stage + (size_t)col * stage_stride, g);
            lds_wave_sync();
            auto dx = [&](int ent, int64_t, int c0) -> Raw {
                return raw_load<T, V>(reinterpret_cast<const T*>(stage + (size_t)ent * stage_stride) + (c0 - ch0));
            };
            const MaxExchange mx{xchg, cs, part};
            uint32_t bits;
            const bool exchange = cs > 1 && full_tail && e.act != DCNN_ACT_NONE && !init;
            if constexpr (PREFETCH_TAIL) {
                if (exchange) bits = tail_finish<T, V, NIT, true>(e, false, lane, dx, ch0, nch, mx, tl);
                else bits = tail_finish<T, V, NIT, false>(e, init != 0, lane, dx, ch0, nch, mx, tl);
            } else {
                if (exchange) bits = act_trunc_tile<T, V, 1, 2, true>(e, false, p32, lane, dx, ch0, nch, COLS, mx);
                else bits = act_trunc_tile<T, V, 1, 2, false>(e, init != 0, p32, lane, dx, ch0, nch, COLS, mx);
            }
            if (full_tail && part == 0 && base < count) {
                if (e.surv) { if (lane == 0) e.surv[tile] = bits; }
                else survivors += __popc(bits);
            }
            lds_wave_sync();
        }
    }
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

template <typename T, int NB>
static dcnn_status launch_conv_nb(dcnn_ctx* ctx, bool init, const ListArgs& l, const ConvArgs& c, const EpilogueArgs& e,
                                  const ConvPlan& p) {
    constexpr int VEC = Elem<T>::VEC;
    const bool vec_out = (e.c % VEC) == 0;
    const bool aligned = ((size_t)c.cin * sizeof(T)) % 16 == 0;
    // Weights that do not fit LDS and a short work list (at most two 4-wave workgroups per compute unit cover it):
    // every wave loads its weight operands itself, several K-steps ahead, instead of one streamed slice per round
    // trip to memory.  Sparse steps with 16-byte aligned channels only.
    const int64_t max_tiles = cdiv(l.max_count > 0 ? l.max_count : 1, kTile);
    const bool direct = p.stream && !init && vec_out && aligned && cdiv(max_tiles * p.cs, kDirectWaves) <= 2 * (int64_t)ctx->num_cu;
    const int waves = direct ? kDirectWaves : p.waves;
    const size_t lds_bytes = direct ? conv_stage_bytes(kDirectWaves, NB, sizeof(T) == 2 ? DCNN_F16 : DCNN_F32) + conv_xchg_bytes(kDirectWaves)
                                    : p.lds_bytes;
    const int tiles_per_iter = waves / p.cs;
    int64_t want = cdiv(l.max_count > 0 ? l.max_count : 1, tiles_per_iter * kTile);
    int64_t per_cu = (int64_t)(kLdsBytes / lds_bytes);
    per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
    if (direct) per_cu = 2;
    int64_t cap = (int64_t)ctx->num_cu * per_cu;
    const int grid = (int)(cdiv(want < cap ? want : cap, kXcd) * kXcd);
    // several passes and fewer workgroups than the chip holds: spread the passes over grid.y
    int ysplit = 1;
    if (p.npass > 1 && grid < cap) {
        const int64_t room = cap / grid;
        ysplit = (int)(room < p.npass ? room : p.npass);
        if (ysplit < 1) ysplit = 1;
    }
    const int pass_split = (int)cdiv(p.npass, ysplit);
    const int grid_y = (int)cdiv(p.npass, pass_split);
    const int ini = init ? 1 : 0;
    hipError_t err = hipSuccess;
    bool launched = false;
#define DCNN_CONV_LAUNCH(V, AL, WM, KS)                                                                          \
    do {                                                                                                         \
        auto kern = conv_mfma_kernel<T, NB, V, AL, WM, KS>;                                                      \
        static bool attr_set = false;                                                                            \
        if (!attr_set) {                                                                                         \
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                      (int)kLdsBytes);                                                           \
            attr_set = (err == hipSuccess);                                                                      \
        }                                                                                                        \
        if (err == hipSuccess)                                                                                   \
            hipLaunchKernelGGL(kern, dim3(grid, grid_y), dim3(waves * kWave), lds_bytes, ctx->stream, l, c, e, ini, p.npass, p.cs, pass_split); \
        launched = true;                                                                                         \
    } while (0)
    // resident weights, vector-aligned channels, one pass, sparse step: the wave-specialised kernel
    const bool dual = c.in2_data != nullptr;
    const size_t ws_lds = conv_ws_lds_bytes(p, sizeof(T) == 2 ? DCNN_F16 : DCNN_F32, c.k, e.c, dual ? c.cin2 : 0);
    const uint64_t in_bytes = (uint64_t)c.n * c.h * c.w * c.cin * sizeof(T);
    const uint64_t in2_bytes = dual ? (uint64_t)c.n * c.h2 * c.w2 * c.cin2 * sizeof(T) : 0;
    const uint64_t out_bytes = (uint64_t)c.n * c.oh * c.ow * e.c * sizeof(T);
    // (a window wider than 1x1, or a 1x1 walk over a list that is not the input's own, needs the tap words)
    const bool ws_taps = l.taps != nullptr || (c.k == 1 && c.stride == 1 && l.list != nullptr && c.in_mask != nullptr);
    const bool ws_ok = vec_out && aligned && ws_lds != 0 && !init && ws_taps && in_bytes <= kWsMaxBytes &&
                       in2_bytes <= kWsMaxBytes && out_bytes <= kWsMaxBytes;
    const bool accum = e.accum_O != nullptr;
    if (dual && (!ws_ok || l.taps == nullptr || e.res_data != nullptr || ((size_t)c.cin2 * sizeof(T)) % 16 != 0))
        return fail(ctx, DCNN_EUNSUPPORTED, "conv %dx%d %d->%d with a fused projection of %d channels: shape not covered", c.k,
                    c.k, c.cin, c.cout, c.cin2);
    if (accum && (!ws_ok || e.res_data != nullptr || e.act == DCNN_ACT_NONE))
        return fail(ctx, DCNN_EUNSUPPORTED, "conv %dx%d %d->%d with a fused final accumulation: shape not covered", c.k, c.k,
                    c.cin, c.cout);
    if (e.xt_flags != nullptr && !ws_ok && !init)
        return fail(ctx, DCNN_EUNSUPPORTED, "conv %dx%d %d->%d: x^T row flags are kept by the wave-specialised kernel only", c.k, c.k,
                    c.cin, c.cout);
    if (ws_ok) {
        const int64_t ws_want = cdiv(l.max_count > 0 ? l.max_count : 1, (kWsProducers / p.cs) * kTile);
        const int64_t ws_cap = ctx->num_cu;                    // 16 waves of up to 128 registers fill a compute unit
        const int ws_grid = (int)(cdiv(ws_want < ws_cap ? ws_want : ws_cap, kXcd) * kXcd);
#define DCNN_WS_LAUNCH(KS, AUX, DUAL)                                                                            \
    do {                                                                                                         \
        auto kern = conv_ws_kernel<T, NB, KS, AUX, DUAL>;                                                        \
        static bool attr_set = false;                                                                            \
        if (!attr_set) {                                                                                         \
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                      (int)kLdsBytes);                                                           \
            attr_set = (err == hipSuccess);                                                                      \
        }                                                                                                        \
        if (err == hipSuccess)                                                                                   \
            hipLaunchKernelGGL(kern, dim3(ws_grid), dim3(kWsWaves * kWave), ws_lds, ctx->stream, l, c, e, p.cs); \
    } while (0)
#define DCNN_WS_PICK(KS)                                                                                         \
    do {                                                                                                         \
        if (dual) { if (accum) DCNN_WS_LAUNCH(KS, 2, true); else DCNN_WS_LAUNCH(KS, 0, true); }                  \
        else if (accum) DCNN_WS_LAUNCH(KS, 2, false);                                                            \
        else if (e.res_data != nullptr) DCNN_WS_LAUNCH(KS, 1, false);                                            \
        else DCNN_WS_LAUNCH(KS, 0, false);                                                                       \
    } while (0)
        if (c.k == 1) DCNN_WS_PICK(1); else DCNN_WS_PICK(3);
#undef DCNN_WS_PICK
#undef DCNN_WS_LAUNCH
        if (err != hipSuccess) return check_hip(ctx, err, "hipFuncSetAttribute(conv_ws_kernel)");
        return check_hip(ctx, hipGetLastError(), "conv_ws_kernel launch");
    }
    // Streamed weights, 1x1 / 3x3 windows whose tap words are known, tensors within 32-bit byte offsets: the
    // register-blocked kernel -- several pixel tiles per wave share every weight operand on long lists, one tile per
    // wave on a deep ring on short ones (it reads tap words instead of testing the window against the mask, and was
    // measured 9-12 % ahead of the direct mode above on 3x3 256->256 with ~5000 listed pixels, equal elsewhere).
    // Short lists with several passes stay with the direct mode, which spreads the passes over the grid.
    const bool blocked = p.stream && !init && (!direct || p.npass == 1) && vec_out && aligned && (c.k == 1 || c.k == 3) && ws_taps &&
                         in_bytes <= kWsMaxBytes && p.w_bytes <= kWsMaxBytes;
    if (blocked) {
        constexpr int TI = NB <= 2 ? 4 : 2;               // pixel tiles per wave: a register block of 128 accumulators
        const size_t b_lds = conv_stage_bytes(kDirectWaves, NB, sizeof(T) == 2 ? DCNN_F16 : DCNN_F32) + conv_xchg_bytes(kDirectWaves);
        const int64_t b_want = cdiv(max_tiles, kDirectWaves / p.cs);
        // TI tiles per wave once that still gives every SIMD of the chip a wave (the list's length is read on the device)
        const int blocked_min_tiles = (int)((int64_t)ctx->num_cu * 4 * TI / p.cs);
        const int64_t b_cap = (int64_t)ctx->num_cu * 2;        // 4 waves of up to 256 registers: two workgroups per compute unit
        const int b_grid = (int)(cdiv(b_want < b_cap ? b_want : b_cap, kXcd) * kXcd);
#define DCNN_BLOCKED_LAUNCH(KS)                                                                                  \
    do {                                                                                                         \
        auto kern = conv_direct_kernel<T, NB, KS, TI>;                                                           \
        static bool attr_set = false;                                                                            \
        if (!attr_set) {                                                                                         \
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                      (int)kLdsBytes);                                                           \
            attr_set = (err == hipSuccess);                                                                      \
        }                                                                                                        \
        if (err == hipSuccess)                                                                                   \
            hipLaunchKernelGGL(kern, dim3(b_grid), dim3(kDirectWaves* kWave), b_lds, ctx->stream, l, c, e, p.npass, p.cs, \
                               blocked_min_tiles);                                                       \
    } while (0)
        if (c.k == 1) DCNN_BLOCKED_LAUNCH(1); else DCNN_BLOCKED_LAUNCH(3);
#undef DCNN_BLOCKED_LAUNCH
        if (err != hipSuccess) return check_hip(ctx, err, "hipFuncSetAttribute(conv_direct_kernel)");
        return check_hip(ctx, hipGetLastError(), "conv_direct_kernel launch");
    }
    // instantiated combinations: the common case (16-byte aligned input pixels, vector-width output
    // channels) is specialised on the window size; odd shapes take the generic-window kernels
    if (vec_out && aligned) {
        if (direct) {
            if (c.k == 1) DCNN_CONV_LAUNCH(VEC, true, 2, 1);
            else if (c.k == 3) DCNN_CONV_LAUNCH(VEC, true, 2, 3);
            else DCNN_CONV_LAUNCH(VEC, true, 2, 0);
        }
        else if (p.stream) DCNN_CONV_LAUNCH(VEC, true, 1, 0);
        else if (c.k == 1) DCNN_CONV_LAUNCH(VEC, true, 0, 1);
        else if (c.k == 3) DCNN_CONV_LAUNCH(VEC, true, 0, 3);
        else DCNN_CONV_LAUNCH(VEC, true, 0, 0);
    } else if (vec_out && !p.stream) {
        DCNN_CONV_LAUNCH(VEC, false, 0, 0);
    } else if (!vec_out && !p.stream) {
        if constexpr (NB <= 2) {
            if (aligned) DCNN_CONV_LAUNCH(1, true, 0, 0); else DCNN_CONV_LAUNCH(1, false, 0, 0);
        }
    }
#undef DCNN_CONV_LAUNCH
    if (!launched)
        return fail(ctx, DCNN_EUNSUPPORTED, "conv %dx%d %d->%d: no kernel for this combination of channel alignment and size",
                    c.k, c.k, c.cin, c.cout);
    if (err != hipSuccess) return check_hip(ctx, err, "hipFuncSetAttribute(conv_mfma_kernel)");
    return check_hip(ctx, hipGetLastError(), "conv_mfma_kernel launch");
}

}  // namespace dcnn
