// Sparse delta convolution whose weights do not fit LDS, long work lists: register-blocked gather-GEMM.
//
// When a layer's packed weights exceed LDS, every wave that multiplies a pixel tile has to fetch the weight
// operands of all K-steps from L2.  With one tile of 32 pixels per wave that is one 16-byte weight vector per
// lane and MFMA -- the L2 and the vector cache, not the matrix cores, set the pace.  Here a wave owns TI pixel
// tiles at once and multiplies every weight operand it has fetched with the gathered operands of all TI tiles
// (a TI*32 x NB*32 register block), which divides the weight traffic per pixel by TI.  No LDS and no barrier in
// the K loop: the operands of the next K-steps are in flight while the current one is multiplied, two
// waves per SIMD cover each other's tails (Section 3.1, Eqs. 4-6; the tail is the one the plain kernel uses).
//
// Addressing is by 32-bit byte offsets against buffer descriptors (tensors below 2 GiB): a lane whose tap is not
// flagged, whose entry lies beyond the list or whose K-step is channel padding gets an offset outside the
// descriptor and reads zeros, so unflagged memory is never touched and the loop has no branches.  Window taps
// that no lane of the wave needs are skipped altogether.  Sparse steps of 1x1 / 3x3 layers with 16-byte aligned
// channels only; which taps an entry needs comes with the work list (one word per entry).
#pragma once

#include "conv_plan.h"

namespace dcnn {

constexpr int kDirectWaves = 4;

// The work of one workgroup with TI pixel tiles per wave and a ring of D operand sets (D - 1 K-steps in flight).
// ROW (3x3, stride 1, padding 1): one gather per window ROW instead of one per tap.  The work list is ascending and
// holds every output pixel with a flagged tap, so if an entry's left tap (dy, 0) is flagged, the output pixel to its
// left is listed too and is the entry just before it -- the lane below holds that very input pixel as ITS centre tap
// (dy, 1).  Left and right operands are therefore the centre column moved by one lane (a DPP wave shift); only the
// first and the last column of a tile, whose neighbours sit in other tiles, fetch theirs, both through ONE extra load
// per tile (the two edges are different lanes).  A third of the gather traffic of a kernel that L2 bounds, and the
// weight operands of a row's three taps are multiplied with the same gathered registers.
template <typename T, int NB, int KS, int TI, int D, bool ROW>
__device__ __forceinline__ void conv_direct_body(const ListArgs& l, const ConvArgs& c, const EpilogueArgs& e, int npass, int cs,
                                                 int64_t count, unsigned char* smem) {
    typedef typename Mma<T>::Vec Vec;
    constexpr int V = Elem<T>::VEC;
    typedef typename RawOf<T, V>::type Raw;
    constexpr int COLS = NB * 32;
    constexpr int ES = (int)sizeof(T);
    constexpr int NW = kDirectWaves;
    constexpr int kNoTap = 31;
    static_assert(sizeof(Vec) == 16, "16-byte operand vectors");

    const int units_per_iter = NW / cs;                        // groups of TI tiles per workgroup iteration
    const int64_t ntiles = (count + kTile - 1) / kTile;
    const WgTileRange r = wg_tile_range((ntiles + units_per_iter * TI - 1) / (units_per_iter * TI));
    if (r.begin >= r.end) return;

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int col = lane % 32, g = lane / 32;
    const int slot = wave / cs, part = wave % cs;
    const int kch = c.kch;
    const int ksteps = KS * KS * kch;
    const bool full_tail = npass == 1;
    constexpr int stage_stride = COLS * ES + kStagePad;
    unsigned char* stage = smem + (size_t)wave * kTile * stage_stride;
    float* xchg = reinterpret_cast<float*>(smem + (size_t)NW * kTile * stage_stride) + (size_t)slot * 2 * cs * kTile;

    const int cin_bytes = c.cin * ES;
    const __amdgpu_buffer_rsrc_t rs_in = ws_rsrc(c.in_data, (uint64_t)c.n * c.h * c.w * cin_bytes);
    const __amdgpu_buffer_rsrc_t rs_w = ws_rsrc(c.wpacked, (uint64_t)npass * cs * ksteps * 2 * COLS * 16);
    const uint32_t wlane = (uint32_t)(g * COLS + col) * 16u;   // this lane's place in a K-step's weight block
    const bool k_exact = kch * 32 == cin_bytes;                // no K-step reaches past the pixel's channels

    auto origin = [&](int p32) {
        // pixel index of tap (0,0) of the entry's window (only used when that tap is in bounds)
        const uint32_t pu = p32 >= 0 ? (uint32_t)p32 : 0u;
        const uint32_t t1 = fast_div(pu, c.div_ow);
        const int ox = (int)(pu - t1 * (uint32_t)c.ow);
        const uint32_t n = fast_div(t1, c.div_oh);
        const int oy = (int)(t1 - n * (uint32_t)c.oh);
        return ((int)n * c.h + oy * c.stride - c.pad) * c.w + ox * c.stride - c.pad;
    };
    auto tile_of = [&](int64_t wt, int ti) { return (wt * units_per_iter + slot) * TI + ti; };
    auto entry = [&](int64_t wt, int ti) { return wt < r.end ? list_pixel(l.list, tile_of(wt, ti) * kTile + col, count) : -1; };
    auto tap_word = [&](int64_t wt, int ti, int p32) -> uint32_t {
        if (l.taps == nullptr) return p32 >= 0 ? 1u : 0u;      // a 1x1 layer on its input's own list: its one tap
        const int64_t j = tile_of(wt, ti) * kTile + col;
        return (wt < r.end && j < count) ? (l.taps[j] & ((1u << (KS * KS)) - 1u)) : 0u;
    };

    int survivors = 0;
    for (int64_t wt = r.begin; wt < r.end; wt += r.step) {
        int p32[TI];
        uint32_t tb[TI], base00[TI];
        uint32_t any = 0;
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            p32[ti] = entry(wt, ti);
            tb[ti] = tap_word(wt, ti, p32[ti]);
            base00[ti] = (uint32_t)origin(p32[ti]) * (uint32_t)cin_bytes + (uint32_t)g * 16u;
            any |= tb[ti];
        }
        uint32_t wave_taps = 0;                                // taps any lane of the wave needs
#pragma unroll
        for (int t = 0; t < KS * KS; ++t)
            if (__ballot((any >> t) & 1)) wave_taps |= 1u << t;
        const int nsteps = __popc(wave_taps) * kch;

        for (int pass = 0; pass < npass; ++pass) {
            const int cgroup = pass * cs + part;               // which group of COLS output channels
            const int ch0 = cgroup * COLS;
            int nch = e.c - ch0;
            nch = nch < 0 ? 0 : (nch > COLS ? COLS : nch);
            f32x16 acc[TI][NB];
#pragma unroll
            for (int ti = 0; ti < TI; ++ti)
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[ti][b][i] = 0.0f;

            const uint32_t wpass = (uint32_t)cgroup * (uint32_t)ksteps;
            if constexpr (ROW) {
                static_assert(KS == 3 && D == 2, "row gathers: 3x3 windows, two operand sets");
                uint32_t rows = 0;                             // window rows any lane of the wave needs
#pragma unroll
                for (int dy = 0; dy < 3; ++dy)
                    if ((wave_taps >> (3 * dy)) & 7u) rows |= 1u << dy;
                const int rsteps = __popc(rows) * kch;
                struct RCur { uint32_t rest; int dy, kc; };    // dy == 3: past the end (gathers zeros, multiplies nothing)
                auto advance = [&](RCur& cu) {
                    if (cu.dy < 3 && ++cu.kc == kch) {
                        cu.kc = 0;
                        cu.rest &= cu.rest - 1;
                        cu.dy = cu.rest ? __builtin_ctz(cu.rest) : 3;
                    }
                };
                const bool first_col = col == 0, last_col = col == kTile - 1;
                struct RSet { Vec xc[TI], xe[TI], wv[3][NB]; };
                auto issue = [&](const RCur& cu, RSet& st) {
                    const bool live = cu.dy < 3;
                    const int dy = live ? cu.dy : 0;
                    const uint32_t uni = (uint32_t)(dy * c.w * cin_bytes + cu.kc * 32);
                    const bool chan_ok = live && (k_exact || (2 * cu.kc + g) * 16 < cin_bytes);
#pragma unroll
                    for (int ti = 0; ti < TI; ++ti) {
                        const uint32_t three = (tb[ti] >> (3 * dy)) & 7u;
                        const uint32_t row0 = base00[ti] + uni;
                        uint32_t offc = (chan_ok && (three & 2u)) ? row0 + (uint32_t)cin_bytes : kOob;
                        uint32_t offe = !chan_ok ? kOob
                                        : (first_col && (three & 1u)) ? row0
                                        : (last_col && (three & 4u)) ? row0 + 2u * (uint32_t)cin_bytes : kOob;
                        asm volatile("" : "+v"(offc));
                        asm volatile("" : "+v"(offe));
                        st.xc[ti] = ws_load16<Vec>(rs_in, offc);
                        st.xe[ti] = ws_load16<Vec>(rs_in, offe);
                    }
                    const uint32_t wave_three = live ? (wave_taps >> (3 * dy)) & 7u : 0u;
#pragma unroll
                    for (int dx = 0; dx < 3; ++dx) {
                        const uint32_t woff = ((wave_three >> dx) & 1u)
                                                  ? wlane + (wpass + (uint32_t)((3 * dy + dx) * kch + cu.kc)) * (uint32_t)(2 * COLS * 16)
                                                  : kOob;
#pragma unroll
                        for (int b = 0; b < NB; ++b)
                            st.wv[dx][b] = ws_load16<Vec>(rs_w, woff == kOob ? kOob : woff + (uint32_t)b * (32u * 16u));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                };
                // the centre column moved by one lane: lane l takes lane l-1 (from_below) or lane l+1; the tile's
                // edge lanes take what they fetched themselves; a lane whose tap is not flagged takes zeros
                auto moved = [&](const Vec& v, bool from_below, bool take, bool edge, const Vec& ev) -> Vec {
                    const u32x4 w = __builtin_bit_cast(u32x4, v), o = __builtin_bit_cast(u32x4, ev);
                    u32x4 rr;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int sft = from_below ? __builtin_amdgcn_update_dpp(0, (int)w[i], 0x138, 0xf, 0xf, true)    // wave_shr:1
                                                   : __builtin_amdgcn_update_dpp(0, (int)w[i], 0x130, 0xf, 0xf, true);   // wave_shl:1
                        rr[i] = edge ? o[i] : (take ? (uint32_t)sft : 0u);
                    }
                    return __builtin_bit_cast(Vec, rr);
                };
                auto mma = [&](const RCur& cu, const RSet& st) {
                    const bool live = cu.dy < 3;
                    const int dy = live ? cu.dy : 0;
                    const uint32_t wave_three = live ? (wave_taps >> (3 * dy)) & 7u : 0u;
#pragma unroll
                    for (int ti = 0; ti < TI; ++ti) {
                        const uint32_t three = live ? (tb[ti] >> (3 * dy)) & 7u : 0u;
                        const Vec xl = moved(st.xc[ti], true, three & 1u, first_col, st.xe[ti]);
                        const Vec xr = moved(st.xc[ti], false, three & 4u, last_col, st.xe[ti]);
#pragma unroll
                        for (int dx = 0; dx < 3; ++dx) {
                            if (!((wave_three >> dx) & 1u)) continue;
#pragma unroll
                            for (int b = 0; b < NB; ++b)
                                Mma<T>::run(acc[ti][b], st.wv[dx][b], dx == 0 ? xl : (dx == 1 ? st.xc[ti] : xr));
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                };
                RSet sa, sb;
                RCur cg{rows, rows ? __builtin_ctz(rows) : 3, 0};
                RCur cm = cg;
                issue(cg, sa); advance(cg);
                for (int s = 0; s < rsteps; s += 2) {
                    issue(cg, sb); advance(cg);
                    mma(cm, sa); advance(cm);
                    issue(cg, sa); advance(cg);
                    mma(cm, sb); advance(cm);
                }
            } else {
            // Wave-uniform cursor over the K-steps that matter: (flagged tap, channel group) pairs in order.
            // Past the end a step gathers zeros and multiplies them with the (valid) first weight block.
            // Every load is issued unconditionally (a lane with nothing to fetch gets an offset outside the
            // descriptor), so the number of loads in flight at each wait is known at compile time.
            struct Cur { uint32_t rest; int t, kc; };
            auto issue = [&](Cur& cu, Vec (&x)[TI], Vec (&wv)[NB]) {
                const bool live = cu.t != kNoTap;
                const int t = live ? cu.t : 0;
                const uint32_t tbit = live ? 1u << t : 0u;
                const int dy = t / KS, dx = t - dy * KS;
                const uint32_t uni = (uint32_t)((dy * c.w + dx) * cin_bytes + cu.kc * 32);
                const bool chan_ok = k_exact || (2 * cu.kc + g) * 16 < cin_bytes;
#pragma unroll
                for (int ti = 0; ti < TI; ++ti) {
                    uint32_t off = (chan_ok && (tb[ti] & tbit)) ? base00[ti] + uni : kOob;
                    asm volatile("" : "+v"(off));              // one load at a computed offset, not a load per case
                    x[ti] = ws_load16<Vec>(rs_in, off);
                }
                const uint32_t woff = wlane + (wpass + (uint32_t)(t * kch + cu.kc)) * (uint32_t)(2 * COLS * 16);
#pragma unroll
                for (int b = 0; b < NB; ++b) wv[b] = ws_load16<Vec>(rs_w, woff + (uint32_t)b * (32u * 16u));
                if (live && ++cu.kc == kch) {
                    cu.kc = 0;
                    cu.rest &= cu.rest - 1;
                    cu.t = cu.rest ? __builtin_ctz(cu.rest) : kNoTap;
                }
                __builtin_amdgcn_sched_barrier(0);             // the scheduler must not sink the loads below the MFMAs
            };
            auto mma = [&](const Vec (&x)[TI], const Vec (&wv)[NB]) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int ti = 0; ti < TI; ++ti) Mma<T>::run(acc[ti][b], wv[b], x[ti]);
                __builtin_amdgcn_sched_barrier(0);
            };
            // ring of D register sets: the operands of D - 1 K-steps travel while one step is multiplied
            Vec x[D][TI], w[D][NB];
            Cur cu{wave_taps, wave_taps ? __builtin_ctz(wave_taps) : kNoTap, 0};
#pragma unroll
            for (int i = 0; i < D - 1; ++i) issue(cu, x[i], w[i]);
            for (int s = 0; s < nsteps; s += D) {
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    issue(cu, x[(j + D - 1) % D], w[(j + D - 1) % D]);
                    mma(x[j], w[j]);
                }
            }
            }

            // ---- tail: this wave's channel slice of each of its tiles -------------------------------
            const MaxExchange mx{xchg, cs, part};
            const bool exchange = cs > 1 && full_tail && e.act != DCNN_ACT_NONE;
#pragma unroll
            for (int ti = 0; ti < TI; ++ti) {
                stage_accumulators<T, NB>(acc[ti], stage + (size_t)col * stage_stride, g);
                lds_wave_sync();
                auto dx = [&](int ent, int64_t, int c0) -> Raw {
                    return raw_load<T, V>(reinterpret_cast<const T*>(stage + (size_t)ent * stage_stride) + (c0 - ch0));
                };
                uint32_t bits;
                if (exchange) bits = act_trunc_tile<T, V, 1, 2, true>(e, false, p32[ti], lane, dx, ch0, nch, COLS, mx);
                else bits = act_trunc_tile<T, V, 1, 2, false>(e, false, p32[ti], lane, dx, ch0, nch, COLS, mx);
                const int64_t tile = tile_of(wt, ti);
                if (full_tail && part == 0 && tile * kTile < count) {
                    if (e.surv) { if (lane == 0) e.surv[tile] = bits; }
                    else survivors += __popc(bits);
                }
                lds_wave_sync();
            }
        }
    }
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

// Lists too short to keep the chip busy with TI tiles per wave run one tile per wave and a deeper ring instead
// (more waves, more loads in flight); the length of the list is only known on the device.
template <typename T, int NB, int KS, int TI>
__global__ __launch_bounds__(kDirectWaves* kWave, 2) void conv_direct_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, int npass, int cs,
                                                                             int blocked_min_tiles) {
    extern __shared__ __align__(16) unsigned char smem[];
    clear_ahead(e);
    const int64_t count = list_count(l);
    if (count >= (int64_t)blocked_min_tiles * kTile) {
        if constexpr (KS == 3 && NB <= 2) {
            // Row gathers pay when most taps of the listed windows are flagged.  Every flagged input pixel is a tap
            // of (up to) nine listed outputs, so flagged inputs / listed outputs IS the mean fraction of flagged taps
            // per window.  Measured on 3x3 128->128, 256x256 maps, uniform-random masks: all taps flagged 0.40 ->
            // 0.30 ms, half of them 0.231 -> 0.243 ms, a tenth 0.127 -> 0.156 ms; hence three quarters.
            // (an input that comes without a count: the rule of the resident-weight kernel, most of the map listed)
            const bool dense_taps = c.in_count ? (int64_t)*c.in_count * 4 >= count * 3
                                               : count * 4 >= (int64_t)c.n * c.oh * c.ow * 3;
            if (c.stride == 1 && c.pad == 1 && dense_taps) {
                conv_direct_body<T, NB, KS, (TI > 3 ? 3 : TI), 2, true>(l, c, e, npass, cs, count, smem);   // 3 tiles: two operand sets of 12 vectors fit beside 96 accumulators
                return;
            }
        }
        conv_direct_body<T, NB, KS, TI, 3, false>(l, c, e, npass, cs, count, smem);
    } else {
        conv_direct_body<T, NB, KS, 1, (NB >= 4 ? 6 : 8), false>(l, c, e, npass, cs, count, smem);
    }
}

}  // namespace dcnn
