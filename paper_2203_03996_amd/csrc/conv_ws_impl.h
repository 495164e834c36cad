// Sparse delta convolution with resident weights, wave-specialised.
//
// A tile of the sparse convolution has two halves with opposite needs.  The gather-GEMM wants many
// short cache-hit loads and the matrix cores; the activation + truncation tail wants a few long
// loads of layer state that come from HBM, and plain vector arithmetic.  One wave that does both in
// turn waits for each memory system in turn, and the registers of both halves limit the compute
// unit to two waves per SIMD.  Here a workgroup of 16 waves splits the roles:
//   producers (waves 0-7)   gather the flagged taps of a tile, multiply on the matrix cores and
//                           leave the rounded result tile in LDS;
//   consumers (waves 8-15)  pick the tile of the PREVIOUS round up from LDS, apply residual /
//                           activation / truncation (Section 3.1, Eqs. 4-6), and write state, output
//                           delta, update mask and survivor word with coalesced 16-byte accesses.
// The result tiles are double-buffered and handed over per tile slot through two LDS counters (tiles staged /
// tiles consumed), so a slot's producers and consumers wait for each other only, never for the whole workgroup.
// Each role needs at most 128 registers: four waves per SIMD, and while the consumers wait for
// HBM the producers keep the matrix cores and the L2 busy.
//
// The channels of a tile are split over `cs` producers (nb*32 output channels each); the consumers
// split the same tile by PIXELS instead (32/cs pixels, all channels), so the per-pixel maximum
// stays inside one wave.
//
// All global traffic uses buffer addressing (32-bit byte offsets against a descriptor): address
// arithmetic is one add per access, and a lane that must not touch memory (tap not flagged, pixel
// beyond the list, pixel truncated) simply gets an offset beyond the descriptor's range, for which
// the hardware returns zeros on loads and drops stores.  No branches, no unflagged memory read.
// A layer may carry a second, 1x1 convolution of another input whose result is added before the
// activation (the projection shortcut of a residual block): the producer runs it as a second short
// K loop on the same tile, so its result never travels through memory.
// Every tensor therefore has to stay below 2 GiB; larger ones run on the plain kernel, as does the
// dense first frame (bias, no truncation).
#pragma once

#include <type_traits>

#include "conv_plan.h"

namespace dcnn {

constexpr int kWsProducers = 8;
constexpr int kWsWaves = 16;
constexpr int kWsSyncBytes = 64;                               // hand-over counters: tiles staged / tiles consumed, per tile slot
constexpr int kWsSpinLimit = 1 << 22;                          // polls after which a wait gives up (never reached: see hand_over)
constexpr int kTapProj = 30;                                   // bit of a tap word: the projection's input pixel is flagged

constexpr int ws_pow2_ceil(int v) { int p = 1; while (p < v) p <<= 1; return p; }

// LDS needed by the wave-specialised kernel; 0 when the shape is not covered by it.
inline size_t conv_ws_lds_bytes(const ConvPlan& p, int dtype, int k, int cout, int cin2 = 0) {
    const int vec = dtype == DCNN_F16 ? 8 : 4;
    if (p.stream || p.npass != 1 || cout % vec != 0 || (k != 1 && k != 3)) return 0;
    const int lpb = ws_pow2_ceil(p.nb * 32 / vec);
    if (p.cs * lpb > kWave) return 0;
    const size_t w2_bytes = (size_t)cdiv(cin2, dtype == DCNN_F16 ? 16 : 8) * 2 * p.cout_pad * 16;   // projection weights
    const size_t bytes = p.w_bytes + w2_bytes + 2 * conv_stage_bytes(kWsProducers, p.nb, dtype) + kWsSyncBytes;
    return bytes <= kLdsBytes ? bytes : 0;
}


// AUX: third per-pixel stream of the tail -- 0 none, 1 residual delta (added before the activation),
// 2 dense accumulated output O of a final layer (O += emitted delta; the delta itself is not stored).
template <typename T, int NB, int KS, int AUX, bool DUAL>
__global__ __launch_bounds__(kWsWaves* kWave) void conv_ws_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, int cs) {
    typedef typename Mma<T>::Vec Vec;
    constexpr int V = Elem<T>::VEC;
    typedef typename RawOf<T, V>::type Raw;
    constexpr bool RES = AUX == 1, ACC = AUX == 2;
    constexpr int COLS = NB * 32;
    constexpr int GK = 4;                                      // K-steps gathered together (one register set)
    // register sets of the gather ring: NSETS-1 groups in flight behind the one being multiplied.  The 3x3 kernel
    // is bound by its producers (nine dependent gather round trips per tile) and takes a third set where the
    // registers allow it; everywhere else two are best (finer groups and deeper rings were measured slower).
    constexpr int NSETS = (KS == 3 && NB <= 2 && AUX == 0 && !DUAL) ? 3 : 2;
    constexpr int NP = kWsProducers;
    constexpr int ES = (int)sizeof(T);
    static_assert(sizeof(Vec) == 16 && sizeof(Raw) == 16, "16-byte channel vectors");
    extern __shared__ __align__(16) unsigned char smem[];
    clear_ahead(e);

    const int tiles_per_iter = NP / cs;
    const int64_t count = list_count(l);
    const WgTileRange r = wg_tile_range((count + tiles_per_iter * kTile - 1) / (tiles_per_iter * kTile));
    if (r.begin >= r.end) return;                              // nothing for this workgroup: skip the weight load
    const int rounds = (int)((r.end - r.begin + r.step - 1) / r.step);

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const bool producer = wave < NP;
    const int ww = producer ? wave : wave - NP;
    const int slot = ww / cs, part = ww % cs;                  // which tile of the round; channel slice / pixel slice
    const int taps = KS * KS, kch = c.kch;
    const int ksteps = taps * kch;
    const int w1_vecs = cs * ksteps * 2 * COLS;
    const int w2_vecs = DUAL ? cs * c.kch2 * 2 * COLS : 0;     // the projection's weights follow the main ones
    const int w_vecs = w1_vecs + w2_vecs;
    Vec* w_lds = reinterpret_cast<Vec*>(smem);
    constexpr int stage_stride = COLS * ES + kStagePad;
    constexpr int stage_tile = kTile * stage_stride;
    unsigned char* stage0 = smem + (size_t)w_vecs * 16;        // [2][NP][32 pixels][stage_stride]
    // Hand-over of result tiles.  A tile slot is the business of its cs producers and cs consumers only, so instead of
    // a workgroup barrier per round (every wave waiting for the slowest of sixteen, round after round) each slot keeps
    // two counters in LDS: `staged` (bumped by a producer once its slice of a tile is in the staging buffer) and
    // `consumed` (bumped by a consumer once it has read its pixels of a tile).  A consumer starts tile r when staged
    // >= cs*(r+1); a producer overwrites the buffer of tile r-2 when consumed >= cs*(r-1).  Tiles 0 and 1 need no
    // wait, every wave bumps its counter once per tile, so by induction over r every wait ends; the poll limit only
    // bounds the damage of a programming error (a kernel that gives wrong results instead of one that never ends).
    uint32_t* staged_ctr = reinterpret_cast<uint32_t*>(stage0 + (size_t)2 * NP * stage_tile) + slot;
    uint32_t* consumed_ctr = staged_ctr + kWsProducers;
    auto bump = [&](uint32_t* ctr) {
        // release at workgroup scope: this wave's LDS accesses so far are complete before the counter moves
        if (lane == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto await = [&](uint32_t* ctr, int target) {
        if (target <= 0) return;
        for (int spin = 0; spin < kWsSpinLimit; ++spin) {
            if ((int)__hip_atomic_load(ctr, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= target) return;
            __builtin_amdgcn_s_sleep(2);
        }
    };
    // pixel of entry `j` of the work list of round `rd` (this wave's tile), -1 beyond the list
    auto tile_of = [&](int rd) { return (r.begin + (int64_t)rd * r.step) * tiles_per_iter + slot; };
    auto list_entry = [&](int rd, int j) { return rd < rounds ? list_pixel(l.list, tile_of(rd) * kTile + j, count) : -1; };

    // The weights travel global -> LDS once per workgroup.  Every wave calls this exactly once, right after it
    // has requested the list entries of its first tiles, so that round trip hides behind the copy.
    // Four loads are in flight per lane before the first is stored: the copy costs a couple of memory round trips
    // instead of one per 16 KiB, which counts in a kernel that runs for ten rounds.
    auto copy_weights = [&](const Vec* src, Vec* dst, int n) {
        constexpr int B = 4, TH = kWsWaves * kWave;
        for (int i0 = threadIdx.x; i0 < n; i0 += B * TH) {
            Vec v[B];
#pragma unroll
            for (int u = 0; u < B; ++u) {
                const int i = i0 + u * TH;
                v[u] = src[i < n ? i : n - 1];
            }
#pragma unroll
            for (int u = 0; u < B; ++u) {
                const int i = i0 + u * TH;
                if (i < n) dst[i] = v[u];
            }
        }
    };
    auto load_weights = [&]() {
        copy_weights(static_cast<const Vec*>(c.wpacked), w_lds, w1_vecs);
        if constexpr (DUAL) copy_weights(static_cast<const Vec*>(c.wpacked2), w_lds + w1_vecs, w2_vecs);
        if (threadIdx.x < 2 * kWsProducers) reinterpret_cast<uint32_t*>(stage0 + (size_t)2 * NP * stage_tile)[threadIdx.x] = 0u;
        lds_block_sync();
    };

    // The only workgroup barrier is the one behind the weight copy; after it the roles meet through the counters.
    if (producer) {
        // =====================================================================================
        // producer: tile -> gathered taps x weights -> rounded result tile in LDS
        // =====================================================================================
        const int col = lane % 32, g = lane / 32;
        const uint64_t in_pixels = (uint64_t)c.n * c.h * c.w;
        const __amdgpu_buffer_rsrc_t rs_in = ws_rsrc(c.in_data, in_pixels * c.cin * ES);
        const int cin_bytes = c.cin * ES;
        const int kgroups = (kch + GK - 1) / GK;               // groups of GK K-steps per tap
        const bool k_exact = kgroups * GK * 32 == cin_bytes;   // no K-step of a group reaches past the pixel's channels
        const bool k_exact2 = kch * 32 == cin_bytes;           // no K-step at all does
        // (one gather per window row pays when most of the map is listed -- the dense mode and high update densities:
        // 4.6 % of the step with everything listed, 1 % at 50 % density; on short lists the tap-by-tap ring with its
        // third set in flight is 1 % ahead)
        const bool row_shift = KS == 3 && !DUAL && NB <= 2 && c.stride == 1 && c.pad == 1 && count * 4 >= (int64_t)c.n * c.oh * c.ow * 3;
        (void)k_exact2; (void)row_shift;
        constexpr int kNoTap = 31;                             // cursor sentinel: no tap has this number
        // Which window taps of a list entry are in bounds and flagged comes with the work list (one
        // word per entry); a 1x1 layer that walks its input's own list has exactly its one tap.
        // Software pipeline over tiles: list entry and tap word of tile n+2 are requested while tile
        // n is processed.
        auto origin = [&](int p32) {
            // pixel index of tap (0,0) of the entry's window (only used when that tap is in bounds)
            const uint32_t pu = p32 >= 0 ? (uint32_t)p32 : 0u;
            const uint32_t t1 = fast_div(pu, c.div_ow);
            const int ox = (int)(pu - t1 * (uint32_t)c.ow);
            const uint32_t n = fast_div(t1, c.div_oh);
            const int oy = (int)(t1 - n * (uint32_t)c.oh);
            return ((int)n * c.h + oy * c.stride - c.pad) * c.w + ox * c.stride - c.pad;
        };
        // the projection's input: pixel (oy*stride2, ox*stride2) of a [n, h2, w2, cin2] map
        const __amdgpu_buffer_rsrc_t rs_in2 = ws_rsrc(c.in2_data, (uint64_t)c.n * c.h2 * c.w2 * c.cin2 * ES);
        const int cin2_bytes = c.cin2 * ES;
        auto origin2 = [&](int p32) {
            const uint32_t pu = p32 >= 0 ? (uint32_t)p32 : 0u;
            const uint32_t t1 = fast_div(pu, c.div_ow);
            const int ox = (int)(pu - t1 * (uint32_t)c.ow);
            const uint32_t n = fast_div(t1, c.div_oh);
            const int oy = (int)(t1 - n * (uint32_t)c.oh);
            return ((int)n * c.h2 + oy * c.stride2) * c.w2 + ox * c.stride2;
        };
        const int kgroups2 = DUAL ? (c.kch2 + GK - 1) / GK : 1;
        (void)rs_in2; (void)cin2_bytes; (void)origin2; (void)kgroups2;
        auto tap_word = [&](int rd, int p32) -> uint32_t {
            if (l.taps == nullptr) return p32 >= 0 ? 1u : 0u;
            const int64_t j = tile_of(rd) * kTile + col;
            return (rd < rounds && j < count) ? l.taps[j] : 0u;
        };
        int p32_next = list_entry(0, col), p32_next2 = list_entry(1, col);
        uint32_t taps_next = tap_word(0, p32_next), taps_next2 = tap_word(1, p32_next2);
        load_weights();
        const Vec* wbase = w_lds + ((size_t)part * ksteps * 2 + g) * COLS + col;
        const Vec* wbase2 = w_lds + w1_vecs + ((size_t)part * (DUAL ? c.kch2 : 0) * 2 + g) * COLS + col;

        for (int rd = 0; rd < rounds; ++rd) {
            {
                bool buffer_free = false;                          // this tile's staging buffer has been waited for
                auto claim_buffer = [&]() {
                    if (!buffer_free) await(consumed_ctr, cs * (rd - 1));
                    buffer_free = true;
                };
                // byte offset of this lane's 16 bytes in tap (0,0), K-step 0
                const int p32_cur = p32_next;
                const uint32_t base00 = (uint32_t)origin(p32_cur) * (uint32_t)cin_bytes + (uint32_t)g * 16u;
                const uint32_t tapbits = taps_next;                // taps this lane needs
                uint32_t wave_taps = 0;                            // taps any lane of the wave needs
#pragma unroll
                for (int t = 0; t < KS * KS; ++t)
                    if (__ballot((tapbits >> t) & 1)) wave_taps |= 1u << t;
                uint32_t base2 = 0;                                // the same for the projection's pixel
                if constexpr (DUAL) {
                    if (__ballot((tapbits >> kTapProj) & 1)) wave_taps |= 1u << kTapProj;
                    base2 = (uint32_t)origin2(p32_cur) * (uint32_t)cin2_bytes + (uint32_t)g * 16u;
                }
                p32_next = p32_next2; taps_next = taps_next2;
                p32_next2 = list_entry(rd + 2, col);
                taps_next2 = tap_word(rd + 2, p32_next2);

                // Wave-uniform cursor over the (tap, group of GK K-steps) pairs that matter: a tap no
                // lane of the wave needs is skipped altogether.  With a projection, its K groups follow
                // as "tap" kTapProj of the same sequence, so its gathers are in flight while the last
                // main group is multiplied.  t == kNoTap once the pairs run out.
                struct Cursor { uint32_t rest; int t, kg; };
                auto first_tap = [](uint32_t m) { return m ? __builtin_ctz(m) : kNoTap; };
                auto advance = [&](Cursor& cu) {
                    if (++cu.kg >= ((DUAL && cu.t == kTapProj) ? kgroups2 : kgroups)) {
                        cu.kg = 0;
                        cu.rest &= cu.rest - 1;
                        cu.t = first_tap(cu.rest);
                    }
                };
                // 16 bytes of input channels per K-step for this lane's pixel; lanes that do not need
                // the tap (or whose channels are padding) get zeros from an out-of-range offset.  Every
                // load is issued unconditionally, so the number in flight is known at compile time and
                // a group's wait never includes the group requested after it.
                auto gather_group = [&](const Cursor& cu, Vec (&x)[GK]) {
                    const bool proj = DUAL && cu.t == kTapProj;
                    const bool tap_ok = (tapbits >> cu.t) & 1;
                    const int dy = cu.t / KS, dx = cu.t % KS;
                    const uint32_t uni = proj ? (uint32_t)(cu.kg * (GK * 32))
                                              : (uint32_t)((dy * c.w + dx) * cin_bytes + cu.kg * (GK * 32));
                    const uint32_t off = tap_ok ? (proj ? base2 : base00) + uni : kOob;
                    const int limit = proj ? cin2_bytes : cin_bytes;
                    const bool exact = proj ? false : k_exact;
                    const __amdgpu_buffer_rsrc_t rs = proj ? rs_in2 : rs_in;
#pragma unroll
                    for (int u = 0; u < GK; ++u) {
                        uint32_t o = off + (uint32_t)u * 32u;
                        if (!exact && (2 * (cu.kg * GK + u) + g) * 16 >= limit) o = kOob;
                        x[u] = ws_load16<Vec>(rs, o);
                    }
                    __builtin_amdgcn_sched_barrier(0);             // the scheduler must not sink the loads below the MFMAs
                };
                f32x16 acc[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
                unsigned char* tile_row = stage0 + (size_t)((rd & 1) * NP + ww) * stage_tile + (size_t)col * stage_stride;
                bool main_staged = false;
                // The weight operands of K-step u+1 are requested from LDS before the MFMAs of step u
                // issue; a K-step past the end multiplies the (valid) last step's weights with zeros.
                auto mma_group = [&](const Cursor& cu, const Vec (&x)[GK]) {
                    const bool proj = DUAL && cu.t == kTapProj;
                    if constexpr (DUAL) {
                        if (proj && !main_staged) {
                            // The main result waits, rounded to the storage type, in the staging tile while
                            // the accumulators are reused: both results are rounded before they are added,
                            // as if each had been stored.
                            claim_buffer();
                            stage_accumulators<T, NB, false>(acc, tile_row, g);
#pragma unroll
                            for (int b = 0; b < NB; ++b)
#pragma unroll
                                for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
                            main_staged = true;
                        }
                    }
                    const int steps = proj ? c.kch2 : kch;
                    const int tap = cu.t == kNoTap ? 0 : cu.t;     // past the end of the sequence: any valid row (it meets zeros)
                    const Vec* wtap = proj ? wbase2 : wbase + (size_t)(tap * kch) * 2 * COLS;
                    Vec wv[2][NB];
                    auto request = [&](int u) {
                        const int kc = cu.kg * GK + u;
                        const Vec* wrow = wtap + (size_t)(kc < steps ? kc : steps - 1) * 2 * COLS;
#pragma unroll
                        for (int b = 0; b < NB; ++b) wv[u & 1][b] = wrow[b * 32];
                    };
                    request(0);
#pragma unroll
                    for (int u = 0; u < GK; ++u) {
                        if (u + 1 < GK) request(u + 1);
                        __builtin_amdgcn_sched_barrier(0);         // keep the requests ahead of the matrix work
#pragma unroll
                        for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wv[u & 1][b], x[u]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                };
                // Ring of NSETS register sets: the gathers of group s+NSETS-1 are issued right before group
                // s is multiplied.  The loop body is straight-line code (groups past the end of the
                // sequence multiply zeros), so every wait counts exactly the loads issued after it.
                bool rows_done = false;
                if constexpr (KS == 3 && !DUAL && NB <= 2) {
                    if (row_shift) {
                        // ---- 3x3, stride 1, padding 1: one gather per window ROW instead of one per tap ---------------
                        // The list is ascending and holds every pixel with a flagged tap, so if this lane's left tap
                        // (dy, 0) is flagged, the pixel to its left is listed too and is the entry just before it: the
                        // lane below holds that very input pixel as ITS centre tap (dy, 1).  The left and right taps of
                        // a row are therefore the centre column moved by one lane; only the first and the last column
                        // of the tile (whose neighbours sit in other tiles) fetch theirs.  A third of the gathers, and
                        // of the cache lines the vector memory pipeline has to look up -- which is what bounds this
                        // kernel.  A lane whose tap is not flagged (or out of bounds) takes zeros, whatever its
                        // neighbour holds.
                        constexpr int RG = 2;                          // K-steps per row group
                        const int rgroups = (kch + RG - 1) / RG;
                        uint32_t rows = 0;
#pragma unroll
                        for (int dy = 0; dy < 3; ++dy)
                            if ((wave_taps >> (3 * dy)) & 7u) rows |= 1u << dy;
                        struct RCur { uint32_t rest; int dy, kg; };
                        auto rfirst = [](uint32_t m) { return m ? __builtin_ctz(m) : 3; };
                        auto radvance = [&](RCur& cu) {
                            if (++cu.kg >= rgroups) { cu.kg = 0; cu.rest &= cu.rest - 1; cu.dy = rfirst(cu.rest); }
                        };
                        const bool first_col = col == 0, last_col = col == kTile - 1;
                        struct RSet { Vec xc[RG], xl[RG], xr[RG]; };
                        auto gather_row = [&](const RCur& cu, RSet& st) {
                            const bool live = cu.dy < 3;
                            const int dy = live ? cu.dy : 0;
                            const uint32_t three = live ? (tapbits >> (3 * dy)) & 7u : 0u;
                            const uint32_t row0 = base00 + (uint32_t)(dy * c.w * cin_bytes + cu.kg * (RG * 32));
                            const uint32_t offc = (three & 2u) ? row0 + (uint32_t)cin_bytes : kOob;
                            const uint32_t offl = (first_col && (three & 1u)) ? row0 : kOob;
                            const uint32_t offr = (last_col && (three & 4u)) ? row0 + 2u * (uint32_t)cin_bytes : kOob;
#pragma unroll
                            for (int u = 0; u < RG; ++u) {
                                const bool pad = !k_exact2 && (2 * (cu.kg * RG + u) + g) * 16 >= cin_bytes;
                                st.xc[u] = ws_load16<Vec>(rs_in, pad ? kOob : offc + (uint32_t)u * 32u);
                                st.xl[u] = ws_load16<Vec>(rs_in, pad ? kOob : offl + (uint32_t)u * 32u);
                                st.xr[u] = ws_load16<Vec>(rs_in, pad ? kOob : offr + (uint32_t)u * 32u);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        };
                        // the centre column moved by one lane: lane l takes lane l-1 (from_below) or l+1
                        auto shifted = [&](const Vec& v, bool from_below, bool take, const Vec& other) -> Vec {
                            const u32x4 w = __builtin_bit_cast(u32x4, v), o = __builtin_bit_cast(u32x4, other);
                            u32x4 r;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int sft = from_below ? __builtin_amdgcn_update_dpp(0, (int)w[i], 0x138, 0xf, 0xf, true)    // wave_shr:1
                                                           : __builtin_amdgcn_update_dpp(0, (int)w[i], 0x130, 0xf, 0xf, true);   // wave_shl:1
                                r[i] = take ? (uint32_t)sft : o[i];
                            }
                            return __builtin_bit_cast(Vec, r);
                        };
                        auto mma_row = [&](const RCur& cu, const RSet& st) {
                            const int dy = cu.dy < 3 ? cu.dy : 0;
                            const uint32_t three = cu.dy < 3 ? (tapbits >> (3 * dy)) & 7u : 0u;
                            const bool take_l = !first_col && (three & 1u), take_r = !last_col && (three & 4u);
                            const uint32_t wave_three = cu.dy < 3 ? (wave_taps >> (3 * dy)) & 7u : 0u;
#pragma unroll
                            for (int u = 0; u < RG; ++u) {
                                const int kc = cu.kg * RG + u;
                                if (kc >= kch) continue;
                                const Vec xl = shifted(st.xc[u], true, take_l, st.xl[u]);
                                const Vec xr = shifted(st.xc[u], false, take_r, st.xr[u]);
#pragma unroll
                                for (int dx = 0; dx < 3; ++dx) {
                                    if (!((wave_three >> dx) & 1u)) continue;
                                    const Vec* wrow = wbase + (size_t)((3 * dy + dx) * kch + kc) * 2 * COLS;
                                    Vec wv[NB];
#pragma unroll
                                    for (int b = 0; b < NB; ++b) wv[b] = wrow[b * 32];
#pragma unroll
                                    for (int b = 0; b < NB; ++b) Mma<T>::run(acc[b], wv[b], dx == 0 ? xl : (dx == 1 ? st.xc[u] : xr));
                                }
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        };
                        RSet ra, rb;
                        RCur rg{rows, rfirst(rows), 0};
                        RCur rm = rg;
                        gather_row(rg, ra); radvance(rg);
                        while (rm.dy < 3) {
                            gather_row(rg, rb); radvance(rg);
                            mma_row(rm, ra); radvance(rm);
                            gather_row(rg, ra); radvance(rg);
                            mma_row(rm, rb); radvance(rm);
                        }
                        rows_done = true;
                    }
                }
                if (!rows_done) {
                Vec x[NSETS][GK];
                Cursor cg{wave_taps, first_tap(wave_taps), 0};     // gathers run ahead of the matrix work
                Cursor cm = cg;
#pragma unroll
                for (int i = 0; i < NSETS - 1; ++i) { gather_group(cg, x[i]); advance(cg); }
                while (cm.t != kNoTap) {
#pragma unroll
                    for (int i = 0; i < NSETS; ++i) {
                        gather_group(cg, x[(i + NSETS - 1) % NSETS]); advance(cg);
                        mma_group(cm, x[i]); advance(cm);
                    }
                }
                }
                claim_buffer();
                if (main_staged) stage_accumulators<T, NB, true>(acc, tile_row, g);
                else stage_accumulators<T, NB, false>(acc, tile_row, g);
                bump(staged_ctr);
            }
        }
    } else {
        // =====================================================================================
        // consumer: result tile of the previous round -> residual / activation / truncation
        // =====================================================================================
        constexpr int LPB = ws_pow2_ceil(COLS / V);            // lanes per pixel and producer slice
        constexpr int NIT = LPB / 2;                           // lane-iterations over this wave's 32/cs pixels
        constexpr int H = (NIT >= 4 && !RES) ? 2 : 1;          // iterations per register set (a residual stream adds a
                                                               // third vector per iteration: single-iteration sets keep
                                                               // that variant within its 128 registers)
        constexpr int NS = NIT / H;                            // sets per tile; two register sets alternate
        static_assert(NIT >= 2 && NS * H == NIT && NS % 2 == 0, "tile iterations split into an even number of sets");
        const int LP = cs * LPB;                               // lanes per pixel (all channels), <= 64
        const int PPI = kWave / LP;                            // pixels per iteration
        const int sub = lane % LP, grp = lane / LP;
        const int spart = sub / LPB, vi = sub % LPB;
        const int c0 = spart * COLS + vi * V;                  // first of this lane's V channels
        const bool ch_on = vi * V < COLS && c0 < e.c;
        const int ent0 = part * (kTile / cs) + grp;            // tile entry of iteration 0
        const uint32_t row_bytes = (uint32_t)e.c * ES;
        const uint32_t ch_bytes = (uint32_t)c0 * ES;
        const uint64_t out_pixels = (uint64_t)c.n * c.oh * c.ow;
        const uint64_t out_bytes = out_pixels * row_bytes;
        const bool stateful = e.act != DCNN_ACT_NONE;
        const __amdgpu_buffer_rsrc_t rs_xA = ws_rsrc(e.xA, out_bytes), rs_xT = ws_rsrc(e.xT, out_bytes);
        const __amdgpu_buffer_rsrc_t rs_out = ws_rsrc(e.out_data, out_bytes);
        const __amdgpu_buffer_rsrc_t rs_res = ws_rsrc(ACC ? e.accum_O : e.res_data, out_bytes);   // the third stream
        const __amdgpu_buffer_rsrc_t rs_rmask = ws_rsrc(e.res_mask, out_pixels);
        const __amdgpu_buffer_rsrc_t rs_omask = ws_rsrc(e.out_mask, out_pixels);
        const bool has_rmask = e.res_mask != nullptr;
        const __amdgpu_buffer_rsrc_t rs_tflag = ws_rsrc(e.xt_flags, out_pixels);
        const bool has_tflag = e.xt_flags != nullptr;
        const bool has_omask = e.out_mask != nullptr;
        const float hi = act_hi(e.act);
        // this lane's 16 bytes in row 0 of the producer slice that holds its channels (lanes without
        // channels read slot 0 and discard it; their stores go nowhere)
        const unsigned char* my_stage = stage0 + (size_t)(slot * cs + spart) * stage_tile + (size_t)(ch_on ? vi : 0) * V * ES;
        int survivors = 0;

        // Per-entry values (list entry, flags) are fetched ONCE per tile, entry lane % 32 per lane, and handed to the
        // lanes that work on an entry by lane shuffles: a vector memory instruction costs its issue slots whatever it
        // moves (a byte per lane as much as a quarter of a 16-byte access), and one per iteration added up to a
        // sixth of this role's memory instructions.
        struct Tile {
            int pix_mine;          // pixel of entry lane % 32 (-1 beyond the list)
            int rflag_mine;        // update flag of the residual stream at that pixel
            int tflag_mine;        // 0: that pixel's x^T row is known to be all zero and is not read
            int pix[NIT];          // pixel of iteration it
            uint32_t off[NIT];     // byte offset of this lane's channels (out of range: nothing to do)
            uint8_t rflag[NIT];
            uint8_t tflag[NIT];
        };
        // derived values of a tile whose list entries have arrived; requests its flags
        auto prepare = [&](Tile& t) {
            const int pm = t.pix_mine;
            t.rflag_mine = 1;
            if constexpr (RES) {
                if (has_rmask) t.rflag_mine = __builtin_amdgcn_raw_buffer_load_b8(rs_rmask, pm >= 0 ? pm : (int)kOob, 0, 0);
            }
            t.tflag_mine = 1;
            if (has_tflag) t.tflag_mine = __builtin_amdgcn_raw_buffer_load_b8(rs_tflag, pm >= 0 ? pm : (int)kOob, 0, 0);
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int p = __shfl(pm, ent0 + it * PPI, kWave);
                t.pix[it] = p;
                t.off[it] = (p >= 0 && ch_on) ? (uint32_t)p * row_bytes + ch_bytes : kOob;
            }
        };
        // the flags have arrived: hand them to the lanes of each iteration
        auto resolve = [&](Tile& t) {
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                t.rflag[it] = (uint8_t)__shfl(t.rflag_mine, ent0 + it * PPI, kWave);
                t.tflag[it] = (uint8_t)__shfl(t.tflag_mine, ent0 + it * PPI, kWave);
            }
        };
        // x^A, x^T and the dense output O are touched once per frame: they stream past the caches (non-temporal), which
        // leaves L2 to the deltas and tap rows that producers and the next kernels re-read.  Measured over the whole
        // step, all three non-temporal is best (4 % against plain accesses).
        auto state_load = [&](__amdgpu_buffer_rsrc_t r, uint32_t o) -> Raw { return ws_load16_nt<Raw>(r, o); };
        auto state_store = [&](__amdgpu_buffer_rsrc_t r, uint32_t o, Raw v) { ws_store16_nt<Raw>(r, o, v); };
        struct Set { Raw ra[H], rt[H], rr[RES ? H : 1]; };
        // loads that do not depend on the convolution result, for the H iterations of set s
        auto load_set = [&](auto sf, const Tile& t, int s, Set& st) {
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const uint32_t o = t.off[s * H + h];
                if constexpr (RES) st.rr[h] = ws_load16<Raw>(rs_res, t.rflag[s * H + h] ? o : kOob);
                if constexpr (decltype(sf)::value) {
                    st.ra[h] = state_load(rs_xA, o);
                    // (not even issued when the flags say that no lane of the wave has anything to read)
                    st.rt[h] = raw_zero<T, V>();
                    if (__builtin_amdgcn_ballot_w64(t.tflag[s * H + h] != 0 && o != kOob))
                        st.rt[h] = state_load(rs_xT, t.tflag[s * H + h] ? o : kOob);
                }
            }
        };
        // arithmetic, decision and stores of set s; returns the survivor bits of its pixels
        auto finish_set = [&](auto sf, auto cf, const Tile& t, int s, const Set& st, const unsigned char* tile_stage) -> uint32_t {
            constexpr bool carry = decltype(cf)::value;            // an update leaves x^A's rounding residue in x^T
            uint32_t bits = 0;
            Raw rd[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                rd[h] = raw_load<T, V>(reinterpret_cast<const T*>(tile_stage + (size_t)(ent0 + (s * H + h) * PPI) * stage_stride));
                if (!ch_on) rd[h] = raw_zero<T, V>();              // lanes without channels must not raise the maximum
            }
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const int it = s * H + h;
                const uint32_t o = t.off[it];
                Raw d = rd[h];
                if constexpr (RES) {
#pragma unroll
                    for (int i = 0; i < V; ++i) raw_set<T, V>(d, i, raw_get<T, V>(rd[h], i) + raw_get<T, V>(st.rr[h], i));
                }
                bool upd = true;
                if constexpr (decltype(sf)::value) {
                    // o_y: the emitted delta -- or, in a final layer, the new dense output.  There O + dy with
                    // O = f(x^A_old) (true after the first frame and kept by every update: f(x^A_old) + f(s) - f(x^A_old))
                    // is f of the new x^A, so O is written without being read, and without the rounding an accumulation
                    // in the storage type would add frame after frame.  f(s) rounded to the storage type IS f of the
                    // rounded s: rounding is monotone and keeps 0 and the upper bound, which are representable.
                    Raw o_a, o_t, o_y, o_r = raw_zero<T, V>();
                    float u = 0.0f;
#pragma unroll
                    for (int i = 0; i < V; ++i) {
                        const float dd = raw_get<T, V>(d, i);
                        const float a = raw_get<T, V>(st.ra[h], i), tt = raw_get<T, V>(st.rt[h], i);
                        const float sum = (a + tt) + dd;
                        const float fs = act_clamp(sum, hi);
                        const float dy = fs - act_clamp(a, hi);
                        u = fmaxf(u, fabsf(dy));
                        raw_set<T, V>(o_a, i, sum);
                        raw_set<T, V>(o_t, i, tt + dd);             // x^T if the pixel is truncated
                        raw_set<T, V>(o_y, i, ACC ? fs : dy);
                        if constexpr (carry) raw_set<T, V>(o_r, i, round_residue<T>(sum));   // x^T if it is updated and keeps it
                    }
                    u = group_max(u, LP);
                    upd = u >= e.eps;
                    const uint32_t o_upd = upd ? o : kOob;
                    state_store(rs_xA, o_upd, o_a);
                    // an update resets x^T to zero (or to the rounding residue of the new x^A): where this lane's x^T
                    // already is all zero bits and stays so nothing needs to be written (most pixels that update every
                    // frame never accumulate anything)
                    {
                        const uint32_t o_t_off = (upd && all_bits_zero(st.rt[h]) && (!carry || all_bits_zero(o_r))) ? kOob : o;
                        if (__builtin_amdgcn_ballot_w64(o_t_off != kOob)) state_store(rs_xT, o_t_off, upd ? o_r : o_t);
                    }
                    if constexpr (ACC) state_store(rs_res, o_upd, o_y);
                    else ws_store16<Raw>(rs_out, o_upd, o_y);
                } else {
                    ws_store16<Raw>(rs_out, o, d);
                }
                const bool lead = t.pix[it] >= 0 && sub == 0;
                if (lead && upd) bits |= 1u << (ent0 + it * PPI);
            }
            return bits;
        };

        auto run = [&](auto sf, auto cf) {
            // Software pipeline.  List entries are requested two tiles ahead, residual flags one tile ahead,
            // and over the sets of consecutive tiles: while set s is finished, the loads of set s+1 (issued
            // one step earlier) and of set s+2 (issued right after) are in flight.
            constexpr bool carry = decltype(cf)::value;
            const int my_first = part * (kTile / cs), my_end = my_first + kTile / cs;    // tile entries this wave owns
            Tile cur, nxt;
            int pix_nn;
            cur.pix_mine = list_entry(0, lane % kTile);
            nxt.pix_mine = list_entry(1, lane % kTile);
            pix_nn = list_entry(2, lane % kTile);
            load_weights();
            prepare(cur);
            prepare(nxt);
            resolve(cur);
            Set set0, set1;
            load_set(sf, cur, 0, set0);
            load_set(sf, cur, 1, set1);
            for (int rd = 1; rd <= rounds; ++rd) {
                // `cur` is the tile produced in round rd-1, `nxt` the one being produced now
                const unsigned char* tile_stage = my_stage + (size_t)(((rd - 1) & 1) * NP) * stage_tile;
                await(staged_ctr, cs * rd);
                uint32_t bits = 0;
    #pragma unroll
                for (int s = 0; s < NS; s += 2) {
                    bits |= finish_set(sf, cf, cur, s, set0, tile_stage);
                    if (s + 2 == NS) resolve(nxt);                 // (its flags were requested a round ago)
                    if (s + 2 < NS) load_set(sf, cur, s + 2, set0); else load_set(sf, nxt, s + 2 - NS, set0);
                    bits |= finish_set(sf, cf, cur, s + 1, set1, tile_stage);
                    if (s + 3 < NS) load_set(sf, cur, s + 3, set1); else load_set(sf, nxt, s + 3 - NS, set1);
                }
                bump(consumed_ctr);                                // (every row of the tile has been read from LDS)
    #pragma unroll
                for (int m = kWave >> 1; m >= 1; m >>= 1) bits |= __shfl_xor(bits, m, kWave);
                if constexpr (decltype(sf)::value) {
                    // Flags of the tile's entries, one store instruction each (entry `lane` by lane `lane`).  The
                    // output mask gets the decision of every listed pixel: whatever it held before (1 from the dilated
                    // flags, or 0 from the clearing a step ahead) does not matter.  x^T row flag: after an update the
                    // row is zero again (unless it keeps residues), after a truncation it holds values.
                    const bool mine = lane >= my_first && lane < my_end && cur.pix_mine >= 0;
                    const bool upd_e = (bits >> (lane & 31)) & 1u;
                    if (has_omask && __builtin_amdgcn_ballot_w64(mine))
                        __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(upd_e ? 1 : 0), rs_omask, mine ? cur.pix_mine : (int)kOob, 0, 0);
                    const int keep = (upd_e && !carry) ? 0 : 1;
                    const bool change = mine && keep != cur.tflag_mine;
                    if (has_tflag && __builtin_amdgcn_ballot_w64(change))
                        __builtin_amdgcn_raw_buffer_store_b8((uint8_t)keep, rs_tflag, change ? cur.pix_mine : (int)kOob, 0, 0);
                }
                const int64_t tile = tile_of(rd - 1);
                if (tile * kTile < count) {
                    if (e.surv) {
                        // this wave owns bits [part*32/cs, (part+1)*32/cs) of the tile's survivor word
                        if (lane == 0) {
                            if (cs == 1) e.surv[tile] = bits;
                            else if (cs == 2) reinterpret_cast<uint16_t*>(e.surv)[tile * 2 + part] = (uint16_t)(bits >> (16 * part));
                            else reinterpret_cast<uint8_t*>(e.surv)[tile * 4 + part] = (uint8_t)(bits >> (8 * part));
                        }
                    } else {
                        survivors += __popc(bits);
                    }
                }
                cur = nxt;
                nxt.pix_mine = pix_nn;
                pix_nn = list_entry(rd + 2, lane % kTile);
                prepare(nxt);
            }
        };
        // layers with an activation keep state (x^A, x^T) and truncate; linear ones pass the delta on
        if (!stateful) run(std::false_type{}, std::false_type{});
        else if (e.carry) run(std::true_type{}, std::true_type{});
        else run(std::true_type{}, std::false_type{});
        // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
        if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
    }
}

}  // namespace dcnn
