// Device-side helpers shared by the kernels: element types, 16-byte channel vectors,
// work-list iteration and the activation + truncation tail.
#pragma once

#include "common.h"

namespace dcnn {

typedef _Float16 f16;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int VEC = 4; };
template <> struct Elem<f16> { static constexpr int VEC = 8; };

// V consecutive channels starting at p, widened to fp32.  V is the full 16-byte vector or 1.
template <typename T, int V> __device__ __forceinline__ void load_vec(const T* p, float (&o)[V]) {
    if constexpr (V == 1) {
        o[0] = (float)p[0];
    } else if constexpr (sizeof(T) == 2) {
        f16x8 v = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = (float)v[i];
    } else {
        f32x4 v = *reinterpret_cast<const f32x4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = v[i];
    }
}

// Round to the storage type (round-to-nearest-even) and store V consecutive channels.
template <typename T, int V> __device__ __forceinline__ void store_vec(T* p, const float (&o)[V]) {
    if constexpr (V == 1) {
        p[0] = (T)o[0];
    } else if constexpr (sizeof(T) == 2) {
        f16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (f16)o[i];
        *reinterpret_cast<f16x8*>(p) = v;
    } else {
        f32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = o[i];
        *reinterpret_cast<f32x4*>(p) = v;
    }
}

// Value as it will read back after a store in the storage type.
template <typename T> __device__ __forceinline__ float round_store(float x) { return (float)(T)x; }
// What the stored value loses: exact in fp32 (the difference of an fp32 number and its rounding to fewer bits).
template <typename T> __device__ __forceinline__ float round_residue(float x) { return x - (float)(T)x; }

// ReLU and ReLU6 as one clamp to [0, hi] (hi = +inf / 6): a single median-of-three instruction,
// exact for every finite x.  Callers compute hi once from the layer's activation.
__device__ __forceinline__ float act_hi(int act) { return act == DCNN_ACT_RELU6 ? 6.0f : INFINITY; }
__device__ __forceinline__ float act_clamp(float x, float hi) { return __builtin_amdgcn_fmed3f(x, 0.0f, hi); }

__device__ __forceinline__ int64_t list_count(const ListArgs& l) {
    return l.count ? (int64_t)(*l.count) : l.count_host;
}

// Work-list tiles are handed out so that consecutive tiles (neighbouring pixels) stay on one
// XCD and share its L2: workgroup b runs on XCD b % 8; XCD x owns a contiguous range of
// workgroup-tiles and its workgroups stride through that range.
struct WgTileRange {
    int64_t begin, end, step;
};
__device__ __forceinline__ WgTileRange wg_tile_range(int64_t n_wg_tiles) {
    const int xcd = blockIdx.x % kXcd, slot = blockIdx.x / kXcd, nslots = gridDim.x / kXcd;
    const int64_t per = (n_wg_tiles + kXcd - 1) / kXcd;
    WgTileRange r;
    r.begin = (int64_t)xcd * per + slot;
    r.end = min((int64_t)(xcd + 1) * per, n_wg_tiles);
    r.step = nslots;
    return r;
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f) {
    return (__umulhi(n, f.m) + n) >> f.s;
}

__device__ __forceinline__ int pow2_ceil(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Raw storage-typed vector of V channels (one 16-byte register quad, or a single element).
template <typename T, int V> struct RawOf;
template <> struct RawOf<f16, 8> { typedef f16x8 type; };
template <> struct RawOf<float, 4> { typedef f32x4 type; };
template <> struct RawOf<f16, 1> { typedef f16 type; };
template <> struct RawOf<float, 1> { typedef float type; };

template <typename T, int V> __device__ __forceinline__ typename RawOf<T, V>::type raw_load(const T* p) {
    return *reinterpret_cast<const typename RawOf<T, V>::type*>(p);
}
template <typename T, int V> __device__ __forceinline__ void raw_store(T* p, typename RawOf<T, V>::type v) {
    *reinterpret_cast<typename RawOf<T, V>::type*>(p) = v;
}
template <typename T, int V> __device__ __forceinline__ typename RawOf<T, V>::type raw_zero() {
    typename RawOf<T, V>::type v;
    if constexpr (V == 1) v = (T)0.0f;
    else {
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = (T)0.0f;
    }
    return v;
}
template <typename T, int V> __device__ __forceinline__ float raw_get(const typename RawOf<T, V>::type& v, int i) {
    if constexpr (V == 1) return (float)v;
    else return (float)v[i];
}
// round-to-nearest-even into the storage type
template <typename T, int V> __device__ __forceinline__ void raw_set(typename RawOf<T, V>::type& v, int i, float x) {
    if constexpr (V == 1) v = (T)x;
    else v[i] = (T)x;
}

// Maximum of a non-negative value over aligned groups of LP lanes (LP a power of two, 2 .. 64), delivered to every
// lane of the group.  Steps within a row of 16 lanes use DPP lane permutations (register to register, a few
// clocks each: two quad swaps, then the half-row and the row mirrored -- after the quad steps every quad holds
// one value, so a mirror serves as well as an exchange); only the steps across rows go through the LDS
// crossbar.  All lanes of the wave must be active.
template <int CTRL> __device__ __forceinline__ float dpp_max_step(float u) {
    const int v = __builtin_bit_cast(int, u);
    const int o = __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, true);
    return fmaxf(u, __builtin_bit_cast(float, o));
}
__device__ __forceinline__ float group_max(float u, int LP) {
    if (LP >= 2) u = dpp_max_step<0xB1>(u);       // quad_perm [1,0,3,2]
    if (LP >= 4) u = dpp_max_step<0x4E>(u);       // quad_perm [2,3,0,1]
    if (LP >= 8) u = dpp_max_step<0x141>(u);      // row_half_mirror
    if (LP >= 16) u = dpp_max_step<0x140>(u);     // row_mirror
    if (LP >= 32) u = fmaxf(u, __shfl_xor(u, 16, kWave));
    if (LP >= 64) u = fmaxf(u, __shfl_xor(u, 32, kWave));
    return u;
}

// LDS-only synchronisation: orders shared-memory traffic without waiting for outstanding global
// loads and stores (a generic fence would drain them and stall the memory pipeline).
// Zeroes e.clear_mask cooperatively: every workgroup of the grid takes a share, before any of them may leave.  A layer
// that walks its input's own list alternates between two output masks; the one its next step will write is cleared
// here, a step ahead, so that step finds zeros wherever it does not write and needs no mask pass of its own.
__device__ __forceinline__ void clear_ahead(const EpilogueArgs& e) {
    if (e.clear_mask == nullptr) return;
    const int64_t n16 = e.clear_bytes / 16;                    // (state pieces are 256-byte aligned)
    const int64_t nthreads = (int64_t)gridDim.x * gridDim.y * blockDim.x;
    const int64_t me = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
    uint4* p16 = reinterpret_cast<uint4*>(e.clear_mask);
    for (int64_t i = me; i < n16; i += nthreads) p16[i] = make_uint4(0u, 0u, 0u, 0u);
    if (me < e.clear_bytes - n16 * 16) e.clear_mask[n16 * 16 + me] = 0;
}

__device__ __forceinline__ void lds_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}
__device__ __forceinline__ void lds_block_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// How several waves that hold different channel slices of the same pixels agree on the
// per-pixel maximum: each writes its partial maxima to LDS, one block barrier, each reads all.
struct MaxExchange {
    float* buf;      // [2][parts][32] floats in LDS (double-buffered by batch parity)
    int parts;       // waves per pixel tile (1: no exchange)
    int part;        // this wave's slice
};

// ---------------------------------------------------------------------------------------------
// Activation + truncation of one tile of 32 work-list entries, executed by one wavefront (or by
// `parts` wavefronts that each own a slice of the channels).
//
// Per pixel (Section 3.1, Eqs. 4-6):  s = (x^A + x^T) + dx;  dy = f(s) - f(x^A);
//   max_c |dy_c| >= eps : x^A <- s, x^T <- 0, emit dy, flag the pixel
//   otherwise           : x^T <- x^T + dx, pixel stays unflagged.
// First frame (init): v = dx (+ dense residual); x^A <- v, x^T <- 0, emit f(v).  (A convolution's bias is part
// of dx: the producer adds it to the fp32 sum before that is rounded to the storage type.)
// act == NONE: the (summed) delta is passed through, no state.
//
// The call handles the channel window [ch0, ch0+nch) of every pixel.  LP consecutive lanes share
// one pixel (each lane owns up to VPL vectors of V channels), so a wave visits 64/LP pixels per
// iteration with coalesced 16-byte accesses; the per-pixel maximum is an LP-lane butterfly,
// followed by the LDS exchange when the pixel's channels are spread over several waves.  The
// kernel is bound by memory latency, not arithmetic: the loads of UB iterations (delta, residual,
// x^A, x^T) are issued back to back before any of them is consumed.  `p_mine` is the pixel of
// entry lane%32 (or -1), so no index-list load sits in front of the address computation.
// `dx(ent, p, c0)` delivers V channels of the first delta stream for tile entry `ent` / pixel p
// as a raw vector already rounded to the storage type.
// Returns the survivor word of the tile (bit e set iff entry e stays flagged) in every lane.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int VPL, int UB, bool XCHG, class Dx>
__device__ __forceinline__ uint32_t act_trunc_tile(const EpilogueArgs& e, bool init, int p_mine, int lane, Dx dx,
                                                  int ch0, int nch, int span, MaxExchange mx) {
    // `span` >= nch fixes how lanes are laid out over a pixel's channels; waves that exchange maxima
    // must use the same span so that they run the same number of batches (and barriers)
    typedef typename RawOf<T, V>::type Raw;
    const int C = e.c;
    const int nvec = (nch + V - 1) / V;
    int LP = pow2_ceil(((span + V - 1) / V + VPL - 1) / VPL);
    LP = LP < 2 ? 2 : (LP > kWave ? kWave : LP);
    const int PPI = kWave / LP;                       // pixels per iteration (<= 32)
    const int sub = lane % LP, grp = lane / LP;
    const int iters = kTile / PPI;
    const T* res = static_cast<const T*>(e.res_data);
    T* xA = static_cast<T*>(e.xA);
    T* xT = static_cast<T*>(e.xT);
    T* out = static_cast<T*>(e.out_data);
    const bool stateful = e.act != DCNN_ACT_NONE;
    const float hi = act_hi(e.act);
    uint32_t bits = 0;
    int batch = 0;

    for (int it0 = 0; it0 < iters; it0 += UB, ++batch) {
        int pix[UB];
        Raw rd[UB][VPL], rr[UB][VPL], ra[UB][VPL], rt[UB][VPL];
        // ---- phase 1: issue every load of the batch ---------------------------------------------
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            const int ent = (it0 + ub) * PPI + grp;
            const int p32 = (it0 + ub) < iters ? __shfl(p_mine, ent & (kTile - 1), kWave) : -1;
            pix[ub] = p32;
            const int64_t p = p32;
            const bool valid = p32 >= 0;
            const bool res_ok = valid && res && (init || e.res_mask == nullptr || e.res_mask[p] != 0);
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const int vi = sub + v * LP;
                const bool on = valid && vi < nvec;
                const int c0 = ch0 + vi * V;
                rd[ub][v] = raw_zero<T, V>(); rr[ub][v] = raw_zero<T, V>();
                ra[ub][v] = raw_zero<T, V>(); rt[ub][v] = raw_zero<T, V>();
                if (!on) continue;
                rd[ub][v] = dx(ent, p, c0);
                if (res_ok) rr[ub][v] = raw_load<T, V>(res + p * C + c0);
                if (stateful && !init) {
                    ra[ub][v] = raw_load<T, V>(xA + p * C + c0);
                    if (xT) rt[ub][v] = raw_load<T, V>(xT + p * C + c0);           // no buffer: truncated values are not kept
                }
            }
        }
        // ---- phase 2: arithmetic and the per-pixel maximum ---------------------------------------
        Raw o_a[UB][VPL], o_t[UB][VPL], o_y[UB][VPL];
        float umax[UB];
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            float u = 0.0f;
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    float d = raw_get<T, V>(rd[ub][v], i);
                    if (init) {
                        if (res) d = round_store<T>(d + raw_get<T, V>(rr[ub][v], i));
                        raw_set<T, V>(o_a[ub][v], i, d);
                        raw_set<T, V>(o_t[ub][v], i, 0.0f);
                        raw_set<T, V>(o_y[ub][v], i, stateful ? act_clamp(d, hi) : d);
                    } else {
                        if (res) d = round_store<T>(d + raw_get<T, V>(rr[ub][v], i));
                        if (stateful) {
                            const float a = raw_get<T, V>(ra[ub][v], i), t = raw_get<T, V>(rt[ub][v], i);
                            const float s = (a + t) + d;
                            const float dy = act_clamp(s, hi) - act_clamp(a, hi);
                            u = fmaxf(u, fabsf(dy));
                            raw_set<T, V>(o_a[ub][v], i, s);
                            raw_set<T, V>(o_t[ub][v], i, t + d);       // x^T if the pixel is truncated
                            raw_set<T, V>(o_y[ub][v], i, dy);
                        } else {
                            raw_set<T, V>(o_a[ub][v], i, 0.0f);
                            raw_set<T, V>(o_t[ub][v], i, 0.0f);
                            raw_set<T, V>(o_y[ub][v], i, d);
                        }
                    }
                }
            }
            if (!init && stateful)
                for (int m = LP >> 1; m >= 1; m >>= 1) u = fmaxf(u, __shfl_xor(u, m, kWave));
            umax[ub] = u;
        }
        if constexpr (XCHG) {
            // every wave of the workgroup passes here the same number of times
            float* slot = mx.buf + (size_t)(batch & 1) * mx.parts * kTile;
#pragma unroll
            for (int ub = 0; ub < UB; ++ub) {
                const int ent = (it0 + ub) * PPI + grp;
                if (sub == 0 && (it0 + ub) < iters) slot[mx.part * kTile + ent] = umax[ub];
            }
            lds_block_sync();
#pragma unroll
            for (int ub = 0; ub < UB; ++ub) {
                const int ent = ((it0 + ub) * PPI + grp) & (kTile - 1);
                float u = 0.0f;
                for (int q = 0; q < mx.parts; ++q) u = fmaxf(u, slot[q * kTile + ent]);
                umax[ub] = u;
            }
        }
        // ---- phase 3: decision and stores --------------------------------------------------------
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            const int64_t p = pix[ub];
            const bool valid = pix[ub] >= 0;
            const int ent = (it0 + ub) * PPI + grp;
            const bool upd = (init || !stateful) ? true : (umax[ub] >= e.eps);
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const int vi = sub + v * LP;
                if (!(valid && vi < nvec)) continue;
                const int64_t off = p * C + ch0 + vi * V;
                if (!stateful) {
                    raw_store<T, V>(out + off, o_y[ub][v]);
                } else if (upd) {
                    raw_store<T, V>(xA + off, o_a[ub][v]);
                    if (xT) {
                        Raw keep = raw_zero<T, V>();
                        if (e.carry && !init) {
                            // the rounding residue of the new x^A, from the same operands in the same order
#pragma unroll
                            for (int i = 0; i < V; ++i) {
                                float d = raw_get<T, V>(rd[ub][v], i);
                                if (res) d = round_store<T>(d + raw_get<T, V>(rr[ub][v], i));
                                const float s = (raw_get<T, V>(ra[ub][v], i) + raw_get<T, V>(rt[ub][v], i)) + d;
                                raw_set<T, V>(keep, i, round_residue<T>(s));
                            }
                        }
                        raw_store<T, V>(xT + off, keep);
                    }
                    raw_store<T, V>(out + off, o_y[ub][v]);
                } else if (xT) {
                    raw_store<T, V>(xT + off, o_t[ub][v]);
                }
            }
            if (valid && sub == 0) {
                if (e.out_mask && !init && mx.part == 0) e.out_mask[p] = upd ? 1 : 0;
                if (upd) bits |= 1u << ent;
            }
        }
    }
    if constexpr (XCHG) lds_block_sync();             // the exchange buffers are free again for the next tile
#pragma unroll
    for (int m = kWave >> 1; m >= 1; m >>= 1) bits |= __shfl_xor(bits, m, kWave);
    return bits;
}

// ---------------------------------------------------------------------------------------------
// The same tail split in two for the convolution kernels: `tail_prefetch` issues the loads that
// do not depend on the convolution result (residual, x^A, x^T of the whole tile) BEFORE the K
// loop, so their latency hides behind the gathers and the matrix work; `tail_finish` consumes
// them once the result tile is staged.  One vector per lane and pixel (VPL = 1), NIT = 32 / (64/LP)
// iterations cover the tile.  Arithmetic, rounding and decisions are exactly those of
// act_trunc_tile.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int NIT> struct TailRegs {
    typename RawOf<T, V>::type rr[NIT], ra[NIT], rt[NIT];
    int pix[NIT];
};

template <typename T, int V, int NIT>
__device__ __forceinline__ void tail_prefetch(const EpilogueArgs& e, bool init, int p_mine, int lane, int ch0, int nch,
                                             TailRegs<T, V, NIT>& r) {
    constexpr int PPI = kTile / NIT, LP = kWave / PPI;
    const int C = e.c;
    const int nvec = (nch + V - 1) / V;
    const int sub = lane % LP, grp = lane / LP;
    const T* res = static_cast<const T*>(e.res_data);
    const T* xA = static_cast<const T*>(e.xA);
    const T* xT = static_cast<const T*>(e.xT);
    const bool stateful = e.act != DCNN_ACT_NONE;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int ent = it * PPI + grp;
        const int p32 = __shfl(p_mine, ent, kWave);
        r.pix[it] = p32;
        const int64_t p = p32;
        const bool on = p32 >= 0 && sub < nvec;
        const int c0 = ch0 + sub * V;
        r.rr[it] = raw_zero<T, V>(); r.ra[it] = raw_zero<T, V>(); r.rt[it] = raw_zero<T, V>();
        if (!on) continue;
        if (res && (init || e.res_mask == nullptr || e.res_mask[p] != 0)) r.rr[it] = raw_load<T, V>(res + p * C + c0);
        if (stateful && !init) {
            r.ra[it] = raw_load<T, V>(xA + p * C + c0);
            if (xT) r.rt[it] = raw_load<T, V>(xT + p * C + c0);
        }
    }
}

template <typename T, int V, int NIT, bool XCHG, class Dx>
__device__ __forceinline__ uint32_t tail_finish(const EpilogueArgs& e, bool init, int lane, Dx dx, int ch0, int nch,
                                               MaxExchange mx, const TailRegs<T, V, NIT>& r) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr int PPI = kTile / NIT, LP = kWave / PPI;
    const int C = e.c;
    const int nvec = (nch + V - 1) / V;
    const int sub = lane % LP, grp = lane / LP;
    const bool has_res = e.res_data != nullptr;
    T* xA = static_cast<T*>(e.xA);
    T* xT = static_cast<T*>(e.xT);
    T* out = static_cast<T*>(e.out_data);
    const bool stateful = e.act != DCNN_ACT_NONE;
    const float hi = act_hi(e.act);
    Raw o_a[NIT], o_t[NIT], o_y[NIT], o_r[NIT];
    float umax[NIT];
    uint32_t bits = 0;
    const bool carry = e.carry && !init;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int ent = it * PPI + grp;
        const bool on = r.pix[it] >= 0 && sub < nvec;
        Raw rd = raw_zero<T, V>();
        if (on) rd = dx(ent, (int64_t)r.pix[it], ch0 + sub * V);
        o_r[it] = raw_zero<T, V>();
        float u = 0.0f;
#pragma unroll
        for (int i = 0; i < V; ++i) {
            float d = raw_get<T, V>(rd, i);
            if (init) {
                if (has_res) d = round_store<T>(d + raw_get<T, V>(r.rr[it], i));
                raw_set<T, V>(o_a[it], i, d);
                raw_set<T, V>(o_t[it], i, 0.0f);
                raw_set<T, V>(o_y[it], i, stateful ? act_clamp(d, hi) : d);
            } else {
                if (has_res) d = round_store<T>(d + raw_get<T, V>(r.rr[it], i));
                if (stateful) {
                    const float a = raw_get<T, V>(r.ra[it], i), t = raw_get<T, V>(r.rt[it], i);
                    const float s = (a + t) + d;
                    const float dy = act_clamp(s, hi) - act_clamp(a, hi);
                    u = fmaxf(u, fabsf(dy));
                    raw_set<T, V>(o_a[it], i, s);
                    raw_set<T, V>(o_t[it], i, t + d);
                    raw_set<T, V>(o_y[it], i, dy);
                    if (carry) raw_set<T, V>(o_r[it], i, round_residue<T>(s));   // x^T of an updated pixel
                } else {
                    raw_set<T, V>(o_a[it], i, 0.0f);
                    raw_set<T, V>(o_t[it], i, 0.0f);
                    raw_set<T, V>(o_y[it], i, d);
                }
            }
        }
        if (!init && stateful)
            for (int m = LP >> 1; m >= 1; m >>= 1) u = fmaxf(u, __shfl_xor(u, m, kWave));
        umax[it] = u;
    }
    if constexpr (XCHG) {
        // every wave of the workgroup passes here once per tile
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            if (sub == 0) mx.buf[mx.part * kTile + it * PPI + grp] = umax[it];
        lds_block_sync();
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            float u = 0.0f;
            for (int q = 0; q < mx.parts; ++q) u = fmaxf(u, mx.buf[q * kTile + it * PPI + grp]);
            umax[it] = u;
        }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int64_t p = r.pix[it];
        const bool valid = r.pix[it] >= 0;
        const int ent = it * PPI + grp;
        const bool upd = (init || !stateful) ? true : (umax[it] >= e.eps);
        if (valid && sub < nvec) {
            const int64_t off = p * C + ch0 + sub * V;
            if (!stateful) {
                raw_store<T, V>(out + off, o_y[it]);
            } else if (upd) {
                raw_store<T, V>(xA + off, o_a[it]);
                if (xT) raw_store<T, V>(xT + off, o_r[it]);
                raw_store<T, V>(out + off, o_y[it]);
            } else if (xT) {
                raw_store<T, V>(xT + off, o_t[it]);
            }
        }
        if (valid && sub == 0) {
            if (e.out_mask && !init && mx.part == 0) e.out_mask[p] = upd ? 1 : 0;
            if (upd) bits |= 1u << ent;
        }
    }
    if constexpr (XCHG) lds_block_sync();             // the exchange buffer is free again for the next tile
#pragma unroll
    for (int m = kWave >> 1; m >= 1; m >>= 1) bits |= __shfl_xor(bits, m, kWave);
    return bits;
}

// Sources of output coordinate o of a bilinear upsampling by the integer factor r (half-pixel centres): the
// sample position (o + 0.5) / r - 0.5 = (2o + 1 - r) / 2r, clamped to the map.  Source i0 always carries weight;
// i1 == i0 when it alone does (w1 = 0), else i1 = i0 + 1 with weight w1.  Integer arithmetic decides, so "no
// weight" is exact.
struct BilinTaps { int i0, i1; float w1; };
__device__ __forceinline__ BilinTaps bilin_taps(int o, int r, int size) {
    BilinTaps t;
    const int num = 2 * o + 1 - r, den = 2 * r;
    if (num <= 0) { t.i0 = t.i1 = 0; t.w1 = 0.0f; return t; }
    const int i0 = num / den, rem = num - i0 * den;
    if (i0 >= size - 1) { t.i0 = t.i1 = size - 1; t.w1 = 0.0f; return t; }
    t.i0 = i0; t.i1 = rem ? i0 + 1 : i0; t.w1 = (float)rem / (float)den;
    return t;
}

// ---- buffer addressing ---------------------------------------------------------------------------
// A load through a buffer descriptor at a byte offset outside the descriptor's range returns zeros and a
// store there is dropped, so "this lane has nothing to do" is an offset, not a branch: every load of a
// phase can be issued back to back.  Offsets are 32 bit: tensors addressed this way stay below 2 GiB.
constexpr uint32_t kOob = 0x80000000u;                         // byte offset no descriptor here reaches
constexpr uint64_t kWsMaxBytes = 0x7fffffffull;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t ws_rsrc(const void* p, uint64_t bytes) {
    // raw buffer (stride 0), 32-bit data format; a null pointer gives an empty range
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, p ? (int)bytes : 0, 0x00020000);
}
template <typename Raw> __device__ __forceinline__ Raw ws_load16(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(Raw, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0));
}
template <typename Raw> __device__ __forceinline__ void ws_store16(__amdgpu_buffer_rsrc_t r, uint32_t off, Raw v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)off, 0, 0);
}
// True iff every bit of the 16-byte vector is zero (+0.0 in every element).
template <typename Raw> __device__ __forceinline__ bool all_bits_zero(Raw v) {
    const u32x4 w = __builtin_bit_cast(u32x4, v);
    return (w[0] | w[1] | w[2] | w[3]) == 0u;
}
// The same with the non-temporal hint, for data that is touched once per frame (accumulated values, truncated
// values, the stored frame, the dense output): it streams past the caches instead of displacing the deltas and
// weights that the next kernels re-read.
constexpr int kAuxNonTemporal = 2;
template <typename Raw> __device__ __forceinline__ Raw ws_load16_nt(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(Raw, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, kAuxNonTemporal));
}
template <typename Raw> __device__ __forceinline__ void ws_store16_nt(__amdgpu_buffer_rsrc_t r, uint32_t off, Raw v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)off, 0, kAuxNonTemporal);
}

// Pixel of work-list entry `j` for the lane that owns it (-1 beyond the end of the list).
__device__ __forceinline__ int list_pixel(const int32_t* list, int64_t j, int64_t count) {
    if (j >= count) return -1;
    return list ? list[j] : (int)j;
}

}  // namespace dcnn
