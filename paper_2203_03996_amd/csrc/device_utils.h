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

__device__ __forceinline__ float act_apply(int act, float x) {
    if (act == DCNN_ACT_RELU) return fmaxf(x, 0.0f);
    if (act == DCNN_ACT_RELU6) return fminf(fmaxf(x, 0.0f), 6.0f);
    return x;
}

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

__device__ __forceinline__ int pow2_ceil(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// ---------------------------------------------------------------------------------------------
// Activation + truncation of one tile of 32 work-list entries, executed by one wavefront.
//
// Per pixel (Section 3.1, Eqs. 4-6):  s = (x^A + x^T) + dx;  dy = f(s) - f(x^A);
//   max_c |dy_c| >= eps : x^A <- s, x^T <- 0, emit dy, flag the pixel
//   otherwise           : x^T <- x^T + dx, pixel stays unflagged.
// First frame (init): v = dx (+ bias) (+ dense residual); x^A <- v, x^T <- 0, emit f(v).
// act == NONE: the (summed) delta is passed through, no state.
//
// LP consecutive lanes share one pixel (each lane owns up to VPL vectors of V channels), so a
// wave visits 64/LP pixels per iteration with fully coalesced 16-byte accesses; the per-pixel
// maximum is an LP-lane butterfly.  `dx(e, p, c0, out, valid_out)` delivers V channels of the
// first delta stream for tile entry e / pixel p, already rounded to the storage type.
// Returns the survivor word of the tile (bit e set iff entry e stays flagged) in every lane.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int VPL, class Dx>
__device__ __forceinline__ uint32_t act_trunc_tile(const EpilogueArgs& e, bool init, const int32_t* list,
                                                  int64_t tile_base, int64_t count, int lane, Dx dx,
                                                  int ch0 = 0, int nch = -1) {
    // [ch0, ch0 + nch) is the window of channels handled by this call (default: all of them);
    // windows are only used for pass-through (act == NONE) tiles, which need no per-pixel maximum
    const int C = e.c;
    if (nch < 0) nch = C;
    const int nvec = (nch + V - 1) / V;
    int LP = pow2_ceil((nvec + VPL - 1) / VPL);
    LP = LP < 2 ? 2 : (LP > kWave ? kWave : LP);
    const int PPI = kWave / LP;                       // pixels per iteration (<= 32)
    const int sub = lane % LP, grp = lane / LP;
    const T* bias = static_cast<const T*>(e.bias);
    const T* res = static_cast<const T*>(e.res_data);
    T* xA = static_cast<T*>(e.xA);
    T* xT = static_cast<T*>(e.xT);
    T* out = static_cast<T*>(e.out_data);
    uint32_t bits = 0;

    for (int it = 0; it < kTile / PPI; ++it) {
        const int ent = it * PPI + grp;
        const int64_t j = tile_base + ent;
        const bool valid = j < count;
        const int64_t p = valid ? (list ? (int64_t)list[j] : j) : 0;
        const bool res_ok = valid && res && (e.res_mask == nullptr || e.res_mask[p] != 0);

        float s[VPL][V], dy[VPL][V], d[VPL][V];
        float u = 0.0f;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int vi = sub + v * LP;
            const bool on = valid && vi < nvec;
            const int c0 = ch0 + vi * V;
#pragma unroll
            for (int i = 0; i < V; ++i) { s[v][i] = 0.0f; dy[v][i] = 0.0f; d[v][i] = 0.0f; }
            if (!on) continue;
            dx(ent, p, c0, d[v]);
            if (init) {
                if (bias) {
                    float b[V];
                    load_vec<T, V>(bias + c0, b);
#pragma unroll
                    for (int i = 0; i < V; ++i) d[v][i] = round_store<T>(d[v][i] + b[i]);
                }
                if (res) {
                    float r[V];
                    load_vec<T, V>(res + p * C + c0, r);
#pragma unroll
                    for (int i = 0; i < V; ++i) d[v][i] = round_store<T>(d[v][i] + r[i]);
                }
#pragma unroll
                for (int i = 0; i < V; ++i) { s[v][i] = d[v][i]; dy[v][i] = act_apply(e.act, d[v][i]); }
                continue;
            }
            if (res) {
                float r[V];
#pragma unroll
                for (int i = 0; i < V; ++i) r[i] = 0.0f;
                if (res_ok) load_vec<T, V>(res + p * C + c0, r);
#pragma unroll
                for (int i = 0; i < V; ++i) d[v][i] = round_store<T>(d[v][i] + r[i]);
            }
            if (e.act != DCNN_ACT_NONE) {
                float a[V], t[V];
                load_vec<T, V>(xA + p * C + c0, a);
                load_vec<T, V>(xT + p * C + c0, t);
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    s[v][i] = (a[i] + t[i]) + d[v][i];
                    dy[v][i] = act_apply(e.act, s[v][i]) - act_apply(e.act, a[i]);
                    u = fmaxf(u, fabsf(dy[v][i]));
                    d[v][i] = t[i] + d[v][i];            // what x^T becomes if the pixel is truncated
                }
            }
        }

        bool upd = true;
        if (!init && e.act != DCNN_ACT_NONE) {
            for (int m = LP >> 1; m >= 1; m >>= 1) u = fmaxf(u, __shfl_xor(u, m, kWave));
            upd = u >= e.eps;
        }

#pragma unroll
        for (int v = 0; v < VPL; ++v) {
            const int vi = sub + v * LP;
            if (!(valid && vi < nvec)) continue;
            const int64_t off = p * C + ch0 + vi * V;
            if (e.act == DCNN_ACT_NONE) {
                store_vec<T, V>(out + off, d[v]);
            } else if (init) {
                store_vec<T, V>(xA + off, s[v]);
                float z[V];
#pragma unroll
                for (int i = 0; i < V; ++i) z[i] = 0.0f;
                store_vec<T, V>(xT + off, z);
                store_vec<T, V>(out + off, dy[v]);
            } else if (upd) {
                store_vec<T, V>(xA + off, s[v]);
                float z[V];
#pragma unroll
                for (int i = 0; i < V; ++i) z[i] = 0.0f;
                store_vec<T, V>(xT + off, z);
                store_vec<T, V>(out + off, dy[v]);
            } else {
                store_vec<T, V>(xT + off, d[v]);
            }
        }
        if (valid && sub == 0) {
            if (e.out_mask && !init) e.out_mask[p] = upd ? 1 : 0;
            if (upd) bits |= 1u << ent;
        }
    }
#pragma unroll
    for (int m = kWave >> 1; m >= 1; m >>= 1) bits |= __shfl_xor(bits, m, kWave);
    return bits;
}

}  // namespace dcnn
