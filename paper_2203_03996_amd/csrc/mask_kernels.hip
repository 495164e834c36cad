// Update-mask propagation and ordered compaction (Section 3.2 "Update mask", Section 3.3).
//
// mask pass  : pixel space; out[o] = OR of the input mask over the in-bounds window taps of o
//              (or the nearest-upsampled input mask), OR a second mask; one count per chunk.
// emit       : pixel space; exclusive prefix over the chunk counts + an in-chunk scan turn the
//              mask into the ascending list of flagged pixels.  No atomics: the list order is
//              fixed, so results are identical from run to run.
//              Optionally also writes, per list entry, the word of window taps that are in bounds and
//              flagged, so the convolution does not have to test the window again.
// emit_sublist: list space; keeps the entries of a work list whose survivor bit is set.
#include "device_utils.h"

namespace dcnn {

constexpr int kMaskThreads = 256;
constexpr int kPxPerThread = kChunk / kMaskThreads;     // 8 consecutive pixels per thread
static_assert(kPxPerThread == 8, "one 64-bit mask word per thread");

__device__ __forceinline__ int block_sum(int v, int* s_red) {
    for (int m = kWave >> 1; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    int t = 0;
    for (int i = 0; i < kMaskThreads / kWave; ++i) t += s_red[i];
    __syncthreads();
    return t;
}

// Exclusive prefix of v over the threads of the block (thread order), and the block total.
__device__ __forceinline__ int block_exclusive_scan(int v, int* s_red, int* total) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int inc = v;
    for (int d = 1; d < kWave; d <<= 1) {
        const int o = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += o;
    }
    if (lane == kWave - 1) s_red[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < kMaskThreads / kWave; ++i) {
        const int s = s_red[i];
        if (i < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// Every non-zero byte of the word becomes 1.
__device__ __forceinline__ uint64_t bytes01(uint64_t w) {
    w |= w >> 4; w |= w >> 2; w |= w >> 1;
    return w & 0x0101010101010101ull;
}

// Flags of input row iy at columns x0-1 .. x0+8 as a bit string (bit j = column x0-1+j), zero outside
// the image.  x0 is a multiple of 8 and the row width a multiple of 8, so the middle is one word.
__device__ __forceinline__ uint32_t row_flags10(const uint8_t* mask, int64_t n, int iy, int x0, int h, int w) {
    if (iy < 0 || iy >= h) return 0;
    const uint8_t* row = mask + (n * h + iy) * w;
    const uint64_t word = bytes01(*reinterpret_cast<const uint64_t*>(row + x0));
    uint32_t bits = (uint32_t)((word * 0x0102040810204080ull) >> 56) << 1;      // byte i -> bit i+1
    if (x0 > 0 && row[x0 - 1]) bits |= 1u;
    if (x0 + 8 < w && row[x0 + 8]) bits |= 1u << 9;
    return bits;
}

// 3x3 window, stride 1, padding 1, rows a multiple of 8 pixels wide: the common dilation, done on
// bit strings instead of byte by byte.
__device__ __forceinline__ bool window3_fast(int k, int stride, int pad, int up, int h, int w, int oh, int ow) {
    return k == 3 && stride == 1 && pad == 1 && up == 1 && (w % 8) == 0 && oh == h && ow == w;
}

// The same window on rows of any width.  The 8 pixels of a thread may then straddle rows, so the flags are taken
// from three spans of 10 consecutive bytes in FLAT pixel order (rows above / at / below, one pixel of margin on
// either side) and each tap is masked by its own bounds test.  All 30 byte loads are independent of each other:
// one round trip to memory instead of one per tap.
__device__ __forceinline__ bool window3_any(int k, int stride, int pad, int up, int h, int w, int oh, int ow) {
    return k == 3 && stride == 1 && pad == 1 && up == 1 && oh == h && ow == w;
}
// bit j: the pixel with flat index first + j exists and is flagged
__device__ __forceinline__ uint32_t span_flags10(const uint8_t* mask, int64_t first, int64_t total) {
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 10; ++j) {
        const int64_t q = first + j;
        const bool in = q >= 0 && q < total;
        const uint8_t f = mask[in ? q : 0];
        if (in && f) bits |= 1u << j;
    }
    return bits;
}
struct Spans3 { uint32_t row[3]; };
__device__ __forceinline__ Spans3 window3_spans(const uint8_t* mask, int64_t p0, int w, int64_t total) {
    Spans3 s;
#pragma unroll
    for (int r = 0; r < 3; ++r) s.row[r] = span_flags10(mask, p0 - 1 + (int64_t)(r - 1) * w, total);
    return s;
}
// taps of pixel p0 + i at (x, y): bit dy*3+dx set iff the tap is inside the map and flagged
__device__ __forceinline__ uint32_t window3_taps(const Spans3& s, int i, int x, int y, int h, int w) {
    uint32_t taps = 0;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        if ((unsigned)(y + dy - 1) >= (unsigned)h) continue;
        uint32_t three = (s.row[dy] >> i) & 7u;
        if (x == 0) three &= ~1u;
        if (x == w - 1) three &= ~4u;
        taps |= three << (3 * dy);
    }
    return taps;
}

// Window taps of the 8 output pixels from p0 on, for a K x K window of any stride and padding: bit ky*K+kx of
// taps[i] is set iff that tap of pixel p0+i lies inside the map and is flagged.  Every load is issued
// unconditionally (a tap outside the map or a pixel beyond the end reads byte 0 of the mask and is masked out),
// so the 8*K*K loads are independent and cost one round trip instead of one each.
template <int K>
__device__ __forceinline__ void window_taps8(const uint8_t* mask, int64_t p0, int64_t out_pixels, int h, int w, int oh, int ow,
                                             int stride, int pad, uint32_t (&taps)[kPxPerThread]) {
    int ox = (int)(p0 % ow);
    const int64_t t = p0 / ow;
    int oy = (int)(t % oh);
    int64_t n = t / oh;
    uint8_t f[kPxPerThread][K * K];
    uint32_t ok[kPxPerThread];
#pragma unroll
    for (int i = 0; i < kPxPerThread; ++i) {
        const bool live = p0 + i < out_pixels;
        const int iy0 = oy * stride - pad, ix0 = ox * stride - pad;
        const int64_t base = (n * h + iy0) * (int64_t)w + ix0;
        uint32_t okm = 0;
#pragma unroll
        for (int ky = 0; ky < K; ++ky)
#pragma unroll
            for (int kx = 0; kx < K; ++kx) {
                const bool in = live && (unsigned)(iy0 + ky) < (unsigned)h && (unsigned)(ix0 + kx) < (unsigned)w;
                f[i][ky * K + kx] = mask[in ? base + (int64_t)ky * w + kx : 0];
                if (in) okm |= 1u << (ky * K + kx);
            }
        ok[i] = okm;
        if (++ox == ow) { ox = 0; if (++oy == oh) { oy = 0; ++n; } }
    }
#pragma unroll
    for (int i = 0; i < kPxPerThread; ++i) {
        uint32_t tp = 0;
#pragma unroll
        for (int j = 0; j < K * K; ++j)
            if (f[i][j]) tp |= 1u << j;
        taps[i] = tp & ok[i];
    }
}

// Flag of the second mask for output pixel p (same shape as the output, or sampled with a stride).
__device__ __forceinline__ bool mask_b_flag(const uint8_t* mask_b, int64_t p, int b_stride, int b_h, int b_w, int oh, int ow) {
    if (b_stride <= 0) return mask_b[p] != 0;
    const int x = (int)(p % ow);
    const int64_t t = p / ow;
    const int y = (int)(t % oh);
    const int64_t n = t / oh;
    return mask_b[(n * b_h + (int64_t)y * b_stride) * b_w + (int64_t)x * b_stride] != 0;
}

struct MaskKernelArgs {
    const uint8_t* mask_in;
    const uint8_t* mask_b;
    uint8_t* mask_out;
    int32_t* chunk_counts;
    int32_t* zero_count;
    int64_t out_pixels;
    int n, h, w, oh, ow, k, stride, pad, up;
    int bilinear;                 // with up > 1: sources of a bilinear upsampling instead of the nearest pixel
    int b_stride, b_h, b_w;       // > 0: mask_b is sampled at (y, x) * b_stride of an [n, b_h, b_w] map
    int kw, pad_w;                // window columns and their padding (rows: k, pad)
};

// Output flags of the 8 pixels from p0 on (byte i of the word: pixel p0+i); with STORE also written to the output mask.
template <bool STORE>
__device__ __forceinline__ uint64_t mask_word(const MaskKernelArgs& a, int64_t p0) {
    uint64_t word = 0;
    if (p0 < a.out_pixels) {
        const bool b_same = a.mask_b == nullptr || a.b_stride <= 0;
        const bool square = a.kw == a.k && a.pad_w == a.pad;
        if (square && a.k == 1 && a.stride == 1 && a.up == 1 && b_same && p0 + kPxPerThread <= a.out_pixels) {
            word = *reinterpret_cast<const uint64_t*>(a.mask_in + p0);
            if (a.mask_b) word |= *reinterpret_cast<const uint64_t*>(a.mask_b + p0);
        } else if (square && b_same && window3_fast(a.k, a.stride, a.pad, a.up, a.h, a.w, a.oh, a.ow)) {
            const int x0 = (int)(p0 % a.w);
            const int64_t t = p0 / a.w;
            const int y = (int)(t % a.h);
            const int64_t n = t / a.h;
            uint32_t any = 0;                                   // bit j: some row has a flag at column x0-1+j
            for (int r = -1; r <= 1; ++r) any |= row_flags10(a.mask_in, n, y + r, x0, a.h, a.w);
            const uint32_t hit = (any | (any >> 1) | (any >> 2)) & 0xffu;   // bit i: window of pixel x0+i has a flag
            for (int i = 0; i < kPxPerThread; ++i) word |= (uint64_t)((hit >> i) & 1u) << (8 * i);
            if (a.mask_b) word |= bytes01(*reinterpret_cast<const uint64_t*>(a.mask_b + p0));
        } else if (square && b_same && window3_any(a.k, a.stride, a.pad, a.up, a.h, a.w, a.oh, a.ow)) {
            const Spans3 sp = window3_spans(a.mask_in, p0, a.w, a.out_pixels);
            int x = (int)(p0 % a.w);
            int y = (int)((p0 / a.w) % a.h);
            for (int i = 0; i < kPxPerThread && p0 + i < a.out_pixels; ++i) {
                if (window3_taps(sp, i, x, y, a.h, a.w)) word |= (uint64_t)1 << (8 * i);
                if (++x == a.w) { x = 0; if (++y == a.h) y = 0; }
            }
            if (a.mask_b) {
                if (p0 + kPxPerThread <= a.out_pixels) word |= bytes01(*reinterpret_cast<const uint64_t*>(a.mask_b + p0));
                else for (int i = 0; p0 + i < a.out_pixels; ++i) word |= (uint64_t)(a.mask_b[p0 + i] ? 1 : 0) << (8 * i);
            }
        } else if (square && a.up == 1 && (a.k == 3 || a.k == 1)) {
            // strided / unpadded 3x3 and 1x1 windows: all taps of the 8 pixels in one batch of loads
            uint32_t taps[kPxPerThread];
            if (a.k == 3) window_taps8<3>(a.mask_in, p0, a.out_pixels, a.h, a.w, a.oh, a.ow, a.stride, a.pad, taps);
            else window_taps8<1>(a.mask_in, p0, a.out_pixels, a.h, a.w, a.oh, a.ow, a.stride, a.pad, taps);
            uint8_t fb[kPxPerThread];
#pragma unroll
            for (int i = 0; i < kPxPerThread; ++i) {
                const int64_t q = p0 + i < a.out_pixels ? p0 + i : p0;
                fb[i] = (a.mask_b && mask_b_flag(a.mask_b, q, a.b_stride, a.b_h, a.b_w, a.oh, a.ow)) ? 1 : 0;
            }
#pragma unroll
            for (int i = 0; i < kPxPerThread; ++i)
                if (p0 + i < a.out_pixels && (taps[i] || fb[i])) word |= (uint64_t)1 << (8 * i);
        } else if (a.up > 1 && !a.bilinear && a.mask_b == nullptr) {
            // nearest upsampling: one source flag per pixel, the 8 loads in one batch
            int ox = (int)(p0 % a.ow);
            const int64_t t = p0 / a.ow;
            int oy = (int)(t % a.oh);
            int64_t n = t / a.oh;
            uint8_t f[kPxPerThread];
#pragma unroll
            for (int i = 0; i < kPxPerThread; ++i) {
                const bool live = p0 + i < a.out_pixels;
                f[i] = a.mask_in[live ? (n * a.h + oy / a.up) * a.w + ox / a.up : 0];
                if (!live) f[i] = 0;
                if (++ox == a.ow) { ox = 0; if (++oy == a.oh) { oy = 0; ++n; } }
            }
#pragma unroll
            for (int i = 0; i < kPxPerThread; ++i)
                if (f[i]) word |= (uint64_t)1 << (8 * i);
        } else {
            int ox = (int)(p0 % a.ow);
            int64_t t = p0 / a.ow;
            int oy = (int)(t % a.oh);
            int64_t n = t / a.oh;
            for (int i = 0; i < kPxPerThread && p0 + i < a.out_pixels; ++i) {
                uint8_t f = 0;
                if (a.up > 1 && a.bilinear) {
                    const BilinTaps ty = bilin_taps(oy, a.up, a.h), tx = bilin_taps(ox, a.up, a.w);
                    const uint8_t* r0 = a.mask_in + (n * a.h + ty.i0) * a.w;
                    const uint8_t* r1 = a.mask_in + (n * a.h + ty.i1) * a.w;
                    f = r0[tx.i0] | r0[tx.i1] | r1[tx.i0] | r1[tx.i1];
                } else if (a.up > 1) {
                    f = a.mask_in[(n * a.h + oy / a.up) * a.w + ox / a.up];
                } else {
                    for (int ky = 0; ky < a.k; ++ky) {
                        const int iy = oy * a.stride - a.pad + ky;
                        if (iy < 0 || iy >= a.h) continue;
                        const uint8_t* row = a.mask_in + (n * a.h + iy) * a.w;
                        for (int kx = 0; kx < a.kw; ++kx) {
                            const int ix = ox * a.stride - a.pad_w + kx;
                            if (ix >= 0 && ix < a.w) f |= row[ix];
                        }
                    }
                }
                if (a.mask_b && mask_b_flag(a.mask_b, p0 + i, a.b_stride, a.b_h, a.b_w, a.oh, a.ow)) f |= 1;
                word |= (uint64_t)(f ? 1 : 0) << (8 * i);
                if (++ox == a.ow) { ox = 0; if (++oy == a.oh) { oy = 0; ++n; } }
            }
        }
        if constexpr (STORE) {
            if (p0 + kPxPerThread <= a.out_pixels) {
                *reinterpret_cast<uint64_t*>(a.mask_out + p0) = word;
            } else {
                for (int i = 0; p0 + i < a.out_pixels; ++i) a.mask_out[p0 + i] = (uint8_t)((word >> (8 * i)) & 1);
            }
        }
    }
    return word;
}

__global__ __launch_bounds__(kMaskThreads) void mask_pass_kernel(MaskKernelArgs a) {
    __shared__ int s_red[kMaskThreads / kWave];
    const int64_t p0 = (int64_t)blockIdx.x * kChunk + (int64_t)threadIdx.x * kPxPerThread;
    const uint64_t word = mask_word<true>(a, p0);
    const int total = block_sum(__popcll(word), s_red);
    if (threadIdx.x == 0) {
        a.chunk_counts[blockIdx.x] = total;
        if (blockIdx.x == 0 && a.zero_count) *a.zero_count = 0;
    }
}

struct EmitArgs {
    const uint8_t* mask;
    const int32_t* chunk_counts;
    int32_t* idx_out;
    int32_t* count_out;
    int64_t pixels;
    const uint8_t* tap_mask;      // input mask the window taps are tested against (with taps_out)
    const uint8_t* mask_b;        // second mask: bit 30 of the tap word
    uint32_t* taps_out;
    int h, w, oh, ow, k, stride, pad;
    int b_stride, b_h, b_w;
};

// The three rows of input flags that the tap words of pixels p0 .. p0+7 are cut from (3x3 windows on rows a
// multiple of 8 wide).  They depend on p0 alone, so they are requested before the scan that fixes the list
// positions instead of after it: one round trip to memory less on the kernel's critical path.
struct EmitRows {
    int mode;                     // 0: none (taps are tested one by one), 1: 3x3/1/1 on rows a multiple of 8 wide,
                                  // 2: 3x3/1/1 on any width, 3: tap words of the 8 pixels (3x3 or 1x1, any stride)
    uint32_t rows[3];
};
__device__ __forceinline__ EmitRows emit_rows(const EmitArgs& a, int64_t p0) {
    EmitRows r;
    r.mode = 0;
    r.rows[0] = r.rows[1] = r.rows[2] = 0;
    if (a.taps_out == nullptr || p0 >= a.pixels) return r;
    if (window3_fast(a.k, a.stride, a.pad, 1, a.h, a.w, a.oh, a.ow) && p0 + kPxPerThread <= a.pixels) {
        r.mode = 1;
        const int x0 = (int)(p0 % a.w);
        const int64_t t = p0 / a.w;
        const int y = (int)(t % a.h);
        const int64_t n = t / a.h;
        for (int i = 0; i < 3; ++i) r.rows[i] = row_flags10(a.tap_mask, n, y + i - 1, x0, a.h, a.w);
    } else if (window3_any(a.k, a.stride, a.pad, 1, a.h, a.w, a.oh, a.ow)) {
        r.mode = 2;
        const Spans3 sp = window3_spans(a.tap_mask, p0, a.w, a.pixels);
        for (int i = 0; i < 3; ++i) r.rows[i] = sp.row[i];
    } else if (a.k == 3 || a.k == 1) {
        // any stride / padding: the tap words of all 8 pixels, 9 bits each, three to a word
        r.mode = 3;
        uint32_t taps[kPxPerThread];
        if (a.k == 3) window_taps8<3>(a.tap_mask, p0, a.pixels, a.h, a.w, a.oh, a.ow, a.stride, a.pad, taps);
        else window_taps8<1>(a.tap_mask, p0, a.pixels, a.h, a.w, a.oh, a.ow, a.stride, a.pad, taps);
#pragma unroll
        for (int i = 0; i < kPxPerThread; ++i) r.rows[i / 3] |= taps[i] << (9 * (i % 3));
    }
    return r;
}

// List entries (and tap words) of the flagged pixels among p0 .. p0+7, written from position `pos` on.
__device__ __forceinline__ void emit_entries(const EmitArgs& a, int64_t p0, uint64_t word, int pos, const EmitRows& er) {
    if (a.taps_out == nullptr) {
        for (int i = 0; i < kPxPerThread; ++i)
            if ((word >> (8 * i)) & 1) a.idx_out[pos++] = (int32_t)(p0 + i);
        return;
    }
    if (word == 0) return;
    if (er.mode == 2) {
        const Spans3 sp{{er.rows[0], er.rows[1], er.rows[2]}};
        int x = (int)(p0 % a.w);
        int y = (int)((p0 / a.w) % a.h);
        for (int i = 0; i < kPxPerThread; ++i) {
            if ((word >> (8 * i)) & 1) {
                a.idx_out[pos] = (int32_t)(p0 + i);
                uint32_t taps = window3_taps(sp, i, x, y, a.h, a.w);
                if (a.mask_b && mask_b_flag(a.mask_b, p0 + i, a.b_stride, a.b_h, a.b_w, a.oh, a.ow)) taps |= 1u << 30;
                a.taps_out[pos] = taps;
                ++pos;
            }
            if (++x == a.w) { x = 0; if (++y == a.h) y = 0; }
        }
        return;
    }
    if (er.mode == 3) {
        for (int i = 0; i < kPxPerThread; ++i) {
            if ((word >> (8 * i)) & 1) {
                a.idx_out[pos] = (int32_t)(p0 + i);
                uint32_t taps = (er.rows[i / 3] >> (9 * (i % 3))) & 0x1ffu;
                if (a.mask_b && mask_b_flag(a.mask_b, p0 + i, a.b_stride, a.b_h, a.b_w, a.oh, a.ow)) taps |= 1u << 30;
                a.taps_out[pos] = taps;
                ++pos;
            }
        }
        return;
    }
    if (er.mode == 1) {
        for (int i = 0; i < kPxPerThread; ++i) {
            if ((word >> (8 * i)) & 1) {
                a.idx_out[pos] = (int32_t)(p0 + i);
                uint32_t taps = ((er.rows[0] >> i) & 7u) | (((er.rows[1] >> i) & 7u) << 3) | (((er.rows[2] >> i) & 7u) << 6);
                if (a.mask_b && mask_b_flag(a.mask_b, p0 + i, a.b_stride, a.b_h, a.b_w, a.oh, a.ow)) taps |= 1u << 30;
                a.taps_out[pos] = taps;
                ++pos;
            }
        }
        return;
    }
    int ox = (int)(p0 % a.ow);
    int64_t t = p0 / a.ow;
    int oy = (int)(t % a.oh);
    int64_t n = t / a.oh;
    for (int i = 0; i < kPxPerThread; ++i) {
        if ((word >> (8 * i)) & 1) {
            uint32_t taps = 0;
            for (int ky = 0, tap = 0; ky < a.k; ++ky) {
                const int iy = oy * a.stride - a.pad + ky;
                for (int kx = 0; kx < a.k; ++kx, ++tap) {
                    const int ix = ox * a.stride - a.pad + kx;
                    if (iy >= 0 && iy < a.h && ix >= 0 && ix < a.w && a.tap_mask[(n * a.h + iy) * a.w + ix]) taps |= 1u << tap;
                }
            }
            if (a.mask_b && mask_b_flag(a.mask_b, p0 + i, a.b_stride, a.b_h, a.b_w, a.oh, a.ow)) taps |= 1u << 30;
            a.idx_out[pos] = (int32_t)(p0 + i);
            a.taps_out[pos] = taps;
            ++pos;
        }
        if (++ox == a.ow) { ox = 0; if (++oy == a.oh) { oy = 0; ++n; } }
    }
}


__global__ __launch_bounds__(kMaskThreads) void emit_kernel(EmitArgs a) {
    __shared__ int s_red[kMaskThreads / kWave];
    const int chunk = blockIdx.x;
    const bool last = chunk == (int)gridDim.x - 1;
    // every load the block needs is requested up front: the counts of the chunks before it, its own flags and
    // the rows its tap words come from
    int part = 0;
    for (int i = threadIdx.x; i < chunk; i += kMaskThreads) part += a.chunk_counts[i];
    const int64_t p0 = (int64_t)chunk * kChunk + (int64_t)threadIdx.x * kPxPerThread;
    uint64_t word = 0;
    if (p0 + kPxPerThread <= a.pixels) {
        word = *reinterpret_cast<const uint64_t*>(a.mask + p0);
    } else {
        for (int i = 0; p0 + i < a.pixels; ++i) word |= (uint64_t)(a.mask[p0 + i] ? 1 : 0) << (8 * i);
    }
    const EmitRows er = emit_rows(a, p0);
    const int prefix = block_sum(part, s_red);
    int total;
    const int pos = prefix + block_exclusive_scan(__popcll(word), s_red, &total);
    if (last && threadIdx.x == 0) *a.count_out = prefix + total;
    emit_entries(a, p0, word, pos, er);
}

// ---- mask pass and list emission in one launch (maps of one chunk) -----------------------------------
// A map of at most kChunk pixels is one workgroup's work: flags, scan and list in one launch.  (Written for any
// number of chunks -- the workgroup of chunk c recomputes the flags of the earlier chunks instead of waiting for
// their counts -- but measured slower than two launches from the second chunk on, as was a variant in which
// workgroups published their counts and waited for the earlier ones with device-scope atomics: 20 us against 12
// on 1 M pixels, 22 against 11 on 55 K.  So was a single workgroup of 1024 threads that owns a whole map of up
// to 16 K pixels, two words of 8 pixels per thread: its chain of dependent memory round trips is longer than two
// short launches back to back -- an 84-layer network on small maps went from 2.10 to 2.48 ms per step.)
constexpr int kFusedMaxChunks = 1;

__global__ __launch_bounds__(kMaskThreads) void mask_emit_kernel(MaskKernelArgs a, EmitArgs e) {
    __shared__ int s_red[kMaskThreads / kWave];
    const int chunk = blockIdx.x;
    const bool last = chunk == (int)gridDim.x - 1;
    int part = 0;
    for (int cc = 0; cc < chunk; ++cc)
        part += __popcll(mask_word<false>(a, (int64_t)cc * kChunk + (int64_t)threadIdx.x * kPxPerThread));
    const int64_t p0 = (int64_t)chunk * kChunk + (int64_t)threadIdx.x * kPxPerThread;
    const uint64_t word = mask_word<true>(a, p0);
    const EmitRows er = emit_rows(e, p0);
    const int prefix = block_sum(part, s_red);
    int total;
    const int loc = block_exclusive_scan(__popcll(word), s_red, &total);
    if (threadIdx.x == 0) {
        if (chunk == 0 && a.zero_count) *a.zero_count = 0;
        if (last) *e.count_out = prefix + total;
    }
    if (total != 0) emit_entries(e, p0, word, prefix + loc, er);
}

// The pass on explicit scratch memory: ws.chunk_counts (one int per chunk; every entry the list emission reads
// has been written by the mask pass of the same call, nothing has to start at zero) and ws.scratch_mask (the
// output mask when the caller does not want one).
static dcnn_status mask_compact_on(dcnn_ctx* ctx, const MaskPassArgs& m, const Workspace& ws) {
    const int64_t out_pixels = (int64_t)m.n * m.oh * m.ow;
    dcnn_status st = DCNN_OK;
    const int nchunks = (int)cdiv(out_pixels, kChunk);
    const uint8_t* emit_mask = m.mask_in;
    // one launch for small maps; large maps keep the two passes
    const bool fused = !m.emit_only && m.idx_out != nullptr && nchunks <= kFusedMaxChunks;
    MaskKernelArgs a{};
    if (!m.emit_only) {
        a.mask_in = m.mask_in; a.mask_b = m.mask_b;
        a.mask_out = m.mask_out ? m.mask_out : ws.scratch_mask;
        a.chunk_counts = ws.chunk_counts;
        a.zero_count = m.zero_count;
        a.out_pixels = out_pixels;
        a.n = m.n; a.h = m.h; a.w = m.w; a.oh = m.oh; a.ow = m.ow;
        a.k = m.k; a.stride = m.stride; a.pad = m.pad;
        a.up = m.up > 1 ? m.up : 1;
        a.bilinear = m.bilinear;
        a.b_stride = m.b_stride; a.b_h = m.b_h; a.b_w = m.b_w;
        a.kw = m.kw > 0 ? m.kw : m.k; a.pad_w = m.kw > 0 ? m.pad_w : m.pad;
        if (!fused) {
            hipLaunchKernelGGL(mask_pass_kernel, dim3(nchunks), dim3(kMaskThreads), 0, ctx->stream, a);
            st = check_hip(ctx, hipGetLastError(), "mask_pass_kernel launch");
            if (st != DCNN_OK) return st;
        }
        emit_mask = a.mask_out;
    }
    if (m.idx_out == nullptr) return DCNN_OK;
    EmitArgs e{emit_mask, ws.chunk_counts, m.idx_out, m.count_out, out_pixels};
    e.tap_mask = m.mask_in; e.taps_out = (m.emit_only || m.up > 1 || m.k * m.k > 25 || m.kw > 0) ? nullptr : m.taps_out;
    e.h = m.h; e.w = m.w; e.oh = m.oh; e.ow = m.ow; e.k = m.k; e.stride = m.stride; e.pad = m.pad;
    e.mask_b = m.mask_b; e.b_stride = m.b_stride; e.b_h = m.b_h; e.b_w = m.b_w;
    if (fused) {
        hipLaunchKernelGGL(mask_emit_kernel, dim3(nchunks), dim3(kMaskThreads), 0, ctx->stream, a, e);
        return check_hip(ctx, hipGetLastError(), "mask_emit_kernel launch");
    }
    hipLaunchKernelGGL(emit_kernel, dim3(nchunks), dim3(kMaskThreads), 0, ctx->stream, e);
    return check_hip(ctx, hipGetLastError(), "emit_kernel launch");
}

dcnn_status launch_mask_compact(dcnn_ctx* ctx, const MaskPassArgs& m) {
    const int64_t out_pixels = (int64_t)m.n * m.oh * m.ow;
    if (out_pixels <= 0 || out_pixels > INT32_MAX) return fail(ctx, DCNN_ESHAPE, "mask pass: bad pixel count");
    Workspace ws;
    dcnn_status st = workspace_view(ctx, out_pixels, &ws);
    if (st != DCNN_OK) return st;
    return mask_compact_on(ctx, m, ws);
}

// ---- statistics: x^T rows read / written by a step (see launch_xt_row_count) --------------------------
__global__ __launch_bounds__(kMaskThreads) void xt_row_count_kernel(int phase, ListArgs l, const uint8_t* flags, uint8_t* before,
                                                                    unsigned long long* io) {
    __shared__ int s_red[kMaskThreads / kWave];
    const int64_t count = list_count(l);
    int local = 0;
    for (int64_t j = (int64_t)blockIdx.x * kMaskThreads + threadIdx.x; j < count; j += (int64_t)gridDim.x * kMaskThreads) {
        const int now = flags[list_pixel(l.list, j, count)] != 0;
        if (phase == 0) { before[j] = (uint8_t)now; local += now; }
        else local += (now | before[j]) ? 1 : 0;
    }
    const int total = block_sum(local, s_red);
    if (threadIdx.x == 0 && total) atomicAdd(io + phase, (unsigned long long)total);
}

// ---- statistics: flagged pixels of a mask whose producer keeps no count -------------------------------------
__global__ __launch_bounds__(256) void mask_sum_kernel(const uint8_t* mask, int64_t pixels, int32_t* out) {
    int mine = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < pixels; i += (int64_t)gridDim.x * blockDim.x)
        mine += mask[i] != 0;
    for (int m = kWave >> 1; m >= 1; m >>= 1) mine += __shfl_xor(mine, m, kWave);
    if (threadIdx.x % kWave == 0 && mine) atomicAdd(out, mine);
}

dcnn_status launch_mask_sum(dcnn_ctx* ctx, const uint8_t* mask, int64_t pixels, int32_t* out) {
    dcnn_status st = launch_fill_i32(ctx, out, 0, 1);
    if (st != DCNN_OK || pixels <= 0) return st;
    const int64_t want = (pixels + 255) / 256;
    const int grid = (int)(want < 1024 ? want : 1024);
    hipLaunchKernelGGL(mask_sum_kernel, dim3(grid), dim3(256), 0, ctx->stream, mask, pixels, out);
    return check_hip(ctx, hipGetLastError(), "mask_sum_kernel launch");
}

dcnn_status launch_xt_row_count(dcnn_ctx* ctx, int phase, const ListArgs& l, const uint8_t* flags, uint8_t* before,
                                unsigned long long* io) {
    const int64_t want = cdiv(l.max_count > 0 ? l.max_count : 1, kMaskThreads);
    const int grid = (int)(want < 1024 ? want : 1024);
    hipLaunchKernelGGL(xt_row_count_kernel, dim3(grid), dim3(kMaskThreads), 0, ctx->stream, phase, l, flags, before, io);
    return check_hip(ctx, hipGetLastError(), "xt_row_count_kernel launch");
}

// ---- library-owned scratch for the entry point that allocates nothing ------------------------------
// One array per GPU the library runs on, held until the process ends: the chunk counts of the largest
// accepted map, followed by a mask for callers that only want the list.
constexpr int64_t kStaticMaxPixels = 4ll << 20;                               // 4 Mi output pixels per call
constexpr size_t kStaticCountBytes = (size_t)(kStaticMaxPixels / kChunk) * sizeof(int32_t);   // 8 KiB
constexpr size_t kStaticScratchBytes = kStaticCountBytes + (size_t)kStaticMaxPixels;          // + 4 MiB of mask
static_assert(kStaticCountBytes % kAlign == 0, "the mask part starts aligned");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of each GPU's copy of `scratch` (the array's name is only a host-side handle for
// hipGetSymbolAddress; kernels and copies get the resolved pointer).
constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices];

hipError_t static_scratch_setup(int dev) {
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (g_scratch_ptr[dev]) return hipSuccess;
    void* p = nullptr;
    const hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));       // resolves for the CURRENT device
    if (err != hipSuccess) return err;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    return hipSuccess;
}

// ---- list-space compaction ---------------------------------------------------------------------
constexpr int kSubTilesPerWg = kMaskThreads / 4;              // 64 tiles (2048 entries) per workgroup

__global__ __launch_bounds__(kMaskThreads) void emit_sublist_kernel(const int32_t* list, const int32_t* count,
                                                                    const uint32_t* surv, int32_t* idx_out,
                                                                    int32_t* count_out) {
    __shared__ int s_red[kMaskThreads / kWave];
    const int64_t n = *count;
    const int64_t ntiles = (n + kTile - 1) / kTile;
    const int64_t nwg = (ntiles + kSubTilesPerWg - 1) / kSubTilesPerWg;
    if (n == 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *count_out = 0;
        return;
    }
    if ((int64_t)blockIdx.x >= nwg) return;
    const int64_t first_tile = (int64_t)blockIdx.x * kSubTilesPerWg;
    int part = 0;
    for (int64_t i = threadIdx.x; i < first_tile; i += kMaskThreads) part += __popc(surv[i]);
    const int prefix = block_sum(part, s_red);
    const int64_t tile = first_tile + threadIdx.x / 4;
    const int quarter = threadIdx.x % 4;
    uint32_t bits = 0;
    if (tile < ntiles) bits = (surv[tile] >> (8 * quarter)) & 0xffu;
    int total;
    int pos = prefix + block_exclusive_scan(__popc(bits), s_red, &total);
    if ((int64_t)blockIdx.x == nwg - 1 && threadIdx.x == 0) *count_out = prefix + total;
    const int64_t j0 = tile * kTile + 8 * quarter;
    for (int i = 0; i < 8; ++i)
        if ((bits >> i) & 1) idx_out[pos++] = list ? list[j0 + i] : (int32_t)(j0 + i);
}

dcnn_status launch_emit_sublist(dcnn_ctx* ctx, const int32_t* list, const int32_t* count, int64_t max_count,
                                const uint32_t* surv, int32_t* idx_out, int32_t* count_out) {
    const int grid = (int)cdiv(cdiv(max_count > 0 ? max_count : 1, kTile), kSubTilesPerWg);
    hipLaunchKernelGGL(emit_sublist_kernel, dim3(grid), dim3(kMaskThreads), 0, ctx->stream, list, count, surv,
                       idx_out, count_out);
    return check_hip(ctx, hipGetLastError(), "emit_sublist_kernel launch");
}

}  // namespace dcnn

using namespace dcnn;

static dcnn_status mask_compact_args(dcnn_ctx* ctx, const char* who, const uint8_t* mask_in_dev, int32_t n, int32_t h, int32_t w,
                                     int32_t k, int32_t stride, int32_t pad, const uint8_t* mask_b_dev, uint8_t* mask_out_dev,
                                     int32_t* idx_out_dev, int32_t* count_out_dev, MaskPassArgs* out) {
    if (!mask_in_dev || !idx_out_dev || !count_out_dev) return fail(ctx, DCNN_EINVAL, "%s: null pointer", who);
    if (n < 1 || h < 1 || w < 1 || k < 1 || k > 15 || stride < 1 || pad < 0 || pad >= k)
        return fail(ctx, DCNN_EINVAL, "%s: bad geometry n=%d h=%d w=%d k=%d stride=%d pad=%d", who, n, h, w, k, stride, pad);
    if (h + 2 * pad < k || w + 2 * pad < k) return fail(ctx, DCNN_ESHAPE, "%s: window larger than the map", who);
    MaskPassArgs m{};
    m.mask_in = mask_in_dev; m.mask_b = mask_b_dev; m.mask_out = mask_out_dev;
    m.idx_out = idx_out_dev; m.count_out = count_out_dev;
    m.n = n; m.h = h; m.w = w;
    m.oh = (h + 2 * pad - k) / stride + 1;
    m.ow = (w + 2 * pad - k) / stride + 1;
    m.k = k; m.stride = stride; m.pad = pad; m.up = 1; m.emit_only = 0;
    *out = m;
    return DCNN_OK;
}

extern "C" {

dcnn_status dcnn_mask_compact(dcnn_ctx* ctx, const uint8_t* mask_in_dev, int32_t n, int32_t h, int32_t w, int32_t k,
                              int32_t stride, int32_t pad, const uint8_t* mask_b_dev, uint8_t* mask_out_dev,
                              int32_t* idx_out_dev, int32_t* count_out_dev) {
    if (!ctx) return DCNN_EINVAL;
    MaskPassArgs m;
    dcnn_status st = mask_compact_args(ctx, "mask_compact", mask_in_dev, n, h, w, k, stride, pad, mask_b_dev, mask_out_dev,
                                       idx_out_dev, count_out_dev, &m);
    if (st != DCNN_OK) return st;
    return launch_mask_compact(ctx, m);
}

dcnn_status dcnn_mask_compact_static(dcnn_ctx* ctx, const uint8_t* mask_in_dev, int32_t n, int32_t h, int32_t w, int32_t k,
                                     int32_t stride, int32_t pad, const uint8_t* mask_b_dev, uint8_t* mask_out_dev,
                                     int32_t* idx_out_dev, int32_t* count_out_dev) {
    if (!ctx) return DCNN_EINVAL;
    MaskPassArgs m;
    dcnn_status st = mask_compact_args(ctx, "mask_compact_static", mask_in_dev, n, h, w, k, stride, pad, mask_b_dev,
                                       mask_out_dev, idx_out_dev, count_out_dev, &m);
    if (st != DCNN_OK) return st;
    const int64_t out_pixels = (int64_t)m.n * m.oh * m.ow;
    if (out_pixels > kStaticMaxPixels)
        return fail(ctx, DCNN_ENOMEM, "mask_compact_static: %lld output pixels exceed the static scratch of %lld pixels; "
                    "use dcnn_mask_compact with a workspace", (long long)out_pixels, (long long)kStaticMaxPixels);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return fail(ctx, DCNN_ESTATE, "mask_compact_static: the context's device %d is not the current device", ctx->device);
    unsigned char* base = g_scratch_ptr[dev];          // resolved by dcnn_ctx_create on this device
    if (!base) return fail(ctx, DCNN_ESTATE, "mask_compact_static: the static scratch was not set up on device %d", dev);
    Workspace ws{};
    ws.chunk_counts = reinterpret_cast<int32_t*>(base);
    ws.scratch_mask = base + kStaticCountBytes;
    ws.max_pixels = kStaticMaxPixels;
    return mask_compact_on(ctx, m, ws);
}

}  // extern "C"
