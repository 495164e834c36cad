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

// ---- sparse-step tail with buffer addressing ---------------------------------------------------
// Activation + truncation (Eqs. 4-6) of one run of tile entries, for the sparse steps of layers whose channel
// count is a multiple of the vector width and whose tensors stay below 2 GiB.  Same arithmetic, rounding and
// decisions as act_trunc_tile; what differs is how memory is reached: every flag a load depends on has been
// fetched for the whole tile beforehand (one round trip, entry lane%32 per lane), and every load and store
// goes through a buffer descriptor with an out-of-range offset where a lane has nothing to do.  A batch of
// UB iterations therefore issues all its loads back to back and costs one round trip to memory.
//
// `Src` delivers the first delta stream: select(ub, ent) runs in wave-uniform control flow and picks the
// per-entry values of iteration ub (lane shuffles); issue(ub, v, c0, on, off) requests the values of the
// lane's vector v; finish(ub, v, c0) returns them, rounded to the storage type.
struct TailRsrc {
    __amdgpu_buffer_rsrc_t res, xA, xT, out, omask;
};

template <typename T, int V, int VPL, int UB, class Src>
__device__ __forceinline__ uint32_t sparse_tile_tail(const EpilogueArgs& e, const TailRsrc& rs, Src& src, int LP, int p_mine,
                                                    int rflag_mine, int ent_first, int ent_end, int nbatch, int lane) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr uint32_t ES = sizeof(T);
    const int PPI = kWave / LP;
    const int sub = lane % LP, grp = lane / LP;
    const int nvec = e.c / V;
    const uint32_t row_bytes = (uint32_t)e.c * ES;
    const bool stateful = e.act != DCNN_ACT_NONE;
    const bool has_res = e.res_data != nullptr;
    const float hi = act_hi(e.act);
    uint32_t bits = 0;
    for (int b = 0; b < nbatch; ++b) {
        int pix[UB];
        uint32_t off[UB][VPL];
        Raw rr[UB][VPL], ra[UB][VPL], rt[UB][VPL];
        // ---- phase 1: every load of the batch ----------------------------------------------------
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            const int ent = ent_first + (b * UB + ub) * PPI + grp;
            const int p_any = __shfl(p_mine, ent & (kTile - 1), kWave);
            const int rf = __shfl(rflag_mine, ent & (kTile - 1), kWave);
            src.select(ub, ent & (kTile - 1));
            const int p = ent < ent_end ? p_any : -1;
            pix[ub] = p;
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const int vi = sub + v * LP;
                const bool on = p >= 0 && vi < nvec;
                const int c0 = vi * V;
                const uint32_t o = on ? (uint32_t)p * row_bytes + (uint32_t)c0 * ES : kOob;
                off[ub][v] = o;
                src.issue(ub, v, c0, on, o);
                rr[ub][v] = ws_load16<Raw>(rs.res, rf ? o : kOob);          // empty descriptor without a second stream
                ra[ub][v] = ws_load16_nt<Raw>(rs.xA, o);                     // empty descriptors without an activation
                rt[ub][v] = ws_load16_nt<Raw>(rs.xT, o);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- phase 2: arithmetic, per-pixel maximum, decision, stores -----------------------------
#pragma unroll
        for (int ub = 0; ub < UB; ++ub) {
            Raw o_a[VPL], o_t[VPL], o_y[VPL], o_r[VPL];
            float u = 0.0f;
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const Raw d0 = src.finish(ub, v, (sub + v * LP) * V);
                o_r[v] = raw_zero<T, V>();
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    float d = raw_get<T, V>(d0, i);
                    if (has_res) d = round_store<T>(d + raw_get<T, V>(rr[ub][v], i));
                    if (stateful) {
                        const float a = raw_get<T, V>(ra[ub][v], i), t = raw_get<T, V>(rt[ub][v], i);
                        const float sum = (a + t) + d;
                        const float dy = act_clamp(sum, hi) - act_clamp(a, hi);
                        u = fmaxf(u, fabsf(dy));
                        raw_set<T, V>(o_a[v], i, sum);
                        raw_set<T, V>(o_t[v], i, t + d);                       // x^T if the pixel is truncated
                        raw_set<T, V>(o_y[v], i, dy);
                        if (e.carry) raw_set<T, V>(o_r[v], i, round_residue<T>(sum));   // x^T if it is updated and keeps the residue
                    } else {
                        raw_set<T, V>(o_y[v], i, d);
                    }
                }
            }
            bool upd = true;
            if (stateful) {
                for (int m = LP >> 1; m >= 1; m >>= 1) u = fmaxf(u, __shfl_xor(u, m, kWave));
                upd = u >= e.eps;
            }
#pragma unroll
            for (int v = 0; v < VPL; ++v) {
                const uint32_t o = off[ub][v];
                if (stateful) {
                    const uint32_t o_upd = upd ? o : kOob;
                    ws_store16_nt<Raw>(rs.xA, o_upd, o_a[v]);
                    // (an x^T that already is all zero bits is not rewritten by an update that leaves zeros)
                    ws_store16_nt<Raw>(rs.xT, (upd && all_bits_zero(rt[ub][v]) && all_bits_zero(o_r[v])) ? kOob : o, upd ? o_r[v] : o_t[v]);
                    ws_store16<Raw>(rs.out, o_upd, o_y[v]);
                } else {
                    ws_store16<Raw>(rs.out, o, o_y[v]);
                }
            }
            const bool lead = pix[ub] >= 0 && sub == 0;
            if (stateful) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(upd ? 1 : 0), rs.omask, lead ? pix[ub] : (int)kOob, 0, 0);
            const int ent = ent_first + (b * UB + ub) * PPI + grp;
            if (lead && upd) bits |= 1u << (ent & (kTile - 1));
        }
    }
#pragma unroll
    for (int m = kWave >> 1; m >= 1; m >>= 1) bits |= __shfl_xor(bits, m, kWave);
    return bits;
}

// How the entries of a tile are spread over waves and batches for a pixel of `nvec` vectors.
struct TailShape {
    int lp;        // lanes per pixel
    int run;       // consecutive tile entries per wave (8, 16 or 32)
    int nbatch;    // batches of UB iterations per wave
};
static TailShape tail_shape(int nvec, int vpl, int ub) {
    TailShape s;
    int lp = 1;
    while (lp < (int)cdiv(nvec, vpl)) lp <<= 1;
    s.lp = lp < 2 ? 2 : (lp > kWave ? kWave : lp);
    const int per_batch = ub * (kWave / s.lp);                 // entries one batch covers
    s.run = per_batch < 8 ? 8 : (per_batch > kTile ? kTile : per_batch);
    s.nbatch = (int)cdiv(s.run, per_batch);
    return s;
}

__device__ __forceinline__ void store_survivors(uint32_t* surv, int64_t tile, int part, int parts, uint32_t bits) {
    if (parts == 1) surv[tile] = bits;
    else if (parts == 2) reinterpret_cast<uint16_t*>(surv)[tile * 2 + part] = (uint16_t)(bits >> (16 * part));
    else reinterpret_cast<uint8_t*>(surv)[tile * 4 + part] = (uint8_t)(bits >> (8 * part));
}

// Activation + truncation (+ add) of a sparse step: the first stream is a stored delta map.
template <typename T, int V, int VPL, int UB> struct ActSrc {
    typedef typename RawOf<T, V>::type Raw;
    __amdgpu_buffer_rsrc_t in;
    int flag_mine;                       // update flag of the first stream at entry lane%32
    int flag[UB];
    Raw d[UB][VPL];
    __device__ __forceinline__ void select(int ub, int ent) { flag[ub] = __shfl(flag_mine, ent, kWave); }
    __device__ __forceinline__ void issue(int ub, int v, int, bool, uint32_t o) { d[ub][v] = ws_load16<Raw>(in, flag[ub] ? o : kOob); }
    __device__ __forceinline__ Raw finish(int ub, int v, int) const { return d[ub][v]; }
};

template <typename T, int V, int VPL, int UB>
__global__ __launch_bounds__(kTileThreads) void act_sparse_kernel(ListArgs l, ActArgs a, EpilogueArgs e, TailShape shape,
                                                                   uint32_t map_bytes, uint32_t pixels) {
    clear_ahead(e);
    const int64_t count = list_count(l);
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    TailRsrc rs;
    rs.res = ws_rsrc(e.res_data, map_bytes); rs.xA = ws_rsrc(e.xA, map_bytes); rs.xT = ws_rsrc(e.xT, map_bytes);
    rs.out = ws_rsrc(e.out_data, map_bytes); rs.omask = ws_rsrc(e.out_mask, pixels);
    const __amdgpu_buffer_rsrc_t rs_rmask = ws_rsrc(e.res_mask, pixels), rs_imask = ws_rsrc(a.in_mask, pixels);
    ActSrc<T, V, VPL, UB> src;
    src.in = ws_rsrc(a.in_data, map_bytes);
    const int parts = kTile / shape.run;
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
        const int p_mine = (j / shape.run == part) ? list_pixel(l.list, base + j, count) : -1;
        const int p_off = p_mine >= 0 ? p_mine : (int)kOob;
        // a stream without a mask is flagged wherever the list points
        const int rflag = e.res_mask ? __builtin_amdgcn_raw_buffer_load_b8(rs_rmask, p_off, 0, 0) : 1;
        src.flag_mine = a.in_mask ? __builtin_amdgcn_raw_buffer_load_b8(rs_imask, p_off, 0, 0) : 1;
        const uint32_t bits = sparse_tile_tail<T, V, VPL, UB>(e, rs, src, shape.lp, p_mine, rflag, part * shape.run,
                                                              (part + 1) * shape.run, shape.nbatch, lane);
        if (e.surv) { if (lane == 0) store_survivors(e.surv, tile, part, parts, bits); }
        else survivors += __popc(bits);
    }
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

// ---- activation + truncation (+ add) of wide pixels on short lists -------------------------------------------
// A pixel of 1024 .. 2048 channels fills a whole wave, so act_sparse_kernel walks the 8 entries of a run one or
// two at a time: four dependent round trips to memory per run, on a handful of waves when the list holds a few
// hundred pixels (the deep stages of a residual backbone: 38 us for 264 pixels of 2048 channels).  Here the four
// waves of a workgroup split the CHANNELS of a run's pixels instead (one vector per lane and pixel), request all
// 8 pixels at once -- one round trip -- and agree on the per-pixel maximum through LDS.  Arithmetic, rounding and
// decisions are those of sparse_tile_tail (Section 3.1, Eqs. 4-6).  Channels a multiple of 4 vectors.
constexpr int kWideRun = 8;                                     // list entries per workgroup unit (a quarter tile)

template <typename T, int V, int VPW>
__global__ __launch_bounds__(kTileThreads) void act_wide_kernel(ListArgs l, ActArgs a, EpilogueArgs e, uint32_t map_bytes, uint32_t pixels) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr uint32_t ES = sizeof(T);
    __shared__ float s_max[2][kWideRun][kTileWaves];
    clear_ahead(e);
    const int64_t count = list_count(l);
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const __amdgpu_buffer_rsrc_t rs_in = ws_rsrc(a.in_data, map_bytes), rs_res = ws_rsrc(e.res_data, map_bytes);
    const __amdgpu_buffer_rsrc_t rs_xA = ws_rsrc(e.xA, map_bytes), rs_xT = ws_rsrc(e.xT, map_bytes);
    const __amdgpu_buffer_rsrc_t rs_out = ws_rsrc(e.out_data, map_bytes), rs_omask = ws_rsrc(e.out_mask, pixels);
    const __amdgpu_buffer_rsrc_t rs_rmask = ws_rsrc(e.res_mask, pixels), rs_imask = ws_rsrc(a.in_mask, pixels);
    const int quarter = e.c / kTileWaves;                      // channels per wave
    const int nvec_q = quarter / V;
    const uint32_t row_bytes = (uint32_t)e.c * ES;
    const bool stateful = e.act != DCNN_ACT_NONE;
    const bool has_res = e.res_data != nullptr;
    const float hi = act_hi(e.act);
    const int64_t ntiles = (count + kTile - 1) / kTile;
    const int64_t units = ntiles * (kTile / kWideRun);
    int survivors = 0;
    int parity = 0;
    for (int64_t unit = blockIdx.x; unit < units; unit += gridDim.x, parity ^= 1) {
        const int64_t tile = unit / (kTile / kWideRun);
        const int part = (int)(unit - tile * (kTile / kWideRun));
        const int64_t base = tile * kTile + part * kWideRun;
        // entry lane % 8 of the run: pixel and the update flags of both streams (one round trip for the run)
        const int p_mine = list_pixel(l.list, base + lane % kWideRun, count);
        const int p_off = p_mine >= 0 ? p_mine : (int)kOob;
        const int rflag_mine = e.res_mask ? __builtin_amdgcn_raw_buffer_load_b8(rs_rmask, p_off, 0, 0) : 1;
        const int iflag_mine = a.in_mask ? __builtin_amdgcn_raw_buffer_load_b8(rs_imask, p_off, 0, 0) : 1;
        int pix[kWideRun];
        uint32_t off[kWideRun][VPW];
        Raw rd[kWideRun][VPW], rr[kWideRun][VPW], ra[kWideRun][VPW], rt[kWideRun][VPW];
#pragma unroll
        for (int ub = 0; ub < kWideRun; ++ub) {
            const int p = __shfl(p_mine, ub, kWave);
            const int rf = __shfl(rflag_mine, ub, kWave), fi = __shfl(iflag_mine, ub, kWave);
            pix[ub] = p;
#pragma unroll
            for (int v = 0; v < VPW; ++v) {
                const int vi = lane + v * kWave;
                const bool on = p >= 0 && vi < nvec_q;
                const uint32_t o = on ? (uint32_t)p * row_bytes + (uint32_t)(wave * quarter + vi * V) * ES : kOob;
                off[ub][v] = o;
                rd[ub][v] = ws_load16<Raw>(rs_in, fi ? o : kOob);
                rr[ub][v] = ws_load16<Raw>(rs_res, rf ? o : kOob);           // empty descriptor without a second stream
                ra[ub][v] = ws_load16_nt<Raw>(rs_xA, o);                      // empty descriptors without an activation
                rt[ub][v] = ws_load16_nt<Raw>(rs_xT, o);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        Raw o_a[kWideRun][VPW], o_t[kWideRun][VPW], o_y[kWideRun][VPW];
        float umax[kWideRun];
#pragma unroll
        for (int ub = 0; ub < kWideRun; ++ub) {
            float u = 0.0f;
#pragma unroll
            for (int v = 0; v < VPW; ++v) {
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    float d = raw_get<T, V>(rd[ub][v], i);
                    if (has_res) d = round_store<T>(d + raw_get<T, V>(rr[ub][v], i));
                    if (stateful) {
                        const float xa = raw_get<T, V>(ra[ub][v], i), t = raw_get<T, V>(rt[ub][v], i);
                        const float sum = (xa + t) + d;
                        const float dy = act_clamp(sum, hi) - act_clamp(xa, hi);
                        u = fmaxf(u, fabsf(dy));
                        raw_set<T, V>(o_a[ub][v], i, sum);
                        // x^T afterwards: the truncated sum, or -- if the pixel updates and keeps it -- x^A's rounding residue
                        raw_set<T, V>(o_t[ub][v], i, t + d);
                        raw_set<T, V>(o_y[ub][v], i, dy);
                    } else {
                        raw_set<T, V>(o_y[ub][v], i, d);
                    }
                }
            }
            if (stateful) u = group_max(u, kWave);
            umax[ub] = u;
        }
        if (stateful) {
            if (lane == 0) {
#pragma unroll
                for (int ub = 0; ub < kWideRun; ++ub) s_max[parity][ub][wave] = umax[ub];
            }
            lds_block_sync();           // (one barrier per unit: the buffers alternate, so a wave that runs ahead writes the other one)
#pragma unroll
            for (int ub = 0; ub < kWideRun; ++ub) {
                float u = 0.0f;
#pragma unroll
                for (int q = 0; q < kTileWaves; ++q) u = fmaxf(u, s_max[parity][ub][q]);
                umax[ub] = u;
            }
        }
        uint32_t bits = 0;
#pragma unroll
        for (int ub = 0; ub < kWideRun; ++ub) {
            const bool upd = stateful ? (umax[ub] >= e.eps) : true;
#pragma unroll
            for (int v = 0; v < VPW; ++v) {
                const uint32_t o = off[ub][v];
                if (stateful) {
                    const uint32_t o_upd = upd ? o : kOob;
                    Raw keep = raw_zero<T, V>();
                    if (e.carry) {
#pragma unroll
                        for (int i = 0; i < V; ++i) {
                            float d = raw_get<T, V>(rd[ub][v], i);
                            if (has_res) d = round_store<T>(d + raw_get<T, V>(rr[ub][v], i));
                            const float sum = (raw_get<T, V>(ra[ub][v], i) + raw_get<T, V>(rt[ub][v], i)) + d;
                            raw_set<T, V>(keep, i, round_residue<T>(sum));
                        }
                    }
                    ws_store16_nt<Raw>(rs_xA, o_upd, o_a[ub][v]);
                    ws_store16_nt<Raw>(rs_xT, (upd && all_bits_zero(rt[ub][v]) && all_bits_zero(keep)) ? kOob : o, upd ? keep : o_t[ub][v]);
                    ws_store16<Raw>(rs_out, o_upd, o_y[ub][v]);
                } else {
                    ws_store16<Raw>(rs_out, o, o_y[ub][v]);
                }
            }
            const bool lead = pix[ub] >= 0 && lane == 0 && wave == 0;
            if (stateful) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(upd ? 1 : 0), rs_omask, lead ? pix[ub] : (int)kOob, 0, 0);
            if (pix[ub] >= 0 && upd) bits |= 1u << (part * kWideRun + ub);
        }
        if (wave == 0 && tile * kTile < count) {               // (a run past the end of the list still clears its byte)
            if (e.surv) { if (lane == 0) store_survivors(e.surv, tile, part, kTile / kWideRun, bits); }
            else survivors += __popc(bits);
        }
    }
    // one atomic per workgroup
    if (e.out_count && !e.surv && wave == 0 && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

// ---- activation + truncation (+ add) ----------------------------------------------------------
template <typename T, int V, int VPL>
__global__ __launch_bounds__(kTileThreads) void act_kernel(ListArgs l, ActArgs a, EpilogueArgs e, int init) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr int UB = (V * VPL >= 16) ? 2 : 4;
    clear_ahead(e);
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
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

template <typename T>
static dcnn_status launch_act_t(dcnn_ctx* ctx, bool init, const ListArgs& l, const ActArgs& a, const EpilogueArgs& e) {
    constexpr int VEC = Elem<T>::VEC;
    const bool vec = (e.c % VEC) == 0;
    const int nvec = vec ? e.c / VEC : e.c;
    const int vpl = (int)cdiv(nvec, kWave);
    // sparse steps over vector channels, tensors below 2 GiB: the buffer-addressed kernel
    const uint64_t map_bytes = (uint64_t)(l.max_count > 0 ? l.max_count : 0) * e.c * sizeof(T);
    // wide pixels on maps of at most 64 K pixels: the channels of a pixel are split over the waves of a workgroup
    if (!init && vec && nvec >= 2 * kWave && nvec % kTileWaves == 0 && nvec <= kWave * kTileWaves && map_bytes > 0 &&
        map_bytes <= kWsMaxBytes && l.max_count <= 65536) {
        const int64_t units = cdiv(l.max_count, kWideRun);
        const int64_t cap = (int64_t)ctx->num_cu * 8;
        const int wgrid = (int)(units < cap ? units : cap);
        const uint32_t mb = (uint32_t)map_bytes, px = (uint32_t)l.max_count;
        hipLaunchKernelGGL((act_wide_kernel<T, VEC, 1>), dim3(wgrid), dim3(kTileThreads), 0, ctx->stream, l, a, e, mb, px);
        return check_hip(ctx, hipGetLastError(), "act_wide_kernel launch");
    }
    if (!init && vec && vpl <= 4 && map_bytes > 0 && map_bytes <= kWsMaxBytes) {
        const int vpl_used = vpl <= 1 ? 1 : (vpl <= 2 ? 2 : 4);
        const int ub = vpl_used == 4 ? 2 : 4;
        const TailShape shape = tail_shape(nvec, vpl_used, ub);
        const int sgrid = list_grid(ctx, l.max_count, kTileWaves * shape.run, 8);
        const uint32_t mb = (uint32_t)map_bytes, px = (uint32_t)l.max_count;
#define DCNN_ACT_SPARSE(VPL, UB) hipLaunchKernelGGL((act_sparse_kernel<T, VEC, VPL, UB>), dim3(sgrid), dim3(kTileThreads), 0, ctx->stream, l, a, e, shape, mb, px)
        if (vpl_used == 1) DCNN_ACT_SPARSE(1, 4);
        else if (vpl_used == 2) DCNN_ACT_SPARSE(2, 4);
        else DCNN_ACT_SPARSE(4, 2);
#undef DCNN_ACT_SPARSE
        return check_hip(ctx, hipGetLastError(), "act_sparse_kernel launch");
    }
    const int grid = list_grid(ctx, l.max_count, kTileWaves * kTile, 8);
    dim3 g(grid), b(kTileThreads);
    const int ini = init ? 1 : 0;
#define DCNN_ACT_LAUNCH(V, VPL) hipLaunchKernelGGL((act_kernel<T, V, VPL>), g, b, 0, ctx->stream, l, a, e, ini)
    if (vec) {
        if (vpl <= 1) DCNN_ACT_LAUNCH(VEC, 1);
        else if (vpl <= 2) DCNN_ACT_LAUNCH(VEC, 2);
        else if (vpl <= 4) DCNN_ACT_LAUNCH(VEC, 4);
        else if (vpl <= 8 && sizeof(T) == 4) {
            if constexpr (sizeof(T) == 4) DCNN_ACT_LAUNCH(VEC, 8);     // (fp32 only: 2048 channels = 8 KB per pixel)
        }
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

// ---- depthwise convolution, sparse steps, 1x1 / 2x2 / 3x3 windows ------------------------------
// The first delta stream is formed on the fly: per tile entry a tap word (bit t: window tap t is inside
// the map and flagged) and the input pixel under tap (0,0) are computed by lane entry%32 up front; the taps
// of a pixel are then requested back to back, an unflagged or padded tap with an out-of-range offset.
// The [k][k][C] weights sit in LDS.
template <typename T, int V, int VPL, int UB, int KS> struct DwSrc {
    typedef typename RawOf<T, V>::type Raw;
    static constexpr int KK = KS * KS;
    __amdgpu_buffer_rsrc_t in;
    const T* w_lds;
    int C, w;                            // channels, input width
    uint32_t row_bytes;
    int word_mine, q_mine;               // of entry lane%32; q = input pixel under tap (0,0), possibly outside
    int word[UB], q[UB];
    Raw x[UB][VPL][KK];
    __device__ __forceinline__ void select(int ub, int ent) {
        word[ub] = __shfl(word_mine, ent, kWave);
        q[ub] = __shfl(q_mine, ent, kWave);
    }
    __device__ __forceinline__ void issue(int ub, int v, int c0, bool on, uint32_t) {
#pragma unroll
        for (int t = 0; t < KK; ++t) {
            const bool ok = on && ((word[ub] >> t) & 1);
            const uint32_t o = ok ? (uint32_t)(q[ub] + (t / KS) * w + t % KS) * row_bytes + (uint32_t)c0 * (uint32_t)sizeof(T) : kOob;
            x[ub][v][t] = ws_load16<Raw>(in, o);
        }
    }
    __device__ __forceinline__ Raw finish(int ub, int v, int c0) const {
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;
        const int cw = c0 < C ? c0 : 0;                          // lanes without channels read weights of channel 0 (result unused)
#pragma unroll
        for (int t = 0; t < KK; ++t) {
            const Raw wv = raw_load<T, V>(w_lds + t * C + cw);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = fmaf(raw_get<T, V>(x[ub][v][t], i), raw_get<T, V>(wv, i), acc[i]);
        }
        Raw o;
#pragma unroll
        for (int i = 0; i < V; ++i) raw_set<T, V>(o, i, acc[i]);
        return o;
    }
};

template <typename T, int V, int VPL, int UB, int KS>
__global__ __launch_bounds__(kTileThreads) void dwconv_sparse_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, TailShape shape,
                                                                      uint32_t in_bytes, uint32_t in_pixels, uint32_t map_bytes,
                                                                      uint32_t pixels) {
    typedef typename RawOf<T, V>::type Raw;
    extern __shared__ __align__(16) unsigned char dw_smem[];
    T* w_lds = reinterpret_cast<T*>(dw_smem);
    {
        const Raw* wsrc = static_cast<const Raw*>(c.wpacked);      // [k][k][C], unpacked
        const int nv = KS * KS * e.c / V;
        for (int i = threadIdx.x; i < nv; i += kTileThreads) reinterpret_cast<Raw*>(w_lds)[i] = wsrc[i];
    }
    __syncthreads();
    const int64_t count = list_count(l);
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    TailRsrc rs;
    rs.res = ws_rsrc(e.res_data, map_bytes); rs.xA = ws_rsrc(e.xA, map_bytes); rs.xT = ws_rsrc(e.xT, map_bytes);
    rs.out = ws_rsrc(e.out_data, map_bytes); rs.omask = ws_rsrc(e.out_mask, pixels);
    const __amdgpu_buffer_rsrc_t rs_rmask = ws_rsrc(e.res_mask, pixels), rs_imask = ws_rsrc(c.in_mask, in_pixels);
    DwSrc<T, V, VPL, UB, KS> src;
    src.in = ws_rsrc(c.in_data, in_bytes);
    src.w_lds = w_lds; src.C = e.c; src.w = c.w; src.row_bytes = (uint32_t)e.c * (uint32_t)sizeof(T);
    const int parts = kTile / shape.run;
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
        const int p_mine = (j / shape.run == part) ? list_pixel(l.list, base + j, count) : -1;
        const int rflag = e.res_mask ? __builtin_amdgcn_raw_buffer_load_b8(rs_rmask, p_mine >= 0 ? p_mine : (int)kOob, 0, 0) : 1;
        // tap word of this lane's entry: all flags of the window requested together
        uint32_t word = 0;
        int q_first = 0;
        {
            const int pp = p_mine >= 0 ? p_mine : 0;
            const int ox = pp % c.ow;
            const int t = pp / c.ow;
            const int oy = t % c.oh, n = t / c.oh;
            const int iy0 = oy * c.stride - c.pad, ix0 = ox * c.stride - c.pad;
            q_first = (n * c.h + iy0) * c.w + ix0;
            uint32_t f[KS * KS];
#pragma unroll
            for (int t2 = 0; t2 < KS * KS; ++t2) {
                const int iy = iy0 + t2 / KS, ix = ix0 + t2 % KS;
                const bool ok = p_mine >= 0 && iy >= 0 && iy < c.h && ix >= 0 && ix < c.w;
                // without a mask (never in a sparse step of a network, possible through the layer interface) every
                // pixel inside the map counts as flagged
                f[t2] = ok ? (c.in_mask ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(rs_imask, q_first + (t2 / KS) * c.w + t2 % KS, 0, 0) : 1u) : 0u;
            }
#pragma unroll
            for (int t2 = 0; t2 < KS * KS; ++t2) word |= f[t2] ? (1u << t2) : 0u;
        }
        src.word_mine = (int)word; src.q_mine = q_first;
        const uint32_t bits = sparse_tile_tail<T, V, VPL, UB>(e, rs, src, shape.lp, p_mine, rflag, part * shape.run,
                                                              (part + 1) * shape.run, shape.nbatch, lane);
        if (e.surv) { if (lane == 0) store_survivors(e.surv, tile, part, parts, bits); }
        else survivors += __popc(bits);
    }
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

// ---- depthwise convolution: the first delta stream is formed on the fly ------------------------
// Work list = flagged OUTPUT pixels.  Every tap's update flag is checked before its values are
// read (unflagged memory is invalid), load and multiply are fused per pixel.
template <typename T, int V, int VPL>
__global__ __launch_bounds__(kTileThreads) void dwconv_kernel(ListArgs l, ConvArgs c, EpilogueArgs e, int init) {
    typedef typename RawOf<T, V>::type Raw;
    constexpr int UB = 2;
    const int64_t count = list_count(l);
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int C = e.c;
    const T* in = static_cast<const T*>(c.in_data);
    const T* wgt = static_cast<const T*>(c.wpacked);           // [k][k][C], unpacked
    // first frame: the bias joins the fp32 sum before its one rounding to the storage type
    const T* bias_f = init ? static_cast<const T*>(e.bias) : nullptr;
    auto dx = [&](int, int64_t p, int c0) -> Raw {
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
        if (bias_f) {
            const Raw bv = raw_load<T, V>(bias_f + c0);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += raw_get<T, V>(bv, i);
        }
        Raw o;
#pragma unroll
        for (int i = 0; i < V; ++i) raw_set<T, V>(o, i, acc[i]);
        return o;
    };
    int survivors = 0;
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
    // one atomic per wave: a counter bumped once per tile by every wave serialises in L2
    if (e.out_count && !e.surv && lane == 0 && survivors) atomicAdd(e.out_count, survivors);
}

template <typename T>
static dcnn_status launch_dwconv_t(dcnn_ctx* ctx, bool init, const ListArgs& l, const ConvArgs& c, const EpilogueArgs& e) {
    constexpr int VEC = Elem<T>::VEC;
    const bool vec = (e.c % VEC) == 0;
    const int nvec = vec ? e.c / VEC : e.c;
    const int vpl = (int)cdiv(nvec, kWave);
    // sparse steps, vector channels, windows up to 3x3, tensors below 2 GiB: the buffer-addressed kernel
    const uint64_t map_bytes = (uint64_t)(l.max_count > 0 ? l.max_count : 0) * e.c * sizeof(T);
    const uint64_t in_pixels = (uint64_t)c.n * c.h * c.w, in_bytes = in_pixels * e.c * sizeof(T);
    const size_t w_bytes = (size_t)c.k * c.k * e.c * sizeof(T);
    if (!init && vec && vpl <= 4 && c.k >= 1 && c.k <= 3 && map_bytes > 0 && map_bytes <= kWsMaxBytes && in_bytes <= kWsMaxBytes &&
        w_bytes <= 64 * 1024) {
        const int vpl_used = vpl <= 1 ? 1 : (vpl <= 2 ? 2 : 4);
        const int ub = 4 / vpl_used;
        const TailShape shape = tail_shape(nvec, vpl_used, ub);
        const int sgrid = list_grid(ctx, l.max_count, kTileWaves * shape.run, 8);
        const uint32_t ib = (uint32_t)in_bytes, ip = (uint32_t)in_pixels, mb = (uint32_t)map_bytes, px = (uint32_t)l.max_count;
#define DCNN_DW_SPARSE(VPL, UB, KS) hipLaunchKernelGGL((dwconv_sparse_kernel<T, VEC, VPL, UB, KS>), dim3(sgrid), dim3(kTileThreads), w_bytes, ctx->stream, l, c, e, shape, ib, ip, mb, px)
#define DCNN_DW_SPARSE_K(VPL, UB)                                                                                  \
    do {                                                                                                           \
        if (c.k == 3) DCNN_DW_SPARSE(VPL, UB, 3);                                                                  \
        else if (c.k == 2) DCNN_DW_SPARSE(VPL, UB, 2);                                                             \
        else DCNN_DW_SPARSE(VPL, UB, 1);                                                                           \
    } while (0)
        if (vpl_used == 1) DCNN_DW_SPARSE_K(1, 4);
        else if (vpl_used == 2) DCNN_DW_SPARSE_K(2, 2);
        else DCNN_DW_SPARSE_K(4, 1);
#undef DCNN_DW_SPARSE_K
#undef DCNN_DW_SPARSE
        return check_hip(ctx, hipGetLastError(), "dwconv_sparse_kernel launch");
    }
    const int grid = list_grid(ctx, l.max_count, kTileWaves * kTile, 8);
    dim3 g(grid), b(kTileThreads);
    const int ini = init ? 1 : 0;
#define DCNN_DW_LAUNCH(V, VPL) hipLaunchKernelGGL((dwconv_kernel<T, V, VPL>), g, b, 0, ctx->stream, l, c, e, ini)
    if (vec) {
        if (vpl <= 1) DCNN_DW_LAUNCH(VEC, 1);
        else if (vpl <= 2) DCNN_DW_LAUNCH(VEC, 2);
        else if (vpl <= 4) DCNN_DW_LAUNCH(VEC, 4);
        else return fail(ctx, DCNN_EUNSUPPORTED, "depthwise conv: %d channels not supported", e.c);
    } else {
        if (vpl <= 1) DCNN_DW_LAUNCH(1, 1);
        else if (vpl <= 2) DCNN_DW_LAUNCH(1, 2);
        else if (vpl <= 4) DCNN_DW_LAUNCH(1, 4);
        else return fail(ctx, DCNN_EUNSUPPORTED, "depthwise conv: %d channels not supported", e.c);
    }
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
                    rf[ub][v] = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(frame + p * C + vi * V));
                    rq[ub][v] = __builtin_nontemporal_load(reinterpret_cast<const Raw*>(P + p * C + vi * V));
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
                        __builtin_nontemporal_store(rf[ub][v], reinterpret_cast<Raw*>(P + p * C + vi * V));
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
        float x[V];
        if (a.bilinear) {
            // up to four sources; an unflagged one counts as zero and is not read
            const BilinTaps ty = bilin_taps(oy, a.factor, a.h), tx = bilin_taps(ox, a.factor, a.w);
#pragma unroll
            for (int i = 0; i < V; ++i) x[i] = 0.0f;
            for (int sy = 0; sy < 2; ++sy) {
                if (sy == 1 && ty.i1 == ty.i0) break;
                const float wy = sy ? ty.w1 : 1.0f - ty.w1;
                const int iy = sy ? ty.i1 : ty.i0;
                for (int sx = 0; sx < 2; ++sx) {
                    if (sx == 1 && tx.i1 == tx.i0) break;
                    const float wgt = wy * (sx ? tx.w1 : 1.0f - tx.w1);
                    const int64_t q = (n * a.h + iy) * a.w + (sx ? tx.i1 : tx.i0);
                    if (a.in_mask && a.in_mask[q] == 0) continue;
                    float s[V];
                    load_vec<T, V>(in + q * C + vi * V, s);
#pragma unroll
                    for (int i = 0; i < V; ++i) x[i] = fmaf(wgt, s[i], x[i]);
                }
            }
        } else {
            const int64_t q = (n * a.h + oy / a.factor) * a.w + ox / a.factor;
            load_vec<T, V>(in + q * C + vi * V, x);
        }
        store_vec<T, V>(out + p * C + vi * V, x);
    }
}

// Global average pooling: workgroup (j, cb) serves list entry j (a stream) and 64 * V channels; wave w sums the
// stream's flagged pixels p = w, w + 4, ... in ascending order, the four partial sums are added in a fixed order:
// the result does not depend on scheduling.
template <typename T, int V>
__global__ __launch_bounds__(256) void gavgpool_kernel(ListArgs l, GapArgs a) {
    __shared__ float s_part[3][kWave][V];
    const int64_t count = list_count(l);
    if ((int64_t)blockIdx.x >= count) return;                  // uniform for the block
    const int64_t n = l.list ? (int64_t)l.list[blockIdx.x] : (int64_t)blockIdx.x;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int c0 = (blockIdx.y * kWave + lane) * V;
    const bool on = c0 < a.c;
    const T* in = static_cast<const T*>(a.in_data) + n * (int64_t)a.hw * a.c;
    const uint8_t* mask = a.in_mask ? a.in_mask + n * (int64_t)a.hw : nullptr;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0f;
    for (int p = wave; p < a.hw; p += 4) {
        if (mask && mask[p] == 0) continue;                    // uniform for the wave
        if (on) {
            float s[V];
            load_vec<T, V>(in + (int64_t)p * a.c + c0, s);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += s[i];
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < V; ++i) s_part[wave - 1][lane][i] = acc[i];
    }
    __syncthreads();
    if (wave == 0 && on) {
        const float inv = 1.0f / (float)a.hw;
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = ((acc[i] + s_part[0][lane][i]) + (s_part[1][lane][i] + s_part[2][lane][i])) * inv;
        store_vec<T, V>(static_cast<T*>(a.out_data) + n * (int64_t)a.c + c0, acc);
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

dcnn_status launch_gavgpool(dcnn_ctx* ctx, int dtype, const ListArgs& l, const GapArgs& a) {
    if (l.max_count < 1 || l.max_count > 65535) return fail(ctx, DCNN_ESHAPE, "global average pooling: %lld streams", (long long)l.max_count);
    const bool f16v = dtype == DCNN_F16 && a.c % 8 == 0, f32v = dtype == DCNN_F32 && a.c % 4 == 0;
    const int v = f16v ? 8 : (f32v ? 4 : 1);
    const dim3 g((unsigned)l.max_count, (unsigned)cdiv(a.c, kWave * v)), b(256);
    if (f16v) hipLaunchKernelGGL((gavgpool_kernel<f16, 8>), g, b, 0, ctx->stream, l, a);
    else if (f32v) hipLaunchKernelGGL((gavgpool_kernel<float, 4>), g, b, 0, ctx->stream, l, a);
    else if (dtype == DCNN_F16) hipLaunchKernelGGL((gavgpool_kernel<f16, 1>), g, b, 0, ctx->stream, l, a);
    else hipLaunchKernelGGL((gavgpool_kernel<float, 1>), g, b, 0, ctx->stream, l, a);
    return check_hip(ctx, hipGetLastError(), "gavgpool_kernel launch");
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

// One wave per row: any non-zero bit among the row's bytes (rows are multiples of 4 bytes for the layers that use it).
__global__ __launch_bounds__(256) void row_flags_kernel(const uint32_t* data, uint8_t* flags, int64_t pixels, int words) {
    const int lane = threadIdx.x % kWave;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * blockDim.x / kWave;
    for (int64_t p = wave; p < pixels; p += nwaves) {
        uint32_t acc = 0;
        for (int i = lane; i < words; i += kWave) acc |= data[p * words + i];
        for (int m = kWave >> 1; m >= 1; m >>= 1) acc |= (uint32_t)__shfl_xor((int)acc, m, kWave);
        if (lane == 0) flags[p] = acc ? 1 : 0;
    }
}

dcnn_status launch_row_flags(dcnn_ctx* ctx, int dtype, const void* data, uint8_t* flags, int64_t pixels, int c) {
    const int64_t row_bytes = (int64_t)c * (int64_t)dtype_size(dtype);
    if (row_bytes % 4 != 0) return fail(ctx, DCNN_EINVAL, "row flags: rows of %lld bytes", (long long)row_bytes);
    const int64_t want = cdiv(pixels, 4);
    const int grid = (int)(want < (int64_t)ctx->num_cu * 8 ? (want > 0 ? want : 1) : (int64_t)ctx->num_cu * 8);
    hipLaunchKernelGGL(row_flags_kernel, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const uint32_t*>(data), flags,
                       pixels, (int)(row_bytes / 4));
    return check_hip(ctx, hipGetLastError(), "row_flags_kernel launch");
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
