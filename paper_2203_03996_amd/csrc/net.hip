// Network executor: a DAG of plain nodes is fused into layers (conv -> add -> activation chains
// become one launch sequence; a 1x1 projection convolution on the other arm of the add is pulled in
// as well), the layers' state is planned into one caller-provided arena, and
// a frame is run by stepping the layers in topological order on the context's stream.
#include <new>
#include <vector>

#include "layer.h"

using namespace dcnn;

namespace {

struct Node {
    dcnn_layer_desc d;
    std::vector<int> in;
    const void* w;
    const void* b;
    int oh, ow, oc;
    std::vector<int> consumers;
};

struct Planned {
    dcnn_layer_desc d;
    std::vector<int> in_nodes;      // producer node of each sparse input
    int out_node;                   // node whose output this layer produces
    const void* w;
    const void* b;
    const void* w2;                 // fused projection
    const void* b2;
    size_t state_off, state_bytes;
    dcnn_layer* layer;
    int lane = 0;                   // which of the network's streams runs the layer (0: the context's own)
    hipEvent_t done = nullptr;      // recorded behind the layer when a layer on another lane consumes its output
};

constexpr int kMaxLanes = 3;       // measured on the four-resolution network at 8 streams: 2 lanes 1.29 ms, 3 lanes 1.12, 4 lanes 1.24 (one: 1.62)

bool is_add(const dcnn_layer_desc& d) { return d.kind == DCNN_ACT && d.act == DCNN_ACT_NONE && d.n_in == 2; }
bool is_plain_act(const dcnn_layer_desc& d) { return d.kind == DCNN_ACT && d.act != DCNN_ACT_NONE && d.n_in == 1; }
bool is_conv(const dcnn_layer_desc& d) { return d.kind == DCNN_CONV || d.kind == DCNN_DWCONV; }

}  // namespace

struct dcnn_net {
    dcnn_ctx* ctx;
    int dtype, n, h, w, c;
    std::vector<Node> nodes;
    std::vector<Planned> plan;
    std::vector<int> layer_of_node;  // plan index producing a node's output, -1 if absorbed midway
    bool finalized = false, bound = false, inited = false;
    size_t arena_bytes = 0;
    // Independent branches on streams of their own (finalize flag bit 2): lane 0 is the caller's context; lanes 1..
    // are copies of it with a stream created here (default priority) and a workspace of their own inside the arena.
    int nlanes = 1;
    size_t lane_ws_off = 0, lane_ws_bytes = 0;
    std::vector<dcnn_ctx*> lane_ctx;        // [nlanes], lane_ctx[0] == ctx
    hipEvent_t ev_start = nullptr;
    std::vector<hipEvent_t> lane_end;       // [nlanes]
};

namespace {

void drop_lanes(dcnn_net* net) {
    for (auto& p : net->plan) {
        if (p.done) (void)hipEventDestroy(p.done);
        p.done = nullptr;
    }
    for (size_t l = 1; l < net->lane_ctx.size(); ++l) {
        if (net->lane_ctx[l]) {
            if (net->lane_ctx[l]->stream) (void)hipStreamDestroy(net->lane_ctx[l]->stream);
            delete net->lane_ctx[l];
        }
    }
    net->lane_ctx.clear();
    for (hipEvent_t e : net->lane_end)
        if (e) (void)hipEventDestroy(e);
    net->lane_end.clear();
    if (net->ev_start) (void)hipEventDestroy(net->ev_start);
    net->ev_start = nullptr;
}

// A failure on a lane leaves its text in that lane's context: hand it to the caller's.
dcnn_status lane_fail(dcnn_net* net, const Planned& p, dcnn_status st) {
    if (p.lane > 0 && p.lane < (int)net->lane_ctx.size() && net->lane_ctx[p.lane])
        memcpy(net->ctx->err, net->lane_ctx[p.lane]->err, sizeof(net->ctx->err));
    return st;
}

// Lanes other than 0 start behind everything the caller's stream holds so far.
dcnn_status lanes_begin(dcnn_net* net) {
    if (net->nlanes <= 1) return DCNN_OK;
    dcnn_ctx* ctx = net->ctx;
    dcnn_status st = check_hip(ctx, hipEventRecord(net->ev_start, ctx->stream), "hipEventRecord");
    for (int l = 1; l < net->nlanes && st == DCNN_OK; ++l)
        st = check_hip(ctx, hipStreamWaitEvent(net->lane_ctx[l]->stream, net->ev_start, 0), "hipStreamWaitEvent");
    return st;
}

// Before a layer runs: wait for the inputs that other lanes produce.  After it: mark its completion if another lane reads it.
dcnn_status lane_wait_inputs(dcnn_net* net, const Planned& p) {
    if (net->nlanes <= 1) return DCNN_OK;
    for (int in : p.in_nodes) {
        const Planned& q = net->plan[net->layer_of_node[in]];
        if (q.lane != p.lane && q.done) {
            dcnn_status st = check_hip(net->ctx, hipStreamWaitEvent(net->lane_ctx[p.lane]->stream, q.done, 0), "hipStreamWaitEvent");
            if (st != DCNN_OK) return st;
        }
    }
    return DCNN_OK;
}
dcnn_status lane_mark_done(dcnn_net* net, const Planned& p) {
    if (!p.done) return DCNN_OK;
    return check_hip(net->ctx, hipEventRecord(p.done, net->lane_ctx[p.lane]->stream), "hipEventRecord");
}

// The caller's stream continues behind every lane.
dcnn_status lanes_end(dcnn_net* net) {
    dcnn_ctx* ctx = net->ctx;
    for (int l = 1; l < net->nlanes; ++l) {
        dcnn_status st = check_hip(ctx, hipEventRecord(net->lane_end[l], net->lane_ctx[l]->stream), "hipEventRecord");
        if (st == DCNN_OK) st = check_hip(ctx, hipStreamWaitEvent(ctx->stream, net->lane_end[l], 0), "hipStreamWaitEvent");
        if (st != DCNN_OK) return st;
    }
    return DCNN_OK;
}

}  // namespace

extern "C" {

dcnn_status dcnn_net_create(dcnn_ctx* ctx, int32_t dtype, int32_t n, int32_t h, int32_t w, int32_t c, dcnn_net** out) {
    if (!ctx) return DCNN_EINVAL;
    if (!out) return fail(ctx, DCNN_EINVAL, "net_create: null output");
    *out = nullptr;
    if (dtype != DCNN_F32 && dtype != DCNN_F16) return fail(ctx, DCNN_EDTYPE, "net_create: bad dtype %d", dtype);
    if (n < 1 || h < 1 || w < 1 || c < 1) return fail(ctx, DCNN_ESHAPE, "net_create: bad input shape");
    dcnn_net* net = new (std::nothrow) dcnn_net();
    if (!net) return fail(ctx, DCNN_ENOMEM, "net_create: host allocation failed");
    net->ctx = ctx; net->dtype = dtype; net->n = n; net->h = h; net->w = w; net->c = c;
    *out = net;
    return DCNN_OK;
}

void dcnn_net_destroy(dcnn_net* net) {
    if (!net) return;
    for (auto& p : net->plan) dcnn_layer_destroy(p.layer);
    drop_lanes(net);
    delete net;
}

dcnn_status dcnn_net_add(dcnn_net* net, const dcnn_layer_desc* desc, const int32_t* inputs, int32_t n_inputs,
                         const void* weights_dev, const void* bias_dev, int32_t* node_id) {
    if (!net) return DCNN_EINVAL;
    dcnn_ctx* ctx = net->ctx;
    if (!desc || !node_id) return fail(ctx, DCNN_EINVAL, "net_add: null argument");
    if (net->finalized) return fail(ctx, DCNN_ESTATE, "net_add: the network is finalized");
    Node nd;
    nd.d = *desc;
    nd.w = weights_dev; nd.b = bias_dev;
    const int id = (int)net->nodes.size();
    if (desc->kind == DCNN_DELTAGEN) {
        if (id != 0 || n_inputs != 0) return fail(ctx, DCNN_EINVAL, "net_add: the input layer must be node 0 without inputs");
        nd.d.n = net->n; nd.d.h = net->h; nd.d.w = net->w; nd.d.c = net->c; nd.d.n_in = 1;
    } else {
        if (id == 0) return fail(ctx, DCNN_EINVAL, "net_add: node 0 must be the input layer (DCNN_DELTAGEN)");
        const int want = (desc->kind == DCNN_ACT) ? desc->n_in : (desc->kind == DCNN_CONCAT ? 2 : 1);
        if (n_inputs != want || !inputs) return fail(ctx, DCNN_EINVAL, "net_add: node %d expects %d inputs, got %d", id, want, n_inputs);
        if (is_conv(*desc) && (desc->act != DCNN_ACT_NONE || desc->n_in != 1))
            return fail(ctx, DCNN_EINVAL, "net_add: add convolutions unfused (act NONE, one input); finalize fuses");
        for (int i = 0; i < n_inputs; ++i) {
            if (inputs[i] < 0 || inputs[i] >= id) return fail(ctx, DCNN_EINVAL, "net_add: node %d input %d out of range", id, inputs[i]);
            if (net->nodes[inputs[i]].d.kind == DCNN_ACCUM) return fail(ctx, DCNN_EINVAL, "net_add: the output layer has no consumers");
            nd.in.push_back(inputs[i]);
        }
        const Node& p0 = net->nodes[inputs[0]];
        nd.d.n = net->n; nd.d.h = p0.oh; nd.d.w = p0.ow; nd.d.c = p0.oc;
        if (n_inputs == 2) {
            const Node& p1 = net->nodes[inputs[1]];
            if (p1.oh != p0.oh || p1.ow != p0.ow || (desc->kind != DCNN_CONCAT && p1.oc != p0.oc))
                return fail(ctx, DCNN_ESHAPE, "net_add: node %d joins [%d,%d,%d] and [%d,%d,%d]", id, p0.oh, p0.ow, p0.oc, p1.oh, p1.ow, p1.oc);
            if (desc->kind == DCNN_CONCAT) { nd.d.n_in = 2; nd.d.cout = p0.oc + p1.oc; }
        }
        if (desc->kind == DCNN_DWCONV) nd.d.cout = nd.d.c;
    }
    nd.d.dtype = net->dtype;
    nd.d.kw = nd.d.kh;
    nd.d.want_idx = 1;
    dcnn_layer_sizes sz;
    dcnn_status st = dcnn_layer_query(&nd.d, &sz);
    if (st != DCNN_OK) return fail(ctx, st, "net_add: node %d has an invalid descriptor", id);
    nd.oh = sz.oh; nd.ow = sz.ow; nd.oc = sz.oc;
    if (is_conv(nd.d) && !weights_dev) return fail(ctx, DCNN_EINVAL, "net_add: convolution node %d without weights", id);
    for (int i : nd.in) net->nodes[i].consumers.push_back(id);
    net->nodes.push_back(nd);
    *node_id = id;
    return DCNN_OK;
}

dcnn_status dcnn_net_finalize(dcnn_net* net, int32_t fuse, size_t* arena_bytes) {
    if (!net) return DCNN_EINVAL;
    dcnn_ctx* ctx = net->ctx;
    if (!arena_bytes) return fail(ctx, DCNN_EINVAL, "net_finalize: null argument");
    if (net->finalized) return fail(ctx, DCNN_ESTATE, "net_finalize: already finalized");
    const int N = (int)net->nodes.size();
    if (N < 2 || net->nodes[N - 1].d.kind != DCNN_ACCUM)
        return fail(ctx, DCNN_EINVAL, "net_finalize: the last node must be the output layer (DCNN_ACCUM)");
    for (int i = 0; i < N - 1; ++i)
        if (net->nodes[i].d.kind == DCNN_ACCUM) return fail(ctx, DCNN_EINVAL, "net_finalize: only the last node may be DCNN_ACCUM");

    std::vector<char> absorbed(N, 0);
    net->layer_of_node.assign(N, -1);
    auto sole_consumer = [&](int i) { return net->nodes[i].consumers.size() == 1 ? net->nodes[i].consumers[0] : -1; };
    char why[256];
    for (int i = 0; i < N; ++i) {
        if (absorbed[i]) continue;
        const Node& nd = net->nodes[i];
        Planned p{};
        p.d = nd.d; p.in_nodes = nd.in; p.out_node = i; p.w = nd.w; p.b = nd.b; p.w2 = nullptr; p.b2 = nullptr; p.layer = nullptr;
        if ((fuse & 1) && is_conv(nd.d)) {
            int cur = i;
            dcnn_layer_desc d = nd.d;
            std::vector<int> ins = nd.in, taken;
            int j = sole_consumer(cur);
            int proj = -1;                       // convolution on the other arm of the add that is pulled in
            if (j >= 0 && !absorbed[j] && is_add(net->nodes[j].d)) {
                const Node& add = net->nodes[j];
                const int other = add.in[0] == cur ? add.in[1] : add.in[0];
                if (other != cur) {
                    d.n_in = 2;
                    ins.push_back(other);
                    taken.push_back(j);
                    cur = j;
                    // the other arm: an unfused 1x1 convolution without padding that feeds only this add and
                    // has not been planned yet (it comes later in node order, or it would be a layer already)
                    const Node& o = net->nodes[other];
                    if (other > i && !absorbed[other] && o.d.kind == DCNN_CONV && o.d.kh == 1 && o.d.pad == 0 &&
                        o.consumers.size() == 1 && o.in.size() == 1)
                        proj = other;
                }
            }
            int k = sole_consumer(cur);
            if (k >= 0 && !absorbed[k] && is_plain_act(net->nodes[k].d)) {
                d.act = net->nodes[k].d.act;
                d.eps = net->nodes[k].d.eps;
                d.no_xT = net->nodes[k].d.no_xT;
                d.xT_residue = net->nodes[k].d.xT_residue;
                taken.push_back(k);
                cur = k;
            }
            if (cur != i && conv_supported(ctx, d.dtype, d.kh, d.c, nd.oc, d.kind == DCNN_DWCONV, true, why, sizeof(why))) {
                for (int a : taken) absorbed[a] = 1;
                p.d = d; p.in_nodes = ins; p.out_node = cur;
                if (proj >= 0 && d.act != DCNN_ACT_NONE && d.kind == DCNN_CONV) {
                    const Node& o = net->nodes[proj];
                    const int64_t px_in = (int64_t)d.n * d.h * d.w, px_in2 = (int64_t)d.n * o.d.h * o.d.w;
                    const int64_t px_out = (int64_t)d.n * nd.oh * nd.ow;
                    if (conv_proj_supported(ctx, d.dtype, d.kh, d.c, o.d.c, nd.oc, px_in * d.c, px_in2 * o.d.c, px_out * nd.oc) &&
                        conv_supported(ctx, d.dtype, 1, o.d.c, nd.oc, 0, false, why, sizeof(why))) {
                        absorbed[proj] = 1;
                        p.d.proj_c = o.d.c; p.d.proj_h = o.d.h; p.d.proj_w = o.d.w; p.d.proj_stride = o.d.stride;
                        p.in_nodes[1] = o.in[0];
                        p.w2 = o.w; p.b2 = o.b;
                    }
                }
            }
        } else if ((fuse & 1) && is_add(nd.d)) {
            int k = sole_consumer(i);
            if (k >= 0 && !absorbed[k] && is_plain_act(net->nodes[k].d)) {
                p.d.act = net->nodes[k].d.act;
                p.d.eps = net->nodes[k].d.eps;
                p.d.no_xT = net->nodes[k].d.no_xT;
                p.d.xT_residue = net->nodes[k].d.xT_residue;
                p.out_node = k;
                absorbed[k] = 1;
            }
        }
        net->plan.push_back(p);
    }
    // run layers in the order of the node whose output they produce (inputs always come earlier)
    for (size_t a = 1; a < net->plan.size(); ++a)
        for (size_t b = a; b > 0 && net->plan[b].out_node < net->plan[b - 1].out_node; --b) std::swap(net->plan[b], net->plan[b - 1]);
    int folded_accum = -1;
    // The output layer behind a convolution + activation that nothing else reads is folded into it: the
    // emitted deltas go straight into the dense output instead of through memory.
    if ((fuse & 1) && net->plan.size() >= 2 && net->plan.back().d.kind == DCNN_ACCUM) {
        Planned& last = net->plan[net->plan.size() - 2];
        const Planned& acc = net->plan.back();
        const dcnn_layer_desc& d = last.d;
        const Node& on = net->nodes[last.out_node];
        if (acc.in_nodes.size() == 1 && acc.in_nodes[0] == last.out_node && on.consumers.size() == 1 &&
            d.kind == DCNN_CONV && d.act != DCNN_ACT_NONE && (d.n_in == 1 || d.proj_c > 0) &&
            conv_ws_supported(ctx, d.dtype, d.kh, d.c, on.oc, (int64_t)d.n * d.h * d.w * d.c, (int64_t)d.n * on.oh * on.ow * on.oc)) {
            last.d.fuse_accum = 1;
            folded_accum = acc.out_node;
            net->plan.pop_back();
        }
    }
    for (size_t a = 0; a < net->plan.size(); ++a) net->layer_of_node[net->plan[a].out_node] = (int)a;
    if (folded_accum >= 0) net->layer_of_node[folded_accum] = (int)net->plan.size() - 1;
    // every sparse input must be the output of a planned layer
    for (auto& p : net->plan)
        for (int in : p.in_nodes)
            if (net->layer_of_node[in] < 0) return fail(ctx, DCNN_EINVAL, "net_finalize: internal: node %d was fused away but is still consumed", in);
    // which outputs need an index list: consumers that walk their input's list as it is
    for (auto& p : net->plan) p.d.want_idx = (fuse & 2) ? 1 : 0;
    for (auto& p : net->plan) {
        if (p.in_nodes.empty()) continue;
        const dcnn_layer_desc& d = p.d;
        const bool walks_input_list = d.kind == DCNN_ACCUM || d.kind == DCNN_MAXPOOL ||
                                      (is_conv(d) && d.kh == 1 && d.stride == 1 && d.n_in == 1) ||
                                      (d.kind == DCNN_ACT && d.n_in == 1);
        if (walks_input_list) net->plan[net->layer_of_node[p.in_nodes[0]]].d.want_idx = 1;
    }
    size_t off = 0;
    for (auto& p : net->plan) {
        dcnn_layer_sizes sz;
        dcnn_status st = dcnn_layer_query(&p.d, &sz);
        if (st != DCNN_OK) return fail(ctx, st, "net_finalize: layer for node %d is invalid", p.out_node);
        p.state_off = off;
        p.state_bytes = sz.state_bytes;
        off += align_up(sz.state_bytes);
    }
    // Lanes: a layer continues the lane of a producer whose lane nothing else has continued yet (a chain stays on
    // one stream); a layer that starts a new branch takes the lane that has been idle longest.
    net->nlanes = 1;
    if (fuse & 4) {
        int tail[kMaxLanes];
        for (int l = 0; l < kMaxLanes; ++l) tail[l] = -1;
        for (size_t a = 0; a < net->plan.size(); ++a) {
            Planned& p = net->plan[a];
            int lane = -1;
            for (int in : p.in_nodes) {
                const int pi = net->layer_of_node[in];
                if (tail[net->plan[pi].lane] == pi) { lane = net->plan[pi].lane; break; }
            }
            if (lane < 0) {
                lane = 0;
                for (int l = 1; l < kMaxLanes; ++l)
                    if (tail[l] < tail[lane]) lane = l;
                if (p.in_nodes.empty()) lane = 0;               // the input layer runs on the caller's stream
            }
            p.lane = lane;
            tail[lane] = (int)a;
            if (lane + 1 > net->nlanes) net->nlanes = lane + 1;
        }
        // A dependency between lanes costs more than a launch (an event recorded on one stream, a wait on the other):
        // a network that is mostly one chain -- a residual backbone whose only side branches are single shortcut
        // convolutions -- was measured slower on lanes (1.91 -> 2.16 ms) and stays on the caller's stream.
        size_t off_main = 0;
        for (const auto& p : net->plan) off_main += p.lane != 0;
        if (off_main * 4 < net->plan.size()) {
            for (auto& p : net->plan) p.lane = 0;
            net->nlanes = 1;
        }
        if (net->nlanes > 1) {
            int64_t max_px = 1;
            for (const Node& nd : net->nodes) {
                const int64_t a = (int64_t)net->n * nd.oh * nd.ow, b = (int64_t)nd.d.n * nd.d.h * nd.d.w;
                max_px = a > max_px ? a : max_px;
                max_px = b > max_px ? b : max_px;
            }
            net->lane_ws_off = off;
            net->lane_ws_bytes = align_up(workspace_bytes(max_px));
            off += (size_t)(net->nlanes - 1) * net->lane_ws_bytes;
        }
    }
    net->arena_bytes = off;
    net->finalized = true;
    *arena_bytes = off;
    return DCNN_OK;
}

dcnn_status dcnn_net_bind(dcnn_net* net, void* arena_dev, size_t arena_bytes) {
    if (!net) return DCNN_EINVAL;
    dcnn_ctx* ctx = net->ctx;
    if (!net->finalized) return fail(ctx, DCNN_ESTATE, "net_bind: finalize first");
    if (net->bound) return fail(ctx, DCNN_ESTATE, "net_bind: already bound");
    if (!arena_dev || (reinterpret_cast<uintptr_t>(arena_dev) % kAlign) != 0)
        return fail(ctx, DCNN_EINVAL, "net_bind: arena missing or not 256-byte aligned");
    if (arena_bytes < net->arena_bytes) return fail(ctx, DCNN_ENOMEM, "net_bind: arena of %zu bytes, need %zu", arena_bytes, net->arena_bytes);
    net->lane_ctx.assign(net->nlanes, nullptr);
    net->lane_ctx[0] = ctx;
    net->lane_end.assign(net->nlanes, nullptr);
    dcnn_status st = DCNN_OK;
    if (net->nlanes > 1) {
        st = check_hip(ctx, hipEventCreateWithFlags(&net->ev_start, hipEventDisableTiming), "hipEventCreate");
        for (int l = 1; l < net->nlanes && st == DCNN_OK; ++l) {
            dcnn_ctx* lc = new (std::nothrow) dcnn_ctx(*ctx);
            if (!lc) { st = fail(ctx, DCNN_ENOMEM, "net_bind: host allocation failed"); break; }
            lc->stream = nullptr;
            lc->ws = static_cast<char*>(arena_dev) + net->lane_ws_off + (size_t)(l - 1) * net->lane_ws_bytes;
            lc->ws_bytes = net->lane_ws_bytes;
            lc->err[0] = 0;
            net->lane_ctx[l] = lc;
            st = check_hip(ctx, hipStreamCreateWithFlags(&lc->stream, hipStreamNonBlocking), "hipStreamCreate");   // default priority
            if (st == DCNN_OK) st = check_hip(ctx, hipEventCreateWithFlags(&net->lane_end[l], hipEventDisableTiming), "hipEventCreate");
        }
        // completion events of layers that a layer on another lane consumes
        for (auto& p : net->plan) {
            if (st != DCNN_OK) break;
            for (int in : p.in_nodes) {
                Planned& q = net->plan[net->layer_of_node[in]];
                if (q.lane != p.lane && !q.done) {
                    st = check_hip(ctx, hipEventCreateWithFlags(&q.done, hipEventDisableTiming), "hipEventCreate");
                    if (st != DCNN_OK) break;
                }
            }
        }
        if (st == DCNN_OK) st = lanes_begin(net);               // weight packing below runs on the lanes' streams
    }
    for (auto& p : net->plan) {
        if (st != DCNN_OK) break;
        st = dcnn::layer_create(net->lane_ctx[p.lane], &p.d, p.w, p.b, p.w2, p.b2, static_cast<char*>(arena_dev) + p.state_off, p.state_bytes, &p.layer);
        if (st != DCNN_OK) st = lane_fail(net, p, st);
    }
    if (st == DCNN_OK) st = lanes_end(net);
    if (st != DCNN_OK) {
        for (auto& q : net->plan) { dcnn_layer_destroy(q.layer); q.layer = nullptr; }
        drop_lanes(net);
        return st;
    }
    net->bound = true;
    return DCNN_OK;
}

dcnn_status dcnn_net_init(dcnn_net* net, const void* frame_dev, void* out_dev) {
    if (!net) return DCNN_EINVAL;
    dcnn_ctx* ctx = net->ctx;
    if (!net->bound) return fail(ctx, DCNN_ESTATE, "net_init: bind an arena first");
    if (!frame_dev) return fail(ctx, DCNN_EINVAL, "net_init: null frame");
    // during the dense first frame every layer writes its dense output into its own (dense-shaped)
    // delta buffer, which the consumers read; afterwards those buffers hold sparse updates again
    dcnn_status st = lanes_begin(net);
    if (st != DCNN_OK) return st;
    for (auto& p : net->plan) {
        const void* ins[2] = {nullptr, nullptr};
        int n_in = 0;
        if (p.d.kind == DCNN_DELTAGEN) {
            ins[0] = frame_dev; n_in = 1;
        } else {
            for (int in : p.in_nodes) ins[n_in++] = net->plan[net->layer_of_node[in]].layer->out_data;
        }
        void* dense_out = p.d.kind == DCNN_ACCUM ? out_dev : p.layer->out_data;
        st = lane_wait_inputs(net, p);
        if (st == DCNN_OK) st = dcnn_layer_init(p.layer, ins, n_in, dense_out);
        if (st == DCNN_OK && p.d.fuse_accum && out_dev) st = launch_copy(net->lane_ctx[p.lane], out_dev, p.layer->buf2, p.layer->buf2_bytes);
        if (st != DCNN_OK) return lane_fail(net, p, st);
        st = lane_mark_done(net, p);
        if (st != DCNN_OK) return st;
    }
    st = lanes_end(net);
    if (st != DCNN_OK) return st;
    net->inited = true;
    return DCNN_OK;
}

dcnn_status dcnn_net_step(dcnn_net* net, const void* frame_dev, void* out_dev) {
    if (!net) return DCNN_EINVAL;
    dcnn_ctx* ctx = net->ctx;
    if (!net->bound) return fail(ctx, DCNN_ESTATE, "net_step: bind an arena first");
    if (!net->inited) return fail(ctx, DCNN_ESTATE, "net_step: no first frame yet (call net_init)");
    if (!frame_dev) return fail(ctx, DCNN_EINVAL, "net_step: null frame");
    dcnn_status st0 = lanes_begin(net);
    if (st0 != DCNN_OK) return st0;
    for (auto& p : net->plan) {
        dcnn_delta views[2];
        const dcnn_delta* ins[2] = {nullptr, nullptr};
        int n_in = 0;
        if (p.d.kind == DCNN_DELTAGEN) {
            views[0] = dcnn_delta{};
            views[0].data = const_cast<void*>(frame_dev);
            views[0].n = net->n; views[0].h = net->h; views[0].w = net->w; views[0].c = net->c; views[0].dtype = net->dtype;
            ins[0] = &views[0]; n_in = 1;
        } else {
            for (int in : p.in_nodes) {
                dcnn_status st = dcnn_layer_output(net->plan[net->layer_of_node[in]].layer, &views[n_in]);
                if (st != DCNN_OK) return st;
                ins[n_in] = &views[n_in];
                ++n_in;
            }
        }
        dcnn_status st = lane_wait_inputs(net, p);
        if (st == DCNN_OK) st = dcnn_layer_step(p.layer, ins, n_in);
        if (st != DCNN_OK) return lane_fail(net, p, st);
        st = lane_mark_done(net, p);
        if (st != DCNN_OK) return st;
    }
    st0 = lanes_end(net);
    if (st0 != DCNN_OK) return st0;
    if (out_dev) {
        dcnn_layer* last = net->plan.back().layer;
        if (last->d.fuse_accum) return launch_copy(ctx, out_dev, last->buf2, last->buf2_bytes);
        return launch_copy(ctx, out_dev, last->buf0, last->buf0_bytes);
    }
    return DCNN_OK;
}

dcnn_status dcnn_net_reset(dcnn_net* net) {
    if (!net) return DCNN_EINVAL;
    if (!net->bound) return fail(net->ctx, DCNN_ESTATE, "net_reset: bind an arena first");
    for (auto& p : net->plan) {
        dcnn_status st = dcnn_layer_reset(p.layer);
        if (st != DCNN_OK) return st;
    }
    net->inited = false;
    return DCNN_OK;
}

dcnn_status dcnn_net_output(const dcnn_net* net, dcnn_delta* out_view) {
    if (!net || !out_view) return DCNN_EINVAL;
    if (!net->bound) return fail(net->ctx, DCNN_ESTATE, "net_output: bind an arena first");
    return dcnn_layer_output(net->plan.back().layer, out_view);
}

int32_t dcnn_net_num_layers(const dcnn_net* net) { return net && net->finalized ? (int32_t)net->plan.size() : 0; }

dcnn_status dcnn_net_layer(const dcnn_net* net, int32_t i, dcnn_layer** layer, int32_t* node_id) {
    if (!net || !layer || !node_id) return DCNN_EINVAL;
    if (!net->bound) return fail(net->ctx, DCNN_ESTATE, "net_layer: bind an arena first");
    if (i < 0 || i >= (int32_t)net->plan.size()) return fail(net->ctx, DCNN_EINVAL, "net_layer: index %d out of range", i);
    *layer = net->plan[i].layer;
    *node_id = net->plan[i].out_node;
    return DCNN_OK;
}

dcnn_status dcnn_net_stats(dcnn_net* net, dcnn_stats* stats_host) {
    if (!net || !stats_host) return DCNN_EINVAL;
    if (!net->bound) return fail(net->ctx, DCNN_ESTATE, "net_stats: bind an arena first");
    for (size_t i = 0; i < net->plan.size(); ++i) {
        dcnn_status st = dcnn_layer_stats(net->plan[i].layer, &stats_host[i]);
        if (st != DCNN_OK) return st;
    }
    return DCNN_OK;
}

}  // extern "C"
