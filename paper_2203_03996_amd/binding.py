"""ctypes binding of libdeltacnn.so: same names as the C ABI, argument marshalling only.

PyTorch is used for device memory (`torch.empty(..., device="cuda")`) and for the HIP
stream; every step of the path runs inside the library's kernels.  There is no CPU
fallback: importing works without a GPU (so the symbol table can be checked), but creating
a context without the built library or without an MI355X raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libdeltacnn.so")

F32, F16 = 0, 1
DELTAGEN, CONV, DWCONV, ACT, MAXPOOL, UPSAMPLE, ACCUM, CONCAT, UPSAMPLE_BILINEAR, GAVGPOOL = range(10)
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2
ACT_CODES = {"none": ACT_NONE, None: ACT_NONE, "relu": ACT_RELU, "relu6": ACT_RELU6}
TORCH_DTYPE = {F32: torch.float32, F16: torch.float16}
DTYPE_CODE = {"f32": F32, "f16": F16}
STATUS_NAMES = ["OK", "EINVAL", "ESHAPE", "EDTYPE", "ESTATE", "ENOMEM", "EHIP", "EUNSUPPORTED"]

EXPORTS = [
    "dcnn_workspace_bytes", "dcnn_ctx_create", "dcnn_ctx_destroy", "dcnn_ctx_sync", "dcnn_status_str",
    "dcnn_last_error", "dcnn_mask_compact", "dcnn_mask_compact_static", "dcnn_layer_query", "dcnn_layer_create", "dcnn_layer_destroy",
    "dcnn_layer_init", "dcnn_layer_step", "dcnn_layer_output", "dcnn_layer_reset", "dcnn_layer_state",
    "dcnn_layer_stats", "dcnn_layer_set_eps", "dcnn_layer_set_timing", "dcnn_layer_set_counting", "dcnn_layer_timing", "dcnn_net_create", "dcnn_net_destroy", "dcnn_net_add", "dcnn_net_finalize",
    "dcnn_net_bind", "dcnn_net_init", "dcnn_net_step", "dcnn_net_reset", "dcnn_net_output",
    "dcnn_net_num_layers", "dcnn_net_layer", "dcnn_net_stats",
]


class DeltaStruct(C.Structure):
    _fields_ = [("data", C.c_void_p), ("mask", C.c_void_p), ("idx", C.c_void_p), ("count", C.c_void_p),
                ("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("c", C.c_int32), ("dtype", C.c_int32)]


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("c", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
                ("cout", C.c_int32), ("act", C.c_int32), ("eps", C.c_float), ("n_in", C.c_int32),
                ("dilate_r", C.c_int32), ("factor", C.c_int32), ("want_idx", C.c_int32),
                ("proj_c", C.c_int32), ("proj_h", C.c_int32), ("proj_w", C.c_int32), ("proj_stride", C.c_int32),
                ("fuse_accum", C.c_int32), ("no_xT", C.c_int32), ("xT_residue", C.c_int32)]


class LayerSizes(C.Structure):
    _fields_ = [("state_bytes", C.c_size_t), ("on", C.c_int32), ("oh", C.c_int32), ("ow", C.c_int32),
                ("oc", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("pixels_in", C.c_int64), ("pixels_in2", C.c_int64), ("pixels_work", C.c_int64),
                ("pixels_out", C.c_int64), ("pixels_total", C.c_int64), ("pixels_in_total", C.c_int64),
                ("pixels_in2_total", C.c_int64),
                ("kind", C.c_int32), ("act", C.c_int32), ("n_in", C.c_int32), ("c_in", C.c_int32),
                ("c_out", C.c_int32), ("k", C.c_int32), ("stride", C.c_int32), ("proj_c", C.c_int32), ("fuse_accum", C.c_int32),
                ("reserved", C.c_int32), ("xT_bytes_read", C.c_int64), ("xT_bytes_written", C.c_int64)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_ if name != "reserved"}


class DcnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libdeltacnn: {STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {text}")
        self.status = status


_lib = None


def load_library() -> C.CDLL:
    """Load the built shared library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                                "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    P = C.POINTER
    lib.dcnn_workspace_bytes.restype = sz
    lib.dcnn_workspace_bytes.argtypes = [C.c_int64]
    lib.dcnn_ctx_create.argtypes = [vp, vp, sz, P(vp)]
    lib.dcnn_ctx_destroy.argtypes = [vp]
    lib.dcnn_ctx_destroy.restype = None
    lib.dcnn_ctx_sync.argtypes = [vp]
    lib.dcnn_status_str.restype = C.c_char_p
    lib.dcnn_status_str.argtypes = [i32]
    lib.dcnn_last_error.restype = C.c_char_p
    lib.dcnn_last_error.argtypes = [vp]
    lib.dcnn_mask_compact.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.dcnn_mask_compact_static.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.dcnn_layer_query.argtypes = [P(LayerDesc), P(LayerSizes)]
    lib.dcnn_layer_create.argtypes = [vp, P(LayerDesc), vp, vp, vp, sz, P(vp)]
    lib.dcnn_layer_destroy.argtypes = [vp]
    lib.dcnn_layer_destroy.restype = None
    lib.dcnn_layer_init.argtypes = [vp, P(vp), i32, vp]
    lib.dcnn_layer_step.argtypes = [vp, P(P(DeltaStruct)), i32]
    lib.dcnn_layer_output.argtypes = [vp, P(DeltaStruct)]
    lib.dcnn_layer_reset.argtypes = [vp]
    lib.dcnn_layer_state.argtypes = [vp, i32, P(vp), P(sz)]
    lib.dcnn_layer_stats.argtypes = [vp, P(Stats)]
    lib.dcnn_layer_set_eps.argtypes = [vp, C.c_float]
    lib.dcnn_layer_set_timing.argtypes = [vp, i32]
    lib.dcnn_layer_set_counting.argtypes = [vp, i32]
    lib.dcnn_layer_timing.argtypes = [vp, P(C.c_float), P(i32)]
    lib.dcnn_net_create.argtypes = [vp, i32, i32, i32, i32, i32, P(vp)]
    lib.dcnn_net_destroy.argtypes = [vp]
    lib.dcnn_net_destroy.restype = None
    lib.dcnn_net_add.argtypes = [vp, P(LayerDesc), P(i32), i32, vp, vp, P(i32)]
    lib.dcnn_net_finalize.argtypes = [vp, i32, P(sz)]
    lib.dcnn_net_bind.argtypes = [vp, vp, sz]
    lib.dcnn_net_init.argtypes = [vp, vp, vp]
    lib.dcnn_net_step.argtypes = [vp, vp, vp]
    lib.dcnn_net_reset.argtypes = [vp]
    lib.dcnn_net_output.argtypes = [vp, P(DeltaStruct)]
    lib.dcnn_net_num_layers.argtypes = [vp]
    lib.dcnn_net_num_layers.restype = i32
    lib.dcnn_net_layer.argtypes = [vp, i32, P(vp), P(i32)]
    lib.dcnn_net_stats.argtypes = [vp, P(Stats)]
    _lib = lib
    return lib


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


@dataclass
class Delta:
    """Device tensors of one sparse update (see dcnn_delta in deltacnn.h)."""
    data: torch.Tensor            # [n,h,w,c]
    mask: torch.Tensor | None     # uint8 [n,h,w]
    idx: torch.Tensor | None      # int32 [n*h*w]
    count: torch.Tensor | None    # int32 [1]

    def struct(self) -> DeltaStruct:
        n, h, w, c = self.data.shape
        code = F16 if self.data.dtype == torch.float16 else F32
        return DeltaStruct(_ptr(self.data), _ptr(self.mask), _ptr(self.idx), _ptr(self.count), n, h, w, c, code)


class Context:
    """dcnn_ctx on torch's current stream, with a torch-allocated workspace."""

    def __init__(self, max_pixels: int, device="cuda"):
        """max_pixels = 0 creates the context without a workspace (enough for mask_compact_static)."""
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("libdeltacnn needs an MI355X (gfx950); no GPU is visible and there is no CPU path")
        self.device = torch.device(device)
        nbytes = self.lib.dcnn_workspace_bytes(int(max_pixels)) if max_pixels > 0 else 0
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8, device=self.device) if nbytes else None
        self.stream = torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        st = self.lib.dcnn_ctx_create(C.c_void_p(self.stream.cuda_stream), C.c_void_p(_ptr(self.workspace)),
                                      nbytes, C.byref(h))
        if st != 0:
            raise DcnnError(st, self.lib.dcnn_status_str(st).decode())
        self.handle = h
        self._bases = []          # tensors whose memory library-returned pointers may point into

    def check(self, st: int):
        if st != 0:
            raise DcnnError(st, self.lib.dcnn_last_error(self.handle).decode())

    def sync(self):
        self.check(self.lib.dcnn_ctx_sync(self.handle))

    def register(self, *tensors):
        for t in tensors:
            if t is not None:
                self._bases.append(t)

    def view(self, ptr: int, nbytes: int, dtype, shape):
        """Torch view of library-returned device memory that lies inside a registered tensor."""
        for b in self._bases:
            lo = b.data_ptr()
            if lo <= ptr and ptr + nbytes <= lo + b.numel() * b.element_size():
                flat = b.reshape(-1).view(torch.uint8)
                return flat[ptr - lo:ptr - lo + nbytes].view(dtype).reshape(shape)
        raise ValueError("pointer does not belong to a registered tensor")

    def delta_view(self, s: DeltaStruct) -> Delta:
        dt = TORCH_DTYPE[s.dtype]
        px = s.n * s.h * s.w
        es = 2 if s.dtype == F16 else 4
        return Delta(self.view(s.data, px * s.c * es, dt, (s.n, s.h, s.w, s.c)),
                     self.view(s.mask, px, torch.uint8, (s.n, s.h, s.w)) if s.mask else None,
                     self.view(s.idx, px * 4, torch.int32, (px,)) if s.idx else None,
                     self.view(s.count, 4, torch.int32, (1,)) if s.count else None)

    def mask_compact(self, mask_in, k=1, stride=1, pad=0, mask_b=None):
        n, h, w = mask_in.shape
        oh, ow = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
        mask_out = torch.empty((n, oh, ow), dtype=torch.uint8, device=self.device)
        idx = torch.empty(n * oh * ow, dtype=torch.int32, device=self.device)
        count = torch.empty(1, dtype=torch.int32, device=self.device)
        self.check(self.lib.dcnn_mask_compact(self.handle, _ptr(mask_in), n, h, w, k, stride, pad, _ptr(mask_b),
                                              _ptr(mask_out), _ptr(idx), _ptr(count)))
        return mask_out, idx, count

    def mask_compact_static(self, mask_in, mask_out, idx, count, k=1, stride=1, pad=0, mask_b=None):
        """dcnn_mask_compact_static: the caller passes every output buffer (mask_out may be None); the call
        itself allocates nothing."""
        n, h, w = mask_in.shape
        self.check(self.lib.dcnn_mask_compact_static(self.handle, _ptr(mask_in), n, h, w, k, stride, pad, _ptr(mask_b),
                                                     _ptr(mask_out), _ptr(idx), _ptr(count)))

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                self.lib.dcnn_ctx_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


def make_desc(kind, dtype, n, h, w, c, k=1, stride=1, pad=0, cout=0, act=ACT_NONE, eps=0.0, n_in=1, dilate_r=0,
              factor=1, want_idx=1, proj=None, fuse_accum=0, no_xT=0, xT_residue=0) -> LayerDesc:
    """proj = (channels, height, width, stride) of the input of a fused 1x1 projection shortcut, or None."""
    pc, ph, pw, ps = proj if proj is not None else (0, 0, 0, 0)
    return LayerDesc(kind, dtype, n, h, w, c, k, k, stride, pad, cout, act, float(eps), n_in, dilate_r, factor,
                     want_idx, pc, ph, pw, ps, fuse_accum, int(no_xT), int(xT_residue))


class Layer:
    """dcnn_layer with torch-allocated state memory."""

    def __init__(self, ctx: Context, desc: LayerDesc, weights: torch.Tensor | None = None,
                 bias: torch.Tensor | None = None):
        self.ctx, self.desc = ctx, desc
        lib = ctx.lib
        sizes = LayerSizes()
        st = lib.dcnn_layer_query(C.byref(desc), C.byref(sizes))
        if st != 0:
            raise DcnnError(st, lib.dcnn_status_str(st).decode())
        self.out_shape = (sizes.on, sizes.oh, sizes.ow, sizes.oc)
        self.state = torch.zeros(sizes.state_bytes, dtype=torch.uint8, device=ctx.device)
        ctx.register(self.state)
        h = C.c_void_p()
        ctx.check(lib.dcnn_layer_create(ctx.handle, C.byref(desc), _ptr(weights), _ptr(bias), _ptr(self.state),
                                        sizes.state_bytes, C.byref(h)))
        self.handle = h
        self._keep = (weights, bias)

    def init(self, dense_in, dense_out=None):
        d = self.desc
        if not dense_in or tuple(dense_in[0].shape) != (d.n, d.h, d.w, d.c):
            raise ValueError(f"dense input 0 must have shape {(d.n, d.h, d.w, d.c)}")
        for t in dense_in:
            if t.dtype != TORCH_DTYPE[d.dtype] or not t.is_contiguous() or not t.is_cuda:
                raise ValueError("dense inputs must be contiguous device tensors of the layer's type")
        arr = (C.c_void_p * len(dense_in))(*[t.data_ptr() for t in dense_in])
        if dense_out is None and self.desc.kind != ACCUM:
            dense_out = torch.empty(self.out_shape, dtype=TORCH_DTYPE[self.desc.dtype], device=self.ctx.device)
        self.ctx.check(self.ctx.lib.dcnn_layer_init(self.handle, arr, len(dense_in), _ptr(dense_out)))
        return dense_out

    def step(self, inputs):
        structs = [d.struct() for d in inputs]
        for d in inputs:
            self.ctx.register(d.data, d.mask, d.idx, d.count)
        arr = (C.POINTER(DeltaStruct) * len(structs))(*[C.pointer(s) for s in structs])
        self.ctx.check(self.ctx.lib.dcnn_layer_step(self.handle, arr, len(structs)))
        return self.output()

    def output(self) -> Delta:
        s = DeltaStruct()
        self.ctx.check(self.ctx.lib.dcnn_layer_output(self.handle, C.byref(s)))
        return self.ctx.delta_view(s)

    def reset(self):
        self.ctx.check(self.ctx.lib.dcnn_layer_reset(self.handle))

    def set_eps(self, eps: float):
        self.ctx.check(self.ctx.lib.dcnn_layer_set_eps(self.handle, float(eps)))

    def state_tensor(self, which: int) -> torch.Tensor:
        p, n = C.c_void_p(), C.c_size_t()
        self.ctx.check(self.ctx.lib.dcnn_layer_state(self.handle, which, C.byref(p), C.byref(n)))
        dt = TORCH_DTYPE[self.desc.dtype]
        d = self.desc
        shape = (d.n, d.h, d.w, d.c) if d.kind in (DELTAGEN, MAXPOOL) else self.out_shape
        return self.ctx.view(p.value, n.value, dt, shape)

    def stats(self) -> dict:
        s = Stats()
        self.ctx.check(self.ctx.lib.dcnn_layer_stats(self.handle, C.byref(s)))
        return s.as_dict()

    def set_timing(self, max_steps: int):
        """Record HIP events around the layer's main kernel for the next `max_steps` steps (0: off)."""
        self.ctx.check(self.ctx.lib.dcnn_layer_set_timing(self.handle, max_steps))

    def timing(self):
        """(summed kernel milliseconds, launches) since the last call."""
        ms, n = C.c_float(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_layer_timing(self.handle, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                self.ctx.lib.dcnn_layer_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


_KIND = {"deltagen": DELTAGEN, "act": ACT, "add": ACT, "maxpool": MAXPOOL, "upsample": UPSAMPLE, "accum": ACCUM}


class Net:
    """dcnn_net built from a topology table (dict with "nodes", "dtype", "h", "w", "c"; see
    the header for node kinds) and a dict {node index: (weights, bias)} of numpy arrays."""

    def __init__(self, ctx: Context, spec: dict, weights: dict, n_streams: int, flags: int = 1):
        self.ctx, self.spec = ctx, spec
        lib = ctx.lib
        self.dtype = DTYPE_CODE[spec["dtype"]]
        tdt = TORCH_DTYPE[self.dtype]
        self.n = int(n_streams)
        h = C.c_void_p()
        ctx.check(lib.dcnn_net_create(ctx.handle, self.dtype, self.n, spec["h"], spec["w"], spec["c"], C.byref(h)))
        self.handle = h
        self._weights = {}
        for i, nd in enumerate(spec["nodes"]):
            kind = nd["kind"]
            wdev = bdev = None
            if kind == "conv":
                wgt, bias = weights[i]
                # one direct round-to-nearest-even to the storage type (numpy's conversion; going through
                # float32 first, as torch's float64 -> float16 does, rounds twice)
                ndt = np.float16 if self.dtype == F16 else np.float32
                wdev = torch.from_numpy(np.ascontiguousarray(np.asarray(wgt).astype(ndt))).to(ctx.device)
                bdev = torch.from_numpy(np.ascontiguousarray(np.asarray(bias).astype(ndt))).to(ctx.device)
                self._weights[i] = (wdev, bdev)
                desc = make_desc(DWCONV if nd["depthwise"] else CONV, self.dtype, 0, 0, 0, 0, k=nd["k"],
                                 stride=nd["stride"], pad=nd["pad"], cout=nd["cout"])
            elif kind == "deltagen":
                desc = make_desc(DELTAGEN, self.dtype, 0, 0, 0, 0, eps=nd["eps"], dilate_r=nd.get("dilate_r", 0))
            elif kind == "act":
                desc = make_desc(ACT, self.dtype, 0, 0, 0, 0, act=ACT_CODES[nd["f"]], eps=nd["eps"], n_in=1,
                                 no_xT=1 if nd.get("no_xT") else 0, xT_residue=1 if nd.get("xT_residue") else 0)
            elif kind == "add":
                desc = make_desc(ACT, self.dtype, 0, 0, 0, 0, act=ACT_NONE, n_in=2)
            elif kind == "concat":
                desc = make_desc(CONCAT, self.dtype, 0, 0, 0, 0, n_in=2)
            elif kind == "maxpool":
                desc = make_desc(MAXPOOL, self.dtype, 0, 0, 0, 0, k=nd["k"], stride=nd["stride"], pad=nd["pad"])
            elif kind == "upsample":
                desc = make_desc(UPSAMPLE, self.dtype, 0, 0, 0, 0, factor=nd["factor"])
            elif kind == "upsample_bilinear":
                desc = make_desc(UPSAMPLE_BILINEAR, self.dtype, 0, 0, 0, 0, factor=nd["factor"])
            elif kind == "gavgpool":
                desc = make_desc(GAVGPOOL, self.dtype, 0, 0, 0, 0)
            elif kind == "accum":
                desc = make_desc(ACCUM, self.dtype, 0, 0, 0, 0)
            else:
                raise ValueError(kind)
            ins = (C.c_int32 * max(1, len(nd["in"])))(*nd["in"])
            nid = C.c_int32()
            ctx.check(lib.dcnn_net_add(self.handle, C.byref(desc), ins, len(nd["in"]), _ptr(wdev), _ptr(bdev),
                                       C.byref(nid)))
            assert nid.value == i
        nbytes = C.c_size_t()
        ctx.check(lib.dcnn_net_finalize(self.handle, flags, C.byref(nbytes)))
        self.arena = torch.zeros(nbytes.value, dtype=torch.uint8, device=ctx.device)
        ctx.register(self.arena)
        ctx.check(lib.dcnn_net_bind(self.handle, _ptr(self.arena), nbytes.value))
        ctx.sync()                      # weights have been packed into the arena
        self.num_layers = lib.dcnn_net_num_layers(self.handle)

    def _check_frame(self, frame: torch.Tensor, out: torch.Tensor | None):
        # the ABI takes bare pointers: a tensor of the wrong size would be read or written out of bounds
        want = (self.n, self.spec["h"], self.spec["w"], self.spec["c"])
        if tuple(frame.shape) != want or frame.dtype != TORCH_DTYPE[self.dtype] or not frame.is_contiguous() or not frame.is_cuda:
            raise ValueError(f"frame must be a contiguous device tensor {want} of {TORCH_DTYPE[self.dtype]}, got "
                             f"{tuple(frame.shape)} {frame.dtype}")
        if out is not None and (out.dtype != TORCH_DTYPE[self.dtype] or not out.is_contiguous() or not out.is_cuda or
                                out.shape[0] != self.n):
            raise ValueError("out must be a contiguous device tensor [n, h, w, c] of the network's type")

    def init(self, frame: torch.Tensor, out: torch.Tensor | None = None):
        self._check_frame(frame, out)
        self.ctx.check(self.ctx.lib.dcnn_net_init(self.handle, _ptr(frame), _ptr(out)))

    def step(self, frame: torch.Tensor, out: torch.Tensor | None = None):
        self._check_frame(frame, out)
        self.ctx.check(self.ctx.lib.dcnn_net_step(self.handle, _ptr(frame), _ptr(out)))

    def reset(self):
        self.ctx.check(self.ctx.lib.dcnn_net_reset(self.handle))

    def output(self) -> Delta:
        s = DeltaStruct()
        self.ctx.check(self.ctx.lib.dcnn_net_output(self.handle, C.byref(s)))
        return self.ctx.delta_view(s)

    def layer_output(self, i: int):
        """(node id, Delta view, raw handle) of layer i of the fused plan."""
        lh, nid = C.c_void_p(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
        s = DeltaStruct()
        self.ctx.check(self.ctx.lib.dcnn_layer_output(lh, C.byref(s)))
        return nid.value, self.ctx.delta_view(s), lh

    def layer_state(self, i: int, which: int):
        lh, nid = C.c_void_p(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
        p, n = C.c_void_p(), C.c_size_t()
        st = self.ctx.lib.dcnn_layer_state(lh, which, C.byref(p), C.byref(n))
        if st != 0:
            return None
        es = 2 if self.dtype == F16 else 4
        return self.ctx.view(p.value, n.value, TORCH_DTYPE[self.dtype], (n.value // es,))

    def stats(self):
        arr = (Stats * self.num_layers)()
        self.ctx.check(self.ctx.lib.dcnn_net_stats(self.handle, arr))
        return [s.as_dict() for s in arr]

    def layer_node(self, i: int) -> int:
        """Node of the topology table whose output planned layer i produces."""
        lh, nid = C.c_void_p(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
        return nid.value

    def set_eps(self, i: int, eps: float):
        """New truncation threshold for planned layer i (input layer or a layer with an activation)."""
        lh, nid = C.c_void_p(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
        self.ctx.check(self.ctx.lib.dcnn_layer_set_eps(lh, float(eps)))

    def set_timing(self, i: int, max_steps: int):
        lh, nid = C.c_void_p(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
        self.ctx.check(self.ctx.lib.dcnn_layer_set_timing(lh, max_steps))

    def set_counting(self, on: bool):
        """Statistics mode for every layer: steps also count the x^T rows read / written (see dcnn_stats)."""
        for i in range(self.num_layers):
            lh, nid = C.c_void_p(), C.c_int32()
            self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
            self.ctx.check(self.ctx.lib.dcnn_layer_set_counting(lh, 1 if on else 0))

    def timing(self, i: int):
        """(summed kernel milliseconds, launches) of layer i since the last call."""
        lh, nid = C.c_void_p(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_net_layer(self.handle, i, C.byref(lh), C.byref(nid)))
        ms, n = C.c_float(), C.c_int32()
        self.ctx.check(self.ctx.lib.dcnn_layer_timing(lh, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                self.ctx.lib.dcnn_net_destroy(self.handle)
                self.handle = None
        except Exception:
            pass
