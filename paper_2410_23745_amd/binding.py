"""ctypes binding of include/syno.h.  Argument marshalling only: every step of the path runs in
the library's kernels; torch supplies device memory and streams."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # loads the HIP runtime the library links against

FWD, BWD_DATA, BWD_WEIGHT = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsyno.so")
_lib = None

EXPORTS = ("syno_plan_create", "syno_plan_destroy", "syno_forward", "syno_backward_data", "syno_backward_weight",
           "syno_backward_weight_static", "syno_plan_workspace_bytes", "syno_plan_shapes", "syno_plan_kernel", "syno_plan_describe",
           "syno_plan_free_size", "syno_debug_mfma_rate", "syno_debug_gather", "syno_debug_gather_host", "syno_status_string",
           "syno_chain_create", "syno_chain_destroy", "syno_chain_stages", "syno_chain_plan",
           "syno_chain_workspace_bytes", "syno_chain_forward", "syno_chain_backward",
           "syno_chain_create_materialized", "syno_chain_weight_stage", "syno_chain_stage_weight")


class _Dim(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("size", ctypes.c_int64)]


class _Prim(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("in_", ctypes.c_int32 * 2), ("out", ctypes.c_int32 * 2),
                ("param", ctypes.c_int64), ("shift_by", ctypes.c_int32), ("shift_coef", ctypes.c_int64)]


class _Options(ctypes.Structure):
    _fields_ = [("kernel_policy", ctypes.c_int32), ("mfma_variant", ctypes.c_int32), ("mfma_rows", ctypes.c_int32),
                ("mfma_taps", ctypes.c_int32), ("dw_workgroups", ctypes.c_int32), ("view_workgroups", ctypes.c_int32),
                ("mfma_splits", ctypes.c_int32), ("clock_probe", ctypes.c_void_p)]


class _Desc(ctypes.Structure):
    _fields_ = [("n_out", ctypes.c_int32), ("out_dims", ctypes.POINTER(_Dim)),
                ("n_prim", ctypes.c_int32), ("prims", ctypes.POINTER(_Prim)),
                ("n_in", ctypes.c_int32), ("input_coords", ctypes.POINTER(ctypes.c_int32)),
                ("n_w", ctypes.c_int32), ("weight_coords", ctypes.POINTER(ctypes.c_int32)),
                ("in_dtype", ctypes.c_int), ("out_dtype", ctypes.c_int),
                ("options", ctypes.POINTER(_Options)),
                ("n_more_weights", ctypes.c_int32), ("more_weight_ranks", ctypes.POINTER(ctypes.c_int32)),
                ("more_weight_coords", ctypes.POINTER(ctypes.c_int32))]


class SynoError(RuntimeError):
    def __init__(self, status: int, what: str):
        msg = load_library().syno_status_string(status)
        super().__init__(f"{what}: {msg.decode() if msg else status}")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsyno.so.  There is no fallback: without the built HIP library nothing runs."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2410_23745_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64p, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)
    lib.syno_plan_create.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(vp)]
    lib.syno_plan_destroy.argtypes = [vp]
    for fn in (lib.syno_forward, lib.syno_backward_data, lib.syno_backward_weight):
        fn.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.syno_backward_weight_static.argtypes = [vp, vp, vp, vp, vp]
    lib.syno_plan_workspace_bytes.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.syno_plan_shapes.argtypes = [vp, i32p, i64p, i32p, i64p, i32p, i64p]
    lib.syno_plan_kernel.argtypes = [vp, ctypes.c_int]
    lib.syno_plan_kernel.restype = ctypes.c_char_p
    lib.syno_plan_describe.argtypes = [vp, ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    lib.syno_plan_free_size.argtypes = [vp, ctypes.c_int, i64p]
    lib.syno_debug_gather.argtypes = [vp, ctypes.c_int, vp, vp, ctypes.c_int64, vp, vp, vp]
    lib.syno_debug_gather_host.argtypes = [vp, ctypes.c_int, vp, vp, ctypes.c_int64, vp, vp]
    lib.syno_debug_mfma_rate.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_int32, vp, i64p, vp]
    lib.syno_status_string.argtypes = [ctypes.c_int]
    lib.syno_status_string.restype = ctypes.c_char_p
    vpp = ctypes.POINTER(vp)
    lib.syno_chain_create.argtypes = [ctypes.POINTER(_Desc), ctypes.c_int32, ctypes.POINTER(vp)]
    lib.syno_chain_destroy.argtypes = [vp]
    lib.syno_chain_create_materialized.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(vp)]
    lib.syno_chain_weight_stage.argtypes = [vp]
    lib.syno_chain_stage_weight.argtypes = [vp, ctypes.c_int32]
    lib.syno_chain_stages.argtypes = [vp]
    lib.syno_chain_plan.argtypes = [vp, ctypes.c_int32]
    lib.syno_chain_plan.restype = vp
    lib.syno_chain_workspace_bytes.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.syno_chain_forward.argtypes = [vp, vp, vpp, vpp, vp, vp, vp]
    lib.syno_chain_backward.argtypes = [vp, vp, vpp, vpp, vp, vp, vpp, vp, vp]
    for name in EXPORTS:
        if name not in ("syno_plan_kernel", "syno_status_string", "syno_chain_plan"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


_TORCH_DTYPE = {0: torch.float32, 1: torch.bfloat16}


def _marshal(desc, options=None):
    """OpDesc-like object (+ a dict of syno_plan_options fields) -> (syno_desc, objects that must stay alive
    while it is used)."""
    dims = (_Dim * max(1, len(desc.out_dims)))()
    names = [str(n).encode() for n, _ in desc.out_dims]
    for i, (_, s) in enumerate(desc.out_dims):
        dims[i].name, dims[i].size = names[i], int(s)
    prims = (_Prim * max(1, len(desc.prims)))()
    for i, p in enumerate(desc.prims):
        prims[i].kind = int(p.kind)
        ins = list(p.ins) + [-1] * (2 - len(p.ins))
        outs = list(p.outs) + [-1] * (2 - len(p.outs))
        prims[i].in_[0], prims[i].in_[1] = ins
        prims[i].out[0], prims[i].out[1] = outs
        prims[i].param, prims[i].shift_by, prims[i].shift_coef = int(p.param), int(p.shift_by), int(p.shift_coef)
    ic = (ctypes.c_int32 * max(1, len(desc.input_coords)))(*desc.input_coords)
    wc = (ctypes.c_int32 * max(1, len(desc.weight_coords)))(*desc.weight_coords)
    opt = _Options(**{k: int(v) for k, v in options.items()}) if options else None
    more = [list(w) for w in (getattr(desc, "more_weights", None) or [])]
    ranks = (ctypes.c_int32 * max(1, len(more)))(*[len(w) for w in more])
    flat = [int(c) for w in more for c in w]
    mc = (ctypes.c_int32 * max(1, len(flat)))(*flat)
    d = _Desc(len(desc.out_dims), dims, len(desc.prims), prims, len(desc.input_coords), ic,
              len(desc.weight_coords), wc, int(desc.in_dtype), int(desc.out_dtype),
              ctypes.pointer(opt) if opt is not None else None, len(more), ranks, mc)
    return d, (dims, names, prims, ic, wc, opt, ranks, mc)


class Plan:
    """Owns one syno_plan.  `desc` is an OpDesc-like object (out_dims, prims, input_coords, weight_coords,
    in_dtype, out_dtype); `options` are fields of syno_plan_options (kernel_policy=1: the generic kernels)."""

    def __init__(self, desc, _borrowed=None, _owner=None, **options):
        lib = load_library()
        if _borrowed is not None:
            handle, self._owned, self._owner = ctypes.c_void_p(_borrowed), False, _owner   # a stage of a chain
        else:
            d, _keep = _marshal(desc, options)
            handle = ctypes.c_void_p()
            st = lib.syno_plan_create(ctypes.byref(d), ctypes.byref(handle))
            if st:
                raise SynoError(st, "syno_plan_create")
            self._owned = True
        self._h = handle
        self.in_dtype = _TORCH_DTYPE[int(desc.in_dtype)]
        self.out_dtype = _TORCH_DTYPE[int(desc.out_dtype)]
        xr, wr, orr = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        xs, ws, os_ = (ctypes.c_int64 * 8)(), (ctypes.c_int64 * 8)(), (ctypes.c_int64 * 8)()
        st = lib.syno_plan_shapes(self._h, ctypes.byref(xr), xs, ctypes.byref(wr), ws, ctypes.byref(orr), os_)
        if st:
            raise SynoError(st, "syno_plan_shapes")
        self.x_shape = tuple(xs[:xr.value])
        self.w_shape = tuple(ws[:wr.value])
        self.out_shape = tuple(os_[:orr.value])
        self._ws = {}

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None and getattr(self, "_owned", False):
            _lib.syno_plan_destroy(h)

    # -- queries ---------------------------------------------------------------------------
    def workspace_bytes(self, which: int) -> int:
        n = ctypes.c_size_t()
        st = load_library().syno_plan_workspace_bytes(self._h, which, ctypes.byref(n))
        if st:
            raise SynoError(st, "syno_plan_workspace_bytes")
        return n.value

    def kernel(self, which: int) -> str:
        s = load_library().syno_plan_kernel(self._h, which)
        return s.decode() if s else ""

    def describe(self, which: int) -> str:
        buf = ctypes.create_string_buffer(512)
        st = load_library().syno_plan_describe(self._h, which, buf, 512)
        if st:
            raise SynoError(st, "syno_plan_describe")
        return buf.value.decode()

    def free_size(self, which: int) -> int:
        n = ctypes.c_int64()
        st = load_library().syno_plan_free_size(self._h, which, ctypes.byref(n))
        if st:
            raise SynoError(st, "syno_plan_free_size")
        return n.value

    # -- compute ---------------------------------------------------------------------------
    @staticmethod
    def _numel(shape) -> int:
        n = 1
        for s in shape:
            n *= int(s)
        return n

    def _arg(self, t: torch.Tensor, shape, dtype, what: str) -> int:
        if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype and t.numel() == self._numel(shape)):
            raise ValueError(f"{what}: need a contiguous {dtype} device tensor with {self._numel(shape)} elements")
        if t.data_ptr() % 16:
            raise ValueError(f"{what}: pointer must be 16-byte aligned")
        return t.data_ptr()

    def _workspace(self, which: int, device, workspace: Optional[torch.Tensor]) -> int:
        need = self.workspace_bytes(which)
        if need == 0:
            return 0
        if workspace is None:
            workspace = self._ws.get((which, device))
            if workspace is None:
                workspace = self._ws[(which, device)] = torch.empty(need, dtype=torch.uint8, device=device)
        if workspace.numel() * workspace.element_size() < need:
            raise ValueError("workspace too small")
        return workspace.data_ptr()

    def _call(self, fn, which, a, a_shape, b, b_shape, out, out_shape, out_dtype, workspace, what):
        pa = self._arg(a, a_shape, self.in_dtype, what + " first input")
        pb = self._arg(b, b_shape, self.in_dtype, what + " second input")
        if out is None:
            out = torch.empty(out_shape if out_shape else (1,), dtype=out_dtype, device=a.device)
        po = self._arg(out, out_shape, out_dtype, what + " output")
        ws = self._workspace(which, a.device, workspace)
        stream = torch.cuda.current_stream(a.device).cuda_stream
        st = fn(self._h, pa, pb, po, ws, stream)
        if st:
            raise SynoError(st, what)
        return out

    def bind(self, which: int, a, b, out, workspace=None):
        """Checks the arguments of call `which` once and returns a function of no arguments that enqueues it on the
        stream that is current NOW (for timing loops: the per-call marshalling is out of the way).  Operand order as
        in forward / backward_data / backward_weight."""
        shapes = ((self.x_shape, self.w_shape, self.out_shape, self.out_dtype),
                  (self.out_shape, self.w_shape, self.x_shape, self.out_dtype),
                  (self.x_shape, self.out_shape, self.w_shape, torch.float32))[which]
        name = ("syno_forward", "syno_backward_data", "syno_backward_weight")[which]
        pa = self._arg(a, shapes[0], self.in_dtype, name + " first input")
        pb = self._arg(b, shapes[1], self.in_dtype, name + " second input")
        po = self._arg(out, shapes[2], shapes[3], name + " output")
        ws = self._workspace(which, a.device, workspace)
        stream = torch.cuda.current_stream(a.device).cuda_stream
        fn, h = getattr(load_library(), name), self._h

        def launch():
            st = fn(h, pa, pb, po, ws, stream)
            if st:
                raise SynoError(st, name)
        return launch

    def forward(self, X, W, out=None, workspace=None):
        return self._call(load_library().syno_forward, FWD, X, self.x_shape, W, self.w_shape, out, self.out_shape,
                          self.out_dtype, workspace, "syno_forward")

    def backward_data(self, G, W, dX=None, workspace=None):
        return self._call(load_library().syno_backward_data, BWD_DATA, G, self.out_shape, W, self.w_shape, dX,
                          self.x_shape, self.out_dtype, workspace, "syno_backward_data")

    def backward_weight(self, X, G, dW=None, workspace=None):
        return self._call(load_library().syno_backward_weight, BWD_WEIGHT, X, self.x_shape, G, self.out_shape, dW,
                          self.w_shape, torch.float32, workspace, "syno_backward_weight")

    def backward_weight_static(self, X, G, dW):
        """syno_backward_weight on the library's static scratch memory; `dW` must be given (nothing is allocated)."""
        px = self._arg(X, self.x_shape, self.in_dtype, "syno_backward_weight_static X")
        pg = self._arg(G, self.out_shape, self.in_dtype, "syno_backward_weight_static G")
        po = self._arg(dW, self.w_shape, torch.float32, "syno_backward_weight_static dW")
        st = load_library().syno_backward_weight_static(self._h, px, pg, po, torch.cuda.current_stream(X.device).cuda_stream)
        if st:
            raise SynoError(st, "syno_backward_weight_static")
        return dW

    def debug_gather_host(self, which: int, t_flat, q_flat):
        """Same maps as `debug_gather`, evaluated on the host (numpy int64 in, numpy int32 out)."""
        import numpy as np
        t = np.ascontiguousarray(t_flat, dtype=np.int64)
        q = np.ascontiguousarray(q_flat, dtype=np.int64)
        if t.shape != q.shape:
            raise ValueError("debug_gather_host: length mismatch")
        a = np.empty(t.shape, dtype=np.int32)
        b = np.empty(t.shape, dtype=np.int32)
        st = load_library().syno_debug_gather_host(self._h, which, t.ctypes.data, q.ctypes.data, t.size,
                                                   a.ctypes.data, b.ctypes.data)
        if st:
            raise SynoError(st, "syno_debug_gather_host")
        return a, b

    def debug_gather(self, which: int, t_flat: torch.Tensor, q_flat: torch.Tensor):
        """Index maps of contraction `which` at the listed (target, free point) pairs; int64 device tensors in,
        two int32 device tensors out (-1 where the term does not exist)."""
        for t in (t_flat, q_flat):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.int64):
                raise ValueError("debug_gather: need contiguous int64 device tensors")
        if t_flat.numel() != q_flat.numel():
            raise ValueError("debug_gather: length mismatch")
        n = t_flat.numel()
        a = torch.empty(n, dtype=torch.int32, device=t_flat.device)
        b = torch.empty(n, dtype=torch.int32, device=t_flat.device)
        stream = torch.cuda.current_stream(t_flat.device).cuda_stream
        st = load_library().syno_debug_gather(self._h, which, t_flat.data_ptr(), q_flat.data_ptr(), n, a.data_ptr(),
                                              b.data_ptr(), stream)
        if st:
            raise SynoError(st, "syno_debug_gather")
        return a, b


def mfma_rate(dtype: int, iters: int = 2000, workgroups: int = 512):
    """(flop, launch) of the library's MFMA-only measurement kernel: `launch()` enqueues it on the current stream."""
    lib = load_library()
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    flop = ctypes.c_int64()
    stream = torch.cuda.current_stream().cuda_stream

    def launch():
        st = lib.syno_debug_mfma_rate(int(dtype), iters, workgroups, out.data_ptr(), ctypes.byref(flop), stream)
        if st:
            raise SynoError(st, "syno_debug_mfma_rate")
    launch()
    return flop.value, launch


class _StageTypes:
    def __init__(self, in_dtype, out_dtype):
        self.in_dtype, self.out_dtype = in_dtype, out_dtype


class Chain:
    """Owns one syno_chain: an operator evaluated as consecutive single-weight stages.  `descs` is a list of
    OpDesc-like objects.  `stages[i]` is a borrowed Plan for queries (shapes, kernel names)."""

    def __init__(self, descs, _materialize=None, **options):
        lib = load_library()
        handle = ctypes.c_void_p()
        if _materialize is not None:
            d, keep = _marshal(_materialize, options)
            st = lib.syno_chain_create_materialized(ctypes.byref(d), ctypes.byref(handle))
            if st:
                raise SynoError(st, "syno_chain_create_materialized")
        else:
            arr = (_Desc * max(1, len(descs)))()
            keep = []
            for i, d in enumerate(descs):
                arr[i], k = _marshal(d, options)
                keep.append(k)
            st = lib.syno_chain_create(arr, len(descs), ctypes.byref(handle))
            if st:
                raise SynoError(st, "syno_chain_create")
        self._h = handle
        n = lib.syno_chain_stages(self._h)
        self.weight_stage = lib.syno_chain_weight_stage(self._h)     # -1: every stage has its own weight
        # per stage: which of the graph's weights it multiplies with (-1: none); W / dW lists are indexed by stage
        self.stage_weight = [lib.syno_chain_stage_weight(self._h, i) for i in range(n)]
        if _materialize is not None:
            # stage i reads the graph's input type; only the last stage writes the graph's output type
            descs = [_StageTypes(_materialize.in_dtype, _materialize.in_dtype if i + 1 < n else _materialize.out_dtype)
                     for i in range(n)]
        self.stages = [Plan(descs[i], _borrowed=lib.syno_chain_plan(self._h, i), _owner=self) for i in range(n)]
        # dX has the first stage's output type; for a materialised graph, the graph's
        self.dx_dtype = _TORCH_DTYPE[int(_materialize.out_dtype)] if _materialize is not None else self.stages[0].out_dtype
        self._ws = {}

    @classmethod
    def materialized(cls, desc, **options):
        """The chain the library's materialised-reduction pass cuts one single-weight pGraph into."""
        return cls(None, _materialize=desc, **options)

    def _own(self, i: int) -> bool:
        return self.stage_weight[i] >= 0

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.syno_chain_destroy(h)

    def workspace_bytes(self, which: int) -> int:
        n = ctypes.c_size_t()
        st = load_library().syno_chain_workspace_bytes(self._h, which, ctypes.byref(n))
        if st:
            raise SynoError(st, "syno_chain_workspace_bytes")
        return n.value

    def _workspace(self, which, device, workspace):
        need = self.workspace_bytes(which)
        if need == 0:
            return 0
        if workspace is None:
            workspace = self._ws.get((which, device))
            if workspace is None:
                workspace = self._ws[(which, device)] = torch.empty(need, dtype=torch.uint8, device=device)
        if workspace.numel() * workspace.element_size() < need:
            raise ValueError("workspace too small")
        return workspace.data_ptr()

    @staticmethod
    def _ptrs(values):
        return (ctypes.c_void_p * max(1, len(values)))(*values)

    def new_activations(self, device):
        """Device buffers for the outputs of all stages but the last."""
        return [torch.empty(p.out_shape, dtype=p.out_dtype, device=device) for p in self.stages[:-1]]

    def forward(self, X, Ws, acts=None, out=None, workspace=None):
        """Returns (out, acts)."""
        first, last = self.stages[0], self.stages[-1]
        px = first._arg(X, first.x_shape, first.in_dtype, "syno_chain_forward X")
        if len(Ws) != len(self.stages):
            raise ValueError("syno_chain_forward: one weight entry per stage (None for a stage without a weight)")
        pw = [p._arg(w, p.w_shape, p.in_dtype, f"syno_chain_forward W[{i}]") if self._own(i) else 0
              for i, (p, w) in enumerate(zip(self.stages, Ws))]
        if acts is None:
            acts = self.new_activations(X.device)
        pa = [p._arg(a, p.out_shape, p.out_dtype, f"syno_chain_forward act[{i}]") for i, (p, a) in
              enumerate(zip(self.stages[:-1], acts))]
        if len(pa) != len(self.stages) - 1:
            raise ValueError("syno_chain_forward: one activation buffer per stage but the last")
        if out is None:
            out = torch.empty(last.out_shape, dtype=last.out_dtype, device=X.device)
        po = last._arg(out, last.out_shape, last.out_dtype, "syno_chain_forward out")
        ws = self._workspace(0, X.device, workspace)
        stream = torch.cuda.current_stream(X.device).cuda_stream
        st = load_library().syno_chain_forward(self._h, px, self._ptrs(pw), self._ptrs(pa), po, ws, stream)
        if st:
            raise SynoError(st, "syno_chain_forward")
        return out, acts

    def backward(self, X, Ws, acts, G, dX=None, dWs=None, want_dx=True, workspace=None):
        """Returns (dX or None, dWs)."""
        first, last = self.stages[0], self.stages[-1]
        px = first._arg(X, first.x_shape, first.in_dtype, "syno_chain_backward X")
        pg = last._arg(G, last.out_shape, last.in_dtype, "syno_chain_backward G")
        if len(Ws) != len(self.stages):
            raise ValueError("syno_chain_backward: one weight entry per stage (None for a stage without a weight)")
        pw = [p._arg(w, p.w_shape, p.in_dtype, f"syno_chain_backward W[{i}]") if self._own(i) else 0
              for i, (p, w) in enumerate(zip(self.stages, Ws))]
        pa = [p._arg(a, p.out_shape, p.out_dtype, f"syno_chain_backward act[{i}]") for i, (p, a) in
              enumerate(zip(self.stages[:-1], acts))]
        if len(pw) != len(self.stages) or len(pa) != len(self.stages) - 1:
            raise ValueError("syno_chain_backward: one weight per stage, one activation per stage but the last")
        if dWs is None:
            dWs = [torch.empty(p.w_shape if p.w_shape else (1,), dtype=torch.float32, device=X.device)
                   if self._own(i) else None for i, p in enumerate(self.stages)]
        pdw = [p._arg(d, p.w_shape, torch.float32, f"syno_chain_backward dW[{i}]") if self._own(i) else 0
               for i, (p, d) in enumerate(zip(self.stages, dWs))]
        pdx = 0
        if want_dx:
            if dX is None:
                dX = torch.empty(first.x_shape, dtype=self.dx_dtype, device=X.device)
            pdx = first._arg(dX, first.x_shape, self.dx_dtype, "syno_chain_backward dX")
        ws = self._workspace(1, X.device, workspace)
        stream = torch.cuda.current_stream(X.device).cuda_stream
        st = load_library().syno_chain_backward(self._h, px, self._ptrs(pw), self._ptrs(pa), pg, pdx,
                                                self._ptrs(pdw), ws, stream)
        if st:
            raise SynoError(st, "syno_chain_backward")
        return (dX if want_dx else None), dWs
