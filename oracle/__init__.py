"""Python face of the CPU checker (`syno_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares nothing with the GPU library: it compiles its own C file with gcc,
marshals an operator description into its own wire format, and works on host arrays in
double precision.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "syno_oracle.c")
_LIB = os.path.join(_HERE, "libsyno_oracle.so")
_lib = None

_I64P = ctypes.POINTER(ctypes.c_int64)
_I32P = ctypes.POINTER(ctypes.c_int32)
_F64P = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the checker with gcc (OpenMP for its outermost loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        for fn in ("oracle_describe", "oracle_forward", "oracle_forward_at", "oracle_backward",
                   "oracle_gather_map", "oracle_threads", "oracle_describe_more", "oracle_forward_multi",
                   "oracle_backward_multi"):
            getattr(_lib, fn).restype = ctypes.c_int
    return _lib


class OracleError(ValueError):
    def __init__(self, code: int):
        names = {-1: "format", -2: "coordinate", -3: "domain", -4: "futile"}
        super().__init__(f"oracle rejected the descriptor: {names.get(code, code)}")
        self.code = code


def _check(rc: int) -> None:
    if rc != 0:
        raise OracleError(rc)


def wire(desc) -> np.ndarray:
    """OpDesc-like object (out_dims, prims, input_coords, weight_coords) -> int64 words."""
    words = [len(desc.out_dims)] + [int(s) for _, s in desc.out_dims]
    words.append(len(desc.prims))
    for p in desc.prims:
        ins = list(p.ins) + [-1] * (2 - len(p.ins))
        outs = list(p.outs) + [-1] * (2 - len(p.outs))
        words += [int(p.kind), ins[0], ins[1], outs[0], outs[1], int(p.param), int(p.shift_by), int(p.shift_coef)]
    words += [len(desc.input_coords)] + [int(c) for c in desc.input_coords]
    words += [len(desc.weight_coords)] + [int(c) for c in desc.weight_coords]
    more = getattr(desc, "more_weights", None) or []
    if more:
        words.append(len(more))
        for w in more:
            words += [len(w)] + [int(c) for c in w]
    return np.asarray(words, dtype=np.int64)


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(t)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def describe(desc):
    """(x_shape, w_shape, reduce_shape) derived from the pGraph."""
    w = wire(desc)
    xr, wr, nr = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    xs, ws = np.zeros(16, np.int64), np.zeros(16, np.int64)
    rs = np.zeros(64, np.int64)
    _check(_load().oracle_describe(_p(w, _I64P), ctypes.c_int64(len(w)), ctypes.byref(xr), _p(xs, _I64P),
                                   ctypes.byref(wr), _p(ws, _I64P), ctypes.byref(nr), _p(rs, _I64P)))
    return tuple(xs[:xr.value].tolist()), tuple(ws[:wr.value].tolist()), tuple(rs[:nr.value].tolist())


def weight_shapes(desc):
    """Shapes of all weights of an operator: the first one, then the further ones (operators with several weights)."""
    w = wire(desc)
    _, ws, _ = describe(desc)
    n, ranks, shapes = ctypes.c_int64(), np.zeros(4, np.int64), np.zeros(64, np.int64)
    _check(_load().oracle_describe_more(_p(w, _I64P), ctypes.c_int64(len(w)), ctypes.byref(n), _p(ranks, _I64P),
                                        _p(shapes, _I64P)))
    return [ws] + [tuple(shapes[16 * k:16 * k + ranks[k]].tolist()) for k in range(n.value)]


def _ptr_array(arrays):
    return (ctypes.c_void_p * len(arrays))(*[a.ctypes.data if a is not None else None for a in arrays])


def forward_multi(desc, X, Ws) -> np.ndarray:
    """out[o] = sum_r X[f] * prod_k W_k[g_k] for an operator with several weights (Fig. 7 of the paper)."""
    w = wire(desc)
    xs, _, _ = describe(desc)
    shapes = weight_shapes(desc)
    X = _f64(X)
    Ws = [_f64(v) for v in Ws]
    assert X.size == int(np.prod(xs)) and len(Ws) == len(shapes)
    assert all(v.size == int(np.prod(s)) for v, s in zip(Ws, shapes)), "weight sizes do not match the pGraph"
    out = np.empty(out_shape(desc), dtype=np.float64)
    _check(_load().oracle_forward_multi(_p(w, _I64P), ctypes.c_int64(len(w)), _p(X, _F64P), _ptr_array(Ws), _p(out, _F64P)))
    return out


def backward_multi(desc, X, Ws, G):
    """(dX, [dW_k]) of L = sum(out*G) for an operator with several weights."""
    w = wire(desc)
    xs, _, _ = describe(desc)
    shapes = weight_shapes(desc)
    X, G = _f64(X), _f64(G)
    Ws = [_f64(v) for v in Ws]
    assert X.size == int(np.prod(xs)) and G.size == int(np.prod(out_shape(desc))) and len(Ws) == len(shapes)
    assert all(v.size == int(np.prod(s)) for v, s in zip(Ws, shapes))
    dX = np.empty(xs, dtype=np.float64)
    dWs = [np.empty(s, dtype=np.float64) for s in shapes]
    _check(_load().oracle_backward_multi(_p(w, _I64P), ctypes.c_int64(len(w)), _p(X, _F64P), _ptr_array(Ws), _p(G, _F64P),
                                         _p(dX, _F64P), _ptr_array(dWs)))
    return dX, dWs


def out_shape(desc):
    return tuple(int(s) for _, s in desc.out_dims)


def forward(desc, X, W) -> np.ndarray:
    w = wire(desc)
    xs, wsh, _ = describe(desc)
    X, W = _f64(X), _f64(W)
    assert X.size == int(np.prod(xs)) and W.size == int(np.prod(wsh)), "tensor sizes do not match the pGraph"
    out = np.empty(out_shape(desc), dtype=np.float64)
    _check(_load().oracle_forward(_p(w, _I64P), ctypes.c_int64(len(w)), _p(X, _F64P), _p(W, _F64P), _p(out, _F64P)))
    return out


def forward_at(desc, X, W, o_flat: Sequence[int]) -> np.ndarray:
    w = wire(desc)
    xs, wsh, _ = describe(desc)
    X, W = _f64(X), _f64(W)
    assert X.size == int(np.prod(xs)) and W.size == int(np.prod(wsh))
    o = np.ascontiguousarray(o_flat, dtype=np.int64)
    assert o.size == 0 or (o.min() >= 0 and o.max() < int(np.prod(out_shape(desc))))
    out = np.empty(o.shape, dtype=np.float64)
    _check(_load().oracle_forward_at(_p(w, _I64P), ctypes.c_int64(len(w)), _p(X, _F64P), _p(W, _F64P),
                                     _p(o, _I64P), ctypes.c_int64(o.size), _p(out, _F64P)))
    return out


def backward(desc, X, W, G, want_dx: bool = True, want_dw: bool = True,
             x_sample: Optional[Sequence[int]] = None, w_sample: Optional[Sequence[int]] = None):
    """(dX, dW).  With x_sample / w_sample (flat indices) only those elements are returned, in order."""
    w = wire(desc)
    xs, wsh, _ = describe(desc)
    X, W, G = _f64(X), _f64(W), _f64(G)
    nx, nw = int(np.prod(xs)), int(np.prod(wsh))
    assert X.size == nx and W.size == nw and G.size == int(np.prod(out_shape(desc)))
    lib = _load()

    def pick(sample, n):
        if sample is None:
            return None, 0
        s = np.asarray(sample, dtype=np.int64)
        assert len(np.unique(s)) == len(s), "sampled indices must be distinct"
        m = np.full(n, -1, dtype=np.int64)
        m[s] = np.arange(len(s), dtype=np.int64)
        return m, len(s)

    xm, nxs = pick(x_sample, nx)
    wm, nws = pick(w_sample, nw)
    dX = np.empty(xs if xm is None else (nxs,), dtype=np.float64) if want_dx else None
    dW = np.empty(wsh if wm is None else (nws,), dtype=np.float64) if want_dw else None
    _check(lib.oracle_backward(_p(w, _I64P), ctypes.c_int64(len(w)), _p(X, _F64P), _p(W, _F64P), _p(G, _F64P),
                               _p(dX, _F64P) if dX is not None else None,
                               _p(dW, _F64P) if dW is not None else None,
                               _p(xm, _I64P) if xm is not None else None, ctypes.c_int64(nxs),
                               _p(wm, _I64P) if wm is not None else None, ctypes.c_int64(nws)))
    return dX, dW


def chain_forward(descs, X, Ws, quantize=None):
    """An operator given as consecutive stages (the result of the materialised-reduction pass of the paper's
    code-generation section; Operator 1 of Fig. 7 is two of them): stage i is evaluated on the output of stage
    i-1, reinterpreted in stage i's input shape (same row-major memory).  Returns every stage's output; the
    last is the operator's.  `quantize`, if given, is applied to each intermediate tensor (the element type the
    intermediate is stored in)."""
    outs = []
    cur = _f64(X)
    for i, (d, W) in enumerate(zip(descs, Ws)):
        cur = forward(d, cur.reshape(-1), W)
        if quantize is not None and i + 1 < len(descs):
            cur = _f64(quantize(cur))
        outs.append(cur)
    return outs


def chain_backward(descs, X, Ws, G, quantize=None):
    """Gradients of L = sum(out*G) through the stages by the chain rule: stage i's gradient with respect to its
    input is the output gradient of stage i-1.  Returns (dX, [dW_i]).  `quantize` is applied to the intermediate
    tensors of the forward sweep and to the intermediate gradients, as in `chain_forward`."""
    acts = [_f64(X)] + chain_forward(descs, X, Ws, quantize)[:-1]
    g = _f64(G)
    dWs = [None] * len(descs)
    for i in range(len(descs) - 1, -1, -1):
        dA, dWs[i] = backward(descs[i], acts[i].reshape(-1), Ws[i], g.reshape(-1))
        g = dA if (quantize is None or i == 0) else _f64(quantize(dA))
    return g, dWs


def gather_map(desc, o_flat, r_flat):
    """Flat offsets into X and W of the listed loop-nest points; both -1 where an Unfold is out of range."""
    w = wire(desc)
    _, _, red = describe(desc)
    o = np.ascontiguousarray(o_flat, dtype=np.int64)
    r = np.ascontiguousarray(r_flat, dtype=np.int64)
    assert o.shape == r.shape
    if o.size:
        assert o.min() >= 0 and o.max() < int(np.prod(out_shape(desc)))
        assert r.min() >= 0 and r.max() < (int(np.prod(red)) if red else 1)
    xo = np.empty(o.shape, dtype=np.int32)
    wo = np.empty(o.shape, dtype=np.int32)
    _check(_load().oracle_gather_map(_p(w, _I64P), ctypes.c_int64(len(w)), _p(o, _I64P), _p(r, _I64P),
                                     ctypes.c_int64(o.size), _p(xo, _I32P), _p(wo, _I32P)))
    return xo, wo


def threads() -> int:
    return int(_load().oracle_threads())
