"""The synthetic workloads: pGraphs of the operators that are evaluated, and
their seeded input tensors.

The operators are written down with the primitives of Table 1 of the paper;
the convolution follows Fig. 2 / Listing 1 (three Reduce, three Share, two
Unfold, C_out matched to the weight), the small examples follow Table 2.
Shapes are ResNet-18 stage shapes; values are i.i.d. from the distribution
each workload names.  These stand in for the image-classification layers the
paper measures on; no dataset is involved.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

from .descriptor import BF16, F32, Builder, OpDesc
from .rng import Stream, bf16_bits_to_f32, to_bf16_bits


# ----------------------------------------------------------------------------
# pGraphs
# ----------------------------------------------------------------------------
def conv2d(N, C, Co, H, W, KH=3, KW=None, in_dtype=F32, out_dtype=F32, w_order=(0, 1, 2, 3), stride=1) -> OpDesc:
    """out[n,co,h,w] = sum_{c,kh,kw} X[n,c,S*h+kh-KH/2,S*w+kw-KW/2] * Wt[co,c,kh,kw]  (S = stride; H, W are the output's
    extents, the input's are S*H, S*W).
    `w_order` lists which of (co, c, kh, kw) each weight axis is, outermost first (weights may be laid out in any
    order: section 6 of the paper lets them be reshaped offline)."""
    KW = KH if KW is None else KW
    b = Builder([("n", N), ("co", Co), ("h", H), ("w", W)],
                name=f"conv{KH}x{KW}{f's{stride}' if stride > 1 else ''}_C{C}_Co{Co}_{H}x{W}_N{N}")
    n, co, h, w = 0, 1, 2, 3
    c = b.reduce(C)
    cx, cw = b.share(c)
    kh = b.reduce(KH)
    khx, khw = b.share(kh)
    kw = b.reduce(KW)
    kwx, kww = b.share(kw)
    hh = b.unfold(b.stride(h, stride) if stride > 1 else h, khx)
    ww = b.unfold(b.stride(w, stride) if stride > 1 else w, kwx)
    waxes = [co, cw, khw, kww]
    return b.finish([n, cx, hh, ww], [waxes[i] for i in w_order], in_dtype, out_dtype)


def flat_window(N, C, Co, A, B, K=3, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """A window over two flattened axes (an Unfold below a Merge, the left side of the paper's Fig. 4(c)):
    out[n,co,i] = sum_{c,j} X[n, c, u div B, u mod B] * Wt[co,c,j] with u = i + j - K/2, zero where u is outside [0, A*B)."""
    b = Builder([("n", N), ("co", Co), ("i", A * B)], name=f"flat_window_k{K}_C{C}_Co{Co}_{A}x{B}_N{N}")
    c = b.reduce(C)
    cx, cw = b.share(c)
    j = b.reduce(K)
    jx, jw = b.share(j)
    q, r = b.merge(b.unfold(2, jx), B)
    return b.finish([0, cx, q, r], [1, cw, jw], in_dtype, out_dtype)


def grouped_shift_unfold(N, C=256, Co=256, H=14, W=14, groups=4, K=3,
                         in_dtype=BF16, out_dtype=F32, w_order=(0, 1, 2, 3)) -> OpDesc:
    """out[n,co,h,w] = sum_{c',k} Wt[co,c',k] * X[n, g*Cg+c', (h+g) mod H, w+k-K/2],  g = co div (Co/groups)."""
    Og, Cg = Co // groups, C // groups
    b = Builder([("n", N), ("co", Co), ("h", H), ("w", W)], name=f"gshift_unfold_C{C}_g{groups}_{H}x{W}_N{N}")
    n, co, h, w = 0, 1, 2, 3
    g, cop = b.merge(co, Og)
    gx, gw = b.share(g)
    c = b.reduce(Cg)
    cx, cw = b.share(c)
    k = b.reduce(K)
    kx, kw = b.share(k)
    cin = b.split(gx, cx)
    hh = b.shift(h, 0, by=gx, coef=1)
    ww = b.unfold(w, kx)
    waxes = [gw, cop, cw, kw]
    return b.finish([n, cin, hh, ww], [waxes[i] for i in w_order], in_dtype, out_dtype)


def strided_depthwise(N, C, H_out, W_out, S=2, K=3, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """out[n,c,h,w] = sum_{kh,kw} Wt[c,kh,kw] * X[n,c,S*h+kh-K/2,S*w+kw-K/2]."""
    b = Builder([("n", N), ("c", C), ("h", H_out), ("w", W_out)], name=f"dw{K}x{K}s{S}_C{C}_{H_out}x{W_out}_N{N}")
    n, c, h, w = 0, 1, 2, 3
    cx, cw = b.share(c)
    kh = b.reduce(K)
    khx, khw = b.share(kh)
    kw = b.reduce(K)
    kwx, kww = b.share(kw)
    hs = b.stride(h, S)
    ws = b.stride(w, S)
    hh = b.unfold(hs, khx)
    ww = b.unfold(ws, kwx)
    return b.finish([n, cx, hh, ww], [cw, khw, kww], in_dtype, out_dtype)


def window_of_sums_1d(H, k=3, s=2, weight=None, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """The example of the paper's materialised-reduction pass: out[i] = sum_{ik,is} X[s*(i+ik-k/2)+is], i < H/s,
    as ONE loop nest.  weight="k": times Wt[ik]; weight="s": times Wt[is]; None: no weight axes."""
    b = Builder([("i", H // s)], name=f"window_of_sums_H{H}_k{k}_s{s}_{weight}")
    ik, i_s = b.reduce(k), b.reduce(s)
    if weight == "k":
        ikx, ikw = b.share(ik)
        return b.finish([b.split(b.unfold(0, ikx), i_s)], [ikw], in_dtype, out_dtype)
    if weight == "s":
        sx, sw = b.share(i_s)
        return b.finish([b.split(b.unfold(0, ik), sx)], [sw], in_dtype, out_dtype)
    return b.finish([b.split(b.unfold(0, ik), i_s)], [], in_dtype, out_dtype)


def pooled_conv2d(N, C, Co, H, W, S=2, K=3, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """A K x K convolution of S x S block sums, written as ONE loop nest with five Reduces:
    out[n,co,h,w] = sum_{c,kh,kw,sh,sw} Wt[co,c,kh,kw] * X[n, c, S*(h+kh-K/2)+sh, S*(w+kw-K/2)+sw]."""
    b = Builder([("n", N), ("co", Co), ("h", H), ("w", W)], name=f"pooled_conv_C{C}_Co{Co}_{H}x{W}_S{S}_N{N}")
    c = b.reduce(C)
    cx, cw = b.share(c)
    kh = b.reduce(K)
    khx, khw = b.share(kh)
    kw = b.reduce(K)
    kwx, kww = b.share(kw)
    sh, sw = b.reduce(S), b.reduce(S)
    hh = b.split(b.unfold(2, khx), sh)
    ww = b.split(b.unfold(3, kwx), sw)
    return b.finish([0, cx, hh, ww], [1, cw, khw, kww], in_dtype, out_dtype)


def shifted_scale(N, C, H, W, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """A pure view with a per-channel weight (no Reduce): out[n,c,h,w] = Wt[c] * X[n, c, h, (w+1) mod W]."""
    b = Builder([("n", N), ("c", C), ("h", H), ("w", W)], name=f"shift_scale_C{C}_{H}x{W}_N{N}")
    cx, cw = b.share(1)
    ws = b.shift(3, 1)
    return b.finish([0, cx, 2, ws], [cw], in_dtype, out_dtype)


def pixel_unshuffle(N, C, H, W, r=2, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """Space-to-depth as a pure view (Table 2's PixelShuffle read the other way), times a one-element weight:
    out[n, c, i, j, h, w] = X[n, c, r*h+i, r*w+j] * Wt[0]."""
    b = Builder([("n", N), ("c", C), ("i", r), ("j", r), ("h", H), ("w", W)], name=f"pixel_unshuffle_C{C}_{H}x{W}_r{r}_N{N}")
    hh = b.split(4, 2)
    ww = b.split(5, 3)
    return b.finish([0, 1, hh, ww], [], in_dtype, out_dtype)


def matmul(M, N, K, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """Table 2: out[i,j] = sum_k X[i,k] * Wt[k,j]."""
    b = Builder([("i", M), ("j", N)], name=f"mm_{M}x{N}x{K}")
    r = b.reduce(K)
    rx, rw = b.share(r)
    return b.finish([0, rx], [rw, 1], in_dtype, out_dtype)


def operator1_stage1(N, Cin, Co, H, W, g=4, s=2, k1=3, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """First stage of Operator 1 (Fig. 7): a 1 x k1 window along w, contracted over the channels of one group
    only; the window iterator k is Shared with the weight but NOT Reduced, so it survives as an output axis.

    Z[n,d,gi,k,h,w] = sum_{c'} X[n, gi*Cg+c', h, w+k-k1/2] * w1[d, gi*Cg+c', k],   Cg = Cin/g, d < Co/g/s."""
    D, Cg = Co // g // s, Cin // g
    b = Builder([("n", N), ("d", D), ("gi", g), ("k", k1), ("h", H), ("w", W)],
                name=f"op1_stage1_C{Cin}_Co{Co}_g{g}_s{s}_{H}x{W}_N{N}")
    n, d, gi, k, h, w = range(6)
    c = b.reduce(Cg)
    cx, cw = b.share(c)
    gx, gw = b.share(gi)
    kx, kw = b.share(k)
    cin = b.split(gx, cx)
    ww = b.unfold(w, kx)
    return b.finish([n, cin, h, ww], [d, gw, cw, kw], in_dtype, out_dtype)


def operator1_graph(N, Cin, Co, H, W, g=4, s=2, k1=3, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """Operator 1 (Fig. 7) as ONE pGraph with two weights:
    out[n,co,h,w] = sum_{d,gi,k,j,c'} X[n, gi*Cg+c', h+j-k1/2, w+k-k1/2] * w1[d,gi,c',k] * w2[co,d,gi,k,j].
    The iterators gi and k reach X and both weights (two Shares each), d reaches the two weights only, j reaches X
    and w2, c' reaches X and w1; co is matched to w2.  w2[co,d,gi,k,j] is the w2[Co, k1*Co/s, k1] of the staged form."""
    D, Cg = Co // g // s, Cin // g
    b = Builder([("n", N), ("co", Co), ("h", H), ("w", W)], name=f"op1_graph_C{Cin}_Co{Co}_g{g}_s{s}_{H}x{W}_N{N}")
    n, co, h, w = range(4)
    d = b.reduce(D)
    d_w1, d_w2 = b.share(d)
    gi = b.reduce(g)
    gi_a, gi_w2 = b.share(gi)
    gi_x, gi_w1 = b.share(gi_a)
    k = b.reduce(k1)
    k_a, k_w2 = b.share(k)
    k_x, k_w1 = b.share(k_a)
    j = b.reduce(k1)
    j_x, j_w2 = b.share(j)
    c = b.reduce(Cg)
    c_x, c_w1 = b.share(c)
    cin = b.split(gi_x, c_x)
    hh = b.unfold(h, j_x)
    ww = b.unfold(w, k_x)
    return b.finish([n, cin, hh, ww], [d_w1, gi_w1, c_w1, k_w1], in_dtype, out_dtype,
                    more_weights=[[co, d_w2, gi_w2, k_w2, j_w2]])


def operator1_stage2(N, Co, H, W, s=2, k1=3, in_dtype=F32, out_dtype=F32) -> OpDesc:
    """Second stage of Operator 1: the first stage's axes (d,gi,k) flattened into k1*Co/s channels, a k1 x 1
    window along h, everything contracted with w2[Co, (k1*Co/s)*k1]."""
    return conv2d(N, k1 * Co // s, Co, H, W, k1, 1, in_dtype, out_dtype)


# ----------------------------------------------------------------------------
# Workloads = pGraph + seeded tensors
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    desc: OpDesc
    x_shape: tuple
    w_shape: tuple
    out_shape: tuple
    X: np.ndarray                 # float32 values (already rounded to bf16 when in_dtype is BF16)
    W: np.ndarray
    G: Optional[np.ndarray]       # upstream gradient, same shape as out (None for forward-only workloads)
    X_bits: Optional[np.ndarray]  # uint16 bf16 patterns when in_dtype is BF16
    W_bits: Optional[np.ndarray]
    G_bits: Optional[np.ndarray]
    flops: int                    # 2 * prod(output iterators) * prod(Reduce sizes)  (section 8 of the paper)


def _finish(desc, xs, ws, os, X, W, G, red) -> Workload:
    Xb = Wb = Gb = None
    if desc.in_dtype == BF16:
        Xb, Wb = to_bf16_bits(X), to_bf16_bits(W)
        X, W = bf16_bits_to_f32(Xb), bf16_bits_to_f32(Wb)
        if G is not None:
            Gb = to_bf16_bits(G)
            G = bf16_bits_to_f32(Gb)
    flops = 2 * int(np.prod(os)) * int(red)
    return Workload(desc, tuple(xs), tuple(ws), tuple(os), X, W, G, Xb, Wb, Gb, flops)


def make_conv(N, C, H, seed=0, bf16=False, Co=None, Wd=None, K=3, with_grad=False, out_bf16=False,
              w_order=(0, 1, 2, 3), stride=1) -> Workload:
    """H, Wd: the output's extents (the input is `stride` times as large)."""
    Co = C if Co is None else Co
    Wd = H if Wd is None else Wd
    desc = conv2d(N, C, Co, H, Wd, K, K, BF16 if bf16 else F32, BF16 if out_bf16 else F32, w_order, stride)
    s = Stream(seed)
    nat = (Co, C, K, K)
    xs, ws, os = (N, C, stride * H, stride * Wd), tuple(nat[i] for i in w_order), (N, Co, H, Wd)
    X = s.normal(xs)
    W = s.uniform_pm(1.0 / np.sqrt(K * K * C), ws)
    G = s.normal(os) if with_grad else None
    return _finish(desc, xs, ws, os, X, W, G, C * K * K)


def make_flat_window(N, C, Co, A, B, K=3, seed=0, bf16=False, with_grad=False) -> Workload:
    desc = flat_window(N, C, Co, A, B, K, BF16 if bf16 else F32, F32)
    s = Stream(seed)
    xs, ws, os = (N, C, A, B), (Co, C, K), (N, Co, A * B)
    X = s.normal(xs)
    W = s.uniform_pm(1.0 / np.sqrt(K * C), ws)
    G = s.normal(os) if with_grad else None
    return _finish(desc, xs, ws, os, X, W, G, C * K)


def make_gshift(N, seeds=(0, 0, 0), with_grad=False, C=256, H=14, Wd=14, groups=4, K=3, out_bf16=False,
                bf16=True, w_order=(0, 1, 2, 3)) -> Workload:
    desc = grouped_shift_unfold(N, C, C, H, Wd, groups, K, BF16 if bf16 else F32, BF16 if out_bf16 else F32, w_order)
    Cg = C // groups
    nat = (groups, Cg, Cg, K)
    # (the natural order [g, co', c', k] is the contiguous Wt[C, Cg, K] the workload names)
    xs, ws, os = (N, C, H, Wd), ((C, Cg, K) if tuple(w_order) == (0, 1, 2, 3) else tuple(nat[i] for i in w_order)), (N, C, H, Wd)
    streams: Dict[int, Stream] = {}

    def st(seed):
        return streams.setdefault(seed, Stream(seed))

    X = st(seeds[0]).normal(xs)
    W = st(seeds[1]).uniform_pm(1.0 / np.sqrt(Cg * K), ws)
    G = st(seeds[2]).normal(os) if with_grad else None
    return _finish(desc, xs, ws, os, X, W, G, Cg * K)


def make_depthwise(N, C, H_in, seed=0, S=2, K=3, with_grad=False) -> Workload:
    Ho = H_in // S
    desc = strided_depthwise(N, C, Ho, Ho, S, K, F32, F32)
    s = Stream(seed)
    xs, ws, os = (N, C, H_in, H_in), (C, K, K), (N, C, Ho, Ho)
    X = s.normal(xs)
    W = s.uniform_pm(1.0 / 3.0, ws)
    G = s.normal(os) if with_grad else None
    return _finish(desc, xs, ws, os, X, W, G, K * K)


@dataclass
class ChainWorkload:
    """An operator evaluated as consecutive stages; the output of one stage is the data input of the next."""
    descs: list
    x_shape: tuple
    w_shapes: list
    inter_shapes: list            # shapes of the tensors between the stages
    out_shape: tuple
    X: np.ndarray
    Ws: list
    G: Optional[np.ndarray]
    X_bits: Optional[np.ndarray]
    Ws_bits: Optional[list]
    G_bits: Optional[np.ndarray]
    flops: int                    # sum over the stages of 2 * prod(output iterators) * prod(Reduce sizes)


def make_operator1(N, C, H, seed=0, bf16=False, Co=None, Wd=None, g=4, s=2, k1=3, with_grad=False,
                   out_f32=False) -> ChainWorkload:
    """Operator 1 of the paper (Fig. 7) as its two materialised stages, on a ResNet-style layer shape.
    Weights ~ U(+-1/sqrt(fan_in)) per stage; the whole chain runs in one element type (out_f32: bf16 inputs and
    intermediate, fp32 result)."""
    Co = C if Co is None else Co
    Wd = H if Wd is None else Wd
    dt = BF16 if bf16 else F32
    D, Cg, C2 = Co // g // s, C // g, k1 * Co // s
    d1 = operator1_stage1(N, C, Co, H, Wd, g, s, k1, dt, dt)
    d2 = operator1_stage2(N, Co, H, Wd, s, k1, dt, F32 if out_f32 else dt)
    st = Stream(seed)
    xs, zs, os = (N, C, H, Wd), (N, D, g, k1, H, Wd), (N, Co, H, Wd)
    w1s, w2s = (D, g, Cg, k1), (Co, C2, k1, 1)
    X = st.normal(xs)
    W1 = st.uniform_pm(1.0 / np.sqrt(Cg), w1s)
    W2 = st.uniform_pm(1.0 / np.sqrt(C2 * k1), w2s)
    G = st.normal(os) if with_grad else None
    Xb = Gb = None
    Wb = None
    if bf16:
        Xb = to_bf16_bits(X)
        X = bf16_bits_to_f32(Xb)
        Wb = [to_bf16_bits(W1), to_bf16_bits(W2)]
        W1, W2 = bf16_bits_to_f32(Wb[0]), bf16_bits_to_f32(Wb[1])
        if G is not None:
            Gb = to_bf16_bits(G)
            G = bf16_bits_to_f32(Gb)
    flops = 2 * int(np.prod(zs)) * Cg + 2 * int(np.prod(os)) * C2 * k1
    return ChainWorkload([d1, d2], xs, [w1s, w2s], [zs], os, X, [W1, W2], G, Xb, Wb, Gb, flops)


RESNET18_STAGES = ((64, 56), (128, 28), (256, 14), (512, 7))


def config0() -> Workload:
    return make_conv(1, 16, 16, seed=0)


def config1(stage: int, bf16: bool, N: int = 32) -> Workload:
    C, H = RESNET18_STAGES[stage]
    return make_conv(N, C, H, seed=0, bf16=bf16)


def config1_train(stage: int, bf16: bool, N: int = 32) -> Workload:
    """configs[1] shapes with an output gradient (seed 0 stream continues into G), for the backward passes."""
    C, H = RESNET18_STAGES[stage]
    return make_conv(N, C, H, seed=0, bf16=bf16, with_grad=True)


def config2(N: int = 32) -> Workload:
    return make_gshift(N, seeds=(0, 0, 0))


def config3(N: int = 64) -> Workload:
    return make_depthwise(N, 128, 56, seed=0)


def config3_train(N: int = 64) -> Workload:
    return make_depthwise(N, 128, 56, seed=0, with_grad=True)


def config4(N: int = 128) -> Workload:
    return make_gshift(N, seeds=(1, 2, 3), with_grad=True)


def operator1(stage: int, bf16: bool, N: int = 32, with_grad: bool = True) -> ChainWorkload:
    """Operator 1 in place of the 3x3 convolution of a ResNet-18 stage (g = 4, s = 2, k1 = 3)."""
    C, H = RESNET18_STAGES[stage]
    return make_operator1(N, C, H, seed=0, bf16=bf16, with_grad=with_grad)


def make_matmul(M, K, N, seed=0, bf16=False, with_grad=False, out_bf16=False) -> Workload:
    """Table 2's matrix multiplication out[i,j] = sum_k X[i,k] * Wt[k,j]; X ~ N(0,1), Wt ~ U(+-1/sqrt(K))."""
    desc = matmul(M, N, K, BF16 if bf16 else F32, BF16 if out_bf16 else F32)
    s = Stream(seed)
    xs, ws, os = (M, K), (K, N), (M, N)
    X = s.normal(xs)
    W = s.uniform_pm(1.0 / np.sqrt(K), ws)
    G = s.normal(os) if with_grad else None
    return _finish(desc, xs, ws, os, X, W, G, K)


def qkv_projection(bf16: bool, tokens: int = 8192, with_grad: bool = True) -> Workload:
    """The matrix product the paper substitutes in GPT-2 (117M: 768 embedding dimensions, Q, K and V projected
    at once): [tokens, 768] x [768, 2304]; 8192 tokens stand for 8 sequences of 1024."""
    return make_matmul(tokens, 768, 2304, seed=0, bf16=bf16, with_grad=with_grad)
