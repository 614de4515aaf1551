"""Pins of the CPU checker against things fixed outside of it: library routines on special
cases, closed forms, integer identities the paper states, brute-force sums written out by
hand, finite differences.  None of these tests touches the GPU library.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from syno_inputs import BF16, F32, Builder, workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def all_points(desc, oracle):
    _, _, red = oracle.describe(desc)
    n_o = int(np.prod(oracle.out_shape(desc)))
    n_r = int(np.prod(red)) if red else 1
    o, r = np.meshgrid(np.arange(n_o), np.arange(n_r), indexing="ij")
    return o.ravel(), r.ravel(), n_o, n_r


# --------------------------------------------------------------------------------------
# Unfold + Share + Reduce = direct convolution (Listing 1, Fig. 2)
# --------------------------------------------------------------------------------------
def direct_conv(X, W):
    """Listing 1 written as seven explicit loops."""
    N, C, H, Wd = X.shape
    Co, _, KH, KW = W.shape
    out = np.zeros((N, Co, H, Wd))
    for n, co, h, w, c, kh, kw in itertools.product(range(N), range(Co), range(H), range(Wd), range(C),
                                                    range(KH), range(KW)):
        y, x = h + kh - KH // 2, w + kw - KW // 2
        if 0 <= y < H and 0 <= x < Wd:
            out[n, co, h, w] += X[n, c, y, x] * W[co, c, kh, kw]
    return out


@pytest.mark.parametrize("N,C,Co,H,W,KH,KW", [
    (1, 1, 1, 2, 2, 3, 3), (2, 3, 2, 5, 4, 3, 3), (1, 2, 3, 4, 6, 1, 1), (1, 2, 2, 6, 5, 5, 3),
    (1, 2, 2, 5, 5, 2, 2), (1, 1, 2, 6, 4, 4, 2), (1, 3, 1, 3, 7, 3, 5)])
def test_conv_equals_seven_loops(oracle, N, C, Co, H, W, KH, KW):
    d = wl.conv2d(N, C, Co, H, W, KH, KW)
    X, Wt = rnd((N, C, H, W), 1), rnd((Co, C, KH, KW), 2)
    np.testing.assert_allclose(oracle.forward(d, X, Wt), direct_conv(X, Wt), rtol=0, atol=1e-13)


def test_conv_config0_equals_library_conv2d(oracle):
    w = wl.config0()
    ref = torch.nn.functional.conv2d(torch.from_numpy(w.X).double(), torch.from_numpy(w.W).double(), padding=1)
    got = oracle.forward(w.desc, w.X, w.W)
    assert got.shape == (1, 16, 16, 16)
    np.testing.assert_allclose(got, ref.numpy(), rtol=0, atol=1e-12)


def test_conv_even_kernel_matches_library_window(oracle):
    # K even: the window is [-K/2, K-1-K/2] with the floored quotient; torch's padded conv gives H+1 rows, the
    # first H of which use exactly that window.
    N, C, Co, H, W, K = 1, 2, 3, 6, 5, 4
    X, Wt = rnd((N, C, H, W), 3), rnd((Co, C, K, K), 4)
    ref = torch.nn.functional.conv2d(torch.from_numpy(X), torch.from_numpy(Wt), padding=K // 2).numpy()[:, :, :H, :W]
    np.testing.assert_allclose(oracle.forward(wl.conv2d(N, C, Co, H, W, K, K), X, Wt), ref, rtol=0, atol=1e-12)


def test_tiny_conv_hand_enumerated(oracle):
    # N=C=Co=1, H=W=2, K=3: every output is an explicit sum of four products.
    X = np.array([[1.0, 2.0], [3.0, 5.0]]).reshape(1, 1, 2, 2)
    W = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)   # W[kh,kw] = 3*kh + kw + 1
    out = oracle.forward(wl.conv2d(1, 1, 1, 2, 2), X, W).reshape(2, 2)
    # out[h,w] = sum_{y,x} X[y,x] * W[y-h+1, x-w+1]
    assert out[0, 0] == 1 * 5 + 2 * 6 + 3 * 8 + 5 * 9
    assert out[0, 1] == 1 * 4 + 2 * 5 + 3 * 7 + 5 * 8
    assert out[1, 0] == 1 * 2 + 2 * 3 + 3 * 5 + 5 * 6
    assert out[1, 1] == 1 * 1 + 2 * 2 + 3 * 4 + 5 * 5


def test_one_hot_input_gives_flipped_stencil(oracle):
    C, Co, H, W = 3, 2, 5, 6
    Wt = rnd((Co, C, 3, 3), 5)
    c, y, x = 1, 2, 3
    X = np.zeros((1, C, H, W))
    X[0, c, y, x] = 1.0
    out = oracle.forward(wl.conv2d(1, C, Co, H, W), X, Wt)
    for co, h, w in itertools.product(range(Co), range(H), range(W)):
        kh, kw = y - h + 1, x - w + 1
        exp = Wt[co, c, kh, kw] if 0 <= kh < 3 and 0 <= kw < 3 else 0.0
        assert out[0, co, h, w] == exp


# --------------------------------------------------------------------------------------
# Closed forms with all-ones tensors: count the taps that fall inside the domain
# --------------------------------------------------------------------------------------
def edge(n, size):
    return 3 - (n == 0) - (n == size - 1)


def test_all_ones_conv(oracle):
    C, H, W = 5, 6, 7
    out = oracle.forward(wl.conv2d(2, C, 3, H, W), np.ones((2, C, H, W)), np.ones((3, C, 3, 3)))
    for h, w in itertools.product(range(H), range(W)):
        assert np.all(out[:, :, h, w] == C * edge(h, H) * edge(w, W))


def test_all_ones_grouped_shift_unfold(oracle):
    d = wl.grouped_shift_unfold(2, 256, 256, 14, 14, 4, 3)
    out = oracle.forward(d, np.ones((2, 256, 14, 14)), np.ones((256, 64, 3)))
    for w in range(14):
        assert np.all(out[:, :, :, w] == 64 * edge(w, 14))     # the cyclic Shift on H never leaves the domain


def test_all_ones_strided_depthwise(oracle):
    d = wl.strided_depthwise(1, 4, 7, 7)
    out = oracle.forward(d, np.ones((1, 4, 14, 14)), np.ones((4, 3, 3)))
    for h, w in itertools.product(range(7), range(7)):
        assert np.all(out[0, :, h, w] == (3 - (h == 0)) * (3 - (w == 0)))


# --------------------------------------------------------------------------------------
# Grouped shift-unfold and strided depthwise against library formulations
# --------------------------------------------------------------------------------------
def test_grouped_shift_unfold_equals_roll_plus_grouped_conv(oracle):
    N, C, H, W, G, K = 2, 8, 5, 6, 4, 3
    Cg = C // G
    d = wl.grouped_shift_unfold(N, C, C, H, W, G, K, F32, F32)
    X, Wt = rnd((N, C, H, W), 6), rnd((C, Cg, K), 7)
    # out[n,co,h,w] = sum W[co,c',k] X[n, g*Cg+c', (h+g)%H, w+k-1]: roll each group's rows up by g, then a 1xK
    # grouped convolution.
    Xr = X.copy()
    for g in range(G):
        Xr[:, g * Cg:(g + 1) * Cg] = np.roll(X[:, g * Cg:(g + 1) * Cg], -g, axis=2)
    ref = torch.nn.functional.conv2d(torch.from_numpy(Xr), torch.from_numpy(Wt.reshape(C, Cg, 1, K)),
                                     padding=(0, 1), groups=G).numpy()
    np.testing.assert_allclose(oracle.forward(d, X, Wt), ref, rtol=0, atol=1e-12)


def test_strided_depthwise_is_stride1_result_sampled(oracle):
    N, C, Hin = 2, 3, 8
    X, Wt = rnd((N, C, Hin, Hin), 8), rnd((C, 3, 3), 9)
    full = torch.nn.functional.conv2d(torch.from_numpy(X), torch.from_numpy(Wt.reshape(C, 1, 3, 3)), padding=1,
                                      groups=C).numpy()
    got = oracle.forward(wl.strided_depthwise(N, C, Hin // 2, Hin // 2), X, Wt)
    np.testing.assert_allclose(got, full[:, :, ::2, ::2], rtol=0, atol=1e-12)


# --------------------------------------------------------------------------------------
# Table 2 examples: mm, AvgPool1d (a sum, no 1/s), PixelShuffle
# --------------------------------------------------------------------------------------
def test_mm_equals_matmul(oracle):
    M, N, K = 5, 7, 6
    X, Wt = rnd((M, K), 10), rnd((K, N), 11)
    np.testing.assert_allclose(oracle.forward(wl.matmul(M, N, K), X, Wt), X @ Wt, rtol=0, atol=1e-13)


def avgpool1d(Hs, s):
    b = Builder([("i", Hs)])
    r = b.reduce(s)
    v = b.split(0, r)
    return b.finish([v], [])


def test_avgpool_is_windowed_sum(oracle):
    Hs, s = 5, 3
    X = rnd((Hs * s,), 12)
    got = oracle.forward(avgpool1d(Hs, s), X, np.ones(1))
    np.testing.assert_allclose(got, X.reshape(Hs, s).sum(1), rtol=0, atol=1e-14)


def pixel_shuffle(H, B):
    b = Builder([("i", H)])
    q, r = b.merge(0, B)
    v = b.split(r, q)
    return b.finish([v], [])


def test_pixel_shuffle_map_matches_paper_formula(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "pixel_shuffle_map.txt")) if l.strip() and l[0] != "#"]
    for H, B, *vals in ([int(t) for t in r] for r in rows):
        d = pixel_shuffle(H, B)
        xo, _ = oracle.gather_map(d, np.arange(H), np.zeros(H, dtype=np.int64))
        assert xo.tolist() == vals
        assert xo.tolist() == [(H // B) * (i % B) + i // B for i in range(H)]
        assert sorted(xo.tolist()) == list(range(H))      # a permutation: nothing dropped, nothing repeated


# --------------------------------------------------------------------------------------
# Split / Merge / Stride integer identities (sections 3 and 6)
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,B", [(12, 3), (12, 4), (7, 7), (8, 1)])
def test_split_of_merge_is_identity(oracle, N, B):
    b = Builder([("i", N)])
    q, r = b.merge(0, B)
    v = b.split(q, r)
    xo, _ = oracle.gather_map(b.finish([v], []), np.arange(N), np.zeros(N, dtype=np.int64))
    assert xo.tolist() == list(range(N))


@pytest.mark.parametrize("G,B", [(3, 4), (5, 2)])
def test_merge_of_split_is_identity(oracle, G, B):
    b = Builder([("i", G), ("j", B)])
    v = b.split(0, 1)
    q, r = b.merge(v, B)
    xo, _ = oracle.gather_map(b.finish([q, r], []), np.arange(G * B), np.zeros(G * B, dtype=np.int64))
    assert xo.tolist() == list(range(G * B))


@pytest.mark.parametrize("A,B,C", [(2, 3, 4), (3, 2, 5), (1, 4, 2)])
def test_merge_above_split_rewrite(oracle, A, B, C):
    # [(C*i+j)/(B*C), (C*i+j)%(B*C)] = [i/B, C*(i%B)+j] for i < A*B, j < C
    b = Builder([("i", A * B), ("j", C)])
    v = b.split(0, 1)
    q, r = b.merge(v, B * C)
    left = b.finish([q, r], [])
    b = Builder([("i", A * B), ("j", C)])
    q, r = b.merge(0, B)
    v = b.split(r, 1)
    right = b.finish([q, v], [])
    n = A * B * C
    z = np.zeros(n, dtype=np.int64)
    assert oracle.describe(left)[0] == oracle.describe(right)[0] == (A, B * C)
    assert oracle.gather_map(left, np.arange(n), z)[0].tolist() == oracle.gather_map(right, np.arange(n), z)[0].tolist()


@pytest.mark.parametrize("A,B,C", [(2, 3, 4), (3, 5, 2)])
def test_stride_mod_identity(oracle, A, B, C):
    # (B*i) % (B*C) = B * (i % C)
    n = A * C
    b = Builder([("i", n)])
    s = b.stride(0, B)
    q, r = b.merge(s, B * C)
    left = b.finish([q, r], [])
    b = Builder([("i", n)])
    q, r = b.merge(0, C)
    s = b.stride(r, B)
    right = b.finish([q, s], [])
    z = np.zeros(n, dtype=np.int64)
    lo = oracle.gather_map(left, np.arange(n), z)[0].tolist()
    assert lo == oracle.gather_map(right, np.arange(n), z)[0].tolist()
    assert lo == [(i // C) * (B * C) + B * (i % C) for i in range(n)]


# --------------------------------------------------------------------------------------
# Shift
# --------------------------------------------------------------------------------------
def shift_chain(N, shifts):
    b = Builder([("i", N)])
    v = 0
    for s in shifts:
        v = b.shift(v, s)
    return b.finish([v], [])


def test_shift_by_one_is_roll(oracle):
    N = 7
    X = rnd((N,), 13)
    got = oracle.forward(shift_chain(N, [1]), X, np.ones(1))
    np.testing.assert_array_equal(got, np.roll(X, -1))          # out[i] = X[(i+1) % N]


def test_shift_plus_minus_is_identity(oracle):
    N = 5
    z = np.zeros(N, dtype=np.int64)
    for s in range(-2 * N, 2 * N + 1):
        xo, _ = oracle.gather_map(shift_chain(N, [s, -s]), np.arange(N), z)
        assert xo.tolist() == list(range(N))
        xo, _ = oracle.gather_map(shift_chain(N, [s]), np.arange(N), z)
        assert xo.tolist() == [(i + s) % N for i in range(N)]   # Python's % is the non-negative remainder
    assert oracle.gather_map(shift_chain(N, [N]), np.arange(N), z)[0].tolist() == list(range(N))


@pytest.mark.parametrize("s,coef", [(0, 1), (3, -1), (-2, 2), (5, 2), (1, -3), (-9, 0)])
def test_shift_by_another_coordinate_is_a_roll_per_slice(oracle, s, coef):
    # out[g,i] = X[g, (i + s + coef*g) mod N]: slice g of X rolled by -(s + coef*g), each slice rolled by hand.
    # A checker that ignored `coef`, its sign, or dropped `s` when `shift_by` is present fails one of the cases.
    Gd, N = 4, 7
    b = Builder([("g", Gd), ("i", N)])
    v = b.shift(1, s, by=0, coef=coef)
    d = b.finish([0, v], [])
    X, Gr = rnd((Gd, N), 40), rnd((Gd, N), 41)
    ref = np.stack([np.roll(X[g], -(s + coef * g)) for g in range(Gd)])
    np.testing.assert_array_equal(oracle.forward(d, X, np.ones(1)), ref)
    # the adjoint of a permutation is its inverse: dX[g] = upstream gradient of slice g rolled the other way
    dX, _ = oracle.backward(d, X, np.ones(1), Gr)
    np.testing.assert_array_equal(dX, np.stack([np.roll(Gr[g], s + coef * g) for g in range(Gd)]))


def test_shift_by_a_reduce_iterator(oracle):
    # out[i] = sum_r X[r, (i + 2 - r) mod N] * Wt[r]: the Shift reads the Reduce iterator (coef = -1, s = 2);
    # checked against explicit loops.
    N, R = 6, 4
    b = Builder([("i", N)])
    r = b.reduce(R)
    rx, rw = b.share(r)
    v = b.shift(0, 2, by=rx, coef=-1)
    d = b.finish([rx, v], [rw])
    X, Wt = rnd((R, N), 42), rnd((R,), 43)
    ref = np.array([sum(X[k, (i + 2 - k) % N] * Wt[k] for k in range(R)) for i in range(N)])
    np.testing.assert_allclose(oracle.forward(d, X, Wt), ref, rtol=0, atol=1e-14)


# --------------------------------------------------------------------------------------
# Expand: the output does not depend on the expanded iterator
# --------------------------------------------------------------------------------------
def test_expand_repeats_output(oracle):
    b = Builder([("i", 3), ("j", 4)])
    b.expand(1)
    d = b.finish([0], [])
    X = rnd((3,), 14)
    got = oracle.forward(d, X, np.ones(1))
    np.testing.assert_array_equal(got, np.repeat(X[:, None], 4, axis=1))
    dX, _ = oracle.backward(d, X, np.ones(1), np.ones((3, 4)))
    np.testing.assert_array_equal(dX, np.full(3, 4.0))


# --------------------------------------------------------------------------------------
# Gradients: exact finite differences of a bilinear map, and the adjoint identities
# --------------------------------------------------------------------------------------
GRAD_CASES = [
    lambda: wl.conv2d(2, 3, 2, 4, 5),
    lambda: wl.grouped_shift_unfold(2, 8, 8, 5, 4, 4, 3, F32, F32),
    lambda: wl.strided_depthwise(2, 3, 3, 4),
    lambda: wl.matmul(3, 4, 5),
]


@pytest.mark.parametrize("mk", GRAD_CASES)
def test_gradients_match_central_differences(oracle, mk):
    d = mk()
    xs, ws, _ = oracle.describe(d)
    X, Wt, G = rnd(xs, 20), rnd(ws, 21), rnd(oracle.out_shape(d), 22)
    dX, dW = oracle.backward(d, X, Wt, G)
    loss = lambda x, w: float((oracle.forward(d, x, w) * G).sum())
    rng = np.random.default_rng(0)
    for _ in range(12):
        i = tuple(rng.integers(0, s) for s in xs)
        e = np.zeros(xs)
        e[i] = 0.5
        assert abs((loss(X + e, Wt) - loss(X - e, Wt)) - dX[i]) < 1e-9
        j = tuple(rng.integers(0, s) for s in ws)
        e = np.zeros(ws)
        e[j] = 0.5
        assert abs((loss(X, Wt + e) - loss(X, Wt - e)) - dW[j]) < 1e-9


@pytest.mark.parametrize("mk", GRAD_CASES)
def test_adjoint_identities(oracle, mk):
    d = mk()
    xs, ws, _ = oracle.describe(d)
    X, Wt, G = rnd(xs, 23), rnd(ws, 24), rnd(oracle.out_shape(d), 25)
    dX, dW = oracle.backward(d, X, Wt, G)
    L = (oracle.forward(d, X, Wt) * G).sum()
    assert abs((dX * X).sum() - L) < 1e-9 * max(1.0, abs(L))
    assert abs((dW * Wt).sum() - L) < 1e-9 * max(1.0, abs(L))


def test_conv_backward_equals_library_autograd(oracle):
    N, C, Co, H, W = 2, 3, 4, 5, 6
    X, Wt, G = rnd((N, C, H, W), 26), rnd((Co, C, 3, 3), 27), rnd((N, Co, H, W), 28)
    xt = torch.from_numpy(X).requires_grad_()
    wt = torch.from_numpy(Wt).requires_grad_()
    (torch.nn.functional.conv2d(xt, wt, padding=1) * torch.from_numpy(G)).sum().backward()
    dX, dW = oracle.backward(wl.conv2d(N, C, Co, H, W), X, Wt, G)
    np.testing.assert_allclose(dX, xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dW, wt.grad.numpy(), rtol=0, atol=1e-12)


def test_strided_backward_leaves_unread_positions_zero(oracle):
    # Stride 2 with a 1-wide window reads only even positions; dX is exactly 0 elsewhere.
    b = Builder([("i", 4)])
    s = b.stride(0, 2)
    d = b.finish([s], [])
    dX, _ = oracle.backward(d, np.ones(8), np.ones(1), np.array([1.0, 2.0, 3.0, 4.0]))
    assert dX.tolist() == [1.0, 0.0, 2.0, 0.0, 3.0, 0.0, 4.0, 0.0]


def test_sampled_backward_equals_full(oracle):
    d = wl.conv2d(2, 3, 2, 4, 5)
    xs, ws, _ = oracle.describe(d)
    X, Wt, G = rnd(xs, 30), rnd(ws, 31), rnd(oracle.out_shape(d), 32)
    dX, dW = oracle.backward(d, X, Wt, G)
    xi, wi = [0, 7, 119, 53], [53, 1, 0]
    sx, sw = oracle.backward(d, X, Wt, G, x_sample=xi, w_sample=wi)
    # the threads' atomic updates land in a different order from run to run
    np.testing.assert_allclose(sx, dX.ravel()[xi], rtol=0, atol=1e-13)
    np.testing.assert_allclose(sw, dW.ravel()[wi], rtol=0, atol=1e-13)
    np.testing.assert_array_equal(oracle.forward_at(d, X, Wt, [5, 0, 31]), oracle.forward(d, X, Wt).ravel()[[5, 0, 31]])


# --------------------------------------------------------------------------------------
# Index-map invariants
# --------------------------------------------------------------------------------------
def test_conv_gather_map_padding_count_and_coverage(oracle):
    N, C, Co, H, W = 1, 2, 2, 5, 7
    d = wl.conv2d(N, C, Co, H, W)
    o, r, n_o, n_r = all_points(d, oracle)
    xo, wo = oracle.gather_map(d, o, r)
    # per (n, co, c): 9*H*W taps of which (3H-2)(3W-2) fall inside the image
    assert int((xo == -1).sum()) == N * Co * C * (9 * H * W - (3 * H - 2) * (3 * W - 2))
    assert np.array_equal(xo == -1, wo == -1)
    assert set(xo[xo >= 0].tolist()) == set(range(N * C * H * W))     # every input element is used
    assert set(wo[wo >= 0].tolist()) == set(range(Co * C * 9))
    # independent formula for the offsets
    n, co, h, w = np.unravel_index(o, (N, Co, H, W))
    c, kh, kw = np.unravel_index(r, (C, 3, 3))
    y, x = h + kh - 1, w + kw - 1
    ok = (y >= 0) & (y < H) & (x >= 0) & (x < W)
    assert np.array_equal(xo, np.where(ok, ((n * C + c) * H + y) * W + x, -1))
    assert np.array_equal(wo, np.where(ok, ((co * C + c) * 3 + kh) * 3 + kw, -1))


def test_grouped_shift_unfold_gather_map_formula(oracle):
    N, C, H, W, G, K = 1, 8, 5, 4, 4, 3
    Cg = C // G
    d = wl.grouped_shift_unfold(N, C, C, H, W, G, K)
    o, r, _, _ = all_points(d, oracle)
    xo, wo = oracle.gather_map(d, o, r)
    n, co, h, w = np.unravel_index(o, (N, C, H, W))
    c, k = np.unravel_index(r, (Cg, K))
    g = co // Cg
    x = w + k - 1
    ok = (x >= 0) & (x < W)
    assert np.array_equal(xo, np.where(ok, ((n * C + g * Cg + c) * H + (h + g) % H) * W + x, -1))
    assert np.array_equal(wo, np.where(ok, (co * Cg + c) * K + k, -1))
    assert set(xo[xo >= 0].tolist()) == set(range(N * C * H * W))


# --------------------------------------------------------------------------------------
# FLOP rule of section 8: 2 * prod(output iterators) * prod(Reduce sizes), padded taps counted
# --------------------------------------------------------------------------------------
def test_flop_rule(oracle):
    exp = {}
    for line in open(os.path.join(GOLDEN, "flops.txt")):
        if line.strip() and line[0] != "#":
            k, v = line.split()
            exp[k] = int(v)
    descs = {
        "config0": wl.conv2d(1, 16, 16, 16, 16),
        "config1_C64": wl.conv2d(32, 64, 64, 56, 56), "config1_C128": wl.conv2d(32, 128, 128, 28, 28),
        "config1_C256": wl.conv2d(32, 256, 256, 14, 14), "config1_C512": wl.conv2d(32, 512, 512, 7, 7),
        "config2": wl.grouped_shift_unfold(32), "config3": wl.strided_depthwise(64, 128, 28, 28),
        "config4": wl.grouped_shift_unfold(128),
    }
    for k, d in descs.items():
        _, _, red = oracle.describe(d)
        assert 2 * int(np.prod(oracle.out_shape(d))) * int(np.prod(red)) == exp[k], k


# --------------------------------------------------------------------------------------
# Operators evaluated in stages: materialised reduction (code-generation section) and Operator 1 (Fig. 7)
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("H,k,s", [(12, 3, 2), (12, 3, 4), (15, 5, 3), (8, 1, 2)])
def test_materialised_reduction_equals_single_loop_nest(oracle, H, k, s):
    """The example of the code-generation section: Y[i] = sum_{ik,is} X[s*(i+ik-k/2)+is] evaluated as one loop
    nest of (H/s)*k*s points equals Z[i'] = sum_is X[s*i'+is] followed by Y[i] = sum_ik Z[i+ik-k/2], and the
    FLOPs drop from k*H to (1+k/s)*H."""
    Hs = H // s
    b = Builder([("i", Hs)])
    ik, i_s = b.reduce(k), b.reduce(s)
    whole = b.finish([b.split(b.unfold(0, ik), i_s)], [])
    b1 = Builder([("i", Hs)])
    st1 = b1.finish([b1.split(0, b1.reduce(s))], [])
    b2 = Builder([("i", Hs)])
    st2 = b2.finish([b2.unfold(0, b2.reduce(k))], [])
    X, one = rnd((H,), 40), np.ones(1)
    ref = oracle.forward(whole, X, one)
    Z, Y = oracle.chain_forward([st1, st2], X, [one, one])
    np.testing.assert_allclose(Z, X.reshape(Hs, s).sum(1), rtol=0, atol=1e-13)
    np.testing.assert_allclose(Y, ref, rtol=0, atol=1e-13)
    points = lambda d: int(np.prod(oracle.out_shape(d))) * int(np.prod(oracle.describe(d)[2]))
    assert points(whole) == k * H
    assert s * (points(st1) + points(st2)) == (s + k) * H


def operator1_single_sum(X, w1, w2, g, k1):
    """Operator 1 as ONE contraction with two weights, every loop written out: the window iterator k indexes X,
    w1 and w2; the second window iterator j indexes X and w2; terms outside the image are dropped."""
    N, Cin, H, W = X.shape
    D, Co, Cg = w1.shape[0], w2.shape[0], Cin // g
    out = np.zeros((N, Co, H, W))
    for n, h, w, d, gi, k, j in itertools.product(range(N), range(H), range(W), range(D), range(g), range(k1),
                                                  range(k1)):
        y, x = h + j - k1 // 2, w + k - k1 // 2
        if not (0 <= y < H and 0 <= x < W):
            continue
        t = 0.0
        for c in range(Cg):
            t += X[n, gi * Cg + c, y, x] * w1[d, gi * Cg + c, k]
        out[n, :, h, w] += t * w2[:, ((d * g + gi) * k1 + k) * k1 + j]
    return out


@pytest.mark.parametrize("N,Cin,Co,H,W,g,s,k1", [(1, 4, 8, 4, 5, 2, 2, 3), (2, 6, 6, 3, 4, 3, 1, 3),
                                                 (1, 4, 4, 5, 3, 1, 2, 1), (1, 2, 4, 6, 6, 2, 1, 5)])
def test_operator1_stages_equal_single_two_weight_sum(oracle, N, Cin, Co, H, W, g, s, k1):
    d1 = wl.operator1_stage1(N, Cin, Co, H, W, g, s, k1)
    d2 = wl.operator1_stage2(N, Co, H, W, s, k1)
    D, C2 = Co // g // s, k1 * Co // s
    X, w1, w2 = rnd((N, Cin, H, W), 41), rnd((D, Cin, k1), 42), rnd((Co, C2 * k1), 43)
    assert oracle.describe(d1)[:2] == ((N, Cin, H, W), (D, g, Cin // g, k1))
    assert oracle.describe(d2)[:2] == ((N, C2, H, W), (Co, C2, k1, 1))
    Z, Y = oracle.chain_forward([d1, d2], X, [w1, w2])
    assert Z.shape == (N, D, g, k1, H, W) and Y.shape == (N, Co, H, W)
    np.testing.assert_allclose(Y, operator1_single_sum(X, w1, w2, g, k1), rtol=0, atol=1e-12)


@pytest.mark.parametrize("N,Cin,Co,H,W,g,s,k1", [(1, 4, 8, 4, 5, 2, 2, 3), (2, 6, 6, 3, 4, 3, 1, 3),
                                                 (1, 4, 4, 5, 3, 1, 2, 1), (1, 2, 4, 6, 6, 2, 1, 5)])
def test_operator1_as_one_graph_with_two_weights(oracle, N, Cin, Co, H, W, g, s, k1):
    """The checker's several-weight path on Operator 1 written as ONE pGraph (five Reduces, seven Shares, two
    weights) against the explicit loops above, and its gradients against central differences (the operator is linear
    in X, in w1 and in w2 separately, so a central difference is exact up to rounding) and the adjoint identities."""
    d = wl.operator1_graph(N, Cin, Co, H, W, g, s, k1)
    D, Cg = Co // g // s, Cin // g
    assert oracle.describe(d)[0] == (N, Cin, H, W)
    assert oracle.weight_shapes(d) == [(D, g, Cg, k1), (Co, D, g, k1, k1)]
    X, w1, w2, G = rnd((N, Cin, H, W), 47), rnd((D, g, Cg, k1), 48), rnd((Co, D, g, k1, k1), 49), rnd((N, Co, H, W), 50)
    out = oracle.forward_multi(d, X, [w1, w2])
    np.testing.assert_allclose(out, operator1_single_sum(X, w1.reshape(D, Cin, k1), w2.reshape(Co, -1), g, k1), rtol=0, atol=1e-12)
    dX, (dw1, dw2) = oracle.backward_multi(d, X, [w1, w2], G)
    loss = lambda x, a, b: float((oracle.forward_multi(d, x, [a, b]) * G).sum())
    L = loss(X, w1, w2)
    for grad, arg in ((dX, 0), (dw1, 1), (dw2, 2)):
        base = [X, w1, w2]
        assert abs((grad * base[arg]).sum() - L) < 1e-9 * max(1.0, abs(L))     # L is linear in each factor
        rng = np.random.default_rng(arg)
        for _ in range(6):
            i = tuple(rng.integers(0, n) for n in base[arg].shape)
            e = np.zeros(base[arg].shape)
            e[i] = 0.5
            hi = [v + e if k == arg else v for k, v in enumerate(base)]
            lo = [v - e if k == arg else v for k, v in enumerate(base)]
            assert abs((loss(*hi) - loss(*lo)) - grad[i]) < 1e-9
    # the single-weight entry points refuse a description with further weights rather than ignore them
    with pytest.raises(oracle.OracleError):
        oracle.forward(d, X, w1)


def test_further_weight_of_ones_changes_nothing(oracle):
    """A second weight that is the constant one leaves the single-weight result: the several-weight loop nest is the
    single-weight one times further factors."""
    one = wl.conv2d(2, 3, 2, 4, 5)
    b = Builder([("n", 2), ("co", 2), ("h", 4), ("w", 5)])
    c = b.reduce(3); cx, cw = b.share(c)
    kh = b.reduce(3); khx, khw = b.share(kh)
    kw = b.reduce(3); kwa, kwv = b.share(kw); kwx, kww = b.share(kwa)
    two = b.finish([0, cx, b.unfold(2, khx), b.unfold(3, kwx)], [1, cw, khw, kww], more_weights=[[kwv]])
    X, Wt = rnd((2, 3, 4, 5), 51), rnd((2, 3, 3, 3), 52)
    v = rnd((3,), 53)
    np.testing.assert_allclose(oracle.forward_multi(two, X, [Wt, np.ones(3)]), oracle.forward(one, X, Wt), rtol=0, atol=1e-13)
    # and a real second weight along kw is the same as scaling the first along that axis
    np.testing.assert_allclose(oracle.forward_multi(two, X, [Wt, v]), oracle.forward(one, X, Wt * v), rtol=0, atol=1e-13)


def test_operator1_equals_library_convolutions(oracle):
    """Stage 1 is, per window position k, a grouped 1x1 convolution of X moved by k-k1/2 along w; stage 2 is a
    k1 x 1 convolution over the flattened (d,gi,k) channels.  Both from the library, in fp64."""
    N, Cin, Co, H, W, g, s, k1 = 2, 8, 16, 6, 7, 4, 2, 3
    D, Cg, C2 = Co // g // s, Cin // g, k1 * Co // s
    X, w1, w2 = rnd((N, Cin, H, W), 44), rnd((D, Cin, k1), 45), rnd((Co, C2 * k1), 46)
    xt = torch.from_numpy(X)
    xp = torch.nn.functional.pad(xt, (k1 // 2, k1 // 2))
    Zt = torch.empty(N, D, g, k1, H, W, dtype=torch.float64)
    for k in range(k1):
        wk = torch.from_numpy(w1[:, :, k]).reshape(D, g, Cg).permute(1, 0, 2).reshape(g * D, Cg, 1, 1)
        zk = torch.nn.functional.conv2d(xp[..., k:k + W], wk, groups=g)          # channels ordered (gi, d)
        Zt[:, :, :, k] = zk.reshape(N, g, D, H, W).permute(0, 2, 1, 3, 4)
    Yt = torch.nn.functional.conv2d(Zt.reshape(N, C2, H, W), torch.from_numpy(w2).reshape(Co, C2, k1, 1),
                                    padding=(k1 // 2, 0))
    d1 = wl.operator1_stage1(N, Cin, Co, H, W, g, s, k1)
    d2 = wl.operator1_stage2(N, Co, H, W, s, k1)
    Z, Y = oracle.chain_forward([d1, d2], X, [w1, w2])
    np.testing.assert_allclose(Z, Zt.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(Y, Yt.numpy(), rtol=0, atol=1e-12)


def test_operator1_chain_gradients_match_central_differences(oracle):
    N, Cin, Co, H, W, g, s, k1 = 1, 4, 8, 4, 5, 2, 2, 3
    descs = [wl.operator1_stage1(N, Cin, Co, H, W, g, s, k1), wl.operator1_stage2(N, Co, H, W, s, k1)]
    shapes = [oracle.describe(d)[1] for d in descs]
    X, G = rnd((N, Cin, H, W), 47), rnd((N, Co, H, W), 48)
    Ws = [rnd(shapes[0], 49), rnd(shapes[1], 50)]
    dX, dWs = oracle.chain_backward(descs, X, Ws, G)
    loss = lambda x, ws: float((oracle.chain_forward(descs, x, ws)[-1] * G).sum())
    rng = np.random.default_rng(1)
    for _ in range(8):
        i = tuple(rng.integers(0, n) for n in X.shape)
        e = np.zeros(X.shape)
        e[i] = 0.5
        assert abs((loss(X + e, Ws) - loss(X - e, Ws)) - dX[i]) < 1e-9       # the loss is linear in X
        for m in range(2):
            j = tuple(rng.integers(0, n) for n in shapes[m])
            e = np.zeros(shapes[m])
            e[j] = 0.5
            up = [w + e if q == m else w for q, w in enumerate(Ws)]
            dn = [w - e if q == m else w for q, w in enumerate(Ws)]
            assert abs((loss(X, up) - loss(X, dn)) - dWs[m][j]) < 1e-9         # and linear in each weight


def test_chain_quantize_hook_rounds_only_intermediates(oracle):
    from syno_inputs.rng import bf16_bits_to_f32, to_bf16_bits
    q = lambda a: bf16_bits_to_f32(to_bf16_bits(np.asarray(a, dtype=np.float32)))
    w = wl.make_operator1(1, 8, 5, g=2, s=2, bf16=True, with_grad=True)
    Z, Y = oracle.chain_forward(w.descs, w.X, w.Ws, quantize=q)
    Z0, _ = oracle.chain_forward(w.descs, w.X, w.Ws)
    np.testing.assert_array_equal(Z, q(Z0).astype(np.float64))
    np.testing.assert_array_equal(Y, oracle.forward(w.descs[1], Z.reshape(-1), w.Ws[1]))
    assert not np.array_equal(Y, q(Y).astype(np.float64))


# --------------------------------------------------------------------------------------
# Descriptor validation
# --------------------------------------------------------------------------------------
def test_rejects_bad_descriptors(oracle):
    b = Builder([("i", 10)])
    q, r = b.merge(0, 3)                     # 3 does not divide 10
    with pytest.raises(oracle.OracleError):
        oracle.describe(b.finish([q, r], []))
    b = Builder([("i", 4), ("j", 4)])         # j never consumed
    with pytest.raises(oracle.OracleError):
        oracle.describe(b.finish([0], []))
    b = Builder([("i", 4)])                   # i consumed twice
    with pytest.raises(oracle.OracleError):
        oracle.describe(b.finish([0, 0], []))
    b = Builder([("i", 4)])                   # a Reduce that reaches nothing
    r = b.reduce(3)
    b.expand(r)
    with pytest.raises(oracle.OracleError):
        oracle.describe(b.finish([0], []))


def test_bf16_inputs_are_what_the_workload_says():
    w = wl.make_gshift(1, seeds=(1, 2, 3), with_grad=True)
    assert w.desc.in_dtype == BF16
    for v, b in ((w.X, w.X_bits), (w.W, w.W_bits), (w.G, w.G_bits)):
        t = torch.from_numpy(v).to(torch.bfloat16)           # already representable: conversion is exact
        assert torch.equal(t.float(), torch.from_numpy(v))
        assert np.array_equal(t.view(torch.int16).numpy().view(np.uint16), b)
    # and the rounding itself agrees with the library's round-to-nearest-even
    raw = np.random.default_rng(5).standard_normal(4096).astype(np.float32)
    from syno_inputs import to_bf16_bits
    lib = torch.from_numpy(raw).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(to_bf16_bits(raw), lib)
