"""GPU parity: the HIP path against the CPU checker on the same seeded inputs, through the C ABI.

Small cases are compared element by element (sizes the checker finishes in seconds, spanning several
tiles and ragged tails); the full-size workloads are compared on sampled outputs where the checker
cannot finish the whole tensor quickly, else in full.  Index maps are compared bit for bit.
"""
import numpy as np
import pytest
import torch

from syno_inputs import BF16, F32, Builder, workloads as wl
from util import TOL_ACC, TOL_CHAIN_BF16, assert_close, plane_samples, rel_l2, to_dev, to_host, tol_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def syno():
    import paper_2410_23745_amd as s
    s.load_library()          # raises if the HIP library has not been built: there is no fallback
    assert torch.cuda.is_available()
    return s


def tile_picks(plan, which, shape):
    """Leading-axis values at the boundaries of the launch's own tiling, for the stratified samples: the images at
    which a block of output rows ends (rows/block of the contraction kernels) and the channels around multiples of
    the MFMA tile and of the channel blocks."""
    import re
    picks = [set() for _ in shape[:-2]]
    if len(shape) < 3:
        return picks
    m = re.search(r"rows/block=(\d+)", plan.describe(which))
    if m and len(shape) == 4:
        tr, rows = int(m.group(1)), shape[0] * shape[2]
        for r in (tr - 1, tr, 2 * tr - 1, 2 * tr, (rows - 1) // tr * tr - 1, (rows - 1) // tr * tr):
            if 0 <= r < rows:
                picks[0].add(r // shape[2])
    for ax in range(1 if len(shape) == 4 else 0, len(shape) - 2):
        for b in (16, 32, 64, 128):
            picks[ax] |= {b - 1, b, shape[ax] - b - 1, shape[ax] - b}
    return picks


def run_all(syno, oracle, w, policy, directions=(0, 1, 2), full=True, n_sample=4096, seed=0, **options):
    """Run the requested directions on the GPU and compare with the checker: relative L2 error and a bound on
    every compared element (util.assert_close).  Without `full` the comparison is on a stratified sample: whole
    image planes at the first, last and tile-boundary images and channels, plus n_sample random elements.
    Returns kernel names."""
    plan = syno.Plan(w.desc, kernel_policy=policy, **options)
    d, tol = w.desc, tol_for(w.desc)
    out_bf16 = d.out_dtype == BF16
    X, W = to_dev(w.X, w.X_bits), to_dev(w.W, w.W_bits)
    aX, aW = np.abs(w.X), np.abs(w.W)
    rng = np.random.default_rng(seed)
    names = [plan.kernel(i) for i in range(3)]
    if 0 in directions:
        print(f"[case] {d.name} fwd kernel={names[0]} policy={policy}", flush=True)
        out = plan.forward(X, W)
        torch.cuda.synchronize()
        got = to_host(out).ravel()
        if full:
            ref, mag = oracle.forward(d, w.X, w.W).ravel(), oracle.forward(d, aX, aW).ravel()
        else:
            idx = plane_samples(w.out_shape, rng, n_sample, tile_picks(plan, 0, w.out_shape))
            ref, mag, got = oracle.forward_at(d, w.X, w.W, idx), oracle.forward_at(d, aX, aW, idx), got[idx]
        e, worst = assert_close(got, ref, mag, plan.free_size(0), out_bf16, "forward", tol)
        print(f"       {got.size} elements: rel-L2 {e:.2e}, worst element at {worst:.2f} of its bound", flush=True)
    if 1 in directions or 2 in directions:
        G = to_dev(w.G, w.G_bits)
        xs = ws = None
        if not full:
            xs = plane_samples(w.x_shape, rng, n_sample, tile_picks(plan, 1, w.x_shape))
            ws = plane_samples(w.w_shape, rng, n_sample, tile_picks(plan, 2, w.w_shape))
        want = (1 in directions, 2 in directions)
        rdx, rdw = oracle.backward(d, w.X, w.W, w.G, *want, x_sample=xs, w_sample=ws)
        mdx, mdw = oracle.backward(d, aX, aW, np.abs(w.G), *want, x_sample=xs, w_sample=ws)
        if 1 in directions:
            print(f"[case] {d.name} bwd-data kernel={names[1]} policy={policy}", flush=True)
            dX = plan.backward_data(G, W)
            torch.cuda.synchronize()
            got = to_host(dX).ravel()
            e, worst = assert_close(got if full else got[xs], rdx, mdx, plan.free_size(1), out_bf16, "backward-data", tol)
            print(f"       {rdx.size} elements: rel-L2 {e:.2e}, worst element at {worst:.2f} of its bound", flush=True)
        if 2 in directions:
            print(f"[case] {d.name} bwd-weight kernel={names[2]} policy={policy}", flush=True)
            dW = plan.backward_weight(X, G)
            torch.cuda.synchronize()
            assert dW.dtype == torch.float32
            got = to_host(dW).ravel()
            e, worst = assert_close(got if full else got[ws], rdw, mdw, plan.free_size(2), False, "backward-weight", tol)
            print(f"       {rdw.size} elements: rel-L2 {e:.2e}, worst element at {worst:.2f} of its bound", flush=True)
    return names


# ------------------------------------------------------------------------------------------------
# small cases, every direction, both the generic kernels (policy 1) and the planner's choice (0)
# ------------------------------------------------------------------------------------------------
def small_cases():
    c = {}
    c["config0"] = lambda: wl.make_conv(1, 16, 16, seed=0, with_grad=True)
    c["conv_f32_ragged"] = lambda: wl.make_conv(3, 24, 13, seed=4, Co=40, Wd=19, with_grad=True)
    c["conv_bf16_ragged"] = lambda: wl.make_conv(3, 40, 13, seed=5, Co=24, Wd=19, bf16=True, with_grad=True)
    c["conv_bf16_out_bf16"] = lambda: wl.make_conv(2, 32, 14, seed=6, bf16=True, with_grad=True, out_bf16=True)
    c["conv_f32_5x5"] = lambda: wl.make_conv(2, 8, 9, seed=7, Co=16, K=5, with_grad=True)
    c["conv_f32_1x1"] = lambda: wl.make_conv(2, 16, 7, seed=8, Co=32, K=1, with_grad=True)
    c["conv_f32_stage3_small_batch"] = lambda: wl.make_conv(2, 512, 7, seed=9, with_grad=True)
    c["conv_bf16_chan_tail"] = lambda: wl.make_conv(2, 80, 10, seed=10, Co=48, bf16=True, with_grad=True)   # 2.5 chunks
    c["conv_f32_wide_rows"] = lambda: wl.make_conv(1, 8, 6, seed=11, Co=8, Wd=60, with_grad=True)
    c["conv_bf16_wide_rows"] = lambda: wl.make_conv(1, 8, 5, seed=12, Co=8, Wd=60, bf16=True, with_grad=True)
    # small images: backward-weight stages several whole images per chunk (the last chunk is short)
    c["conv_bf16_7x7_five_images"] = lambda: wl.make_conv(5, 24, 7, seed=13, Co=40, bf16=True, with_grad=True)
    c["conv_bf16_5x4_five_images"] = lambda: wl.make_conv(5, 16, 5, seed=14, Co=16, Wd=4, bf16=True, with_grad=True)
    c["conv_f32_5x4_five_images"] = lambda: wl.make_conv(5, 16, 5, seed=15, Co=16, Wd=4, with_grad=True)   # one staging item per row
    # backward-weight kernels whose wave halves alternate between multiplying and staging: images cut into chunks with
    # a short last one, channel counts that end inside a tile, whole-row items (14- and 7-pixel rows), items of 4 in
    # two batches, items of 2
    c["conv_f32_14wide_30rows"] = lambda: wl.make_conv(3, 40, 30, seed=20, Co=72, Wd=14, with_grad=True)
    c["conv_f32_28wide_20rows"] = lambda: wl.make_conv(2, 24, 20, seed=21, Co=24, Wd=28, with_grad=True)
    c["conv_f32_10wide"] = lambda: wl.make_conv(2, 16, 9, seed=22, Co=16, Wd=10, with_grad=True)
    c["conv_bf16_14x14_three_images"] = lambda: wl.make_conv(3, 24, 14, seed=23, Co=40, bf16=True, with_grad=True)
    c["conv_bf16_7x7_eleven_images"] = lambda: wl.make_conv(11, 40, 7, seed=24, Co=72, bf16=True, with_grad=True)
    # a Stride below the window (the downsampling convolutions of a ResNet stage): forward on the contraction kernel
    c["conv_f32_3x3_stride2"] = lambda: wl.make_conv(3, 24, 7, seed=25, Co=40, Wd=9, stride=2, with_grad=True)
    c["conv_bf16_3x3_stride2"] = lambda: wl.make_conv(3, 40, 7, seed=26, Co=24, Wd=9, stride=2, bf16=True, with_grad=True)
    c["conv_f32_1x1_stride2"] = lambda: wl.make_conv(5, 40, 4, seed=27, Co=48, Wd=6, K=1, stride=2, with_grad=True)
    c["conv_bf16_1x1_stride2"] = lambda: wl.make_conv(5, 72, 4, seed=28, Co=48, Wd=6, K=1, stride=2, bf16=True, with_grad=True)
    c["conv_f32_3x3_stride3"] = lambda: wl.make_conv(2, 16, 5, seed=29, Co=24, Wd=9, stride=3, with_grad=True)
    # a window over two flattened axes (Unfold below a Merge): the two halves of the Merge lie side by side in X, so the
    # planner reads them as one long row and the contraction kernels take all three passes
    c["flat_window_f32"] = lambda: wl.make_flat_window(3, 24, 40, 6, 10, seed=31, with_grad=True)
    c["flat_window_bf16"] = lambda: wl.make_flat_window(3, 40, 24, 14, 14, seed=32, bf16=True, with_grad=True)
    c["flat_window_f32_k5_C80"] = lambda: wl.make_flat_window(2, 80, 40, 7, 7, K=5, seed=33, with_grad=True)
    c["gshift_bf16"] = lambda: wl.make_gshift(3, seeds=(1, 2, 3), with_grad=True)
    c["gshift_bf16_small_groups"] = lambda: wl.make_gshift(2, seeds=(4, 5, 6), with_grad=True, C=96, H=9, Wd=11, groups=3)
    c["gshift_f32"] = lambda: wl.make_gshift(2, seeds=(7, 8, 9), with_grad=True, C=64, H=6, Wd=10, groups=2, bf16=False)
    # weights laid out in other axis orders (the planner sends these to the same tuned kernels: element-gathered
    # fp32 weight staging, packing and transposition from arbitrary strides, strided writes of the weight gradient)
    for tag, wo in (("c_co_kh_kw", (1, 0, 2, 3)), ("kh_kw_c_co", (2, 3, 1, 0)), ("co_kw_kh_c", (0, 3, 2, 1))):
        c[f"conv_f32_w_{tag}"] = lambda wo=wo: wl.make_conv(3, 24, 13, seed=16, Co=40, Wd=19, with_grad=True, w_order=wo)
        c[f"conv_bf16_w_{tag}"] = lambda wo=wo: wl.make_conv(3, 40, 13, seed=17, Co=24, Wd=19, bf16=True, with_grad=True,
                                                             w_order=wo)
    c["conv_f32_w_kh_kw_c_co_C128"] = lambda: wl.make_conv(2, 128, 28, seed=18, with_grad=True, w_order=(2, 3, 1, 0))
    c["conv_bf16_w_c_co_kh_kw_C128"] = lambda: wl.make_conv(2, 128, 28, seed=19, bf16=True, with_grad=True, w_order=(1, 0, 2, 3))
    c["gshift_bf16_w_permuted"] = lambda: wl.make_gshift(2, seeds=(4, 5, 6), with_grad=True, C=96, H=9, Wd=11, groups=3,
                                                         w_order=(2, 0, 3, 1))
    c["gshift_f32_w_permuted"] = lambda: wl.make_gshift(2, seeds=(7, 8, 9), with_grad=True, C=128, H=28, Wd=28, groups=1,
                                                        bf16=False, w_order=(3, 2, 0, 1))
    c["depthwise_f32"] = lambda: wl.make_depthwise(3, 20, 30, seed=2, with_grad=True)
    c["depthwise_f32_odd"] = lambda: wl.make_depthwise(2, 7, 18, seed=3, with_grad=True)
    c["depthwise_f32_even"] = lambda: wl.make_depthwise(2, 5, 28, seed=4, with_grad=True)      # stream kernels, all passes
    c["depthwise_f32_even_ragged"] = lambda: wl.make_depthwise(3, 4, 20, seed=5, with_grad=True)  # last strip 3 rows
    c["depthwise_f32_stride1"] = lambda: wl.make_depthwise(2, 6, 12, seed=6, S=1, with_grad=True)       # forward streams
    c["depthwise_f32_stride1_odd"] = lambda: wl.make_depthwise(2, 3, 10, seed=7, S=1, with_grad=True)   # rows not vector-aligned
    return c


@pytest.mark.parametrize("policy", [1, 0])
@pytest.mark.parametrize("name", list(small_cases()))
def test_small_cases_all_directions(syno, oracle, name, policy):
    run_all(syno, oracle, small_cases()[name](), policy)


@pytest.mark.parametrize("seed", range(32))
def test_random_convolution_shapes(syno, oracle, seed):
    """Seeded draws over batch, channels (ragged against every tile and chunk size), image extents, window, stride and
    element type, all three passes against the checker: whatever tiling the planner picks for a shape nobody chose by
    hand."""
    rng = np.random.default_rng(1000 + seed)
    K, stride, bf16 = int(rng.choice([1, 3])), int(rng.choice([1, 1, 2])), bool(rng.integers(2))
    N, C, Co = int(rng.integers(1, 6)), int(rng.choice([3, 8, 20, 40, 72, 96, 136])), int(rng.choice([5, 16, 24, 40, 80, 130]))
    H, Wd = int(rng.integers(3, 16)), int(rng.integers(4, 22))
    w = wl.make_conv(N, C, H, seed=2000 + seed, bf16=bf16, Co=Co, Wd=Wd, K=K, stride=stride, with_grad=True)
    names = run_all(syno, oracle, w, 0)
    assert all(n.startswith("mfma_contraction") for n in names), names


@pytest.mark.parametrize("seed", range(16))
def test_random_grouped_shift_unfold_shapes(syno, oracle, seed):
    """The grouped shift-unfold operator over seeded draws of groups, channels per group, extents, window and element
    type: cyclic row shifts per group, ragged channel blocks, all three passes."""
    rng = np.random.default_rng(7000 + seed)
    groups, K, bf16 = int(rng.choice([1, 2, 3, 4])), int(rng.choice([1, 3])), bool(rng.integers(2))
    Cg = int(rng.choice([8, 16, 24, 40, 64, 72]))
    N, H, Wd = int(rng.integers(1, 5)), int(rng.integers(3, 15)), int(rng.integers(4, 20))
    w = wl.make_gshift(N, seeds=(7100 + seed, 7200 + seed, 7300 + seed), with_grad=True, C=Cg * groups, H=H, Wd=Wd,
                       groups=groups, K=K, bf16=bf16)
    names = run_all(syno, oracle, w, 0)
    assert all(n.startswith("mfma_contraction") for n in names), names


@pytest.mark.parametrize("seed", range(8))
def test_random_operator1_shapes(syno, oracle, seed):
    rng = np.random.default_rng(8000 + seed)
    g, s, k1 = int(rng.choice([2, 4])), int(rng.choice([2, 4])), int(rng.choice([3, 5]))
    C = g * s * int(rng.choice([1, 2, 3]))
    w = wl.make_operator1(int(rng.integers(1, 4)), C, int(rng.integers(4, 13)), seed=8100 + seed, bf16=bool(rng.integers(2)),
                          Co=int(rng.choice([8, 16, 24])), Wd=int(rng.integers(5, 17)), g=g, s=s, k1=k1, with_grad=True)
    run_chain(syno, oracle, w, 0)


@pytest.mark.parametrize("KH,KW,bf16", [(5, 1, False), (5, 1, True), (1, 5, False), (3, 1, True), (1, 3, False)])
def test_one_sided_windows(syno, oracle, KH, KW, bf16):
    """Windows along one image axis only, 3 and 5 wide (the second stage of Operator 1 is k1 x 1): all three passes on
    the contraction kernels; the weight gradient keeps one set of accumulators per tap."""
    N, C, Co, H, Wd = 3, 40, 24, 9, 12
    d = wl.conv2d(N, C, Co, H, Wd, KH, KW, BF16 if bf16 else F32, F32)
    st = wl.Stream(90 + KH * 10 + KW)
    xs, ws, os_ = (N, C, H, Wd), (Co, C, KH, KW), (N, Co, H, Wd)
    w = wl._finish(d, xs, ws, os_, st.normal(xs), st.uniform_pm(1.0 / np.sqrt(C * KH * KW), ws), st.normal(os_), C * KH * KW)
    names = run_all(syno, oracle, w, 0)
    assert all(n.startswith("mfma_contraction") for n in names), names


def random_valid_graphs(seed, n):
    """Seeded random primitive graphs (the generator of the host sanitizer test) that the checker accepts and the
    library plans, with at least one X axis."""
    import random
    from test_host_sanitizers import random_graph
    rng = random.Random(seed)
    out = []
    for _ in range(n):
        d = random_graph(rng)
        try:
            xs, ws, _ = oracle_mod().describe(d)
        except Exception:
            continue
        if not xs or (d.in_dtype == F32 and d.out_dtype == BF16):
            continue          # (fp32 inputs with a bf16 result: no bar is stated for that pair)
        out.append(d)
    return out


def oracle_mod():
    import oracle
    return oracle


@pytest.mark.parametrize("seed", list(range(5150, 5162)))
def test_random_primitive_graphs(syno, oracle, seed):
    """Whatever the planner makes of arbitrary valid pGraphs (Split, Merge, Shift with and without a read coordinate,
    Expand, Unfold, Stride, Reduce, Share in random order, random element types): all three passes against the
    checker.  About a third of them are pure views and run on the view kernels (stream, scatter, gathers); the rest
    exercise the index-program kernels on graphs nobody wrote by hand."""
    fast = 0
    for i, d in enumerate(random_valid_graphs(seed, 150)):
        try:
            plan = syno.Plan(d)
        except syno.SynoError:
            continue                       # valid but outside what the library lowers (reported as unsupported)
        xs, ws, _ = oracle.describe(d)
        os_ = oracle.out_shape(d)
        st = wl.Stream(seed * 1000 + i)
        w = wl._finish(d, xs, ws if ws else (1,), os_, st.normal(xs), st.uniform_pm(2.0, ws if ws else (1,)), st.normal(os_), 1)
        print(f"[graph {seed}/{i}] {[plan.kernel(k) for k in range(3)]} X{xs} W{ws} out{os_}", flush=True)
        names = run_all(syno, oracle, w, 0)
        fast += sum(n != "generic_index_program" for n in names)
    assert fast > 30


def random_view_graph(rng):
    """A random Reduce-free, Unfold-free graph over a few larger output axes: Share, Split, Merge, Shift (constant, or by
    another coordinate), Stride and Expand in random order - sized so that runs of four, long sliced sums and zero-filled
    gaps all occur."""
    n_out = rng.randint(2, 4)
    b = Builder([(f"o{i}", rng.choice([3, 4, 8, 12, 16, 28, 56])) for i in range(n_out)])
    live = list(range(n_out))
    size = {i: sz for i, (_, sz) in enumerate(b.desc.out_dims)}
    wcoords = []
    for _ in range(rng.randint(1, 6)):
        kind = rng.choice(["share", "share", "split", "merge", "shift", "stride", "expand"])
        if not live:
            break
        if kind == "share":
            c = live.pop(rng.randrange(len(live))); x, w = b.share(c); size[x] = size[w] = size[c]; live.append(x); wcoords.append(w)
        elif kind == "split" and len(live) >= 2:
            i = live.pop(rng.randrange(len(live))); j = live.pop(rng.randrange(len(live)))
            v = b.split(i, j); size[v] = size[i] * size[j]; live.append(v)
        elif kind == "merge":
            c = live.pop(rng.randrange(len(live)))
            B = rng.choice([k for k in range(1, size[c] + 1) if size[c] % k == 0])
            q, r = b.merge(c, B); size[q], size[r] = size[c] // B, B; live += [q, r]
        elif kind == "shift":
            c = live.pop(rng.randrange(len(live)))
            v = b.shift(c, rng.randint(-5, 5)); size[v] = size[c]; live.append(v)
        elif kind == "stride":
            c = live.pop(rng.randrange(len(live))); S = rng.choice([2, 3]); v = b.stride(c, S); size[v] = S * size[c]; live.append(v)
        elif kind == "expand" and len(live) >= 2:
            b.expand(live.pop(rng.randrange(len(live))))
    rng.shuffle(live)
    rng.shuffle(wcoords)
    dt = rng.choice([(F32, F32), (BF16, F32), (BF16, BF16)])
    return b.finish(live, wcoords, dt[0], dt[1])


@pytest.mark.parametrize("seed", list(range(6200, 6208)))
def test_random_views_at_larger_sizes(syno, oracle, seed):
    import random
    rng = random.Random(seed)
    ran = 0
    for i in range(40):
        d = random_view_graph(rng)
        try:
            xs, ws, _ = oracle.describe(d)
            plan = syno.Plan(d)
        except Exception:
            continue
        os_ = oracle.out_shape(d)
        if not xs or max(int(np.prod(xs)), int(np.prod(os_))) > (1 << 20):
            continue
        # (some of these gradients are ONE sum over 10^4 to 10^6 products of either sign: the gather kernels add in fp64)
        st = wl.Stream(seed * 1000 + i)
        w = wl._finish(d, xs, ws if ws else (1,), os_, st.normal(xs), st.uniform_pm(2.0, ws if ws else (1,)), st.normal(os_), 1)
        print(f"[view {seed}/{i}] {[plan.describe(k) for k in range(3)]} X{xs} W{ws} out{os_}", flush=True)
        names = run_all(syno, oracle, w, 0)
        ran += sum(n == "bandwidth_view" for n in names)
    assert ran >= 20


@pytest.mark.parametrize("seed", range(12))
def test_random_matmul_shapes(syno, oracle, seed):
    rng = np.random.default_rng(3000 + seed)
    M, K = int(rng.integers(5, 300)), int(rng.integers(4, 260))
    N = int(rng.choice([7, 13, 24, 40, 56, 64])) * int(rng.integers(1, 9))
    w = wl.make_matmul(M, K, N, seed=4000 + seed, bf16=bool(rng.integers(2)), with_grad=True)
    names = run_all(syno, oracle, w, 0)
    assert names[0] == names[2] == "mfma_contraction_transposed", names


@pytest.mark.parametrize("variant,rows,order", [(0, 4, (1, 0, 2, 3)), (1, 3, (2, 3, 1, 0)), (2, 2, (0, 3, 2, 1)), (0, 1, (0, 1, 2, 3)),
                                                (3, 4, (0, 1, 2, 3)), (11, 2, (0, 1, 2, 3))])
def test_conv_f32_named_tile_variants(syno, oracle, variant, rows, order):
    """Tile variants the planner's cost model does not pick at small sizes, named through the plan options:
    the element-gathered weight staging (variants 0-2, any weight layout) and two of the 16-byte-staged ones."""
    w = wl.make_conv(3, 24, 13, seed=20 + variant, Co=72, Wd=19, with_grad=True, w_order=order)
    plan = syno.Plan(w.desc, mfma_variant=variant + 1, mfma_rows=rows)
    assert f"variant={variant} rows/block={rows} " in plan.describe(syno.FWD)
    run_all(syno, oracle, w, 0, directions=(0, 1), mfma_variant=variant + 1, mfma_rows=rows)


@pytest.mark.parametrize("bf16,variant,rows,K", [(False, 3, 10, 3), (False, 0, 5, 3), (False, 11, 9, 1), (True, 0, 10, 3),
                                                 (True, 6, 6, 3), (True, 2, 11, 1), (True, 3, 7, 1)])
def test_strided_conv_blocks_across_images(syno, oracle, bf16, variant, rows, K):
    """Stride 2 below the window, with tiles of several output rows that start and end inside images (4 rows per image):
    every image boundary inside a tile changes the slot of the rows after it by KH - 2."""
    w = wl.make_conv(5, 40, 4, seed=60 + variant, Co=40, Wd=9, K=K, stride=2, bf16=bf16)
    plan = syno.Plan(w.desc, mfma_variant=variant + 1, mfma_rows=rows)
    assert f"variant={variant} rows/block={rows} " in plan.describe(syno.FWD), plan.describe(syno.FWD)
    assert run_all(syno, oracle, w, 0, directions=(0,), mfma_variant=variant + 1, mfma_rows=rows)[0].startswith("mfma_contraction")


@pytest.mark.parametrize("variant,rows", [(0, 4), (1, 5), (3, 3), (4, 2), (5, 1), (6, 4), (7, 4), (8, 2), (9, 3)])
def test_conv_bf16_named_tile_variants(syno, oracle, variant, rows):
    C = 40 if variant == 6 else 72          # (variant 6 holds the whole reduction in one chunk: at most 64 channels)
    w = wl.make_conv(3, C, 13, seed=30 + variant, Co=40, Wd=19, bf16=True, with_grad=True, w_order=(0, 1, 2, 3))
    plan = syno.Plan(w.desc, mfma_variant=variant + 1, mfma_rows=rows)
    assert f"variant={variant} rows/block={rows} " in plan.describe(syno.FWD)
    # variants 1, 8 and 9 (and the single-chunk one) read forward-layout weights themselves in backward-data too
    assert ("weights=direct" in plan.describe(syno.BWD_DATA)) == (variant in (1, 6, 8, 9)), plan.describe(syno.BWD_DATA)
    run_all(syno, oracle, w, 0, directions=(0, 1), mfma_variant=variant + 1, mfma_rows=rows)


ROWS_CASES = {
    # (workload, rows per tile): the row-streaming bf16 kernel on shapes its default choice does not reach
    "ragged_tiles_two_blocks": (lambda: wl.make_conv(3, 40, 13, seed=40, Co=72, Wd=19, bf16=True, with_grad=True), 5),
    "channel_tail_packed": (lambda: wl.make_conv(2, 36, 11, seed=41, Co=20, Wd=16, bf16=True, with_grad=True), 4),
    "permuted_weights": (lambda: wl.make_conv(2, 24, 9, seed=42, Co=40, Wd=12, bf16=True, with_grad=True, w_order=(2, 3, 1, 0)), 3),
    "several_tiles_per_workgroup": (lambda: wl.make_conv(40, 16, 12, seed=43, Co=16, Wd=8, bf16=True, with_grad=True), 1),
    "gshift_several_tiles": (lambda: wl.make_gshift(80, seeds=(4, 5, 6), with_grad=True, C=96, H=9, Wd=12, groups=3), 2),
    "gshift_bf16_out": (lambda: wl.make_gshift(3, seeds=(7, 8, 9), with_grad=True, C=128, H=10, Wd=14, groups=2, out_bf16=True), 4),
    "one_by_one": (lambda: wl.make_conv(3, 48, 9, seed=44, Co=80, Wd=20, K=1, bf16=True, with_grad=True), 6),
}


DW_HALVES_CASES = ["conv_f32_14wide_30rows", "conv_f32_28wide_20rows", "conv_f32_10wide", "conv_f32_stage3_small_batch",
                   "conv_bf16_14x14_three_images", "conv_bf16_7x7_eleven_images", "conv_f32_ragged"]


@pytest.mark.parametrize("workgroups", [1, 3])
@pytest.mark.parametrize("name", DW_HALVES_CASES)
def test_backward_weight_with_several_chunks_per_workgroup(syno, oracle, name, workgroups):
    """The backward-weight kernels whose wave halves take turns: with the pixel axis split over few workgroups each one
    walks over several chunks (both halves multiply, stage and meet at the end), an odd count among them."""
    w = small_cases()[name]()
    plan = syno.Plan(w.desc, dw_workgroups=workgroups)
    text = plan.describe(syno.BWD_WEIGHT)
    chunks, splits = (int(text.split(k + "=")[1].split()[0]) for k in ("chunks", "splits"))
    if workgroups == 1:
        assert splits == 1 and chunks > 1, text
    run_all(syno, oracle, w, 0, directions=(2,), dw_workgroups=workgroups)


@pytest.mark.parametrize("name", list(ROWS_CASES))
def test_conv_bf16_row_streaming_kernel(syno, oracle, name):
    mk, rows = ROWS_CASES[name]
    w = mk()
    plan = syno.Plan(w.desc, mfma_variant=-1, mfma_rows=rows)
    assert f"row-streaming rows/block={rows} " in plan.describe(syno.FWD), plan.describe(syno.FWD)
    if "several_tiles" in name:
        for which in (syno.FWD, syno.BWD_DATA):
            assert "row-streaming" in plan.describe(which) and "tiles/workgroup=1 " not in plan.describe(which)
    run_all(syno, oracle, w, 0, directions=(0, 1), mfma_variant=-1, mfma_rows=rows)


def test_table2_examples_and_odd_graphs(syno, oracle):
    rng = np.random.default_rng(11)
    from test_abi import pixel_unshuffle_conv
    for d in (wl.matmul(37, 29, 45), pixel_unshuffle_conv()):
        xs, ws, _ = oracle.describe(d)
        X, W = rng.standard_normal(xs).astype(np.float32), rng.standard_normal(ws).astype(np.float32)
        G = rng.standard_normal(oracle.out_shape(d)).astype(np.float32)
        w = wl.Workload(d, xs, ws, oracle.out_shape(d), X, W, G, None, None, None, 0)
        run_all(syno, oracle, w, 0)


def test_stride_backward_writes_zeros(syno, oracle):
    # Stride 2 under a 1-wide window: odd rows and columns of dX receive no term and must be written as 0.
    b = Builder([("n", 2), ("c", 5), ("h", 6), ("w", 7)])
    cx, cw = b.share(1)
    hs, ws_ = b.stride(2, 2), b.stride(3, 2)
    d = b.finish([0, cx, hs, ws_], [cw])
    plan = syno.Plan(d)
    G = torch.randn(plan.out_shape, device="cuda")
    W = torch.randn(plan.w_shape, device="cuda")
    dX = torch.full(plan.x_shape, 7.0, device="cuda")
    plan.backward_data(G, W, dX=dX)
    torch.cuda.synchronize()
    ref, _ = oracle.backward(d, np.zeros(plan.x_shape), to_host(W), to_host(G), True, False)
    assert rel_l2(to_host(dX), ref) <= 1e-6
    assert float(dX[:, :, 1::2, :].abs().max()) == 0.0 and float(dX[:, :, :, 1::2].abs().max()) == 0.0


# ------------------------------------------------------------------------------------------------
# index maps on the device, bit exact
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("mk", [lambda: wl.config0().desc, lambda: wl.grouped_shift_unfold(32),
                                lambda: wl.strided_depthwise(64, 128, 28, 28),
                                lambda: wl.conv2d(32, 512, 512, 7, 7)])
def test_device_gather_map_bit_exact(syno, oracle, mk):
    d = mk()
    plan = syno.Plan(d)
    n_o, n_r = int(np.prod(plan.out_shape)), plan.free_size(syno.FWD)
    if n_o * n_r <= (1 << 20):
        o, r = (a.ravel() for a in np.meshgrid(np.arange(n_o), np.arange(n_r), indexing="ij"))
    else:
        rng = np.random.default_rng(1)
        o, r = rng.integers(0, n_o, 1 << 20), rng.integers(0, n_r, 1 << 20)
    xo, wo = oracle.gather_map(d, o, r)
    a, b = plan.debug_gather(syno.FWD, torch.from_numpy(o).cuda(), torch.from_numpy(r).cuda())
    assert np.array_equal(a.cpu().numpy(), xo) and np.array_equal(b.cpu().numpy(), wo)
    # the device and the host evaluation of the gradient maps agree as well
    for which, n_t in ((syno.BWD_DATA, int(np.prod(plan.x_shape))), (syno.BWD_WEIGHT, int(np.prod(plan.w_shape)))):
        rng = np.random.default_rng(2 + which)
        t, q = rng.integers(0, n_t, 1 << 16), rng.integers(0, plan.free_size(which), 1 << 16)
        a, b = plan.debug_gather(which, torch.from_numpy(t).cuda(), torch.from_numpy(q).cuda())
        ha, hb = plan.debug_gather_host(which, t, q)
        assert np.array_equal(a.cpu().numpy(), ha) and np.array_equal(b.cpu().numpy(), hb)


def device_gradient_terms(syno, plan, which, targets):
    """All terms the device enumerates for the listed target elements of dX (which = 1) or dW (which = 2), as rows
    (o, x, w) of flat offsets into out, X and W."""
    F = plan.free_size(which)
    t, q = (v.ravel() for v in np.meshgrid(np.asarray(targets, dtype=np.int64), np.arange(F, dtype=np.int64), indexing="ij"))
    a, b = plan.debug_gather(which, torch.from_numpy(t).cuda(), torch.from_numpy(q).cuda())
    a, b = a.cpu().numpy().astype(np.int64), b.cpu().numpy().astype(np.int64)
    ok = a >= 0
    assert np.array_equal(ok, b >= 0)
    a, b, t = a[ok], b[ok], t[ok]
    return np.stack([a, t, b] if which == syno.BWD_DATA else [a, b, t], axis=1)


GRADIENT_MAP_SMALL = [
    lambda: wl.config0().desc,
    lambda: wl.grouped_shift_unfold(2, 64, 64, 14, 14, 4, 3),
    lambda: wl.strided_depthwise(2, 8, 14, 14),
    lambda: wl.conv2d(1, 32, 32, 7, 7),
    lambda: wl.conv2d(2, 6, 10, 5, 9, 3, 3, F32, F32, (2, 3, 1, 0)),
    lambda: wl.matmul(24, 40, 56),
]


@pytest.mark.parametrize("mk", GRADIENT_MAP_SMALL)
def test_device_gradient_maps_equal_checker_term_sets(syno, oracle, mk):
    """Every term (o, x, w) of the checker's loop nest, grouped by x (backward-data) and by w (backward-weight), against
    what the device enumerates for every target element: the same set, each term once."""
    d = mk()
    plan = syno.Plan(d)
    n_o, n_r = int(np.prod(plan.out_shape)), plan.free_size(syno.FWD)
    o, r = (a.ravel() for a in np.meshgrid(np.arange(n_o), np.arange(n_r), indexing="ij"))
    xo, wo = oracle.gather_map(d, o, r)
    ok = xo >= 0
    terms = np.stack([o[ok], xo[ok].astype(np.int64), wo[ok].astype(np.int64)], axis=1)
    terms = terms[np.lexsort(terms.T[::-1])]
    for which, n_t in ((syno.BWD_DATA, int(np.prod(plan.x_shape))), (syno.BWD_WEIGHT, int(np.prod(plan.w_shape)))):
        got = device_gradient_terms(syno, plan, which, np.arange(n_t))
        got = got[np.lexsort(got.T[::-1])]
        assert got.shape == terms.shape and np.array_equal(got, terms), f"direction {which}"


@pytest.mark.parametrize("mk", [lambda: wl.grouped_shift_unfold(32), lambda: wl.strided_depthwise(64, 128, 28, 28),
                                lambda: wl.conv2d(32, 512, 512, 7, 7), lambda: wl.conv2d(32, 64, 64, 56, 56)])
def test_device_gradient_maps_full_size_against_checker(syno, oracle, mk):
    """At the benchmark shapes the whole term set does not fit, so for sampled targets: (1) no term twice, (2) as many
    terms as the checker counts (its scatter-form gradients of all-ones tensors count the terms per element), and (3)
    sampled terms are terms of the checker's loop nest (some Reduce point of that output has exactly these offsets)."""
    d = mk()
    plan = syno.Plan(d)
    xs, ws, red = oracle.describe(d)
    n_r = int(np.prod(red)) if red else 1
    rng = np.random.default_rng(7)
    nx, nw = int(np.prod(xs)), int(np.prod(ws))
    budget = 1 << 22
    tx = plane_samples(xs, rng, 64)
    tx = rng.choice(tx, min(tx.size, max(8, budget // plan.free_size(syno.BWD_DATA))), replace=False)
    tw = np.unique(np.concatenate([[0, nw - 1], rng.integers(0, nw, max(2, min(64, budget // plan.free_size(syno.BWD_WEIGHT))))]))
    ones = lambda shape: np.ones(shape)
    cnt_x, cnt_w = oracle.backward(d, ones(xs), ones(ws), ones(oracle.out_shape(d)), x_sample=np.sort(tx), w_sample=tw)
    for which, targets, cnt in ((syno.BWD_DATA, np.sort(tx), cnt_x), (syno.BWD_WEIGHT, tw, cnt_w)):
        got = device_gradient_terms(syno, plan, which, targets)
        assert np.unique(got, axis=0).shape[0] == got.shape[0], "a term is enumerated twice"
        col = 1 if which == syno.BWD_DATA else 2
        per_target = np.array([(got[:, col] == t).sum() for t in targets]) if targets.size <= 256 else None
        if per_target is not None:
            assert np.array_equal(per_target, cnt.astype(np.int64)), "term counts differ from the checker's"
        else:
            assert got.shape[0] == int(cnt.sum())
        pick = got[rng.choice(got.shape[0], min(got.shape[0], 2048), replace=False)]
        oo, rr = (v.ravel() for v in np.meshgrid(pick[:, 0], np.arange(n_r), indexing="ij"))
        xo, wo = oracle.gather_map(d, oo, rr)
        hit = (xo.reshape(-1, n_r) == pick[:, 1:2]) & (wo.reshape(-1, n_r) == pick[:, 2:3])
        assert hit.any(axis=1).all(), "the device enumerates a term the loop nest does not have"


# ------------------------------------------------------------------------------------------------
# the full-size workloads, in the configuration the benchmark times
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("stage", [0, 1, 2, 3])
def test_config1_full_size_sampled(syno, oracle, stage, bf16):
    run_all(syno, oracle, wl.config1(stage, bf16), 0, directions=(0,), full=False)


def test_config2_full_size(syno, oracle):
    run_all(syno, oracle, wl.config2(), 0, directions=(0,), full=True)


def test_config3_full_size(syno, oracle):
    run_all(syno, oracle, wl.config3(), 0, directions=(0,), full=True)


def test_config4_full_size_training_step(syno, oracle):
    run_all(syno, oracle, wl.config4(), 0, directions=(0, 1, 2), full=False, n_sample=8192)


def test_config3_full_size_backward_sampled(syno, oracle):
    names = run_all(syno, oracle, wl.config3_train(), 0, directions=(1, 2), full=False, n_sample=4096)
    assert names[1] == names[2] == "bandwidth_depthwise"


@pytest.mark.parametrize("stage", [0, 1, 2, 3])
@pytest.mark.parametrize("bf16", [False, True])
def test_config1_full_size_backward_sampled(syno, oracle, stage, bf16):
    """Backward passes of the conv-equivalent operator at the benchmark shapes (sampled against the checker)."""
    run_all(syno, oracle, wl.config1_train(stage, bf16), 0, directions=(1, 2), full=False, n_sample=2048)


# ------------------------------------------------------------------------------------------------
# operators evaluated in stages (Operator 1, Fig. 7)
# ------------------------------------------------------------------------------------------------
def chain_tol(desc):
    """rel-L2 bar of a staged operator: fp32 stages only accumulate (1e-5); bf16 stages also round every stored
    intermediate to nearest even, and where the two sides' fp32/fp64 sums straddle a rounding boundary the stored
    values differ by one bf16 ulp, which the next stage carries on (well inside the 2e-2 the inputs' type allows)."""
    return TOL_CHAIN_BF16 if desc.in_dtype == BF16 else TOL_ACC


def run_chain(syno, oracle, w, policy):
    """Forward and backward sweeps of a chain against the checker's chain, every tensor in full."""
    from syno_inputs.rng import bf16_bits_to_f32, to_bf16_bits
    bf16 = w.descs[0].in_dtype == BF16
    q = (lambda a: bf16_bits_to_f32(to_bf16_bits(np.asarray(a, dtype=np.float32)))) if bf16 else None
    tol = chain_tol(w.descs[0])
    chain = syno.Chain(w.descs, kernel_policy=policy)
    names = [[p.kernel(i) for i in range(3)] for p in chain.stages]
    print(f"[case] {w.descs[0].name} + {w.descs[1].name} kernels={names} policy={policy}", flush=True)
    X, G = to_dev(w.X, w.X_bits), to_dev(w.G, w.G_bits)
    Ws = [to_dev(v, b) for v, b in zip(w.Ws, w.Ws_bits or [None] * len(w.Ws))]
    out, acts = chain.forward(X, Ws)
    torch.cuda.synchronize()
    ref = oracle.chain_forward(w.descs, w.X, w.Ws, quantize=q)
    for i, a in enumerate(acts):
        e = rel_l2(to_host(a), ref[i])
        assert e <= tol, f"stage {i} output rel-L2 {e:.3e} > {tol}"
    e = rel_l2(to_host(out), ref[-1])
    print(f"       chain output rel-L2 {e:.2e}", flush=True)
    assert e <= tol, f"chain output rel-L2 {e:.3e} > {tol}"
    print(f"[case] {w.descs[0].name} backward sweep", flush=True)
    dX, dWs = chain.backward(X, Ws, acts, G)
    torch.cuda.synchronize()
    rdx, rdws = oracle.chain_backward(w.descs, w.X, w.Ws, w.G, quantize=q)
    e = rel_l2(to_host(dX), rdx)
    print(f"       chain dX rel-L2 {e:.2e}", flush=True)
    assert e <= tol, f"chain dX rel-L2 {e:.3e} > {tol}"
    for i, (d, r) in enumerate(zip(dWs, rdws)):
        assert d.dtype == torch.float32
        e = rel_l2(to_host(d), r)
        print(f"       chain dW[{i}] rel-L2 {e:.2e}", flush=True)
        assert e <= tol, f"chain dW[{i}] rel-L2 {e:.3e} > {tol}"
    # without dX: the weights' gradients are the same, and nothing else is needed
    _, dWs2 = chain.backward(X, Ws, acts, G, want_dx=False)
    torch.cuda.synchronize()
    for a, b in zip(dWs, dWs2):
        assert torch.equal(a, b)
    return names


def test_operator1_bf16_stages_fp32_result(syno, oracle):
    """bf16 inputs and intermediate, fp32 result: the gradient between the stages is bf16 (what the first stage
    reads), although the second stage's own backward-data type would be its fp32 output type."""
    w = wl.make_operator1(3, 24, 13, seed=23, bf16=True, Co=32, Wd=19, g=4, s=2, with_grad=True, out_f32=True)
    run_chain(syno, oracle, w, 0)
    run_chain(syno, oracle, w, 1)


@pytest.mark.parametrize("policy", [1, 0])
@pytest.mark.parametrize("bf16", [False, True])
def test_operator1_small(syno, oracle, bf16, policy):
    run_chain(syno, oracle, wl.make_operator1(3, 24, 13, seed=21, bf16=bf16, Co=32, Wd=19, g=4, s=2, with_grad=True),
              policy)
    run_chain(syno, oracle, wl.make_operator1(2, 16, 9, seed=22, bf16=bf16, Co=16, Wd=10, g=2, s=1, with_grad=True),
              policy)


@pytest.mark.parametrize("k1", [3, 5])
@pytest.mark.parametrize("dt", ["f32", "bf16", "bf16_f32out"])
@pytest.mark.parametrize("shape", [
    (3, 16, 16, 5, 12, 4, 2),      # runs of 4 pixels, fewer runs than one workgroup's lanes
    (2, 40, 40, 6, 10, 2, 1),      # runs of 2 (of 1 for the 5-wide window); D = 20 and Cg = 20: several tiles of each, ragged
    (2, 12, 24, 4, 7, 3, 2),       # single pixels (odd width); D = 4, Cg = 4
    (5, 8, 8, 17, 16, 1, 1),       # one group; more runs than one workgroup
])
def test_share_window_stage_small(syno, oracle, shape, dt, k1):
    """The first stage of Operator 1 by itself on the streaming kernels (3- and 5-wide windows), all three passes,
    element by element."""
    N, Cin, Co, H, W, g, s = shape
    i_dt = F32 if dt == "f32" else BF16
    o_dt = BF16 if dt == "bf16" else F32
    d = wl.operator1_stage1(N, Cin, Co, H, W, g, s, k1, i_dt, o_dt)
    xs, ws, _ = oracle.describe(d)
    os_ = oracle.out_shape(d)
    st = wl.Stream(31)
    w = wl._finish(d, xs, ws, os_, st.normal(xs), st.uniform_pm(0.5, ws), st.normal(os_), Cin // g)
    names = run_all(syno, oracle, w, 0)
    assert names == ["bandwidth_share_window"] * 3


def test_share_window_bf16_rounding_is_nearest_even(syno, oracle):
    """With Cg = 2 and the weights 1 and 2^-9 every sum x0 + x1/512 of two bf16 values is exact in fp32 (or
    rounded once, identically, by the fused multiply-add), so the stored bf16 must be the round-to-nearest-even
    of the checker's value, bit for bit."""
    from syno_inputs.rng import to_bf16_bits
    N, H, W = 2, 6, 16
    d = wl.operator1_stage1(N, 2, 1, H, W, 1, 1, 3, BF16, BF16)
    xs, ws, _ = oracle.describe(d)
    st = wl.Stream(33)
    Xb = to_bf16_bits(st.normal(xs))
    Wv = np.empty(ws, dtype=np.float32)
    Wv[0, 0, 0, :], Wv[0, 0, 1, :] = 1.0, 2.0 ** -9
    Wb = to_bf16_bits(Wv)
    from syno_inputs.rng import bf16_bits_to_f32
    ref = oracle.forward(d, bf16_bits_to_f32(Xb), Wv)
    plan = syno.Plan(d)
    assert plan.kernel(0) == "bandwidth_share_window"
    out = plan.forward(to_dev(None, Xb), to_dev(None, Wb))
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, to_bf16_bits(ref.astype(np.float32)))


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("stage", [0, 3])
def test_operator1_full_size(syno, oracle, stage, bf16):
    """Operator 1 in place of a ResNet-18 stage's convolution, N = 32: the first stage (C = 64, 56 x 56: the shape
    the benchmark's detail times) and the last (C = 512, 7 x 7: odd width, 64 x 128 weights per group and window
    position, several tiles of each in the first-stage kernels)."""
    names = run_chain(syno, oracle, wl.operator1(stage, bf16), 0)
    assert names[0] == ["bandwidth_share_window"] * 3


# ------------------------------------------------------------------------------------------------
# the materialised-reduction pass: one loop nest in, stages out, same result as the loop nest
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dt", ["f32", "bf16", "bf16_f32out"])
@pytest.mark.parametrize("mk", [
    lambda i, o: wl.window_of_sums_1d(120, 3, 2, None, i, o),
    lambda i, o: wl.window_of_sums_1d(90, 5, 3, "k", i, o),
    lambda i, o: wl.window_of_sums_1d(64, 3, 4, "s", i, o),
    lambda i, o: wl.pooled_conv2d(3, 24, 40, 13, 10, 2, 3, i, o),
])
def test_materialised_chain_equals_the_single_loop_nest(syno, oracle, mk, dt):
    """The checker evaluates the graph as written (one loop nest); the library cuts it into stages."""
    d = mk(F32 if dt == "f32" else BF16, BF16 if dt == "bf16" else F32)
    chain = syno.Chain.materialized(d)
    assert len(chain.stages) >= 2
    xs, ws, _ = oracle.describe(d)
    os_ = oracle.out_shape(d)
    st = wl.Stream(51)
    w = wl._finish(d, xs, ws if ws else (1,), os_, st.normal(xs), st.uniform_pm(0.5, ws if ws else (1,)), st.normal(os_), 1)
    tol = chain_tol(d)
    print(f"[case] {d.name} {dt}: {len(chain.stages)} stages, weight in stage {chain.weight_stage}, kernels "
          f"{[p.kernel(0) for p in chain.stages]}", flush=True)
    X, W, G = to_dev(w.X, w.X_bits), to_dev(w.W, w.W_bits), to_dev(w.G, w.G_bits)
    Ws = [W if i == chain.weight_stage else None for i in range(len(chain.stages))]
    out, acts = chain.forward(X, Ws)
    torch.cuda.synchronize()
    e = rel_l2(to_host(out), oracle.forward(d, w.X, w.W))
    assert e <= tol, f"forward rel-L2 {e:.3e} > {tol}"
    dX, dWs = chain.backward(X, Ws, acts, G)
    torch.cuda.synchronize()
    rdx, rdw = oracle.backward(d, w.X, w.W, w.G)
    e = rel_l2(to_host(dX), rdx)
    assert e <= tol, f"dX rel-L2 {e:.3e} > {tol}"
    assert all((g is None) == (i != chain.weight_stage) for i, g in enumerate(dWs))
    e = rel_l2(to_host(dWs[chain.weight_stage]), rdw)
    assert e <= tol, f"dW rel-L2 {e:.3e} > {tol}"


@pytest.mark.parametrize("dt", ["f32", "bf16", "bf16_f32out"])
@pytest.mark.parametrize("shape", [(3, 24, 32, 13, 19, 4, 2, 3), (2, 16, 16, 9, 10, 2, 1, 3), (2, 8, 8, 6, 7, 1, 2, 5)])
def test_operator1_single_graph_with_two_weights(syno, oracle, shape, dt):
    """Operator 1 handed over as ONE pGraph with two weights: the library's materialised-reduction pass cuts it into
    the two single-weight stages of the paper's listing; the checker evaluates the single two-weight loop nest."""
    N, Cin, Co, H, W, g, s_, k1 = shape
    d = wl.operator1_graph(N, Cin, Co, H, W, g, s_, k1, F32 if dt == "f32" else BF16, BF16 if dt == "bf16" else F32)
    with pytest.raises(syno.SynoError) as e:
        syno.Plan(d)                    # several weights: only as stages
    assert e.value.status == 4
    chain = syno.Chain.materialized(d)
    assert len(chain.stages) == 2 and chain.stage_weight == [0, 1]
    D, Cg = Co // g // s_, Cin // g
    assert chain.stages[0].w_shape == (D, g, Cg, k1) and chain.stages[1].w_shape == (Co, D, g, k1, k1)
    if k1 == 3:      # the cut-off stages are laid out like the hand-written ones and run on the same kernels
        fam = "mfma_contraction_f32" if dt == "f32" else "mfma_contraction_bf16"
        assert [p.kernel(0) for p in chain.stages] == ["bandwidth_share_window", fam]
    st = wl.Stream(71)
    from syno_inputs.rng import bf16_bits_to_f32, to_bf16_bits
    q = (lambda a: bf16_bits_to_f32(to_bf16_bits(np.asarray(a, dtype=np.float32)))) if dt != "f32" else (lambda a: np.asarray(a, dtype=np.float32))
    X, G = q(st.normal((N, Cin, H, W))), q(st.normal((N, Co, H, W)))
    w1, w2 = q(st.uniform_pm(1.0 / np.sqrt(Cg), (D, g, Cg, k1))), q(st.uniform_pm(1.0 / np.sqrt(D * g * k1 * k1), (Co, D, g, k1, k1)))
    dev = lambda a: to_dev(a, to_bf16_bits(a) if dt != "f32" else None)
    Xd, Gd, Ws = dev(X), dev(G), [dev(w1), dev(w2)]
    tol = chain_tol(d)
    out, acts = chain.forward(Xd, Ws)
    torch.cuda.synchronize()
    e_out = rel_l2(to_host(out), oracle.forward_multi(d, X, [w1, w2]))
    dX, dWs = chain.backward(Xd, Ws, acts, Gd)
    torch.cuda.synchronize()
    rdx, rdws = oracle.backward_multi(d, X, [w1, w2], G)
    errs = [e_out, rel_l2(to_host(dX), rdx)] + [rel_l2(to_host(a), b) for a, b in zip(dWs, rdws)]
    print(f"[case] {d.name} {dt}: kernels {[p.kernel(0) for p in chain.stages]} rel-L2 out/dX/dW1/dW2 = "
          + "/".join(f"{v:.2e}" for v in errs), flush=True)
    assert max(errs) <= tol, errs


# ------------------------------------------------------------------------------------------------
# pure views (no Reduce) and small gather-and-add operators: the table-driven streaming kernel forwards, index
# programs backwards
# ------------------------------------------------------------------------------------------------
def view_cases():
    def expand_stride(i, o):
        # out[n,r,k] = X[n, 3*k] * Wt[k]: Expand over r, Stride 3 under a Shared iterator
        b = Builder([("n", 3), ("r", 4), ("k", 8)])
        kx, kw = b.share(2)
        b.expand(1)
        return b.finish([0, b.stride(kx, 3)], [kw], i, o)

    def expand_long(i, o):
        # out[a,r,s] = X[a] * Wt[a]: 96 * 128 copies per element, so both gradients are long sums sliced over workgroups
        b = Builder([("a", 37), ("r", 96), ("s", 128)])
        ax, aw = b.share(0)
        b.expand(1)
        b.expand(2)
        return b.finish([ax], [aw], i, o)

    def stride_gaps_odd(i, o):
        # out[a,k] = X[3*a, k] * Wt[k]: two of three rows of X are never read (zero gradient); X has 105 elements, an
        # odd number, so a bf16 dX ends in half a word
        b = Builder([("a", 7), ("k", 5)])
        kx, kw = b.share(1)
        return b.finish([b.stride(0, 3), kx], [kw], i, o)

    def pixel_shuffle(i, o):
        # Table 2's PixelShuffle: out[n,c,H,W] = X[n, c, H%r, W%r, H/r, W/r] * Wt[c]
        b = Builder([("n", 2), ("c", 3), ("H", 6), ("W", 10)])
        cx, cw = b.share(1)
        hq, hr = b.merge(2, 2)
        wq, wr = b.merge(3, 2)
        return b.finish([0, cx, hr, wr, hq, wq], [cw], i, o)

    def shift_of_digit(i, o):
        # a Shift applied to one digit of an output axis: X[(h/4), ((h%4)+3) mod 4, w]
        b = Builder([("h", 12), ("w", 8)])
        q, r = b.merge(0, 4)
        return b.finish([q, b.shift(r, 3), 1], [], i, o)

    def block_sums(i, o):
        # out[n,c,h,w] = Wt[c] * sum_{sh,sw} X[n, c, 2h+sh, 3w+sw]: 6 sum points per output
        b = Builder([("n", 2), ("c", 5), ("h", 4), ("w", 8)])
        cx, cw = b.share(1)
        sh, sw = b.reduce(2), b.reduce(3)
        return b.finish([0, cx, b.split(2, sh), b.split(3, sw)], [cw], i, o)

    return {
        "block_sums": block_sums,
        "small_matmul": lambda i, o: wl.matmul(9, 3, 7, i, o),     # 3 columns: not folded into a convolution
        "shift_scale_v4": lambda i, o: wl.shifted_scale(3, 5, 7, 12, i, o),
        "shift_scale_v1": lambda i, o: wl.shifted_scale(2, 3, 5, 7, i, o),
        "pixel_unshuffle": lambda i, o: wl.pixel_unshuffle(2, 3, 5, 8, 2, i, o),
        "pixel_unshuffle_r3": lambda i, o: wl.pixel_unshuffle(1, 2, 4, 5, 3, i, o),
        "expand_stride": expand_stride, "pixel_shuffle": pixel_shuffle, "shift_of_digit": shift_of_digit,
        "expand_long": expand_long, "stride_gaps_odd": stride_gaps_odd,
    }


@pytest.mark.parametrize("dt", ["f32", "bf16", "bf16_f32out"])
@pytest.mark.parametrize("name", list(view_cases()))
def test_pure_views_small(syno, oracle, name, dt):
    i_dt = F32 if dt == "f32" else BF16
    o_dt = BF16 if dt == "bf16" else F32
    d = view_cases()[name](i_dt, o_dt)
    xs, ws, _ = oracle.describe(d)
    os_ = oracle.out_shape(d)
    st = wl.Stream(61)
    w = wl._finish(d, xs, ws if ws else (1,), os_, st.normal(xs), st.uniform_pm(2.0, ws if ws else (1,)), st.normal(os_), 1)
    names = run_all(syno, oracle, w, 0)
    assert names[0] == "bandwidth_view"
    # one-to-one views scatter their backward-data through the same tables; the others sum or leave gaps
    one_to_one = name in ("shift_scale_v4", "shift_scale_v1", "pixel_unshuffle", "pixel_unshuffle_r3", "pixel_shuffle",
                          "shift_of_digit")
    # the others (an Expand sums, a Stride leaves gaps, sum points) and every weight gradient gather through the tables
    assert names[1] == names[2] == "bandwidth_view"
    plan = syno.Plan(d)
    assert plan.describe(1).endswith("scatter") == one_to_one and "gather" in plan.describe(2)
    if one_to_one:   # every element of dX is written: nothing of a pre-filled buffer survives
        plan = syno.Plan(d)
        G, W = to_dev(w.G, w.G_bits), to_dev(w.W, w.W_bits)
        dX = plan.backward_data(G, W)
        dX2 = torch.full_like(dX, 7.0)
        plan.backward_data(G, W, dX=dX2)
        torch.cuda.synchronize()
        assert torch.equal(dX, dX2)


def test_pure_view_full_size(syno, oracle):
    """The shapes the benchmark's detail times (102.8 MB in and out), all three passes, in full against the checker
    (the weight gradients are one sum of 200704 products per channel, and one of 25.7 million)."""
    for d in (wl.shifted_scale(64, 128, 56, 56), wl.pixel_unshuffle(64, 128, 28, 28, 2)):
        xs, ws, _ = oracle.describe(d)
        st = wl.Stream(62)
        w = wl._finish(d, xs, ws if ws else (1,), oracle.out_shape(d), st.normal(xs), st.uniform_pm(2.0, ws if ws else (1,)),
                       st.normal(oracle.out_shape(d)), 1)
        assert run_all(syno, oracle, w, 0, full=True) == ["bandwidth_view"] * 3


# ------------------------------------------------------------------------------------------------
# matrix products (Table 2) run as 1x1 convolutions with the operands' roles exchanged
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("M,K,N", [(37, 45, 29), (130, 72, 112), (64, 200, 640), (9, 16, 7 * 13)])
def test_matmul_small(syno, oracle, M, K, N, bf16):
    names = run_all(syno, oracle, wl.make_matmul(M, K, N, seed=41, bf16=bf16, with_grad=True), 0)
    assert names == ["mfma_contraction_transposed"] * 3


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("splits", [2, 3])
def test_contraction_with_split_reduction(syno, oracle, bf16, splits):
    """Several workgroups per output tile, each summing a range of the channel chunks (the last range is shorter, and
    with 80 channels the last bf16 chunk is incomplete); the partial results are added by a second kernel."""
    w = wl.make_conv(2, 80, 12, seed=47, bf16=bf16, Co=96, with_grad=True)
    plan = syno.Plan(w.desc, mfma_splits=splits)
    for which in (0, 1):
        assert f"reduction-splits={splits}" in plan.describe(which), plan.describe(which)
        assert plan.workspace_bytes(which) >= splits * 2 * (96, 80)[which] * 12 * 12 * 4
    names = run_all(syno, oracle, w, 0, directions=(0, 1), mfma_splits=splits)
    assert all(n.startswith("mfma_contraction") for n in names[:2])
    m = wl.make_matmul(136, 200, 640, seed=48, bf16=bf16, with_grad=True)
    assert "reduction-splits" in syno.Plan(m.desc, mfma_splits=splits).describe(2)
    assert run_all(syno, oracle, m, 0, mfma_splits=splits) == ["mfma_contraction_transposed"] * 3


@pytest.mark.parametrize("M,K,N", [(130, 72, 112), (40, 7 * 9, 200)])
def test_matmul_small_bf16_result(syno, oracle, M, K, N):
    """With a bf16 result type the forward product and dX (the product G * W^T on a transposed copy of W) stay on
    the contraction kernel; dW, which is fp32 inside, is left to the bandwidth-bound kernels."""
    names = run_all(syno, oracle, wl.make_matmul(M, K, N, seed=43, bf16=True, with_grad=True, out_bf16=True), 0)
    # (63 sum points still count as a few: that product's dW gathers through the view tables, a thread per element)
    assert names == ["mfma_contraction_transposed", "mfma_contraction_transposed",
                     "bandwidth_view" if K <= 64 else "generic_index_program"]


@pytest.mark.parametrize("N,C,Co,H,bf16", [(48, 768, 768, 7, False), (128, 64, 64, 56, False), (16, 2048, 512, 7, False),
                                          (64, 256, 512, 14, True)])
def test_tile_order_across_xcds_sampled(syno, oracle, N, C, Co, H, bf16):
    """Shapes whose tiles are dealt to the XCDs in rectangles of several kinds: more tiles than are resident at once
    (walked rows of tiles first where the weights outgrow an L2, panels first otherwise), a rectangle per reduction
    split, different splits forward and backward.  Every tile must still be computed exactly once: sampled outputs
    (image borders, tile boundaries, uniform draws) against the checker."""
    w = wl.make_conv(N, C, H, seed=61, bf16=bf16, Co=Co, with_grad=True)
    plan = syno.Plan(w.desc)
    assert all("tiles-per-xcd=" in plan.describe(which) for which in (0, 1)), plan.describe(0)
    if (N, C) == (48, 768):
        assert "(rows first)" in plan.describe(0)
    names = run_all(syno, oracle, w, 0, directions=(0, 1), full=False, n_sample=1024)
    assert all(n.startswith("mfma_contraction") for n in names[:2])


@pytest.mark.parametrize("bf16", [False, True])
def test_qkv_projection_full_size_sampled(syno, oracle, bf16):
    names = run_all(syno, oracle, wl.qkv_projection(bf16), 0, full=False, n_sample=2048)
    assert names == ["mfma_contraction_transposed"] * 3


def test_rejects_wrong_arguments(syno):
    plan = syno.Plan(wl.conv2d(1, 4, 4, 5, 5))
    X = torch.zeros(plan.x_shape, device="cuda")
    W = torch.zeros(plan.w_shape, device="cuda")
    with pytest.raises(ValueError):
        plan.forward(X[:, :2], W)
    with pytest.raises(ValueError):
        plan.forward(X.to(torch.bfloat16), W)
    lib = syno.load_library()
    assert lib.syno_forward(plan._h, None, W.data_ptr(), X.data_ptr(), None, None) == 1
