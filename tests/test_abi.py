"""Host-side checks of the GPU library: it loads, exports what the header declares, rejects bad
graphs, and its lowered index maps (forward and both gradients) agree with the CPU checker bit
for bit.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from syno_inputs import BF16, F32, Builder, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def syno():
    import paper_2410_23745_amd as s
    if not os.path.exists(s.library_path()):
        from paper_2410_23745_amd import build
        build.build()
    s.load_library()
    return s


def test_library_exports_every_declared_symbol(syno):
    header = open(os.path.join(ROOT, "include", "syno.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(syno_[a-z_]+)\s*\(", header))
    assert {"syno_plan_create", "syno_forward", "syno_backward_data", "syno_backward_weight",
            "syno_plan_destroy"} <= declared
    lib = ctypes.CDLL(syno.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), name


def test_status_strings(syno):
    lib = syno.load_library()
    assert lib.syno_status_string(0) == b"ok"
    assert all(lib.syno_status_string(i) for i in range(8))


def test_rejects_invalid_graphs(syno):
    b = Builder([("i", 10)])
    q, r = b.merge(0, 3)
    with pytest.raises(syno.SynoError) as e:
        syno.Plan(b.finish([q, r], []))
    assert e.value.status == 2
    b = Builder([("i", 4), ("j", 4)])
    with pytest.raises(syno.SynoError):
        syno.Plan(b.finish([0], []))                 # j never consumed
    b = Builder([("i", 4)])
    with pytest.raises(syno.SynoError):
        syno.Plan(b.finish([0, 0], []))              # i consumed twice
    b = Builder([("i", 4)])
    r = b.reduce(3)
    b.expand(r)
    with pytest.raises(syno.SynoError):
        syno.Plan(b.finish([0], []))                 # Reduce straight into Expand
    b = Builder([("i", 1 << 20), ("j", 1 << 12)])
    v = b.split(0, 1)
    with pytest.raises(syno.SynoError) as e:
        syno.Plan(b.finish([v], []))                 # 2^32 elements
    assert e.value.status == 4
    for size, fits in ((1 << 18, True), (1 << 20, False)):   # backward-data sums i x r points per element: 2^30, 2^32
        b = Builder([("i", size), ("k", 2)])
        r = b.reduce(1 << 12)
        b.expand(0)
        if fits:
            syno.Plan(b.finish([1], [r]))
        else:
            with pytest.raises(syno.SynoError) as e:
                syno.Plan(b.finish([1], [r]))
            assert e.value.status == 4


def test_shapes_match_the_checker(syno, oracle):
    for d in (wl.conv2d(2, 3, 4, 5, 6), wl.grouped_shift_unfold(2), wl.strided_depthwise(2, 4, 7, 7), wl.matmul(3, 4, 5)):
        p = syno.Plan(d)
        xs, ws, red = oracle.describe(d)
        assert p.x_shape == xs and p.w_shape == ws and p.out_shape == oracle.out_shape(d)
        assert p.free_size(syno.FWD) == int(np.prod(red))


def pixel_unshuffle_conv():
    """A graph outside the convolution-like form: Merge above Unfold, Stride, Expand, two Shifts."""
    b = Builder([("n", 2), ("co", 3), ("h", 6), ("e", 2)])
    c = b.reduce(4)
    cx, cw = b.share(c)
    k = b.reduce(3)
    kx, kw = b.share(k)
    u = b.unfold(2, kx)          # h + k - 1 : 6
    q, r = b.merge(u, 2)         # (u/2, u%2) : 3, 2
    s = b.shift(q, -1)
    t = b.stride(r, 3)           # 3*(u%2) : 6
    t2 = b.shift(t, 2, by=s, coef=1)
    b.expand(3)
    return b.finish([0, cx, s, t2], [1, cw, kw])


CASES = [
    lambda: wl.conv2d(2, 3, 4, 5, 6),
    lambda: wl.conv2d(1, 2, 2, 4, 5, 4, 2),
    lambda: wl.grouped_shift_unfold(2, 8, 8, 5, 4, 4, 3),
    lambda: wl.strided_depthwise(2, 3, 3, 4),
    lambda: wl.matmul(3, 4, 5),
    pixel_unshuffle_conv,
]


@pytest.mark.parametrize("mk", CASES)
def test_index_maps_bit_exact_against_checker(syno, oracle, mk):
    d = mk()
    p = syno.Plan(d)
    _, _, red = oracle.describe(d)
    n_o, n_r = int(np.prod(p.out_shape)), int(np.prod(red)) if red else 1
    o, r = (a.ravel() for a in np.meshgrid(np.arange(n_o), np.arange(n_r), indexing="ij"))
    xo, wo = oracle.gather_map(d, o, r)
    a, b = p.debug_gather_host(syno.FWD, o, r)
    assert np.array_equal(a, xo) and np.array_equal(b, wo)
    ok = xo >= 0
    terms = sorted(zip(o[ok].tolist(), xo[ok].tolist(), wo[ok].tolist()))
    # The gradients enumerate the same set of terms (o, x, w), grouped by x or by w; the order inside a group is
    # the planner's own, so compare as sorted sets: every term once, none invented.
    for which, n_t in ((syno.BWD_DATA, int(np.prod(p.x_shape))), (syno.BWD_WEIGHT, int(np.prod(p.w_shape)))):
        t, q = (v.ravel() for v in np.meshgrid(np.arange(n_t), np.arange(p.free_size(which)), indexing="ij"))
        a, b = p.debug_gather_host(which, t, q)
        v = a >= 0
        assert np.array_equal(v, b >= 0)
        got = zip(a[v].tolist(), t[v].tolist(), b[v].tolist()) if which == syno.BWD_DATA else \
            zip(a[v].tolist(), b[v].tolist(), t[v].tolist())
        assert sorted(got) == terms


def test_out_of_range_points_yield_minus_one(syno):
    p = syno.Plan(wl.conv2d(1, 2, 2, 3, 3))
    a, b = p.debug_gather_host(syno.FWD, [0, 18, -1, 0], [0, 0, 0, 18])
    assert a[1] == -1 and a[2] == -1 and a[3] == -1 and b[2] == -1


def test_kernel_choice(syno):
    names = lambda d: [syno.Plan(d).kernel(i) for i in range(3)]
    assert all(n == "generic_index_program" for n in names(wl.matmul(3, 3, 70)))     # 3 columns: too narrow to fold
    assert names(wl.matmul(3, 3, 5)) == ["bandwidth_view"] * 3   # 5 sum points; the gradients gather through the same tables
    assert all(n == "generic_index_program" for n in names(pixel_unshuffle_conv()))
    # the benchmarked workloads run on the tuned families, not on the index-program kernels
    for stage in range(4):
        C, H = wl.RESNET18_STAGES[stage]
        assert names(wl.conv2d(32, C, C, H, H))[:2] == ["mfma_contraction_f32"] * 2
        assert names(wl.conv2d(32, C, C, H, H, 3, 3, BF16, F32))[:2] == ["mfma_contraction_bf16"] * 2
    # weights in any axis order stay on the tuned kernels, in all three passes
    for wo in ((1, 0, 2, 3), (2, 3, 1, 0), (0, 3, 2, 1)):
        assert names(wl.conv2d(3, 24, 40, 13, 19, 3, 3, F32, F32, wo)) == ["mfma_contraction_f32"] * 3
        assert names(wl.conv2d(3, 40, 24, 13, 19, 3, 3, BF16, F32, wo)) == ["mfma_contraction_bf16"] * 3
        assert names(wl.conv2d(2, 128, 128, 28, 28, 3, 3, F32, F32, wo)) == ["mfma_contraction_f32"] * 3
    assert names(wl.grouped_shift_unfold(2, 96, 96, 9, 11, 3, 3, BF16, F32, (2, 0, 3, 1))) == ["mfma_contraction_bf16"] * 3
    assert names(wl.conv2d(1, 16, 16, 16, 16))[0] == "mfma_contraction_f32"
    assert names(wl.grouped_shift_unfold(32)) == ["mfma_contraction_bf16"] * 3
    assert names(wl.grouped_shift_unfold(128)) == ["mfma_contraction_bf16"] * 3
    assert names(wl.strided_depthwise(64, 128, 28, 28))[0] == "bandwidth_depthwise"
    p = syno.Plan(wl.grouped_shift_unfold(128))
    # 64 channels per group: forward and backward-data read the weights as they lie in memory, no workspace;
    # backward-weight keeps its split partials there
    assert p.workspace_bytes(syno.FWD) == 0 and p.workspace_bytes(syno.BWD_DATA) == 0
    assert p.workspace_bytes(syno.BWD_WEIGHT) > 0
    # more channels than one chunk holds: backward-data of a 3x3 window takes its weights from the forward layout as
    # they lie (bf16 and fp32 alike); weights in another axis order are packed (bf16) or transposed (fp32) into the
    # workspace, and so are the bf16 weights of other windows
    p = syno.Plan(wl.conv2d(32, 128, 128, 28, 28, 3, 3, BF16, F32))
    assert p.workspace_bytes(syno.FWD) == 0 and p.workspace_bytes(syno.BWD_DATA) == 0 and "weights=direct" in p.describe(syno.BWD_DATA)
    q = syno.Plan(wl.conv2d(32, 128, 128, 28, 28, 3, 3, BF16, F32, (1, 0, 2, 3)))
    assert q.workspace_bytes(syno.BWD_DATA) > 0 and "weights=packed" in q.describe(syno.BWD_DATA)
    q = syno.Plan(wl.conv2d(32, 128, 128, 28, 28, 1, 1, BF16, F32))
    assert q.workspace_bytes(syno.BWD_DATA) > 0 and "weights=packed" in q.describe(syno.BWD_DATA)
    q = syno.Plan(wl.conv2d(32, 128, 128, 28, 28))
    assert q.workspace_bytes(syno.BWD_DATA) == 0 and "turned-while-staged" in q.describe(syno.BWD_DATA)
    q = syno.Plan(wl.conv2d(32, 128, 128, 28, 28, 3, 3, F32, F32, (1, 0, 2, 3)))
    assert q.workspace_bytes(syno.BWD_DATA) == 128 * 128 * 9 * 4 and "transposed-copy" in q.describe(syno.BWD_DATA)
    assert "grid=" in p.describe(syno.FWD)
    # per-plan options: the generic kernels on request; a named tile variant of the contraction kernel
    generic = syno.Plan(wl.strided_depthwise(2, 4, 7, 7), kernel_policy=1)
    assert all(generic.kernel(i) == "generic_index_program" for i in range(3))
    d = wl.conv2d(2, 128, 128, 28, 28)
    for variant, rows in ((0, 4), (1, 8), (3, 4)):
        p = syno.Plan(d, mfma_variant=variant + 1, mfma_rows=rows)
        assert f"variant={variant} rows/block={rows} " in p.describe(syno.FWD)
    assert "splits=2 " in syno.Plan(wl.grouped_shift_unfold(128), dw_workgroups=8).describe(syno.BWD_WEIGHT)


def test_chain_plans_operator1_on_the_host(syno):
    w = wl.make_operator1(2, 16, 12, g=4, s=2)
    chain = syno.Chain(w.descs)
    assert len(chain.stages) == 2
    assert chain.stages[0].x_shape == w.x_shape and chain.stages[0].out_shape == w.inter_shapes[0]
    assert chain.stages[0].w_shape == w.w_shapes[0] and chain.stages[1].w_shape == w.w_shapes[1]
    assert chain.stages[1].out_shape == w.out_shape
    lib = syno.load_library()
    assert lib.syno_chain_stages(chain._h) == 2 and lib.syno_chain_plan(chain._h, 2) is None
    # backward workspace: both intermediate-gradient buffers plus the largest stage workspace
    inter = int(np.prod(w.inter_shapes[0])) * 4
    stage_ws = max(p.workspace_bytes(k) for p in chain.stages for k in (1, 2))
    assert chain.workspace_bytes(1) >= 2 * inter + stage_ws
    assert chain.workspace_bytes(0) == max(p.workspace_bytes(0) for p in chain.stages)


def test_chain_rejects_stages_that_do_not_fit(syno):
    a, b = wl.conv2d(1, 4, 6, 5, 5), wl.conv2d(1, 5, 4, 5, 5)          # 6 channels out, 5 channels in
    with pytest.raises(syno.SynoError):
        syno.Chain([a, b])
    c = wl.conv2d(1, 6, 4, 5, 5, in_dtype=BF16)                          # element types differ
    with pytest.raises(syno.SynoError):
        syno.Chain([a, c])
    with pytest.raises(syno.SynoError):
        syno.Chain([])


def test_unreduced_window_goes_to_the_streaming_family(syno):
    stage1 = wl.operator1_stage1(2, 16, 16, 8, 8, g=4, s=2)
    p = syno.Plan(stage1)
    assert [p.kernel(i) for i in range(3)] == ["bandwidth_share_window"] * 3
    assert p.workspace_bytes(0) == 0 and p.workspace_bytes(1) == 0 and p.workspace_bytes(2) > 0
    # 5-wide windows are in the family too; a 7-wide one and an fp32 -> bf16 stage are valid but not: index-program kernels
    assert [syno.Plan(wl.operator1_stage1(2, 16, 16, 8, 8, g=4, s=2, k1=5)).kernel(i) for i in range(3)] == ["bandwidth_share_window"] * 3
    assert syno.Plan(wl.operator1_stage1(2, 16, 16, 8, 8, g=4, s=2, k1=7)).kernel(0) == "generic_index_program"
    assert syno.Plan(wl.operator1_stage1(2, 16, 16, 8, 8, 4, 2, 3, F32, BF16)).kernel(0) == "generic_index_program"
    # the same window Reduced is the convolution-like form, not this one
    assert syno.Plan(wl.conv2d(2, 16, 16, 8, 8, 1, 3)).kernel(0).startswith("mfma")


def test_window_over_flattened_axes_is_a_contraction(syno):
    # Unfold below a Merge whose halves are adjacent axes of X: one long row for the convolution-like analysis
    p = syno.Plan(wl.flat_window(2, 16, 24, 6, 10, 3))
    assert p.x_shape == (2, 16, 6, 10) and p.out_shape == (2, 24, 60)
    assert [p.kernel(i) for i in range(3)] == ["mfma_contraction_f32"] * 3
    # rows longer than a workgroup tile (512 pixels) are left to the index-program kernels
    assert syno.Plan(wl.flat_window(2, 16, 24, 28, 28, 3)).kernel(0) == "generic_index_program"
    # the halves in the other order are a transposition, not one axis
    b = Builder([("n", 2), ("co", 24), ("i", 60)])
    c = b.reduce(16); cx, cw = b.share(c)
    j = b.reduce(3); jx, jw = b.share(j)
    q, r = b.merge(b.unfold(2, jx), 10)
    assert syno.Plan(b.finish([0, cx, r, q], [1, cw, jw])).kernel(0) == "generic_index_program"


def test_strided_convolution_runs_on_the_contraction_kernels(syno):
    for K in (3, 1):
        p = syno.Plan(wl.conv2d(2, 16, 24, 6, 6, K, stride=2))
        assert p.x_shape == (2, 16, 12, 12) and p.out_shape == (2, 24, 6, 6)
        # forward gathers the strided window into LDS; the gradients run at stride 1 on the stride's phase planes
        assert [p.kernel(i) for i in range(3)] == ["mfma_contraction_f32", "mfma_contraction_phases", "mfma_contraction_phases"]
        assert "depth-to-space" in p.describe(1) and "space-to-depth" in p.describe(2)
        # workspaces: the re-ordered weights and the phase planes of dX; the phase planes of X and the stride-1 gradient
        # (the 1x1 window only reads phase (0,0): the sub-sampled X and dX instead of all four phase planes)
        win, phases = (3, 4) if K == 3 else (1, 1)
        assert p.workspace_bytes(1) >= 4 * (phases * 16 * 24 * win * win + 2 * phases * 16 * 6 * 6)
        assert p.workspace_bytes(2) >= 4 * (2 * phases * 16 * 6 * 6 + 24 * phases * 16 * win * win)
        assert p.workspace_bytes(2) < 4 * (2 * 16 * 12 * 12 + 24 * 64 * 9) * (1 if K == 3 else 0) + (1 << 16) * (K == 1) + (1 << 30) * (K == 3)
    assert syno.Plan(wl.conv2d(2, 16, 24, 6, 6, 3, in_dtype=BF16, stride=2)).kernel(0) == "mfma_contraction_bf16"
    # an index-program-only plan keeps every pass there
    q = syno.Plan(wl.conv2d(2, 16, 24, 6, 6, 3, stride=2), kernel_policy=1)
    assert [q.kernel(i) for i in range(3)] == ["generic_index_program"] * 3


def test_contraction_tiles_are_dealt_to_the_xcds_in_rectangles(syno):
    """Host logic of the tile order: the 8 XCDs split a plane's tiles m x n so that the fewest bytes cross the fabric
    (the source is fetched n times, the weights m times), a plane whose tile count is not a multiple of 8 keeps the
    plain order, and a rectangle too large to be resident at once is walked so that the operand the XCD keeps coming
    back to fits its L2."""
    import re

    def split(desc):
        m = re.search(r"tiles-per-xcd=(\d+)x(\d+)(\(rows first\))?", desc)
        return (int(m.group(1)), int(m.group(2)), bool(m.group(3))) if m else None

    # the benchmark's four stages, 256 tiles each: source-heavy stages give every XCD its own rows and all panels,
    # weight-heavy ones go to a 2-D split
    expect = {(64, 56): (32, 1), (128, 28): (8, 4), (256, 14): (8, 4), (512, 7): (8, 4)}
    for (C, H), tiles in expect.items():
        plan = syno.Plan(wl.conv2d(32, C, C, H, H, 3, 3))
        for which in (0, 1):
            assert split(plan.describe(which))[:2] == tiles, plan.describe(which)
    # weights of 21 MB against 7 MB of source, more tiles than fit at once: rows of tiles first
    assert split(syno.Plan(wl.conv2d(48, 768, 768, 7, 7, 3, 3)).describe(0))[2]
    # 3 x 3 = 9 tiles: no rectangles
    small = syno.Plan(wl.conv2d(3, 40, 72, 9, 12, 3, 3))
    assert "grid=" in small.describe(0) and split(small.describe(0)) is None


def test_matmul_is_planned_as_a_convolution_with_exchanged_roles(syno):
    p = syno.Plan(wl.matmul(96, 2304, 768))
    assert [p.kernel(i) for i in range(3)] == ["mfma_contraction_transposed"] * 3
    assert "1x1 convolution" in p.describe(0)
    assert p.x_shape == (96, 768) and p.w_shape == (768, 2304) and p.out_shape == (96, 2304)
    # dX = G * W^T is a product of its own: forward contraction on a transposed copy of W at the head of the workspace
    assert "transposed copy of W" in p.describe(1) and p.workspace_bytes(1) >= 768 * 2304 * 4
    # a bf16 result type leaves dW on the index-program kernel (its result must be fp32 inside)
    q = syno.Plan(wl.matmul(96, 2304, 768, BF16, BF16))
    assert q.kernel(0) == q.kernel(1) == "mfma_contraction_transposed" and q.kernel(2) == "generic_index_program"
    # too few reduction columns to fold W^T into image rows: dX stays the convolution's weight gradient
    assert "transposed copy" not in syno.Plan(wl.matmul(64, 128, 3)).describe(1)
    # a prime number of columns above 64 cannot be folded into image rows
    assert syno.Plan(wl.matmul(8, 127, 80)).kernel(0) == "generic_index_program"


def test_materialised_reduction_pass_cuts_where_it_saves_work(syno):
    # the paper's example: (H/s)*k*s points become H/s*s + H/s*k
    for weight, stage_of_weight, w_shapes in ((None, 1, [(), ()]), ("k", 1, [(), (3,)]), ("s", 0, [(2,), ()])):
        c = syno.Chain.materialized(wl.window_of_sums_1d(12, 3, 2, weight))
        assert len(c.stages) == 2 and c.weight_stage == stage_of_weight
        assert [p.x_shape for p in c.stages] == [(12,), (6,)] and [p.out_shape for p in c.stages] == [(6,), (6,)]
        assert [p.w_shape for p in c.stages] == w_shapes
    # nothing to gain on a plain convolution: one stage, which keeps the weight
    c = syno.Chain.materialized(wl.conv2d(2, 8, 8, 6, 6))
    assert len(c.stages) == 1 and c.weight_stage == 0
    # block sums under a convolution: rows, then columns, then the convolution on the contraction kernels
    c = syno.Chain.materialized(wl.pooled_conv2d(2, 8, 8, 6, 6))
    assert len(c.stages) == 3 and c.weight_stage == 2
    assert [p.out_shape for p in c.stages] == [(2, 8, 6, 12), (2, 8, 6, 6), (2, 8, 6, 6)]
    assert c.stages[2].kernel(0) == "mfma_contraction_f32" and c.stages[2].w_shape == (8, 8, 3, 3)
    # a Shift that reads another coordinate is left whole
    assert len(syno.Chain.materialized(wl.grouped_shift_unfold(2, 16, 16, 6, 6, 2)).stages) == 1


def test_reduce_free_graphs_go_to_the_view_kernel_forwards(syno):
    for d in (wl.shifted_scale(2, 8, 6, 6), wl.pixel_unshuffle(2, 4, 3, 4, 2)):
        p = syno.Plan(d)
        # one-to-one views: backward-data is the scatter of the same tables; backward-weight is one sum per weight
        # element over the output axes that do not select it (72 and 192 products here: a thread per element)
        assert p.kernel(0) == p.kernel(1) == p.kernel(2) == "bandwidth_view"
        assert p.workspace_bytes(0) == p.workspace_bytes(1) == p.workspace_bytes(2) == 0
    # long sums are sliced over workgroups: slice sums and one target index per weight element in the workspace
    p = syno.Plan(wl.shifted_scale(4, 8, 16, 16))
    assert p.kernel(2) == "bandwidth_view" and p.workspace_bytes(2) >= 4 * (8 + 8)
    # not one-to-one: an Expand repeats X (its gradient sums over the repeats), a Stride leaves elements of X unread
    # (their gradient is zero): gathers through the same tables, zero-filled first where there are gaps
    b = Builder([("i", 6), ("j", 4)])
    b.expand(1)
    p = syno.Plan(b.finish([0], []))
    assert p.kernel(0) == p.kernel(1) == "bandwidth_view"
    b = Builder([("i", 6)])
    p = syno.Plan(b.finish([b.stride(0, 2)], []))
    assert p.kernel(0) == p.kernel(1) == "bandwidth_view"
    # an Expand and a Stride whose sizes cancel: as many X elements as outputs, still not one-to-one
    b = Builder([("i", 6), ("j", 2)])
    b.expand(1)
    p = syno.Plan(b.finish([b.stride(0, 2)], []))
    assert p.x_shape == (12,) and p.kernel(1) == "bandwidth_view" and "gather targets=6 products/target=2" in p.describe(1)
    assert "zero-filled-first" in p.describe(1) and syno.Plan(wl.shifted_scale(2, 8, 6, 6)).describe(1).endswith("scatter")
    # a Shared iterator whose two copies both reach X (a diagonal: X[i,i], or folded into one axis, X[3i+i]) next to
    # an iterator that only reaches the weight would also have as many X elements as outputs; such graphs are
    # refused as a whole, because backward-data would have to fix one coordinate from two places
    for fold in (False, True):
        b = Builder([("i", 3), ("j", 3)])
        i1, i2 = b.share(0)
        with pytest.raises(syno.SynoError) as e:
            syno.Plan(b.finish([b.split(i1, i2)] if fold else [i1, i2], [1]))
        assert e.value.status == 4
    # a Shift whose amount depends on another output axis is not separable: index program
    b = Builder([("g", 4), ("h", 6)])
    gx, gw = b.share(0)
    d = b.finish([gx, b.shift(1, 0, by=gx, coef=1)], [gw])
    assert syno.Plan(d).kernel(0) == "generic_index_program"


def test_chain_entry_points_reject_bad_arguments_on_the_host(syno):
    lib = syno.load_library()
    chain = syno.Chain([wl.conv2d(1, 4, 4, 5, 5)])
    null = ctypes.c_void_p()
    n = ctypes.c_size_t()
    assert lib.syno_chain_workspace_bytes(chain._h, 2, ctypes.byref(n)) == 3          # selector out of range
    assert lib.syno_chain_workspace_bytes(None, 0, ctypes.byref(n)) == 1
    assert lib.syno_chain_stages(None) == 0 and lib.syno_chain_weight_stage(None) == -1
    assert lib.syno_chain_weight_stage(chain._h) == -1                                 # every stage has its own weight
    # NULL tensors are refused before anything is launched
    assert lib.syno_chain_forward(chain._h, None, None, None, None, None, None) == 1
    assert lib.syno_chain_backward(chain._h, None, None, None, None, None, None, None, None) == 1
    h = ctypes.c_void_p()
    assert lib.syno_chain_create(None, 1, ctypes.byref(h)) == 1
    assert lib.syno_chain_create_materialized(None, ctypes.byref(h)) == 1
    # an invalid graph is reported by the pass as by plan creation
    b = Builder([("i", 4)])
    bad = b.finish([0, 0], [])                                                         # coordinate consumed twice
    with pytest.raises(syno.SynoError):
        syno.Chain.materialized(bad)


def test_random_graphs_index_maps_against_checker(syno, oracle):
    """Seeded random primitive graphs: wherever both sides accept a graph, the forward index map agrees bit for bit
    and both gradient enumerations list the checker's terms, each once.  A graph the checker rejects is rejected by
    the library as well."""
    import random
    from test_host_sanitizers import random_graph
    rng = random.Random(7)
    both = 0
    for _ in range(400):
        d = random_graph(rng)
        try:
            xs, ws, red = oracle.describe(d)
            valid = True
        except oracle.OracleError:
            valid = False
        try:
            p = syno.Plan(d)
        except syno.SynoError as e:
            assert e.status in (2, 4) and (valid or e.status == 2)      # invalid graphs: INVALID_DESC, not UNSUPPORTED
            continue
        assert valid, "the library accepted a graph the checker rejects"
        n_o, n_r = int(np.prod(p.out_shape)), int(np.prod(red)) if red else 1
        if n_o * n_r > 200000:
            continue
        both += 1
        assert p.x_shape == xs and p.w_shape == ws
        o, r = (a.ravel() for a in np.meshgrid(np.arange(n_o), np.arange(n_r), indexing="ij"))
        xo, wo = oracle.gather_map(d, o, r)
        a, b = p.debug_gather_host(syno.FWD, o, r)
        assert np.array_equal(a, xo) and np.array_equal(b, wo)
        ok = xo >= 0
        terms = sorted(zip(o[ok].tolist(), xo[ok].tolist(), wo[ok].tolist()))
        for which, n_t in ((syno.BWD_DATA, int(np.prod(p.x_shape))), (syno.BWD_WEIGHT, int(np.prod(p.w_shape)))):
            if n_t * p.free_size(which) > 400000:
                continue
            t, q = (v.ravel() for v in np.meshgrid(np.arange(n_t), np.arange(p.free_size(which)), indexing="ij"))
            a, b = p.debug_gather_host(which, t, q)
            v = a >= 0
            got = zip(a[v].tolist(), t[v].tolist(), b[v].tolist()) if which == syno.BWD_DATA else \
                zip(a[v].tolist(), b[v].tolist(), t[v].tolist())
            assert sorted(got) == terms
    assert both >= 100


def test_two_weight_graph_is_cut_into_single_weight_stages(syno, oracle):
    """Operator 1 as one pGraph with two weights (host only): refused as a single plan, cut by the materialised-
    reduction pass into the stage that multiplies with w1 (it takes the Shares feeding w1 along) and the stage that
    multiplies with w2; the stages' shapes are the checker's weight shapes."""
    d = wl.operator1_graph(2, 16, 16, 6, 8, 4, 2, 3)
    with pytest.raises(syno.SynoError) as e:
        syno.Plan(d)
    assert e.value.status == 4
    chain = syno.Chain.materialized(d)
    assert chain.stage_weight == [0, 1] and chain.weight_stage == 0
    shapes = oracle.weight_shapes(d)
    assert [p.w_shape for p in chain.stages] == shapes
    assert chain.stages[0].x_shape == (2, 16, 6, 8) and chain.stages[1].out_shape == (2, 16, 6, 8)
    assert chain.stages[0].out_shape == chain.stages[1].x_shape
    # the stored tensor is laid out [n, d, gi, k, h, w]: batch, the weight's own iterator, channel digit, window iterator,
    # image axes; that is the layout of the hand-written first stage, so both stages land on the fast kernels (the second
    # one as a convolution over the three reduced axes taken as one channel axis)
    assert chain.stages[0].out_shape == (2, 2, 4, 3, 6, 8)
    assert [p.kernel(k) for p in chain.stages for k in range(3)] == ["bandwidth_share_window"] * 3 + ["mfma_contraction_f32"] * 3
    # multiply-adds: the two stages together cost less than the single loop nest
    pts = lambda p: int(np.prod(p.out_shape)) * p.free_size(syno.FWD)
    single = 2 * 16 * 6 * 8 * (2 * 4 * 3 * 3 * 4)
    assert sum(pts(p) for p in chain.stages) < single
    # a chain given as explicit stages names each stage's own weight
    w = wl.make_operator1(2, 16, 12, g=4, s=2)
    assert syno.Chain(w.descs).stage_weight == [0, 1]
    # Shares written the other way round (the copy for w1 handed out first) do not come apart: refused, not mis-cut
    b = Builder([("i", 6)])
    r = b.reduce(4)
    ra, rw1 = b.share(r)
    rx, rw2 = b.share(ra)
    k = b.reduce(3)
    kx, kw2 = b.share(k)
    two = b.finish([rx, b.unfold(0, kx)], [rw1], more_weights=[[rw2, kw2]])
    try:
        c = syno.Chain.materialized(two)
        assert all(sw in (-1, 0, 1) for sw in c.stage_weight) and sorted(x for x in c.stage_weight if x >= 0) == [0, 1]
    except syno.SynoError as e2:
        assert e2.status == 4


def test_adjacent_reduced_axes_count_as_one_channel_axis(syno):
    """A convolution whose input channels are written as three adjacent reduced axes, in the same order in X and in
    the weight, has the same bytes as the plain convolution and is lowered like it; with the axes in different orders
    on the two sides it is not."""
    from syno_inputs.descriptor import Builder

    def conv_split_channels(w_order):
        b = Builder([("n", 2), ("o", 16), ("h", 9), ("w", 10)])
        n, o, h, w = range(4)
        pairs = [b.share(b.reduce(sz)) for sz in (2, 4, 3)]           # (X copy, W copy) of d, gi, k
        jx, jw = b.share(b.reduce(3))
        hh = b.unfold(h, jx)
        xs = [p[0] for p in pairs]
        ws = [pairs[i][1] for i in w_order]
        return b.finish([n] + xs + [hh, w], [o] + ws + [jw], 0, 0)

    same = syno.Plan(conv_split_channels((0, 1, 2)))
    assert same.x_shape == (2, 2, 4, 3, 9, 10) and same.w_shape == (16, 2, 4, 3, 3)
    assert [same.kernel(k) for k in range(3)] == ["mfma_contraction_f32"] * 3
    other = syno.Plan(conv_split_channels((1, 0, 2)))
    assert [other.kernel(k) for k in range(3)] == ["generic_index_program"] * 3
