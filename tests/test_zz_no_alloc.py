"""The allocation-free backward-weight entry point (static scratch memory inside the library) against
syno_backward_weight with a caller's workspace, through the C ABI: same bits, on consecutive calls of shrinking size."""
import numpy as np
import pytest
import torch

from syno_inputs import workloads as wl
from util import assert_close, to_dev, to_host, tol_for

pytestmark = pytest.mark.gpu

LIMIT = 32 << 20


@pytest.fixture(scope="module")
def syno():
    import paper_2410_23745_amd as s
    s.load_library()
    assert torch.cuda.is_available()
    return s


# each family whose backward-weight keeps partial sums in scratch memory: a larger operator first, then a smaller one
SEQUENCES = {
    "gshift_bf16": [lambda: wl.make_gshift(16, seeds=(1, 2, 3), with_grad=True),
                    lambda: wl.make_gshift(3, seeds=(4, 5, 6), with_grad=True, C=96, H=9, Wd=11, groups=3)],
    "conv_f32": [lambda: wl.make_conv(4, 64, 28, seed=3, with_grad=True),
                 lambda: wl.make_conv(3, 24, 13, seed=4, Co=40, Wd=19, with_grad=True)],
    "conv_bf16": [lambda: wl.make_conv(8, 128, 14, seed=5, bf16=True, with_grad=True),
                  lambda: wl.make_conv(5, 24, 7, seed=13, Co=40, bf16=True, with_grad=True)],
    "depthwise_f32": [lambda: wl.make_depthwise(4, 16, 56, seed=6, with_grad=True),
                      lambda: wl.make_depthwise(2, 5, 28, seed=7, with_grad=True)],
}


@pytest.mark.parametrize("name", list(SEQUENCES))
def test_static_scratch_backward_weight_equals_the_workspace_call(syno, oracle, name):
    for k, mk in enumerate(SEQUENCES[name]):
        w = mk()
        plan = syno.Plan(w.desc)
        need = plan.workspace_bytes(syno.BWD_WEIGHT)
        print(f"[case] {w.desc.name}: kernel={plan.kernel(2)} scratch needed {need} B", flush=True)
        assert 0 < need <= LIMIT
        X, G = to_dev(w.X, w.X_bits), to_dev(w.G, w.G_bits)
        ref = plan.backward_weight(X, G)
        dW = torch.full(plan.w_shape, float("nan"), dtype=torch.float32, device=X.device)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        plan.backward_weight_static(X, G, dW)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        assert torch.equal(ref, dW), f"call {k}: the static-scratch result differs from the workspace call's"
        # and both are the checker's gradient
        _, rdw = oracle.backward(w.desc, w.X, w.W, w.G, False, True)
        _, mdw = oracle.backward(w.desc, np.abs(w.X), np.abs(w.W), np.abs(w.G), False, True)
        assert_close(to_host(dW), rdw, mdw, plan.free_size(2), False, "backward-weight (static scratch)", tol_for(w.desc))


def test_static_scratch_rejects_what_does_not_fit(syno):
    d = wl.conv2d(4, 512, 512, 7, 7)
    plan = syno.Plan(d, dw_workgroups=1024)          # more splits than the planner would take: 4 x 9.4 MB of partials
    assert plan.workspace_bytes(syno.BWD_WEIGHT) > LIMIT
    X = torch.zeros(plan.x_shape, device="cuda")
    G = torch.zeros(plan.out_shape, device="cuda")
    dW = torch.zeros(plan.w_shape, device="cuda")
    with pytest.raises(syno.SynoError) as e:
        plan.backward_weight_static(X, G, dW)
    assert e.value.status == 7
    assert syno.load_library().syno_backward_weight_static(plan._h, None, G.data_ptr(), dW.data_ptr(), None) == 1
