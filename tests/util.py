"""Helpers shared by the tests: moving seeded workloads to the device, the error metric."""
import numpy as np
import torch

from syno_inputs import BF16

# Parity bars: relative L2 error of the GPU result against the fp64 checker on identical inputs.
TOL_F32 = 1e-5      # fp32 inputs, fp32 accumulation
TOL_BF16 = 2e-2     # bf16 inputs, fp32 accumulation (any output type)


def tol_for(desc):
    return TOL_BF16 if desc.in_dtype == BF16 else TOL_F32


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def to_dev(values, bits, dev="cuda:0"):
    """fp32 values (or bf16 bit patterns when given) -> device tensor of the workload's input type."""
    if bits is not None:
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)
    return torch.from_numpy(np.ascontiguousarray(values, dtype=np.float32)).to(dev)


def to_host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)
