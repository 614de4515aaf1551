"""Helpers shared by the tests: moving seeded workloads to the device, the error metrics and their bars."""
import numpy as np
import torch

from syno_inputs import BF16

# Contractual bars: relative L2 error of the GPU result against the fp64 checker on identical inputs.
TOL_F32 = 1e-5      # fp32 inputs, fp32 accumulation
TOL_BF16 = 2e-2     # bf16 inputs, fp32 accumulation (any output type)

# Working bars, derived from the arithmetic.  Both sides read the same input values (bf16 inputs are rounded once,
# on the host) and a product of two bf16 or two fp32 values is exact in the fp64 checker, so the only error of an
# fp32 result is the fp32 accumulation; a bf16 result adds one rounding to nearest even on the store.
U32 = 2.0 ** -24               # unit roundoff of fp32
TOL_ACC = 1e-5                 # rel-L2 of any fp32 result (fp32 or bf16 inputs alike)
TOL_BF16_STORE = 4e-3          # rel-L2 of a bf16 result: half an ulp is at most 2^-8 of the value, 2^-9/sqrt(3) on average
TOL_CHAIN_BF16 = 6e-3          # rel-L2 through stages whose intermediates are stored as bf16 (one-ulp flips carried on)
RTOL_BF16_STORE = 2.0 ** -8    # per element: half a bf16 ulp relative to the value
ACC_FACTOR = 4.0               # per element: |error| <= ACC_FACTOR * sqrt(terms) * U32 * sum|terms|
                               # (a random walk of roundings, each at most U32 of a partial sum that never exceeds the
                               # sum of magnitudes, with a safety factor; one dropped or doubled term of typical size
                               # sum|terms|/terms is far outside it for every reduction length used here)


def tol_for(desc):
    """The contractual outer bar for this operator's input type."""
    return TOL_BF16 if desc.in_dtype == BF16 else TOL_F32


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def assert_close(got, ref, mag, n_terms, result_bf16, what, outer_tol):
    """The parity bar for one result tensor (or a sample of it).

    got, ref : GPU values and checker values of the same elements
    mag      : per element, the sum of the magnitudes of its terms (the checker run on |inputs|)
    n_terms  : upper bound of the number of terms per element
    Checks the relative L2 error against the working bar (and the contractual one) and every element against
    |got - ref| <= ACC_FACTOR*sqrt(n_terms)*U32*mag (+ half a bf16 ulp of the value for a bf16 result)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    mag = np.asarray(mag, dtype=np.float64).ravel()
    assert got.shape == ref.shape == mag.shape, (got.shape, ref.shape, mag.shape)
    e = rel_l2(got, ref)
    bar = TOL_BF16_STORE if result_bf16 else TOL_ACC
    assert e <= bar and e <= outer_tol, f"{what}: rel-L2 {e:.3e} > {min(bar, outer_tol):.1e}"
    acc = ACC_FACTOR * np.sqrt(max(int(n_terms), 1)) * U32 * mag
    bound = acc * (1.0 + RTOL_BF16_STORE) + RTOL_BF16_STORE * np.abs(ref) if result_bf16 else acc
    bound = bound + 1e-37      # (elements without any term are exactly 0 on both sides)
    err = np.abs(got - ref)
    bad = np.flatnonzero(err > bound)
    if bad.size:
        i = bad[np.argmax(err[bad] / bound[bad])]
        raise AssertionError(f"{what}: {bad.size} of {got.size} elements outside the per-element bound; worst at "
                             f"sample {i}: got {got[i]!r} want {ref[i]!r} |err| {err[i]:.3e} bound {bound[i]:.3e}")
    return e, float(np.max(err / bound)) if got.size else 0.0


def to_dev(values, bits, dev="cuda:0"):
    """fp32 values (or bf16 bit patterns when given) -> device tensor of the workload's input type."""
    if bits is not None:
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)
    return torch.from_numpy(np.ascontiguousarray(values, dtype=np.float32)).to(dev)


def to_host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def plane_samples(shape, rng, n_random, lead_picks=None):
    """Flat indices of a stratified sample of a tensor whose last two axes are an image plane and whose leading
    axes select the plane: whole planes for the first, the last and a middle index of every leading axis (all
    image borders, the rows where consecutive images meet, the first and last tile of any tiling over rows,
    channels or images) plus `n_random` uniformly drawn elements.  `lead_picks` adds values per leading axis
    (tile boundaries of the launch that is being checked)."""
    shape = tuple(int(s) for s in shape)
    if len(shape) >= 3:
        lead, plane = shape[:-2], shape[-2] * shape[-1]
    else:                      # matrices: whole rows; vectors: the random draw only
        lead, plane = shape[:-1], shape[-1]
    if not lead:
        return np.unique(rng.integers(0, plane, n_random))
    picks = []
    for ax, s in enumerate(lead):
        v = {0, 1, s // 2, s - 2, s - 1}
        if lead_picks and ax < len(lead_picks) and lead_picks[ax]:
            v |= set(int(p) for p in lead_picks[ax])
        picks.append(sorted(p for p in v if 0 <= p < s))
    grids = np.meshgrid(*picks, indexing="ij") if picks else []
    base = np.zeros(grids[0].size if grids else 1, dtype=np.int64)
    stride = plane
    for ax in range(len(lead) - 1, -1, -1):
        base += grids[ax].ravel().astype(np.int64) * stride
        stride *= lead[ax]
    idx = (base[:, None] + np.arange(plane, dtype=np.int64)[None, :]).ravel()
    total = int(np.prod(shape))
    return np.unique(np.concatenate([idx, rng.integers(0, total, n_random)]))
