"""Helpers of the GPU-vs-oracle parity tests (tolerances, device transfer)."""
import numpy as np
import torch

from paper_2509_26277_amd import workloads

RTOL = {"f32": 1e-4, "bf16": 2e-2}   # values: centroids, gamma, beta, corrected
# Centroids are double-precision sums divided once and rounded to fp32 (6e-8), whatever the row dtype: where the
# library and the oracle average the SAME partition they are compared at this, far inside RTOL, so that a single row
# lost from a sum of a hundred thousand shows.
CENTROID_RTOL = 1e-6
TIE_GAP = 1e-5                        # assignments: rows below this relative top-2 gap are exempt


def dev_matrix(x_f32, dtype):
    """numpy fp32 matrix -> device tensor of the workload dtype (bf16: the values must
    already be bf16-representable, as the generators guarantee)."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).cuda()
    bits = workloads.f32_to_bf16_bits(x_f32)
    assert (workloads.bf16_bits_to_f32(bits) == x_f32).all(), "input is not bf16-representable"
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host_matrix(t):
    """device tensor -> numpy float64"""
    return t.detach().float().cpu().numpy().astype(np.float64)


def f32_round(a):
    """float64 array rounded to float32 and widened again (what the GPU is handed)"""
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def check_values(got, want, rtol, what):
    """|got - want| <= rtol * max(|want|, rms(want)) element-wise."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    rms = float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    bound = rtol * np.maximum(np.abs(want), rms) + 1e-30
    err = np.abs(got - want)
    worst = np.unravel_index(np.argmax(err / bound), err.shape) if err.size else None
    assert (err <= bound).all(), (
        f"{what}: {int((err > bound).sum())} of {err.size} outside rtol={rtol}; worst at {worst}: "
        f"got {got[worst]!r} want {want[worst]!r} (rms {rms:.3g})")


def check_assignments(got, want, d1, d2, what):
    """identical, except rows whose oracle top-2 gap (d2 - d1) / d2 is below TIE_GAP"""
    got = np.asarray(got)
    want = np.asarray(want)
    bad = np.flatnonzero(got != want)
    if bad.size == 0:
        return 0
    gap = (d2[bad] - d1[bad]) / np.maximum(d2[bad], np.finfo(np.float64).tiny)
    hard = bad[gap >= TIE_GAP]
    assert hard.size == 0, (
        f"{what}: {hard.size} rows differ with a clear gap, e.g. row {hard[0]}: got {got[hard[0]]} want "
        f"{want[hard[0]]} d1={d1[hard[0]]!r} d2={d2[hard[0]]!r}")
    return bad.size


def check_assignments_lazy(got, want, lq, centroids, what):
    """check_assignments with the oracle's two smallest distances computed only for the rows that differ
    (`centroids`: the ones `want` was taken against)."""
    import oracle
    got = np.asarray(got)
    want = np.asarray(want)
    bad = np.flatnonzero(got != want)
    if bad.size == 0:
        return 0
    a, d1, d2 = oracle.assign(np.ascontiguousarray(lq[bad]), centroids, want_distances=True)
    assert (a == want[bad]).all(), f"{what}: `want` was not taken against these centroids"
    check_assignments(got[bad], want[bad], d1, d2, what)
    return bad.size
