"""GPU-vs-oracle parity of the low-precision deployment (cat_params_to_bf16, cat_apply_lp).

The rounding of the parameters is a quantised code: the library's must equal the oracle's bit for bit (the oracle
rounds from the definition of the format).  Inference then runs on identical stored values on both sides, so the
assignments follow the tie-gap rule and the corrected rows the tolerance of their storage type: 1e-4 for fp32 output,
2e-2 for bfloat16 output (one unit in the last place of bfloat16 is 2^-8 of the value: the library rounds its fp32
result, the oracle its double result, and the two can land on neighbouring bfloat16 values)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import cat_apply, cat_apply_lp, cat_params_to_bf16, workloads
from paper_2509_26277_amd.binding import CAT_PATH_AUTO, CAT_PATH_STREAM, CatError, select_path

from parity_util import RTOL, check_assignments_lazy, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_path_after():
    yield
    select_path(CAT_PATH_AUTO)


def _model(seed, N, D, K, dt="f32"):
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((K, D)) * 1.5
    lab = rng.integers(0, K, N)
    x = (cent[lab] + 0.7 * rng.standard_normal((N, D))).astype(np.float32)
    if dt == "bf16":
        x = workloads.round_to_bf16(x)
    gamma = rng.uniform(0.7, 1.3, (K, D))
    beta = 0.3 * rng.standard_normal((K, D))
    return x, cent, gamma, beta


def _stored(cent, gamma, beta):
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return cat_params_to_bf16(f(cent)), cat_params_to_bf16(f(gamma)), cat_params_to_bf16(f(beta))


def test_rounding_is_the_oracles_bit_for_bit():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(200000) * 10.0 ** rng.integers(-6, 7, 200000),
                        (np.arange(-512, 512) + 0.5) * 2.0 ** -8 + 1.0, [0.0, -0.0, 1.0, -1.0]]).astype(np.float32)
    got = cat_params_to_bf16(torch.from_numpy(x).cuda())
    assert got.dtype == torch.bfloat16
    assert (got.double().cpu().numpy() == oracle.to_bf16(x.astype(np.float64))).all()


@pytest.mark.parametrize("N,D,K,alpha,bf16_out", [
    (3000, 64, 6, 1.0, True),
    (3000, 64, 6, 0.6, True),
    (2500, 256, 30, 0.6, False),     # stored parameters, fp32 rows out
    (4099, 512, 100, 1.0, True),     # one-part operand instance, rows not a multiple of the tile
    (1777, 1000, 16, 0.25, True),    # ragged last vector of a row
    (1500, 37, 4, 0.6, True),        # no instance of the fused kernel: assign first, map by the labels
    (900, 2052, 20, 1.0, True),      # rows longer than the fused kernel holds
    (1200, 48, 300, 0.6, True),      # more clusters than the matrix-core kernels take
])
def test_inference_on_stored_parameters(N, D, K, alpha, bf16_out):
    x, cent, gamma, beta = _model(N + D + K, N, D, K)
    xd = dev_matrix(x, "f32")
    cq, gq, bq = _stored(cent, gamma, beta)
    out, a = cat_apply_lp(xd, cq, gq, bq, alpha=alpha, bf16_out=bf16_out)
    assert out.dtype == (torch.bfloat16 if bf16_out else torch.float32)
    o_out, o_a, (ocq, ogq, obq) = oracle.apply_lp(x, cent.astype(np.float32), gamma.astype(np.float32),
                                                  beta.astype(np.float32), alpha=alpha, bf16_out=bf16_out)
    assert (cq.double().cpu().numpy() == ocq).all() and (gq.double().cpu().numpy() == ogq).all()
    a = a.cpu().numpy()
    check_assignments_lazy(a, o_a, x, ocq, "assignments")
    same = a == o_a
    check_values(host_matrix(out)[same], o_out[same], RTOL["bf16" if bf16_out else "f32"], "corrected")
    if bf16_out:
        # within one bfloat16 step of the oracle's value everywhere (not only 2e-2), and mostly the same value
        g, w = host_matrix(out)[same], o_out[same]
        assert (np.abs(g - w) <= np.abs(w) * 2.0 ** -7 + 1e-30).all()
        assert (g == w).mean() > 0.98


def test_bf16_rows_and_the_streaming_path():
    x, cent, gamma, beta = _model(3, 2000, 136, 9, "bf16")
    xd = dev_matrix(x, "bf16")
    cq, gq, bq = _stored(cent, gamma, beta)
    o_out, o_a, (ocq, _, _) = oracle.apply_lp(x, cent.astype(np.float32), gamma.astype(np.float32), beta.astype(np.float32), alpha=0.6)
    for path in (CAT_PATH_AUTO, CAT_PATH_STREAM):
        select_path(path)
        out, a = cat_apply_lp(xd, cq, gq, bq, alpha=0.6)
        a = a.cpu().numpy()
        check_assignments_lazy(a, o_a, x, ocq, "assignments")
        check_values(host_matrix(out)[a == o_a], o_out[a == o_a], RTOL["bf16"], "corrected")


def test_same_as_cat_apply_on_the_expanded_parameters():
    """fp32 out: bit for bit what cat_apply gives on the stored values widened to fp32; bf16 out: those values rounded."""
    x, cent, gamma, beta = _model(8, 5000, 512, 128)
    xd = dev_matrix(x, "f32")
    cq, gq, bq = _stored(cent, gamma, beta)
    ref, a_ref = cat_apply(xd, cq.float(), gq.float(), bq.float())
    out32, a32 = cat_apply_lp(xd, cq, gq, bq, bf16_out=False)
    assert torch.equal(out32, ref) and torch.equal(a32, a_ref)
    out16, a16 = cat_apply_lp(xd, cq, gq, bq, bf16_out=True, want_assignments=False)
    assert a16 is None
    assert torch.equal(out16, cat_params_to_bf16(ref))


def test_all_rows_of_the_inference_workload_sampled():
    w = workloads.make("cfg5")
    x = w["lq"]
    xd = dev_matrix(x, "f32")
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    cq, gq, bq = cat_params_to_bf16(f(w["centroids"])), cat_params_to_bf16(f(w["gamma"])), cat_params_to_bf16(f(w["beta"]))
    out, a = cat_apply_lp(xd, cq, gq, bq, alpha=1.0, bf16_out=True)
    rows = np.random.default_rng(5).choice(w["N"], 200000, replace=False)
    rows.sort()
    o_out, o_a, (ocq, _, _) = oracle.apply_lp(np.ascontiguousarray(x[rows]), w["centroids"].astype(np.float32),
                                              w["gamma"].astype(np.float32), w["beta"].astype(np.float32))
    idx = torch.from_numpy(rows).cuda()
    ga = a[idx].cpu().numpy()
    check_assignments_lazy(ga, o_a, np.ascontiguousarray(x[rows]), ocq, "assignments")
    same = ga == o_a
    check_values(host_matrix(out[idx])[same], o_out[same], RTOL["bf16"], "corrected")
    # properties that hold on all rows: the labels are those of cat_apply on the stored centroids
    ref_a = cat_apply(xd, cq.float(), gq.float(), bq.float(), out=torch.empty_like(xd))[1]
    assert torch.equal(a, ref_a)


def test_bad_arguments_are_refused():
    x = torch.zeros((64, 8), device="cuda")
    p = torch.zeros((2, 8), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        cat_apply_lp(x, p.float(), p, p)
    with pytest.raises(CatError):
        cat_apply_lp(x, p, p, p, alpha=float("nan"))
