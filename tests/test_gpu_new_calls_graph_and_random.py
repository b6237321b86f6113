"""The calls added beside cat_fit / cat_apply (cat_fit_bounds, cat_fit_multi_k, cat_apply_lp): captured into a HIP graph
and replayed, and seeded random shapes against the oracle.

Capture: none of them allocates, synchronises, reads anything back or uses a memset node; how many rows a bound-based
pass evaluates, and whether a pass has anything to do at all, is decided on the device, so one captured graph must give
the eager results on every replay, with eager work in between."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_apply_lp, cat_fit, cat_fit_multi_k, cat_params_to_bf16, workloads

from parity_util import CENTROID_RTOL, RTOL, check_assignments_lazy, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


def _mixture(seed, N, D, C, dt, spread=2.0):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((C, D)) * spread
    lab = rng.integers(0, C, N)
    y = (centres[lab] + rng.standard_normal((N, D))).astype(np.float32)
    x = (y * rng.uniform(0.6, 1.4, D).astype(np.float32) + 0.2 * rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y


def _same(got, ref, key):
    """integer outputs and centroids bit for bit; gamma / beta to rounding (their sums go through atomics)"""
    if key in ("gamma", "beta"):
        torch.testing.assert_close(got, ref, rtol=1e-5, atol=1e-6)
    else:
        assert torch.equal(got, ref), key


def _capture(run):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on a side stream, as torch asks for
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        outs = run()
    return g, outs


def test_new_calls_capture_into_a_hip_graph_and_replay():
    N, D, K, iters = 6000, 64, 6, 9
    x, y = _mixture(1, N, D, 6, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    lib = binding.load_library()
    ws_b = torch.empty(lib.cat_fit_bounds_workspace_bytes(N, D, K, iters, binding.CAT_F32), dtype=torch.uint8, device="cuda")
    Ks = [3, 17, 6]
    ks = (binding.ctypes.c_int32 * 3)(*Ks)
    ws_m = torch.empty(lib.cat_fit_multi_k_workspace_bytes(N, D, ks, 3, iters, binding.CAT_F32), dtype=torch.uint8, device="cuda")
    ws_l = torch.empty(lib.cat_apply_lp_workspace_bytes(N, D, K, binding.CAT_F32), dtype=torch.uint8, device="cuda")
    out16 = torch.empty((N, D), dtype=torch.bfloat16, device="cuda")

    def run():
        b = cat_fit(xd, yd, K, iters, seed=5, workspace=ws_b, bounds=True)
        m = cat_fit_multi_k(xd, yd, Ks, iters, seed=5, workspace=ws_m)
        cq, gq, bq = (cat_params_to_bf16(b[k]) for k in ("centroids", "gamma", "beta"))
        o, a = cat_apply_lp(xd, cq, gq, bq, alpha=0.6, bf16_out=True, out=out16, workspace=ws_l)
        return b, m, o, a

    b0, m0, o0, a0 = run()
    torch.cuda.synchronize()
    keys = ("centroids", "gamma", "beta", "assignments", "counts")
    ref_b = {k: b0[k].clone() for k in keys + ("rows_evaluated",)}
    ref_m = [{k: r[k].clone() for k in keys} for r in m0]
    ref_o, ref_a = o0.clone(), a0.clone()
    assert int(ref_b["rows_evaluated"][3:-1].min()) < N  # the captured loop does leave rows out
    g, (b, m, o, a) = _capture(run)
    for _ in range(3):
        for t in [b[k] for k in keys] + [r[k] for r in m for k in keys] + [o, a, b["rows_evaluated"]]:
            t.zero_()  # eager work between the replays; also proves that a replay rewrites every output
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in keys + ("rows_evaluated",):
            _same(b[k], ref_b[k], k)
        for r, rr in zip(m, ref_m):
            for k in keys:
                _same(r[k], rr[k], k)
        # (the stored parameters are bfloat16 roundings of gamma / beta: a last-bit difference there moves an entry by a
        # bfloat16 step at most)
        assert torch.equal(a, ref_a)
        torch.testing.assert_close(o.float(), ref_o.float(), rtol=2e-2, atol=1e-2)


def _cases(n_cases=16, seed=20251128):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n_cases):
        dt = "bf16" if rng.random() < 0.3 else "f32"
        step = 8 if dt == "bf16" else 4
        D = int(rng.integers(1, 70)) * step
        K = int(rng.integers(1, 60))
        N = int(rng.integers(max(K, 300), K + 3000))
        iters = int(rng.integers(4, 10))
        out.append((i, dt, N, D, K, iters))
    return out


@pytest.mark.parametrize("case,dt,N,D,K,iters", _cases())
def test_random_shape_bounds_multi_k_low_precision(case, dt, N, D, K, iters):
    x, y = _mixture(9000 + case, N, D, max(2, min(K, 7)), dt, spread=1.5)
    if N > 8:
        x[N // 3] = x[N // 3 + 1]  # duplicated rows: exact ties between candidates
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    o = oracle.fit_bounds(x, y, K, iters, seed=case)
    b = cat_fit(xd, yd, K, iters, seed=case, bounds=True)
    a = b["assignments"].cpu().numpy()
    exempt = check_assignments_lazy(a, o["assignments"], x, o["centroids"], "bounds fit")
    if exempt == 0:
        assert (b["counts"].cpu().numpy() == o["counts"]).all()
        check_values(host_matrix(b["centroids"]), o["centroids"], CENTROID_RTOL, "centroids")
        check_values(host_matrix(b["gamma"]), o["gamma"], RTOL[dt], "gamma")
        check_values(host_matrix(b["beta"]), o["beta"], RTOL[dt], "beta")
    # the same count inside a list of three: the entry equals the bound-based fit bit for bit
    Ks = [max(1, K // 2), K, min(N, K + 5)]
    m = cat_fit_multi_k(xd, yd, Ks, iters, seed=case)
    for key in ("centroids", "assignments", "counts", "gamma", "beta"):
        _same(m[1][key], b[key], key)
    om = oracle.fit(x, y, Ks[2], iters, seed=case)
    check_assignments_lazy(m[2]["assignments"].cpu().numpy(), om["assignments"], x, om["centroids"], "third entry of the list")
    # low-precision inference with the fitted parameters
    if dt == "f32":
        cq, gq, bq = (cat_params_to_bf16(b[k]) for k in ("centroids", "gamma", "beta"))
        out, al = cat_apply_lp(xd, cq, gq, bq, alpha=0.6, bf16_out=True)
        o_out, o_a, (ocq, _, _) = oracle.apply_lp(x, host_matrix(b["centroids"]).astype(np.float32), host_matrix(b["gamma"]).astype(np.float32),
                                                  host_matrix(b["beta"]).astype(np.float32), alpha=0.6)
        al = al.cpu().numpy()
        check_assignments_lazy(al, o_a, x, ocq, "low-precision inference")
        same = al == o_a
        check_values(host_matrix(out)[same], o_out[same], RTOL["bf16"], "corrected")
