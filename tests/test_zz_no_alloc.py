"""cat_apply_static (the entry point that allocates nothing) against cat_apply, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2509_26277_amd import binding, cat_apply, cat_apply_static, workloads

pytestmark = pytest.mark.gpu


def _params(K, D, seed):
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((K, D)).astype(np.float32)
    gamma = rng.uniform(0.8, 1.2, (K, D)).astype(np.float32)
    beta = (0.3 * rng.standard_normal((K, D))).astype(np.float32)
    return cent, gamma, beta


def _rows(N, cent, seed, dtype):
    rng = np.random.default_rng(seed)
    x = (cent[rng.integers(0, cent.shape[0], N)] + rng.standard_normal((N, cent.shape[1]))).astype(np.float32)
    if dtype == "bf16":
        x = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(x))
        bits = workloads.f32_to_bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


@pytest.mark.parametrize("dtype,D,K", [("f32", 512, 128), ("f32", 1000, 16), ("bf16", 256, 48), ("f32", 37, 5),
                                        ("f32", 1001, 16), ("bf16", 1002, 16)])
def test_two_calls_in_a_row_match_cat_apply(dtype, D, K):
    """Two calls in a row on the one built-in scratch array, the second on a smaller input with other parameters
    (fewer rows, fewer clusters): each must equal cat_apply with a caller workspace bit for bit."""
    torch.cuda.set_device(0)
    shapes = [(6000 + 37, K, 1.0), (1000 + 5, max(1, K // 2), 0.6)]
    for call, (N, k, alpha) in enumerate(shapes):
        cent, gamma, beta = _params(k, D, 100 + call)
        lq = _rows(N, cent, 200 + call, dtype)
        c, g, b = (torch.from_numpy(a).cuda() for a in (cent, gamma, beta))
        want, want_a = cat_apply(lq, c, g, b, alpha=alpha)
        out = torch.full_like(lq, float("nan"))
        a = torch.full((N,), -7, dtype=torch.int32, device="cuda")
        got, got_a = cat_apply_static(lq, c, g, b, alpha=alpha, out=out, assignments=a)
        torch.cuda.synchronize()
        assert torch.equal(got_a, want_a), f"call {call}: assignments differ"
        assert torch.equal(got.view(torch.int16 if dtype == "bf16" else torch.int32),
                           want.view(torch.int16 if dtype == "bf16" else torch.int32)), f"call {call}: corrected differs"


def test_without_assignments_and_on_the_streaming_path():
    torch.cuda.set_device(0)
    cent, gamma, beta = _params(7, 96, 3)
    lq = _rows(3001, cent, 4, "f32")
    c, g, b = (torch.from_numpy(a).cuda() for a in (cent, gamma, beta))
    for path in (binding.CAT_PATH_AUTO, binding.CAT_PATH_STREAM):
        binding.select_path(path)
        try:
            want, _ = cat_apply(lq, c, g, b, alpha=0.25)
            got, none = cat_apply_static(lq, c, g, b, alpha=0.25)
            torch.cuda.synchronize()
        finally:
            binding.select_path(binding.CAT_PATH_AUTO)
        assert none is None
        assert torch.equal(got, want)


def test_sizes_beyond_the_array_are_refused():
    torch.cuda.set_device(0)
    lib = binding.load_library()
    limit = lib.cat_apply_static_max_workspace_bytes()
    assert limit == 8 << 20
    K, D, N = 256, 2048, 512
    assert binding.cat_apply_workspace_bytes(N, D, K) > limit
    lq = torch.zeros((N, D), device="cuda")
    p = torch.zeros((K, D), device="cuda")
    with pytest.raises(binding.CatError) as e:
        cat_apply_static(lq, p, p, p)
    assert e.value.status == 2 and "cat_apply_static" in str(e.value)
    # the largest cluster count that still fits at this D goes through
    k_ok = max(k for k in range(1, K + 1) if binding.cat_apply_workspace_bytes(N, D, k) <= limit)
    cent, gamma, beta = _params(k_ok, D, 9)
    c, g, b = (torch.from_numpy(a).cuda() for a in (cent, gamma, beta))
    lq = _rows(N, cent, 10, "f32")
    want, want_a = cat_apply(lq, c, g, b)
    a = torch.empty((N,), dtype=torch.int32, device="cuda")
    got, got_a = cat_apply_static(lq, c, g, b, assignments=a)
    torch.cuda.synchronize()
    assert torch.equal(got_a, want_a) and torch.equal(got, want)
