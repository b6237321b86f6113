"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, its seeded-row rule agrees with the oracle's
independent implementation, and every argument error is reported as a status
before anything is launched."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2509_26277_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2509_26277_amd import build
        build.build(verbose=False)
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    with open(os.path.join(ROOT, "include", "cat.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = set(re.findall(r"\b(cat_[a-z0-9_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_init_indices_agree_with_the_oracle(lib):
    for N, K, seed in [(37, 30, 99), (4096, 4, 0), (65536, 16, 1002), (1024, 1024, 7), (5, 1, 2**64 - 1),
                       (4194304, 128, 1005)]:
        got = binding.cat_init_indices(N, K, seed)
        assert got == oracle.init_indices(N, K, seed).tolist()
        assert len(set(got)) == K


def test_workspace_sizes(lib):
    assert binding.cat_fit_workspace_bytes(65536, 1000, 16, binding.CAT_F32) >= 4 * 16 * 1000 * 8
    assert binding.cat_apply_workspace_bytes(65536, 1000, 16, binding.CAT_F32) >= 2 * 16 * 1000 * 4
    assert binding.cat_fit_workspace_bytes(8, 4, 16, binding.CAT_F32) == 0      # K > N
    assert binding.cat_fit_workspace_bytes(8, 0, 2, binding.CAT_F32) == 0       # D < 1
    assert binding.cat_fit_workspace_bytes(8, 3, 2, binding.CAT_BF16) == 0      # odd D, bf16
    assert binding.cat_fit_workspace_bytes(8, 4, 2, 7) == 0                     # unknown dtype
    assert binding.cat_apply_workspace_bytes(4096, 8, 2000, binding.CAT_F32) == 0  # K > CAT_MAX_K


FAKE = 0x7F0000001000  # never dereferenced: every case below fails validation first


def _fit(lib, **kw):
    a = dict(lq=FAKE, fp=FAKE, N=64, D=8, K=4, iters=2, seed=0, dt=0, init=None, cent=FAKE, gamma=FAKE, beta=FAKE,
             assign=FAKE, counts=None, inertia=None, ws=FAKE, ws_bytes=0, stream=None)
    a.update(kw)
    return lib.cat_fit(a["lq"], a["fp"], a["N"], a["D"], a["K"], a["iters"], a["seed"], a["dt"], a["init"], a["cent"],
                       a["gamma"], a["beta"], a["assign"], a["counts"], a["inertia"], a["ws"], a["ws_bytes"], a["stream"])


def test_fit_argument_errors(lib):
    INVALID, WORKSPACE = 1, 3
    assert _fit(lib, lq=None) == INVALID and b"lq is NULL" in lib.cat_last_error()
    assert _fit(lib, fp=None) == INVALID
    assert _fit(lib, cent=None) == INVALID
    assert _fit(lib, assign=None) == INVALID
    assert _fit(lib, K=65) == INVALID          # K > N
    assert _fit(lib, K=0) == INVALID
    assert _fit(lib, N=0) == INVALID
    assert _fit(lib, D=0) == INVALID
    assert _fit(lib, iters=-1) == INVALID and b"negative" in lib.cat_last_error()
    assert _fit(lib, dt=5) == INVALID
    assert _fit(lib, dt=1, D=7) == INVALID     # bf16 rows must be 4-byte aligned
    assert _fit(lib, lq=FAKE + 4) == INVALID and b"aligned" in lib.cat_last_error()
    assert _fit(lib, ws=None) == WORKSPACE
    assert _fit(lib, ws=FAKE + 16, ws_bytes=1 << 30) == WORKSPACE
    assert _fit(lib, ws_bytes=128) == WORKSPACE and b"need" in lib.cat_last_error()


def test_apply_and_step_argument_errors(lib):
    INVALID, WORKSPACE = 1, 3
    f = ctypes.c_float
    assert lib.cat_apply(None, 64, 8, 4, 0, FAKE, FAKE, FAKE, f(1.0), FAKE, None, FAKE, 0, None) == INVALID
    assert lib.cat_apply(FAKE, 64, 8, 4, 0, FAKE, FAKE, FAKE, f(1.0), FAKE, None, FAKE, 0, None) == INVALID  # aliasing
    assert b"alias" in lib.cat_last_error()
    assert lib.cat_apply(FAKE, 64, 8, 4, 0, FAKE, FAKE, FAKE, f(float("nan")), FAKE + 4096, None, FAKE, 0,
                         None) == INVALID
    assert lib.cat_apply(FAKE, 64, 8, 4, 0, FAKE, FAKE, FAKE, f(1.0), FAKE + 4096, None, FAKE, 16, None) == WORKSPACE
    assert lib.cat_assign(FAKE, 64, 8, 4, 0, None, FAKE, None, None, FAKE, 0, None) == INVALID
    assert lib.cat_assign(FAKE, 64, 8, 4, 0, FAKE, FAKE, None, None, FAKE, 0, None) == WORKSPACE
    assert lib.cat_update(FAKE, None, 64, 8, 4, 0, FAKE, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.cat_update(FAKE, FAKE, 64, 8, 4, 0, FAKE, FAKE, None, FAKE, 0, None) == WORKSPACE
    assert lib.cat_stats(FAKE, FAKE, FAKE, 64, 8, 4, 0, None, None, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.cat_stats(FAKE, FAKE, FAKE, 64, 8, 4, 0, None, FAKE, FAKE, None, FAKE, 0, None) == WORKSPACE
    assert lib.cat_select_path(9) == INVALID and lib.cat_select_path(0) == 0
    buf = (ctypes.c_int64 * 4)()
    assert lib.cat_init_indices(3, 4, 0, buf) == INVALID
    assert lib.cat_init_indices(8, 4, 0, None) == INVALID
