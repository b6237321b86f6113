"""Seeded synthetic inputs for the CAT hot path.

This module only draws numbers.  It holds none of the method's arithmetic (no
distances, no assignment, no means/variances, no affine fit) and is the one
piece of code that both the GPU tests/benchmark and the CPU oracle's tests may
share.  It depends on numpy alone.

The paper applies CAT to ImageNet-1K calibration logits (d = 1000 classes, up to
100,000 fitting samples, 1..256 clusters; Sec. 4 Setup, Sec. 5 ablations, Sec. 6).
Neither that data set nor the networks are available here, so the five workloads
below stand in for it: same shapes, same qualitative structure (a clusterable LQ
cloud whose relation to FP is a per-cluster, per-channel affine map plus
quantisation-like noise).

    cfg1  N=4,096     D=64    K=4    fp32  planted mixture, 20 Lloyd iterations
    cfg2  N=65,536    D=1000  K=16   fp32  logit-shaped, heavy tails, 30 iterations
    cfg3  N=1,048,576 D=256   K=32   fp32  post-ReLU feature map, 4-level LQ, 15 iterations
    cfg4  N=262,144   D=2048  K=64   bf16  Zipf(1.1)-skewed cluster sizes, 20 iterations
    cfg5  N=4,194,304 D=512   K=128  fp32  inference only, parameters drawn from the seed

"N(0, v)" is read as variance v (so N(0, 0.5) has std 0.7071 and N(0, 0.1) has
std 0.3162).  Every generator takes ``n_rows`` so that tests can run a
structure-preserving, smaller copy of a workload.
"""
from dataclasses import dataclass

import numpy as np

_ROW_CHUNK = 1 << 16  # rows drawn at a time, bounds the temporaries


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    D: int
    K: int
    iters: int
    dtype: str  # "f32" | "bf16"
    kind: str  # "fit" | "apply"


CONFIGS = {
    "cfg1": Config("cfg1", 4096, 64, 4, 20, "f32", "fit"),
    "cfg2": Config("cfg2", 65536, 1000, 16, 30, "f32", "fit"),
    "cfg3": Config("cfg3", 1048576, 256, 32, 15, "f32", "fit"),
    "cfg4": Config("cfg4", 262144, 2048, 64, 20, "bf16", "fit"),
    "cfg5": Config("cfg5", 4194304, 512, 128, 0, "f32", "apply"),
    # cfg2 with one more channel: rows that are not whole 16-byte groups (the shapes the matrix-core kernels do not
    # take as they lie); not one of the five listed workloads, measured beside them
    "cfg2u": Config("cfg2u", 65536, 1001, 16, 30, "f32", "fit"),
}


def seed_of(name):
    return 1000 + list(CONFIGS).index(name) + 1


# ---------------------------------------------------------------------------
# bf16 helpers (storage format only: round-to-nearest-even of an fp32 value to
# its upper 16 bits, and the exact widening back)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x):
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(u):
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x):
    """fp32 array holding the values a bf16 copy of ``x`` would hold."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ---------------------------------------------------------------------------
# shared pieces
# ---------------------------------------------------------------------------
def _affine_distortion(rng, K, D):
    g = rng.uniform(0.5, 1.5, size=(K, D)).astype(np.float32)
    b = (rng.standard_normal((K, D)) * np.sqrt(0.5)).astype(np.float32)
    return g, b


def _uniform_labels(rng, N, K):
    return rng.integers(0, K, size=N, dtype=np.int32)


def _zipf_labels(rng, N, K, s):
    p = 1.0 / np.arange(1, K + 1, dtype=np.float64) ** s
    p /= p.sum()
    return rng.choice(K, size=N, p=p).astype(np.int32)


def _chunks(N):
    for lo in range(0, N, _ROW_CHUNK):
        yield lo, min(N, lo + _ROW_CHUNK)


# ---------------------------------------------------------------------------
# the five workloads
# ---------------------------------------------------------------------------
def planted_mixture(N, D, K, seed, zipf=None, bf16=False):
    """cfg1 / cfg4 structure.

    mu_k ~ N(0, 4 I); FP = mu_k + N(0, I); LQ = g_k * FP + b_k + N(0, 0.05^2),
    g_k ~ U(0.5, 1.5), b_k ~ N(0, 0.5) per channel.  Labels i.i.d. uniform, or
    with probabilities proportional to k^-zipf.
    """
    rng = np.random.default_rng(seed)
    mu = (rng.standard_normal((K, D)) * 2.0).astype(np.float32)
    g, b = _affine_distortion(rng, K, D)
    labels = _uniform_labels(rng, N, K) if zipf is None else _zipf_labels(rng, N, K, zipf)
    fp = np.empty((N, D), dtype=np.float32)
    lq = np.empty((N, D), dtype=np.float32)
    for lo, hi in _chunks(N):
        lab = labels[lo:hi]
        f = mu[lab] + rng.standard_normal((hi - lo, D), dtype=np.float32)
        q = g[lab] * f + b[lab] + np.float32(0.05) * rng.standard_normal((hi - lo, D), dtype=np.float32)
        fp[lo:hi] = f
        lq[lo:hi] = q
    if bf16:
        fp = round_to_bf16(fp)
        lq = round_to_bf16(lq)
    return dict(lq=lq, fp=fp, labels=labels, mu=mu, g=g, b=b, noise_std=0.05)


def logit_mixture(N, D, K, seed):
    """cfg2 structure: FP = mu_k + Student-t(df=4) noise, mu_k ~ N(0, 3^2 I);
    LQ = g_k * FP + b_k + U(-1/2, 1/2) (coarse rounding noise)."""
    rng = np.random.default_rng(seed)
    mu = (rng.standard_normal((K, D)) * 3.0).astype(np.float32)
    g, b = _affine_distortion(rng, K, D)
    labels = _uniform_labels(rng, N, K)
    fp = np.empty((N, D), dtype=np.float32)
    lq = np.empty((N, D), dtype=np.float32)
    for lo, hi in _chunks(N):
        lab = labels[lo:hi]
        f = mu[lab] + rng.standard_t(4.0, size=(hi - lo, D)).astype(np.float32)
        q = g[lab] * f + b[lab] + rng.uniform(-0.5, 0.5, size=(hi - lo, D)).astype(np.float32)
        fp[lo:hi] = f
        lq[lo:hi] = q
    return dict(lq=lq, fp=fp, labels=labels, mu=mu, g=g, b=b)


def relu_feature_map(N, D, K, seed):
    """cfg3 structure: FP = max(0, mu_k + N(0, I)), mu_k ~ N(-1, 2^2 I); LQ = FP
    snapped to 4 uniform levels on [0, 9] (step 3), then g_k * . + b_k.  Many
    (cluster, channel) pairs are constant in LQ while FP still varies."""
    rng = np.random.default_rng(seed)
    mu = (rng.standard_normal((K, D)) * 2.0 - 1.0).astype(np.float32)
    g, b = _affine_distortion(rng, K, D)
    labels = _uniform_labels(rng, N, K)
    top, step = np.float32(9.0), np.float32(3.0)
    fp = np.empty((N, D), dtype=np.float32)
    lq = np.empty((N, D), dtype=np.float32)
    for lo, hi in _chunks(N):
        lab = labels[lo:hi]
        f = np.maximum(mu[lab] + rng.standard_normal((hi - lo, D), dtype=np.float32), np.float32(0.0))
        lev = np.rint(np.minimum(f, top) / step) * step
        fp[lo:hi] = f
        lq[lo:hi] = g[lab] * lev + b[lab]
    return dict(lq=lq, fp=fp, labels=labels, mu=mu, g=g, b=b)


def inference_stream(N, D, K, seed):
    """cfg5 structure: centroids ~ N(0, I), gamma ~ U(0.8, 1.2), beta ~ N(0, 0.1);
    rows = centroid of a uniformly drawn component + N(0, I)."""
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((K, D), dtype=np.float32)
    gamma = rng.uniform(0.8, 1.2, size=(K, D)).astype(np.float32)
    beta = (rng.standard_normal((K, D)) * np.sqrt(0.1)).astype(np.float32)
    labels = _uniform_labels(rng, N, K)
    lq = np.empty((N, D), dtype=np.float32)
    for lo, hi in _chunks(N):
        lq[lo:hi] = cent[labels[lo:hi]] + rng.standard_normal((hi - lo, D), dtype=np.float32)
    return dict(lq=lq, labels=labels, centroids=cent, gamma=gamma, beta=beta)


def make(name, n_rows=None, seed=None):
    """Draw workload ``name`` ('cfg1'..'cfg5', 'cfg2u'); ``n_rows`` overrides N."""
    c = CONFIGS[name]
    N = c.N if n_rows is None else int(n_rows)
    s = seed_of(name) if seed is None else seed
    if name == "cfg1":
        w = planted_mixture(N, c.D, c.K, s)
    elif name in ("cfg2", "cfg2u"):
        w = logit_mixture(N, c.D, c.K, s)
    elif name == "cfg3":
        w = relu_feature_map(N, c.D, c.K, s)
    elif name == "cfg4":
        w = planted_mixture(N, c.D, c.K, s, zipf=1.1, bf16=True)
    elif name == "cfg5":
        w = inference_stream(N, c.D, c.K, s)
    else:
        raise KeyError(name)
    w.update(name=name, N=N, D=c.D, K=c.K, iters=c.iters, dtype=c.dtype, kind=c.kind, seed=s)
    return w
