"""Seeded synthetic inputs shaped like the paper's workloads.

This module is shared by the tests, the oracle-side checks and the benchmark.  It
holds no arithmetic of the method itself (no quantizer, no MatMul): it only draws
tensors and chooses which output channels are declared salient.

Recipe (stand-in for the real Llama / Qwen / Mistral weights and the calibration
text the paper uses, Sec. 4.1, none of which is available offline):
  x  fp16 [M,K]   ~ N(0,1), then round(1% of K) input channels scaled by 20 (outliers)
  W  fp16 [N,K]   ~ N(0,sigma), then `n_outlier_rows` rows scaled by 4
  salient rows    the n8 rows with the largest modelled output error of 4-bit
                  rounding (uniform-noise model, see select_salient), n8 = 10% of N
"""
from dataclasses import dataclass

import numpy as np

G = 128  # quantization group size used throughout the paper (Sec. 4.1)

# (K, N) of the linear layers of one decoder block, fused the way serving engines run them.
LLAMA3_8B = {
    "qkv": (4096, 6144),
    "o": (4096, 4096),
    "gate_up": (4096, 28672),
    "down": (14336, 4096),
}
LLAMA31_70B = {
    "qkv": (8192, 10240),
    "o": (8192, 8192),
    "gate_up": (8192, 57344),
    "down": (28672, 8192),
}
SIGMA = {"8b": 0.02, "70b": 0.015}


def _rng(seed, *tags) -> np.random.Generator:
    """Counter-based generator keyed by (seed, tags); independent streams per tensor."""
    key = [int(seed) & 0xFFFFFFFF]
    for t in tags:
        if isinstance(t, str):
            h = 2166136261
            for ch in t.encode():
                h = ((h ^ ch) * 16777619) & 0xFFFFFFFF
            key.append(h)
        else:
            key.append(int(t) & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(key)))


def make_x(M: int, K: int, seed: int = 0, tag: str = "x") -> np.ndarray:
    """Activations: N(0,1) with 1% of the input channels (same channels for every
    token) 20x larger."""
    r = _rng(seed, tag, M, K)
    x = r.standard_normal((M, K), dtype=np.float32)
    n_out = int(round(0.01 * K))
    if n_out:
        ch = _rng(seed, tag + "/outlier-channels", K).choice(K, size=n_out, replace=False)
        x[:, ch] *= 20.0
    return x.astype(np.float16)


def make_w(N: int, K: int, sigma: float = 0.02, n_outlier_rows: int = 64, seed: int = 0,
           tag: str = "w") -> np.ndarray:
    """Weights: N(0,sigma); `n_outlier_rows` random rows get 4x the std."""
    r = _rng(seed, tag, N, K)
    W = np.empty((N, K), np.float16)
    step = max(1, (1 << 24) // max(K, 1))
    for r0 in range(0, N, step):
        r1 = min(N, r0 + step)
        W[r0:r1] = (r.standard_normal((r1 - r0, K), dtype=np.float32) * np.float32(sigma)).astype(np.float16)
    n_out = min(n_outlier_rows, N)
    if n_out:
        rows = _rng(seed, tag + "/outlier-rows", N).choice(N, size=n_out, replace=False)
        W[rows] = (W[rows].astype(np.float32) * 4.0).astype(np.float16)
    return W


def n8_for(N: int, frac: float = 0.10) -> int:
    """Number of 8-bit channels for a share `frac` of N (round half to even)."""
    return int(np.clip(np.rint(frac * N), 0, N))


def select_salient(W: np.ndarray, n8: int, seed: int = 0, n_cal: int = 128) -> np.ndarray:
    """Pick the n8 output channels declared salient (sorted ascending).

    The paper ranks channels by a gradient-based loss estimate (Sec. 3.2), which needs
    a model and calibration data.  The stand-in ranks rows by a modelled output error
    of 4-bit rounding: a uniform quantizer with step (range/15) adds noise of variance
    step^2/12 to each weight, so the error energy of row n on calibration tokens X is
    proportional to  sum_g range[n,g]^2 * sum_{k in g} mean_t X[t,k]^2.
    No quantizer runs here; the choice only decides WHICH rows are 8-bit."""
    N, K = W.shape
    if n8 <= 0:
        return np.zeros(0, np.int32)
    if n8 >= N:
        return np.arange(N, dtype=np.int32)
    return np.sort(salience_order(W, seed, n_cal)[:n8]).astype(np.int32)


def salience_order(W: np.ndarray, seed: int = 0, n_cal: int = 128) -> np.ndarray:
    """All output channels of W, most salient first, by the modelled 4-bit output error that
    select_salient describes (equal scores: lower index first).  One ranking serves every 8-bit
    share of the same weights."""
    N, K = W.shape
    xc = make_x(n_cal, K, seed, tag="x_cal").astype(np.float32)
    energy = (xc * xc).mean(axis=0).reshape(K // G, G).sum(axis=1)          # [K/G]
    score = np.zeros(N, np.float64)
    step = max(1, (1 << 24) // K)
    for r0 in range(0, N, step):
        blk = W[r0:r0 + step].astype(np.float32).reshape(-1, K // G, G)
        rng_ = np.maximum(blk.max(axis=2), 0) - np.minimum(blk.min(axis=2), 0)
        score[r0:r0 + step] = (rng_.astype(np.float64) ** 2) @ energy.astype(np.float64)
    return np.lexsort((np.arange(N), -score))           # descending score, ties -> lower index


@dataclass
class LayerInputs:
    name: str
    K: int
    N: int
    n8: int
    W: np.ndarray            # fp16 [N,K]
    salient_idx: np.ndarray  # int32 [n8], ascending


def make_layer(name: str, K: int, N: int, sigma: float = 0.02, frac8: float = 0.10,
               n_outlier_rows: int = 64, seed: int = 0) -> LayerInputs:
    W = make_w(N, K, sigma, n_outlier_rows, seed, tag="w/" + name)
    n8 = n8_for(N, frac8)
    sal = select_salient(W, n8, seed)
    return LayerInputs(name, K, N, n8, W, sal)


def model_layers(model: str = "8b"):
    """[(name, K, N, sigma, n_outlier_rows)] for one decoder block of the named model.
    70B: the number of outlier rows is not stated by the workload description; N/64 is used."""
    if model == "8b":
        return [(n, k, nn, SIGMA["8b"], 64) for n, (k, nn) in LLAMA3_8B.items()]
    if model == "70b":
        return [(n, k, nn, SIGMA["70b"], nn // 64) for n, (k, nn) in LLAMA31_70B.items()]
    raise ValueError(model)


def uneven_fractions(n_layers: int = 32, seed: int = 0, mean: float = 0.10, cap: float = 0.40):
    """Per-linear 8-bit shares for a stack of `n_layers` blocks x 4 linears, drawn from a
    Dirichlet so that the channel-weighted mean share is `mean` and no layer exceeds `cap`
    (the paper's measured per-layer spread, Appendix table of per-layer 8-bit share, is
    wider still).  Returns {(layer, name): share}."""
    names = list(LLAMA3_8B)
    sizes = np.array([LLAMA3_8B[n][1] for n in names] * n_layers, np.float64)
    r = _rng(seed, "uneven", n_layers)
    f = r.dirichlet(np.full(sizes.size, 0.6))
    f = f / f.max() * cap                                   # in [0, cap]
    for _ in range(50):                                     # rescale to the target mean under the cap
        cur = (f * sizes).sum() / sizes.sum()
        f = np.minimum(f * (mean / cur), cap)
    out = {}
    for i in range(sizes.size):
        out[(i // len(names), names[i % len(names)])] = float(f[i])
    return out
