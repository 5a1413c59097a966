"""Helpers shared by the GPU parity tests: move oracle results to the device, the error gates
(row norm and per element), row sampling for large token counts, cached full-size layers."""
import functools

import numpy as np
import torch

import paper_2412_14590_amd as mx
from oracle import ref
from paper_2412_14590_amd import synth

G = 128
TOL = 2e-3   # max relative error of a row of y, normalised by the row's L2 norm (workload target)
U32 = 2.0 ** -24   # unit roundoff of fp32


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pack_from_oracle(L: ref.QuantizedLayer) -> mx.PackedLayer:
    """Inject the oracle's codes into the library's packed layout."""
    q8 = dev(L.q8) if L.n8 else None
    s8 = dev(L.s8) if L.n8 else None
    q4 = dev(L.q4) if L.n4 else None
    s4 = dev(L.s4) if L.n4 else None
    z4 = dev(L.z4) if L.n4 else None
    return mx.pack_weights(q8, s8, q4, s4, z4, dev(L.perm), L.K, L.w8_group)


def row_rel_err(y_gpu: np.ndarray, y_ref: np.ndarray) -> float:
    a = y_gpu.astype(np.float64)
    b = y_ref.astype(np.float64)
    num = np.linalg.norm(a - b, axis=1)
    den = np.linalg.norm(b, axis=1)
    den = np.where(den == 0, 1.0, den)
    return float((num / den).max())


def weight_scales_in_channel_order(L: ref.QuantizedLayer) -> np.ndarray:
    """s_w [N, K/128] float64 in ORIGINAL channel order (an 8-bit channel with one scale repeats it)."""
    ng = L.K // L.G
    sw = np.empty((L.N, ng), np.float64)
    if L.n8:
        s8 = L.s8.astype(np.float64)
        sw[L.perm[:L.n8]] = s8 if s8.shape[1] == ng else np.repeat(s8, ng, axis=1)
    if L.n4:
        sw[L.perm[L.n8:]] = L.s4.astype(np.float64)
    return sw


def elementwise_bound(y64: np.ndarray, P: np.ndarray, xs: np.ndarray, L: ref.QuantizedLayer) -> np.ndarray:
    """Largest |y_kernel - y64| a correct kernel can show, per element.

    The kernels form v = sum_g float(P_g) s_w s_a in fp32 and round v to fp16 once.  Per group they
    round at most three times (the tiled and the decode kernels once, in a fused multiply-add;
    once more where s_w s_a is formed first; the one-thread-per-output kernel multiplies twice and
    adds), once for a token scale applied at the end, and up to 16 more times where partial sums
    of several waves or K chunks meet.  Every rounding is relative 2^-24 of a term or partial sum
    no larger than A = sum_g |P_g| s_w s_a, so |v - y64| <= delta = 3 (K/128 + 16) 2^-24 A, and the
    fp16 rounding adds half a unit in the last place of fp16 at |y64| + delta.  y64 is the
    oracle's fp64 sum (its own rounding, 2^-53 A, is far below delta)."""
    ng = L.K // L.G
    sw = weight_scales_in_channel_order(L)
    sa = xs.astype(np.float64)
    if sa.shape[1] == 1:
        sa = np.repeat(sa, ng, axis=1)
    A = np.empty(y64.shape, np.float64)
    for r0 in range(0, y64.shape[0], 8):          # row chunks: P is [rows, N, ng]
        r1 = min(y64.shape[0], r0 + 8)
        A[r0:r1] = np.einsum("mng,ng,mg->mn", np.abs(P[r0:r1]).astype(np.float64), sw, sa[r0:r1], optimize=True)
    delta = 3.0 * (ng + 16) * U32 * A
    v = np.abs(y64) + delta
    e = np.floor(np.log2(np.maximum(v, 2.0 ** -14)))       # fp16 binade (subnormals share the spacing of 2^-14)
    return 2.0 ** (e - 11) + delta


def check_against_oracle(y_gpu: np.ndarray, xq: np.ndarray, xs: np.ndarray, L: ref.QuantizedLayer, tag: str = ""):
    """y_gpu (fp16, the rows of xq) against the oracle: the workload's row-norm gate AND a bound on
    every element (elementwise_bound).  Returns (oracle partial sums P, row error) for further checks."""
    y_ref, y64 = ref.mixed_linear(xq, xs, L, want_f64=True)
    P = ref.group_partials(xq, L)
    err = row_rel_err(y_gpu, y_ref)
    assert err <= TOL, (tag, err)
    bound = elementwise_bound(y64, P, xs, L)
    yg = y_gpu.astype(np.float64)
    fits = np.abs(y64) + bound < 65504.0          # beyond that fp16 overflows to inf: covered by a test of its own
    excess = np.where(fits, np.abs(yg - y64) / bound, 0.0)
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 1.0, (tag, "element", worst, "gpu", yg[worst], "oracle fp64", y64[worst], "bound", bound[worst])
    return P, err


def stratified_rows(M: int, seed: int) -> np.ndarray:
    """Token rows to check at large M: one (seeded) per tile of 32 tokens - the tile of one MFMA and
    of one wave of the smallest block - plus the first and last row of every block of 128 tokens."""
    rng = np.random.default_rng(seed)
    rows = {0, M - 1}
    for t in range(0, M, 32):
        rows.add(min(M - 1, t + int(rng.integers(0, 32))))
    for b in range(0, M, 128):
        rows.add(b)
        rows.add(min(M - 1, b + 127))
    return np.array(sorted(rows))


def make_case(M, K, N, n8, seed, w8_group=None, act_group=None, sigma=0.02, n_outlier_rows=None):
    """Seeded inputs + oracle quantization for one layer."""
    if n_outlier_rows is None:
        n_outlier_rows = min(64, max(1, N // 64))
    W = synth.make_w(N, K, sigma, n_outlier_rows, seed)
    sal = synth.select_salient(W, n8, seed)
    L = ref.quantize_weights(W, sal, G, w8_group)
    x = synth.make_x(M, K, seed) if M else np.zeros((0, K), np.float16)
    xq, xs = ref.quantize_act(x, act_group) if M else (np.zeros((0, K), np.int8), np.zeros((0, 1), np.float16))
    return W, sal, L, x, xq, xs


@functools.lru_cache(maxsize=2)
def full_size_layer(model: str, name: str, frac8: float = 0.10, seed: int = 1, w8_group=None):
    """A full-size layer of the workload list: (inputs, the oracle's quantized layer, the GPU's packed
    layer, quantized on the GPU from the same fp16 weights).  Cached: drawing and quantizing a
    layer on the host costs more than the checks that use it."""
    K, N = (synth.LLAMA3_8B if model == "8b" else synth.LLAMA31_70B)[name]
    n_out = 64 if model == "8b" else N // 64
    lay = synth.make_layer(name, K, N, sigma=synth.SIGMA[model], frac8=frac8, n_outlier_rows=n_out, seed=seed)
    L = ref.quantize_weights(lay.W, lay.salient_idx, G, w8_group)
    PL = mx.quantize_weights(dev(lay.W), lay.salient_idx, w8_group)
    return lay, L, PL
