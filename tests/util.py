"""Helpers shared by the GPU parity tests: move oracle results to the device, error metric."""
import numpy as np
import torch

import paper_2412_14590_amd as mx
from oracle import ref
from paper_2412_14590_amd import synth

G = 128
TOL = 2e-3   # max relative error of a row of y, normalised by the row's L2 norm (workload target)


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
