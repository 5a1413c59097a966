"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the mistake it is meant to catch.  The fixed points are: values the
paper prints (tests/golden/paper_constants.txt), closed forms, invariants of the
method (Sec. 2 quantizer, Sec. 3.1.1 disjoint output features, Sec. 3.3 two-step
dequantization), numpy's fp16 conversions, and a brute-force fp64
dequantize-then-matmul."""
import os

import numpy as np
import pytest

from oracle import ref
from paper_2412_14590_amd import synth

G = 128
HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    with open(os.path.join(HERE, "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [t.strip() for t in line.split("=")]
                out[k] = v
    return out


def f16(a):
    return np.asarray(a, dtype=np.float16)


def dequant_w(L):
    """fp64 dequantized weights in ORIGINAL channel order, straight from the codes."""
    ng = L.K // L.G
    W = np.zeros((L.N, L.K), np.float64)
    if L.n8:
        s8 = np.repeat(L.s8.astype(np.float64), L.w8_group, axis=1)
        W[L.perm[:L.n8]] = L.q8.astype(np.float64) * s8
    if L.n4:
        s4 = np.repeat(L.s4.astype(np.float64), L.G, axis=1)
        z4 = np.repeat(L.z4.astype(np.float64), L.G, axis=1)
        W[L.perm[L.n8:]] = (L.q4.astype(np.float64) - z4) * s4
    assert ng * L.G == L.K
    return W


def dequant_x(xq, xs):
    K = xq.shape[1]
    return xq.astype(np.float64) * np.repeat(xs.astype(np.float64), K // xs.shape[1], axis=1)


# ----------------------------------------------------------------- fp16 I/O --

def test_fp16_decode_exhaustive_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = ref.half_to_double(bits)
    want = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    assert np.array_equal(got[m], want[m])
    assert np.array_equal(np.signbit(got[m]), np.signbit(want[m]))


def test_fp16_round_from_double_vs_numpy_including_ties_and_subnormals():
    allh = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    fin = allh[np.isfinite(allh)]
    fin = np.sort(fin)
    mids = (fin[:-1] + fin[1:]) / 2          # exact ties between neighbours
    rng = np.random.default_rng(1)
    rnd = rng.standard_normal(300000) * 10.0 ** rng.uniform(-9, 5.2, 300000)
    near = np.concatenate([np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf)])
    v = np.concatenate([fin, mids, near, rnd, [65519.99, 65520.0, 70000.0, -1e9, 0.0, -0.0]])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = ref.double_to_half(v)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- quantizers --

def test_act_quant_closed_form_ties_to_even_and_range():
    # amax = 127 -> scale exactly 1.0, so codes are round-half-even of the values.
    vals = [127.0, -64.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.499, 126.5, -126.5, 0.0]
    x = np.zeros((1, 128), np.float16)
    x[0, :len(vals)] = f16(vals)
    xq, xs = ref.quantize_act(x)
    assert xs.shape == (1, 1) and float(xs[0, 0]) == 1.0
    want = [127, -64, 0, 2, 2, 0, -2, -2, 3, 126, -126, 0]
    # 3.499 is not fp16-representable: fp16(3.499) = 3.498..., below the tie -> 3
    assert float(f16(3.499)) < 3.5
    assert xq[0, :len(vals)].tolist() == want
    assert np.all(xq[0, len(vals):] == 0)


def test_act_quant_invariants_random():
    x = synth.make_x(37, 512, seed=3)
    for ag in (512, 128):
        xq, xs = ref.quantize_act(x, ag)
        s = np.repeat(xs.astype(np.float64), ag, axis=1)
        xf = x.astype(np.float64)
        assert xq.min() >= -127 and xq.max() <= 127
        # every element reconstructs to within half a step (division is correctly rounded
        # in fp32, so allow a relative 2^-22 on top)
        assert np.all(np.abs(xq * s - xf) <= s * (0.5 + 1e-6))
        # the largest element of each block lands on +-127
        blk = np.abs(xf).reshape(37, -1, ag)
        am = blk.argmax(axis=2)
        codes = np.take_along_axis(np.abs(xq.astype(np.int32)).reshape(37, -1, ag), am[..., None], axis=2)
        assert np.all(codes == 127)
        # scale is fp16(amax/127) computed in fp32
        want_s = (blk.max(axis=2).astype(np.float32) / np.float32(127)).astype(np.float16)
        assert np.array_equal(xs, want_s)


def test_act_quant_power_of_two_scaling_leaves_codes_unchanged():
    x = synth.make_x(5, 256, seed=4)
    x = (x.astype(np.float32) * 0.125).astype(np.float16)      # keep clear of fp16 overflow
    xq1, xs1 = ref.quantize_act(x)
    x2 = (x.astype(np.float32) * 8.0).astype(np.float16)        # exact in fp16
    xq2, xs2 = ref.quantize_act(x2)
    assert np.array_equal(xq1, xq2)
    assert np.array_equal(xs2.astype(np.float32), xs1.astype(np.float32) * 8.0)


def test_degenerate_blocks_get_unit_scale_and_zero_codes():
    x = np.zeros((2, 256), np.float16)
    x[1, 0] = np.float16(6e-8)             # smallest subnormal: amax/127 rounds to 0 in fp16
    xq, xs = ref.quantize_act(x)
    assert np.all(xs.astype(np.float32) == 1.0) and np.all(xq == 0)
    q, s, z = ref.quantize_w4(np.zeros((3, 256), np.float16))
    assert np.all(q == 0) and np.all(z == 0) and np.all(s.astype(np.float32) == 1.0)
    q, s = ref.quantize_w8(np.zeros((3, 256), np.float16))
    assert np.all(q == 0) and np.all(s.astype(np.float32) == 1.0)


def test_w4_exact_grid_reproduces_itself():
    # A group whose values are exactly the 16 levels s*(i - z): codes must be i, zero point z.
    for s_true, z_true in ((0.25, 5), (0.0078125, 0), (2.0, 15), (0.5, 8)):
        levels = (np.arange(16) - z_true) * s_true
        w = np.tile(levels, 8)[None, :].astype(np.float16)      # one group of 128
        q, s, z = ref.quantize_w4(w)
        assert float(s[0, 0]) == s_true and int(z[0, 0]) == z_true
        assert np.array_equal(q[0], np.tile(np.arange(16), 8))


def test_w4_ties_and_asymmetric_zero_point():
    # values 0..15 plus two ties: scale 1, zero point 0, ties go to even
    w = np.zeros((1, 128), np.float16)
    w[0, :16] = np.arange(16)
    w[0, 16:20] = f16([2.5, 3.5, 0.5, 14.5])
    q, s, z = ref.quantize_w4(w)
    assert float(s[0, 0]) == 1.0 and int(z[0, 0]) == 0
    assert q[0, 16:20].tolist() == [2, 4, 0, 14]
    # range [-5,10]: zero point 5, codes = value + 5
    w = np.zeros((1, 128), np.float16)
    w[0, :16] = np.arange(16) - 5
    q, s, z = ref.quantize_w4(w)
    assert float(s[0, 0]) == 1.0 and int(z[0, 0]) == 5
    assert q[0, :16].tolist() == list(range(16)) and np.all(q[0, 16:] == 5)
    # all-positive group: the range is widened to contain 0, so z = 0 and nothing clips
    w = np.full((1, 128), 3.0, np.float16)
    w[0, 0] = 7.5
    q, s, z = ref.quantize_w4(w)
    assert int(z[0, 0]) == 0 and float(s[0, 0]) == 0.5 and q[0, 0] == 15 and q[0, 1] == 6


def test_w4_invariants_random():
    W = synth.make_w(48, 512, seed=5, n_outlier_rows=4)
    q, s, z = ref.quantize_w4(W)
    assert q.max() <= 15 and z.max() <= 15            # uint4 codes and zero points (Sec. 3.3)
    d = q.astype(np.int32) - np.repeat(z.astype(np.int32), G, axis=1)
    assert d.min() >= -15 and d.max() <= 15           # (W_q - z) fits int8 without overflow (Sec. 3.3)
    sf = np.repeat(s.astype(np.float64), G, axis=1)
    err = np.abs(d * sf - W.astype(np.float64))
    # inside the representable range the error is at most half a step; the fp16 rounding of
    # the scale can push the extreme element out by at most 15 * 2^-11 of a step.
    assert np.all(err <= sf * (0.5 + 15 * 2.0 ** -11 + 1e-6))
    # scale is fp16((max0 - min0)/15) in fp32
    Wf = W.astype(np.float32).reshape(48, -1, G)
    rngv = np.maximum(Wf.max(axis=2), 0) - np.minimum(Wf.min(axis=2), 0)
    assert np.array_equal(s, (rngv / np.float32(15)).astype(np.float16))
    # the group minimum maps to code 0; the maximum to 15, or 14 when the zero point and the
    # maximum both round down (rne(a) + rne(15 - a) is 14, 15 or 16 before the clamp)
    assert np.all(q.reshape(48, -1, G).min(axis=2) == 0)
    assert np.all(q.reshape(48, -1, G).max(axis=2) >= 14)


def test_w8_invariants_per_channel_and_per_group():
    W = synth.make_w(16, 512, seed=6, n_outlier_rows=2)
    for g in (512, 128):
        q, s = ref.quantize_w8(W, g)
        assert s.shape == (16, 512 // g)
        sf = np.repeat(s.astype(np.float64), g, axis=1)
        assert np.abs(q.astype(np.int32)).max() == 127
        assert np.all(np.abs(q * sf - W.astype(np.float64)) <= sf * (0.5 + 1e-6))
        Wf = np.abs(W.astype(np.float32)).reshape(16, -1, g).max(axis=2)
        assert np.array_equal(s, (Wf / np.float32(127)).astype(np.float16))


# ---------------------------------------------------------- feature ordering --

def test_feature_perm_order_and_errors():
    perm = ref.feature_perm(8, [6, 1, 3])
    assert perm.tolist() == [1, 3, 6, 0, 2, 4, 5, 7]     # 8-bit ascending, then 4-bit ascending
    assert ref.feature_perm(4, []).tolist() == [0, 1, 2, 3]
    assert ref.feature_perm(3, [2, 0, 1]).tolist() == [0, 1, 2]
    with pytest.raises(ValueError):
        ref.feature_perm(4, [1, 1])
    with pytest.raises(ValueError):
        ref.feature_perm(4, [4])


# ------------------------------------------------ partial sums and the linear --

def small_layer(N=7, K=256, n8=2, seed=7, w8_group=None):
    W = synth.make_w(N, K, seed=seed, n_outlier_rows=1)
    sal = synth.select_salient(W, n8, seed)
    return W, sal, ref.quantize_weights(W, sal, G, w8_group)


def test_one_hot_and_all_ones_activations_read_out_codes():
    W, sal, L = small_layer()
    K, N = L.K, L.N
    # one-hot at k: P[m, n, g(k)] = integer weight at k, other groups 0 (wrong index/transposed
    # operand shows here)
    ks = [0, 5, 127, 128, 255]
    xq = np.zeros((len(ks), K), np.int8)
    for i, k in enumerate(ks):
        xq[i, k] = 1
    P = ref.group_partials(xq, L)
    Wi = np.zeros((N, K), np.int32)
    Wi[L.perm[:L.n8]] = L.q8
    Wi[L.perm[L.n8:]] = L.q4.astype(np.int32) - np.repeat(L.z4.astype(np.int32), G, axis=1)
    for i, k in enumerate(ks):
        want = np.zeros((N, K // G), np.int32)
        want[:, k // G] = Wi[:, k]
        assert np.array_equal(P[i], want)
    # all ones: P = sum over the group of (q - z)  (a dropped zero point shows here)
    P1 = ref.group_partials(np.ones((1, K), np.int8), L)[0]
    assert np.array_equal(P1, Wi.reshape(N, K // G, G).sum(axis=2))


@pytest.mark.parametrize("n8", [0, 2, 7])
@pytest.mark.parametrize("variant", ["baseline", "paper"])
def test_linear_equals_bruteforce_fp64_dequantize_then_matmul(n8, variant):
    # Sec. 3.5 closed form: sum_g P * s_w * s_a == (A_q s_a) (W_q - z) s_w.  n8 = 0 and n8 = N
    # are the all-4-bit / all-8-bit degenerate layers (the 0% and 100% settings of Sec. 4.1).
    act_group, w8_group = (256, None) if variant == "baseline" else (128, 128)
    W, sal, L = small_layer(N=7, K=256, n8=n8, seed=11, w8_group=w8_group)
    x = synth.make_x(3, 256, seed=11)
    xq, xs = ref.quantize_act(x, act_group)
    y, y64 = ref.mixed_linear(xq, xs, L, want_f64=True)
    want = dequant_x(xq, xs) @ dequant_w(L).T
    assert np.allclose(y64, want, rtol=1e-12, atol=1e-12)
    assert np.array_equal(y.view(np.uint16), want.astype(np.float16).view(np.uint16)) or \
        np.array_equal(y.view(np.uint16), y64.astype(np.float16).view(np.uint16))
    # integer partials against an integer matmul per group
    P = ref.group_partials(xq, L)
    Wi = np.zeros((L.N, L.K), np.int64)
    Wi[L.perm[:L.n8]] = L.q8
    Wi[L.perm[L.n8:]] = L.q4.astype(np.int64) - np.repeat(L.z4.astype(np.int64), G, axis=1)
    for g in range(L.K // G):
        sl = slice(g * G, (g + 1) * G)
        assert np.array_equal(P[:, :, g], xq[:, sl].astype(np.int64) @ Wi[:, sl].T)


def test_partials_stay_inside_fast_i2f_window():
    gd = golden()
    assert int(gd["i2f_group_k"]) == G
    W, sal, L = small_layer(N=16, K=512, n8=4, seed=12)
    # worst-case activations
    xq = np.where(np.random.default_rng(0).random((4, 512)) < 0.5, -127, 127).astype(np.int8)
    P = ref.group_partials(xq, L)
    assert np.abs(P).max() <= G * 127 * 127 < 2 ** (int(gd["i2f_window_log2"]) - 1)


def test_output_feature_permutation_only_permutes_columns():
    # Sec. 3.1.1: output features are disjoint sub-problems.
    N, K = 12, 256
    W = synth.make_w(N, K, seed=13, n_outlier_rows=2)
    sal = np.array([1, 4, 9], np.int32)
    x = synth.make_x(4, K, seed=13)
    xq, xs = ref.quantize_act(x)
    y = ref.mixed_linear(xq, xs, ref.quantize_weights(W, sal))
    sigma = np.random.default_rng(2).permutation(N)       # new row i = old row sigma[i]
    inv = np.argsort(sigma)
    y2 = ref.mixed_linear(xq, xs, ref.quantize_weights(W[sigma], np.sort(inv[sal]).astype(np.int32)))
    assert np.array_equal(y2.view(np.uint16), y[:, sigma].view(np.uint16))


def test_moving_one_row_between_parts_changes_only_that_column():
    N, K = 10, 256
    W = synth.make_w(N, K, seed=14, n_outlier_rows=1)
    x = synth.make_x(3, K, seed=14)
    xq, xs = ref.quantize_act(x)
    ya = ref.mixed_linear(xq, xs, ref.quantize_weights(W, [2, 5]))
    yb = ref.mixed_linear(xq, xs, ref.quantize_weights(W, [2, 5, 7]))
    diff = np.any(ya.view(np.uint16) != yb.view(np.uint16), axis=0)
    assert diff[7] and not np.any(np.delete(diff, 7))


def test_quantized_linear_is_within_the_rounding_error_bound_of_the_exact_product():
    # |x - xq*sa| <= sa/2 and |w - wq| <= sw/2 (+ fp16-scale slack) elementwise, hence
    # |y - x.w| <= sum_k |x| ew + |w| ex + ex ew.  A wrong scale or sign breaks the bound.
    N, K, M = 24, 512, 6
    W = synth.make_w(N, K, seed=15, n_outlier_rows=2)
    sal = synth.select_salient(W, 5, 15)
    L = ref.quantize_weights(W, sal)
    x = synth.make_x(M, K, seed=15)
    xq, xs = ref.quantize_act(x)
    _, y64 = ref.mixed_linear(xq, xs, L, want_f64=True)
    exact = x.astype(np.float64) @ W.astype(np.float64).T
    ex = np.repeat(xs.astype(np.float64), K, axis=1) * 0.5001
    ew = np.zeros((N, K))
    ew[L.perm[:L.n8]] = np.repeat(L.s8.astype(np.float64), L.w8_group, axis=1) * 0.5001
    ew[L.perm[L.n8:]] = np.repeat(L.s4.astype(np.float64), G, axis=1) * (0.5 + 15 * 2.0 ** -11 + 1e-4)
    bound = np.abs(x.astype(np.float64)) @ ew.T + ex @ np.abs(W.astype(np.float64)).T + ex @ ew.T
    assert np.all(np.abs(y64 - exact) <= bound)
    # and the error is far from trivial-zero: the bound is not vacuous
    assert np.abs(y64 - exact).max() > 0


def test_error_shrinks_as_more_rows_go_8bit():
    # mirrors the ordering of the 0/10/20/50/100% rows of the perplexity table (Sec. 4.2)
    N, K, M = 64, 512, 16
    W = synth.make_w(N, K, seed=16, n_outlier_rows=6)
    x = synth.make_x(M, K, seed=16)
    xq, xs = ref.quantize_act(x)
    exact = dequant_x(xq, xs) @ W.astype(np.float64).T        # isolate the weight error
    errs = []
    for n8 in (0, 6, 13, 32, 64):
        L = ref.quantize_weights(W, synth.select_salient(W, n8, 16))
        _, y64 = ref.mixed_linear(xq, xs, L, want_f64=True)
        errs.append(np.linalg.norm(y64 - exact))
    assert all(a > b for a, b in zip(errs, errs[1:])), errs


def test_fast_i2f_identity_from_the_paper_holds_on_the_partial_sum_range():
    # Sec. 3.3: as_float(i + 0x4b400000) - as_float(0x4b400000) == float(i) inside the window.
    gd = golden()
    magic = int(gd["i2f_magic_hex"], 16)
    assert np.array([magic], np.uint32).view(np.float32)[0] == 12582912.0
    lim = G * 127 * 127
    i = np.concatenate([np.arange(-lim, -lim + 1000), np.arange(-1000, 1000), np.arange(lim - 1000, lim + 1),
                        np.random.default_rng(3).integers(-lim, lim, 100000)]).astype(np.int32)
    f = (i + np.int32(magic)).view(np.float32) - np.float32(12582912.0)
    assert np.array_equal(f, i.astype(np.float32))
    # and it breaks outside the 2^23 window, as the paper's range argument says
    bad = np.array([2 ** 22 + 5], np.int32)
    assert ((bad + np.int32(magic)).view(np.float32) - np.float32(12582912.0))[0] != np.float32(bad[0])


def test_paper_roofline_constants():
    gd = golden()
    assert round(float(gd["a100_int8_tops"]) * 1e3 / float(gd["a100_hbm_gbs"])) == int(gd["a100_ridge_op_per_byte"])
    assert float(gd["a100_int8_tops"]) / float(gd["a100_fp32_tflops"]) == float(gd["a100_tc_to_simt_ratio"])
    assert 1 + 2 / G == float(gd["w8a8_bytes_per_weight_G128"])
    assert 0.5 + 2.5 / G == float(gd["w4a8_bytes_per_weight_G128"])


def test_config0_shape_runs_and_matches_bruteforce_on_sampled_columns():
    # The single-layer workload: M=1, K=N=4096, 410 int8 rows.  Full oracle run, checked on a column sample.
    lay = synth.make_layer("o", 4096, 4096, seed=0)
    assert lay.n8 == 410 and len(lay.salient_idx) == 410
    L = ref.quantize_weights(lay.W, lay.salient_idx)
    x = synth.make_x(1, 4096, seed=0)
    xq, xs = ref.quantize_act(x)
    y, y64 = ref.mixed_linear(xq, xs, L, want_f64=True)
    cols = np.random.default_rng(5).choice(4096, 64, replace=False)
    want = dequant_x(xq, xs) @ dequant_w(L)[cols].T
    assert np.allclose(y64[:, cols], want, rtol=1e-12, atol=1e-12)
    # the 64 planted outlier rows are all among the salient ones
    Wn = np.linalg.norm(lay.W.astype(np.float32), axis=1)
    top64 = np.argsort(-Wn)[:64]
    assert np.all(np.isin(top64, lay.salient_idx))


# ------------------------------------------------ global precision search (Sec. 3.2) --

def _salience_by_hand(W, Gd):
    """Eq. 4 for one sample, re-derived from the quantizer's codes in plain fp64 numpy."""
    q, s, z = ref.quantize_w4(W)
    N, K = W.shape
    deq = (q.astype(np.float64).reshape(N, K // 128, 128) - z.astype(np.float64)[:, :, None]) * \
        s.astype(np.float64)[:, :, None]
    s1 = (Gd.astype(np.float64) * (deq.reshape(N, K) - W.astype(np.float64))).sum(axis=1)
    return np.abs(s1 + 0.5 * s1 * s1), s1


def test_salience_is_zero_when_the_weights_sit_on_the_4bit_grid():
    # every group holds the 16 levels 0, 0.5, ..., 7.5: quantization reproduces it exactly
    W = np.tile(np.arange(16, dtype=np.float16) * np.float16(0.5), (3, 16))       # [3, 256]
    Gd = synth.make_x(3, 256, seed=5, tag="g").astype(np.float16)
    sal, s1 = ref.channel_salience(W, Gd)
    assert np.all(s1 == 0) and np.all(sal == 0)


def test_salience_closed_form_first_and_second_order_terms():
    # one group with range [0, 15] (scale 1, zero point 0) and one element at 7.25 -> code 7,
    # quantization error -0.25; the gradient is non-zero only there
    W = np.zeros((1, 128), np.float16)
    W[0, 1], W[0, 2] = 15.0, 7.25
    for g, s1_want, sal_want in [(1.0, -0.25, 0.21875),      # |-0.25 + 0.03125|
                                 (8.0, -2.0, 0.0),           # |-2 + 2|: first and second order cancel
                                 (-8.0, 2.0, 4.0),           # |2 + 2|
                                 (4.0, -1.0, 0.5)]:          # |-1 + 0.5|
        Gd = np.zeros((1, 128), np.float16)
        Gd[0, 2] = g
        sal, s1 = ref.channel_salience(W, Gd)
        assert s1[0] == s1_want and sal[0] == sal_want, (g, s1, sal)


def test_salience_equals_the_formula_evaluated_by_hand_and_averages_over_samples():
    W = synth.make_w(37, 512, seed=11, n_outlier_rows=3)
    g1 = (synth.make_x(37, 512, seed=12, tag="g1") * 0.05).astype(np.float16)
    g2 = (synth.make_x(37, 512, seed=13, tag="g2") * 5.0).astype(np.float16)     # large: the square term matters
    for g in (g1, g2):
        sal, s1 = ref.channel_salience(W, g)
        want, s1_want = _salience_by_hand(W, g)
        assert np.allclose(s1, s1_want, rtol=1e-12, atol=1e-15) and np.allclose(sal, want, rtol=1e-12, atol=1e-15)
    assert np.any(np.abs(_salience_by_hand(W, g2)[1]) > 0.5)
    both, _ = ref.channel_salience(W, [g1, g2])
    assert np.allclose(both, 0.5 * (_salience_by_hand(W, g1)[0] + _salience_by_hand(W, g2)[0]), rtol=1e-12)
    # a channel's salience depends on its own row only
    p = np.random.default_rng(2).permutation(37)
    assert np.array_equal(ref.channel_salience(W[p], g1[p])[0], ref.channel_salience(W, g1)[0][p])


def test_global_selection_takes_the_top_t_over_all_layers_with_ties_to_the_earlier_channel():
    rng = np.random.default_rng(9)
    layers = [rng.integers(0, 6, n).astype(np.float32) * 0.25 for n in (7, 1, 30, 12)]   # many equal values
    flat = np.concatenate(layers)
    for T in (0, 1, 5, 17, flat.size):
        got = ref.select_salient(layers, T)
        order = sorted(range(flat.size), key=lambda i: (-flat[i], i))[:T]
        o = 0
        for lay, idx in zip(layers, got):
            want = sorted(i - o for i in order if o <= i < o + lay.size)
            assert idx.tolist() == want
            o += lay.size
        assert sum(len(i) for i in got) == T
    assert [a.tolist() for a in ref.select_salient([np.float32([3, 1, 2]), np.float32([2, 5])], 3)] == [[0, 2], [1]]
    with pytest.raises(ValueError):
        ref.select_salient(layers, flat.size + 1)
