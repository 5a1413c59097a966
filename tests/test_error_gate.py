"""CPU checks of the per-element gate the GPU parity tests apply to fp16 outputs
(util.elementwise_bound): fp32 emulations of the orders in which the kernels add the group terms
stay inside it, and a single wrong (channel, group) partial - which the row-norm gate of the
workload lets through - breaks it.  The mistake is planted in a copy of the oracle's partials."""
import numpy as np

from oracle import ref
from util import TOL, elementwise_bound, make_case, row_rel_err, weight_scales_in_channel_order


def emulate(P, sw, sa, order):
    """y fp16 from int32 partials the way a kernel would: fp32 throughout, one rounding to fp16."""
    M, N, ng = P.shape
    Pf = P.astype(np.float32)
    sw = sw.astype(np.float32)
    sa = np.repeat(sa.astype(np.float32), ng // sa.shape[1], axis=1)
    if order == "fma_then_token_scale":        # acc += P s_w per group (product exact in the fma), token scale last
        acc = np.zeros((M, N), np.float64)
        for g in range(ng):
            acc = (acc + Pf[:, :, g].astype(np.float64) * sw[None, :, g].astype(np.float64)).astype(np.float32).astype(np.float64)
        v = (acc.astype(np.float32) * sa[:, :1]).astype(np.float32)
    elif order == "scale_product_first":       # s = s_w s_a rounded, then fma
        acc = np.zeros((M, N), np.float64)
        for g in range(ng):
            s = (sw[None, :, g] * sa[:, g:g + 1]).astype(np.float32)
            acc = (acc + Pf[:, :, g].astype(np.float64) * s.astype(np.float64)).astype(np.float32).astype(np.float64)
        v = acc.astype(np.float32)
    else:                                      # three roundings per term, groups in reverse order
        acc = np.zeros((M, N), np.float32)
        for g in reversed(range(ng)):
            t = (Pf[:, :, g] * sw[None, :, g]).astype(np.float32)
            t = (t * sa[:, g:g + 1]).astype(np.float32)
            acc = (acc + t).astype(np.float32)
        v = acc
    return v.astype(np.float16)


def case(variant):
    ag, wg = (None, None) if variant == "baseline" else (128, 128)
    _, _, L, _, xq, xs = make_case(6, 2048, 96, 10, seed=91, w8_group=wg, act_group=ag)
    y_ref, y64 = ref.mixed_linear(xq, xs, L, want_f64=True)
    P = ref.group_partials(xq, L)
    return L, xs, y_ref, y64, P


def test_fp32_emulations_of_the_kernels_orders_stay_inside_the_bound():
    for variant in ("baseline", "paper"):
        L, xs, y_ref, y64, P = case(variant)
        bound = elementwise_bound(y64, P, xs, L)
        sw = weight_scales_in_channel_order(L)
        for order in ("fma_then_token_scale", "scale_product_first", "three_roundings_reversed"):
            if order == "fma_then_token_scale" and variant == "paper":
                continue
            y = emulate(P, sw, xs, order)
            assert np.all(np.abs(y.astype(np.float64) - y64) <= bound), (variant, order)
        # the oracle's own fp16 result is inside it with room to spare
        assert np.all(np.abs(y_ref.astype(np.float64) - y64) <= bound)


def test_one_wrong_group_partial_breaks_the_element_gate_but_not_the_row_norm_gate():
    L, xs, y_ref, y64, P = case("baseline")
    bound = elementwise_bound(y64, P, xs, L)
    sw = weight_scales_in_channel_order(L)
    bad = P.copy()
    bad[2, 40, 7] += 3          # one partial of one (token, channel, group) off by three
    y = emulate(bad, sw, xs, "fma_then_token_scale")
    assert row_rel_err(y, y_ref) <= TOL                       # the workload's gate does not see it
    excess = np.abs(y.astype(np.float64) - y64) / bound
    assert excess[2, 40] > 1.0 and (np.delete(excess[2], 40) <= 1.0).all()


def test_bound_is_half_an_fp16_ulp_where_the_sum_has_no_cancellation():
    # a single group, one exact term: the bound is the fp16 rounding alone (plus a relative 1e-5)
    L, xs, y_ref, y64, P = case("baseline")
    b = elementwise_bound(np.array([[1.0, 3.0, 1000.0, 2.0 ** -20]]), np.zeros((1, 4, L.K // 128), np.int32), xs[:1],
                          type("Layer", (), dict(K=L.K, G=128, N=4, n8=0, n4=4, perm=np.arange(4), s8=L.s8[:0], s4=L.s4[:4]))())
    assert np.allclose(b, [2.0 ** -11, 2.0 ** -10, 2.0 ** -2, 2.0 ** -25])
