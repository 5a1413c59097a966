"""The entry point that allocates nothing (mixllm_mixed_linear_fp16_static, scratch in a device array of
the library) against the entry point that takes a workspace, through the C ABI: the same kernels, so
the outputs must be bit-identical, call after call, also when a smaller input follows a larger one and
finds the larger one's leftovers in the scratch area."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2412_14590_amd as mx
from paper_2412_14590_amd import synth

from util import check_against_oracle, dev, make_case, pack_from_oracle
from oracle import ref

pytestmark = pytest.mark.gpu

STATIC_BYTES = 8 * 1024 * 1024 + 256 * 1024


def call_both(x, PL, act_group=None):
    """(y of the workspace entry point, y of the static one); the static call is made with the caching
    allocator's statistics watched: it must not allocate."""
    M, K = x.shape
    d = PL.desc(M, act_group)
    need = mx.query_sizes(M, K, PL.N, PL.n8, act_group, PL.w8_group)["workspace_bytes"]
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    y1 = torch.zeros((M, PL.N), dtype=torch.float16, device="cuda")
    y2 = torch.zeros((M, PL.N), dtype=torch.float16, device="cuda")
    L = mx.lib()
    p = lambda t: C.c_void_p(t.data_ptr()) if t.numel() else None
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.mixllm_mixed_linear_fp16(C.byref(d), p(x), p(PL.w4), p(PL.w8), p(PL.s4), p(PL.s8), p(PL.z4), p(PL.perm), p(y1),
                                    p(ws), C.c_size_t(ws.numel()), st)
    assert rc == 0
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    rc = L.mixllm_mixed_linear_fp16_static(C.byref(d), p(x), p(PL.w4), p(PL.w8), p(PL.s4), p(PL.s8), p(PL.z4), p(PL.perm),
                                           p(y2), st)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    return y1, y2


def test_static_scratch_entry_point_matches_the_workspace_entry_point_call_after_call():
    # two kernels (quantizer into the scratch area, then the linear): 300 tokens, then 40 - the second,
    # smaller call finds the first one's codes and scales beyond its own
    _, _, L, x_big, xq_big, xs_big = make_case(300, 1024, 272, 27, seed=81)
    PL = pack_from_oracle(L)
    y1, y2 = call_both(dev(x_big), PL)
    assert torch.equal(y1, y2)
    check_against_oracle(y2.cpu().numpy(), xq_big, xs_big, L, "static, 300 tokens")
    x_small = synth.make_x(40, 1024, seed=82)
    y1, y2 = call_both(dev(x_small), PL)
    assert torch.equal(y1, y2)
    xq, xs = ref.quantize_act(x_small)
    check_against_oracle(y2.cpu().numpy(), xq, xs, L, "static, 40 tokens after 300")
    # and back to a larger one, with scales per (token, group) this time (the scale area moves)
    _, _, Lp, x3, xq3, xs3 = make_case(130, 1024, 272, 27, seed=83, w8_group=128, act_group=128)
    PLp = pack_from_oracle(Lp)
    y1, y2 = call_both(dev(x3), PLp, act_group=128)
    assert torch.equal(y1, y2)
    check_against_oracle(y2.cpu().numpy(), xq3, xs3, Lp, "static, 130 tokens, group-wise scales")


def test_static_scratch_entry_point_single_kernel_shapes_and_decode():
    # one token (the decode kernel quantizes by itself: the scratch area is not touched), and 16
    # tokens of a long row (quantizer + decode kernel through the scratch area)
    for M, K in ((1, 4096), (16, 4096), (4, 14336)):
        _, _, L, x, xq, xs = make_case(M, K, 530, 53, seed=84 + M)
        PL = pack_from_oracle(L)
        y1, y2 = call_both(dev(x), PL)
        assert torch.equal(y1, y2)
        check_against_oracle(y2.cpu().numpy(), xq, xs, L, ("static", M, K))


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_leaves_y_alone():
    # 2048 tokens of K = 4096 fit (8 MiB of codes + the scales); 2049 do not
    for ag in (None, 128):
        need = mx.query_sizes(2048, 4096, 64, 6, act_group=ag)
        assert (need["xq_bytes"] + 255) // 256 * 256 + (need["xscale_bytes"] + 255) // 256 * 256 <= STATIC_BYTES
    _, _, L, _, _, _ = make_case(0, 4096, 64, 6, seed=85)
    PL = pack_from_oracle(L)
    x = torch.zeros((2112, 4096), dtype=torch.float16, device="cuda")
    y = torch.full((2112, 64), 7.0, dtype=torch.float16, device="cuda")
    with pytest.raises(mx.MixllmError) as e:
        mx.linear_fp16_static(x, PL, y)
    assert e.value.status == -3                      # MIXLLM_EWORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())                    # nothing ran
    # the largest shape that fits runs, and agrees with the workspace entry point
    xb = dev(synth.make_x(2048, 4096, seed=86))
    y1, y2 = call_both(xb, PL)
    assert torch.equal(y1, y2)
