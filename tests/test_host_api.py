"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments before touching the device, and its size accounting and
feature permutation are right."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2412_14590_amd as mx
from paper_2412_14590_amd import binding
from oracle import ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "mixllm.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mixllm_[a-z0-9_]+)\s*\(", src)))


def test_library_loads_and_exports_every_declared_symbol():
    L = mx.lib()
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), n
    assert mx.abi_version() >= 2


def test_query_sizes_matches_the_layout_arithmetic_and_paper_footprints():
    K, N, n8 = 4096, 4096, 410
    s = mx.query_sizes(3, K, N, n8)
    n4, n8p, n4p, ngp = N - n8, 416, 3696, 32
    assert n4p >= n4 and n8p >= n8
    assert s["w8_bytes"] == n8p * K and s["w4_bytes"] == n4p * K // 2
    assert s["scales4_bytes"] == n4p * ngp * 2 and s["zeros4_bytes"] == n4p * ngp // 2
    assert s["scales8_bytes"] == n8p * 2 and s["perm_bytes"] == 4 * N
    assert s["xq_bytes"] == 3 * K and s["xscale_bytes"] == 6 and s["y_bytes"] == 3 * N * 2
    assert s["workspace_bytes"] == 3 * K + 256      # xq, then xscale, each rounded up to 256 bytes
    # per stored weight the 4-bit part costs 0.5 + 2.5/G bytes and the group-wise 8-bit part
    # 1 + 2/G bytes (Sec. 3.5, memory traffic)
    assert (s["w4_bytes"] + s["scales4_bytes"] + s["zeros4_bytes"]) / (n4p * K) == 0.5 + 2.5 / 128
    sp = mx.query_sizes(3, K, N, n8, act_group=128, w8_group=128)
    assert (sp["w8_bytes"] + sp["scales8_bytes"]) / (n8p * K) == 1 + 2 / 128
    assert sp["xscale_bytes"] == 3 * (K // 128) * 2
    # metadata rows are padded to a multiple of 8 groups
    s2 = mx.query_sizes(0, 384, 32, 0)
    assert s2["scales4_bytes"] == 32 * 8 * 2 and s2["zeros4_bytes"] == 32 * 4


@pytest.mark.parametrize("kw,code", [
    (dict(M=1, K=4000, N=64, n8=0), -2),            # K not a multiple of the group
    (dict(M=1, K=256, N=64, n8=65), -1),            # n8 > N
    (dict(M=-1, K=256, N=64, n8=0), -1),
    (dict(M=1, K=256, N=64, n8=0, act_group=64), -2),
    (dict(M=1, K=256, N=64, n8=0, w8_group=256 * 2), -2),
    (dict(M=1, K=131072 + 128, N=64, n8=0), -2),    # beyond the K an int32 sum over all of K is safe for
])
def test_bad_descriptors_are_rejected(kw, code):
    d = binding._desc(**kw)
    s = binding._Sizes()
    assert mx.lib().mixllm_query_sizes(C.byref(d), C.byref(s)) == code


def test_null_and_misaligned_pointers_are_rejected_before_any_launch():
    L = mx.lib()
    d = binding._desc(4, 256, 64, 8)
    # null everything
    assert L.mixllm_mixed_linear(C.byref(d), None, None, None, None, None, None, None, None, None, None, 0, None) == -1
    assert L.mixllm_quantize_activations(C.byref(d), None, None, None, None) == -1
    assert L.mixllm_debug_group_partials(C.byref(d), None, None, None, None, None, None, 0, None) == -1
    assert L.mixllm_debug_channel_sums(C.byref(d), None, None, None, None, None, None, None, None, None, 0, None) == -1
    # misaligned (fake, never dereferenced: validation fails first)
    fake = 0x1000
    # the list of 8-bit channels is a device pointer: null with n8 > 0, or not 4-byte aligned
    assert L.mixllm_quantize_weights(C.byref(d), fake, None, fake, fake, fake, fake, fake, fake, None) == -1
    assert L.mixllm_quantize_weights(C.byref(d), fake, fake + 2, fake, fake, fake, fake, fake, fake, None) == -1
    # the integer sums over the groups come from the generic and the tiled kernel only: refused, nothing launched
    assert L.mixllm_debug_channel_sums(C.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, fake, 2, None) == -2
    # the 128 x 128 block shape is not built for activation scales per (token, group)
    dg = binding._desc(300, 256, 64, 8, act_group=128)
    assert L.mixllm_mixed_linear_path(C.byref(dg), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, 0, 10, None) == -2
    assert L.mixllm_quantize_activations(C.byref(d), fake + 2, fake, fake, None) == -1
    # bad path value
    assert L.mixllm_mixed_linear_path(C.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, 0, 11, None) == -1
    # the decode path refuses M > 16; M = 0 is a no-op that succeeds without a device
    d0 = binding._desc(0, 256, 64, 8)
    assert L.mixllm_mixed_linear(C.byref(d0), None, None, None, None, None, None, None, None, None, None, 0, None) == 0
    assert L.mixllm_status_string(-2).decode().startswith("unsupported")


def test_precision_search_calls_validate_on_the_host():
    L = mx.lib()
    d = binding._desc(0, 256, 8, 0)
    buf = (C.c_uint8 * 8192)()
    addr = (C.addressof(buf) + 15) & ~15                       # 16-byte aligned host address: never dereferenced
    vp = C.c_void_p
    # salience: null / misaligned pointers, K not a multiple of the group
    assert L.mixllm_channel_salience(C.byref(d), None, vp(addr), C.c_float(1), 0, vp(addr), None) == -1
    assert L.mixllm_channel_salience(C.byref(d), vp(addr + 2), vp(addr), C.c_float(1), 0, vp(addr), None) == -1
    bad = binding._desc(0, 200, 8, 0)
    assert L.mixllm_channel_salience(C.byref(bad), vp(addr), vp(addr), C.c_float(1), 0, vp(addr), None) == -2
    empty = binding._desc(0, 256, 0, 0)
    assert L.mixllm_channel_salience(C.byref(empty), None, None, C.c_float(1), 0, None, None) == 0
    # selection: layer list, T, workspace
    off = (C.c_int64 * 3)(0, 5, 9)
    need = L.mixllm_select_salient_workspace(2)
    assert need > 0 and L.mixllm_select_salient_workspace(0) == 0
    args = lambda o, nl, T, ws, wb: L.mixllm_select_salient(vp(addr), C.cast(o, vp), nl, C.c_int64(T), vp(addr), vp(addr),
                                                            ws, C.c_size_t(wb), None)
    assert args(off, 0, 1, vp(addr), need) == -1                 # no layers
    assert args(off, 2, 10, vp(addr), need) == -1                # T beyond the number of channels
    assert args(off, 2, -1, vp(addr), need) == -1
    assert args((C.c_int64 * 3)(0, 5, 4), 2, 1, vp(addr), need) == -1      # offsets not ascending
    assert args((C.c_int64 * 3)(1, 5, 9), 2, 1, vp(addr), need) == -1      # offsets do not start at 0
    assert args(off, 2, 3, None, need) == -1
    assert args(off, 2, 3, vp(addr), need - 1) == -3             # MIXLLM_EWORKSPACE


def test_feature_perm_matches_oracle_and_rejects_bad_lists():
    rng = np.random.default_rng(0)
    for N, n8 in ((8, 3), (100, 0), (100, 100), (4096, 410)):
        sal = rng.choice(N, n8, replace=False).astype(np.int32)
        got = mx.build_feature_perm(N, sal)
        assert np.array_equal(got, ref.feature_perm(N, sal))
        assert np.array_equal(np.sort(got), np.arange(N))
        assert np.all(np.diff(got[:n8]) > 0) and np.all(np.diff(got[n8:]) > 0)
    with pytest.raises(mx.MixllmError):
        mx.build_feature_perm(4, [1, 1])
    with pytest.raises(mx.MixllmError):
        mx.build_feature_perm(4, [7])


def test_product_path_does_not_import_the_oracle():
    # the library binding and the input generator must stand alone
    for f in ("binding.py", "synth.py", "__init__.py", "build.py"):
        src = open(os.path.join(ROOT, "paper_2412_14590_amd", f)).read()
        assert "oracle" not in src.replace("oracle-side", ""), f


def test_build_scan_flags_a_register_used_between_its_hand_issued_load_and_the_wait():
    from paper_2412_14590_amd import build
    ok = """
	;;#ASMSTART
	global_load_dwordx2 v[104:105], v119, s[98:99]
	;;#ASMEND
	v_add_u32_e32 v1, v2, v3
	;;#ASMSTART
	s_waitcnt vmcnt(6)
	;;#ASMEND
	v_lshrrev_b32_e32 v128, 16, v104
"""
    build.check_hand_issued_loads(ok, "ok")
    bad = ok.replace("v_add_u32_e32 v1, v2, v3", "v_lshrrev_b32_e32 v128, 16, v104")
    with pytest.raises(RuntimeError):
        build.check_hand_issued_loads(bad, "bad")
    # a branch ends the judged region (the two arms of a conditional load are not one sequence),
    # and a direct-to-LDS load has no destination register
    branchy = ok.replace("v_add_u32_e32 v1, v2, v3", "s_branch .LBB1_2\n.LBB1_1:\n\tv_mov_b32_e32 v104, 0")
    build.check_hand_issued_loads(branchy, "branchy")
    lds = ok.replace("global_load_dwordx2 v[104:105], v119, s[98:99]", "global_load_lds_dwordx4 v104, s[98:99]")
    build.check_hand_issued_loads(lds.replace("v_add_u32_e32 v1, v2, v3", "v_mov_b32_e32 v104, 0"), "lds")
