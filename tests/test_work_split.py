"""Host-side check of how the weight-streaming kernels split a layer over blocks and waves.

The library reports its launch plan through mixllm_debug_work_split (no GPU needed); the lane ->
(tile, channel) formulas of the kernels are restated here in plain Python, and for a range of
shapes every channel row of both precisions must be owned by exactly one valid lane, every tile
index a lane addresses must exist (clamped lanes included), and a block's LDS cell area must
cover its virtual tiles.  A mismatch between the host plan and the device formulas would
otherwise only show as a memory fault on the GPU."""
import ctypes as C

import pytest

import paper_2412_14590_amd as mx
from paper_2412_14590_amd import binding

NW = 8


def plan(path, M, K, N, n8):
    out = (C.c_int32 * 16)()
    d = binding._desc(M, K, N, n8)
    rc = mx.lib().mixllm_debug_work_split(C.byref(d), path, C.cast(out, C.c_void_p))
    return rc, list(out)


def tiles(N, n8):
    return (n8 + 15) // 16, (N - n8 + 15) // 16


def check_decode_split_part(ntiles, nblk, tcap):
    """linear_decode_split.hip: whole tiles round robin, the rest in quarter tiles."""
    if ntiles == 0:
        assert nblk == 0
        return
    assert 1 <= nblk <= 4 * ntiles
    rounds = ntiles // nblk
    left_base = 4 * rounds * nblk
    left = 4 * ntiles - left_base
    seen = set()
    for b in range(nblk):
        L_lo, L_hi = left * b // nblk, left * (b + 1) // nblk
        assert L_hi - L_lo <= 4
        nvt = rounds + (1 if L_hi > L_lo else 0)
        assert 1 <= nvt <= tcap
        for vt in range(nvt):
            full = vt < rounds
            u0 = 4 * (b + nblk * vt) if full else left_base + L_lo
            cnt = 4 if full else L_hi - L_lo
            base_tile = u0 >> 2
            for c in range(16):
                uc = u0 + min(c >> 2, cnt - 1)
                row = (uc >> 2) * 16 + 4 * (uc & 3) + (c & 3)
                rel = row - base_tile * 16
                assert 0 <= rel < 32 and (uc >> 2) < ntiles and base_tile + (rel >> 4) < ntiles
                if (c >> 2) < cnt:
                    assert row not in seen
                    seen.add(row)
    assert len(seen) == 16 * ntiles


def check_mid_part(ntiles, nblk, qv):
    """linear_mid.hip: contiguous shares of quarter tiles, qv quarters per virtual tile."""
    if ntiles == 0:
        assert nblk == 0
        return
    assert 1 <= nblk <= 4 * ntiles and qv in (1, 2, 4)
    nunits = 4 * ntiles
    seen = set()
    for b in range(nblk):
        Q_lo, Q_hi = nunits * b // nblk, nunits * (b + 1) // nblk
        nvt = (Q_hi - Q_lo + qv - 1) // qv
        assert nvt >= 1
        for vt_raw in range((nvt + NW - 1) // NW * NW):        # idle waves of the last round clamp to the last tile
            has = vt_raw < nvt
            u0 = Q_lo + qv * min(vt_raw, nvt - 1)
            cnt = min(qv, Q_hi - u0)
            assert cnt >= 1
            base_tile = u0 >> 2
            for c in range(16):
                uc = u0 + min(c >> 2, cnt - 1)
                row = (uc >> 2) * 16 + 4 * (uc & 3) + (c & 3)
                rel = row - base_tile * 16
                assert 0 <= rel < 32 and (uc >> 2) < ntiles and base_tile + (rel >> 4) < ntiles
                if has and (c >> 2) < cnt:
                    assert row not in seen
                    seen.add(row)
    assert len(seen) == 16 * ntiles


def check_windowed_chunk_lists(nvt, nquads, nwin, wq):
    """linear_decode_split.hip, activations staged window by window: the eight waves' chunk lists, located the
    way the kernel does it (window by subtraction, virtual tile by multiplication with ceil(2^32 / columns)),
    visit every (virtual tile, chunk column) once, every chunk inside the window its wave is in."""
    wql = nquads - (nwin - 1) * wq
    assert 1 <= wql <= wq
    magic = {c: ((1 << 32) + c - 1) // c for c in (wq, wql)}
    seen = set()
    for wave in range(8):
        share = lambda chunks: (chunks - wave + 7) // 8 if wave < chunks else 0
        cnt_w, cnt_l = share(nvt * wq), share(nvt * wql)
        for i in range((nwin - 1) * cnt_w + cnt_l):
            win, ii = 0, i
            while win < nwin - 1 and ii >= cnt_w:
                ii -= cnt_w
                win += 1
            j = wave + 8 * ii
            cols = wql if win == nwin - 1 else wq
            vt = j if cols == 1 else (j * magic[cols]) >> 32
            q = win * wq + (j - vt * cols)
            assert vt == j // cols and 0 <= vt < nvt and win * wq <= q < min(nquads, (win + 1) * wq)
            assert (vt, q) not in seen
            seen.add((vt, q))
    assert len(seen) == nvt * nquads


SHAPES = [(28672, 8192, 819), (4096, 4096, 410), (4096, 6144, 614), (4096, 28672, 2867), (14336, 4096, 410), (8192, 10240, 1024),
          (8192, 57344, 5734), (256, 7, 2), (384, 70, 70), (1024, 530, 0), (640, 50, 5), (128, 16, 16), (512, 4097, 1),
          (4096, 14336, 10178), (2048, 2070, 207), (128, 33, 3)]


@pytest.mark.parametrize("K,N,n8", SHAPES)
def test_decode_split_plan_covers_every_channel_once(K, N, n8):
    t8, t4 = tiles(N, n8)
    for M in (1, 4, 5, 9, 12, 16):
        rc, p = plan(mx.PATH_DECODE_SPLIT, M, K, N, n8)
        if M * K > 131072 and M <= 4:
            assert rc == -2            # the activations do not fit the LDS stage: not covered, not an error path
            continue
        if rc == -2:                   # fits, but only with several blocks per CU each staging > 64 KB
            assert 65536 < M * K <= 131072
            continue
        assert rc == 0, (M, K, N, n8)
        nblk8, nblk4, tcap, lds, nwin, wq = p[:6]
        assert lds <= 160 * 1024
        nquads = (K // 128 + 3) // 4
        if M * K > 131072:             # staged window by window in two buffers: one block per CU, whole pieces of 1 KB per row
            assert nblk8 + nblk4 <= 256 and wq in (16, 12, 8, 4, 2) and nwin == -(-nquads // wq) >= 2
            assert lds >= 2 * M * (wq * 512 + 16) + tcap * 8 * 4 * 256
            for nvt in range(1, tcap + 1):
                check_windowed_chunk_lists(nvt, nquads, nwin, wq)
        else:
            assert (nwin, wq) == (1, nquads)
        check_decode_split_part(t8, nblk8, tcap)
        check_decode_split_part(t4, nblk4, tcap)


@pytest.mark.parametrize("K,N,n8", SHAPES)
def test_mid_plan_covers_every_channel_once(K, N, n8):
    t8, t4 = tiles(N, n8)
    for M in (17, 33, 64):
        rc, p = plan(mx.PATH_MID, M, K, N, n8)
        assert rc == 0, (M, K, N, n8)
        nblk8, nblk4, qv8, qv4, lds = p[:5]
        assert lds <= 160 * 1024
        check_mid_part(t8, nblk8, qv8)
        check_mid_part(t4, nblk4, qv4)
    assert plan(mx.PATH_MID, 65, K, N, n8)[0] == -2


def check_prefill_grid(M, K, N, n8, act_group=None):
    """linear_prefill.hip: blocks are dealt round robin to 8 XCDs; per XCD a contiguous range of 4-bit
    logical ids, then of 8-bit ids; ids walk the tile grid in bands of `band` token tiles (channel
    tile outer, token tile inner).  Restated here: every (token tile, channel tile) of either part
    must be taken by exactly one block, and no block may name a tile outside the grid."""
    out = (C.c_int32 * 16)()
    d = binding._desc(M, K, N, n8, act_group, None)
    rc = mx.lib().mixllm_debug_work_split(C.byref(d), mx.PATH_PREFILL, C.cast(out, C.c_void_p))
    assert rc == 0
    BM, BN, nbm, nb8, nb4, blocks, band, lds, kparts, groups_per_part, BM8, nbm8, band8 = list(out)[:13]
    t8, t4 = tiles(N, n8)
    # K split over blocks (when the caller brings the scratch): whole groups of 4 quantization groups per
    # part, the parts cover K exactly, no part is empty; only layers with a long K are split, into at
    # most about two blocks per CU in all, and the parts' sums stay under 16 MB
    ng = K // 128
    assert 1 <= kparts <= 8 and groups_per_part % 4 == 0
    assert (kparts - 1) * groups_per_part < ng <= kparts * groups_per_part
    if kparts > 1:
        ntile = nbm * nb4 + nbm8 * nb8
        assert ng >= 64 and groups_per_part >= 8 and ntile * kparts <= 2 * 256 + ntile // 2
        assert kparts * M * (t8 + t4) * 16 * 4 <= 16 << 20
    assert BM <= 32 or M > 32
    assert BM in (32, 64, 128) and BN == 128
    assert nbm == -(-M // BM) and nb8 == -(-t8 * 16 // BN) and nb4 == -(-t4 * 16 // BN)
    # in a launch of 128 x 128 blocks at most four rounds of blocks long (two blocks per CU at a time) the
    # 8-bit part runs in tiles half as tall, banded over the same token rows
    assert BM8 == (64 if BM == 128 and nbm * (nb8 + nb4) <= 8 * 256 else BM)
    assert nbm8 == -(-M // BM8) and 1 <= band8 <= min(4 * BM // BM8, nbm8)
    assert 1 <= band <= min(4, nbm) and lds <= 80 * 1024 and blocks % 8 == 0
    # the shape rule: the largest block tile whose grid still has about one block per CU or more
    nbn = nb8 + nb4
    if act_group == 128:
        assert BM <= 64
    per4, per8 = -(-nbm * nb4 // 8), -(-nbm8 * nb8 // 8)
    assert blocks == 8 * (per4 + per8)
    seen = set()
    for b in range(blocks):
        xcd, i = b & 7, b >> 3
        part8 = i >= per4
        nb, nbm_p, band_p = (nb8, nbm8, band8) if part8 else (nb4, nbm, band)
        L = xcd * per8 + (i - per4) if part8 else xcd * per4 + i
        if L >= nbm_p * nb:
            continue
        bd = L // (band_p * nb)
        w = min(band_p, nbm_p - bd * band_p)
        r = L - bd * band_p * nb
        bn, bm = r // w, bd * band_p + r % w
        assert 0 <= bm < nbm_p and 0 <= bn < nb, (b, bm, bn)
        key = (part8, bm, bn)
        assert key not in seen
        seen.add(key)
    assert len(seen) == nbm * nb4 + nbm8 * nb8
    return BM


@pytest.mark.parametrize("K,N,n8", SHAPES)
def test_prefill_grid_covers_every_tile_once(K, N, n8):
    sizes = set()
    for M in (1, 31, 64, 65, 128, 200, 256, 512, 1000, 2048, 8192):
        sizes.add(check_prefill_grid(M, K, N, n8))
        check_prefill_grid(M, K, N, n8, act_group=128)
    assert sizes <= {32, 64, 128}


def test_prefill_block_tile_follows_the_grid_size():
    # Llama-3-8B shapes on a 256-CU part (the fallback count without a GPU is also 256): small grids take
    # small block tiles, the large prefill batches the 128 x 128 tile
    assert check_prefill_grid(64, 4096, 4096, 410) == 32
    assert check_prefill_grid(256, 4096, 4096, 410) == 32
    assert check_prefill_grid(512, 4096, 4096, 410) == 64
    assert check_prefill_grid(2048, 4096, 4096, 410) == 128
    assert check_prefill_grid(128, 4096, 28672, 2867) == 128
    assert check_prefill_grid(2048, 4096, 28672, 2867, act_group=128) == 64
