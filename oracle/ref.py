"""ctypes front end of the C oracle (canonical layouts, numpy arrays in and out).

Test infrastructure only.  fp16 tensors are numpy float16 arrays; they cross into C
as their uint16 bit patterns.  The only arithmetic done here in numpy is row
gathering (splitting W into its 8-bit and 4-bit rows)."""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.oracle_feature_perm.restype = C.c_int
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _i64(v):
    return C.c_int64(int(v))


def _h(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a.view(np.uint16)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def half_to_double(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, np.float64)
    lib().oracle_half_to_double(_p(bits), _i64(bits.size), _p(out))
    return out


def double_to_half(v: np.ndarray) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, np.uint16)
    lib().oracle_double_to_half(_p(v), _i64(v.size), _p(out))
    return out


def feature_perm(N: int, salient_idx) -> np.ndarray:
    sal = np.ascontiguousarray(salient_idx, dtype=np.int32)
    perm = np.empty(N, np.int32)
    rc = lib().oracle_feature_perm(_i64(N), _i64(sal.size), _p(sal), _p(perm))
    if rc != 0:
        raise ValueError("salient_idx must hold distinct indices in [0,N)")
    return perm


def quantize_act(x: np.ndarray, act_group: int = None):
    xb = _h(x)
    M, K = xb.shape
    act_group = K if act_group is None else int(act_group)
    assert K % act_group == 0
    xq = np.empty((M, K), np.int8)
    xs = np.empty((M, K // act_group), np.uint16)
    lib().oracle_quantize_act(_p(xb), _i64(M), _i64(K), _i64(act_group), _p(xq), _p(xs))
    return xq, xs.view(np.float16)


def quantize_w8(W: np.ndarray, w8_group: int = None):
    wb = _h(W)
    R, K = wb.shape
    w8_group = K if w8_group is None else int(w8_group)
    assert K % w8_group == 0
    q = np.empty((R, K), np.int8)
    s = np.empty((R, K // w8_group), np.uint16)
    lib().oracle_quantize_w8(_p(wb), _i64(R), _i64(K), _i64(w8_group), _p(q), _p(s))
    return q, s.view(np.float16)


def quantize_w4(W: np.ndarray, G: int = 128):
    wb = _h(W)
    R, K = wb.shape
    assert K % G == 0
    q = np.empty((R, K), np.uint8)
    s = np.empty((R, K // G), np.uint16)
    z = np.empty((R, K // G), np.uint8)
    lib().oracle_quantize_w4(_p(wb), _i64(R), _i64(K), _i64(G), _p(q), _p(s), _p(z))
    return q, s.view(np.float16), z


class QuantizedLayer:
    """Canonical quantized weights of one layer (what the offline step produces)."""

    def __init__(self, N, K, G, w8_group, perm, q8, s8, q4, s4, z4):
        self.N, self.K, self.G, self.w8_group = N, K, G, w8_group
        self.perm, self.q8, self.s8, self.q4, self.s4, self.z4 = perm, q8, s8, q4, s4, z4
        self.n8 = q8.shape[0]
        self.n4 = q4.shape[0]


def quantize_weights(W: np.ndarray, salient_idx, G: int = 128, w8_group: int = None) -> QuantizedLayer:
    """Split W's rows into the 8-bit set (salient_idx) and the 4-bit rest, quantize both."""
    W = np.ascontiguousarray(W)
    N, K = W.shape
    w8_group = K if w8_group is None else int(w8_group)
    perm = feature_perm(N, salient_idx)
    n8 = len(np.atleast_1d(np.asarray(salient_idx, dtype=np.int32)))
    q8, s8 = quantize_w8(W[perm[:n8]], w8_group)
    q4, s4, z4 = quantize_w4(W[perm[n8:]], G)
    return QuantizedLayer(N, K, G, w8_group, perm, q8, s8, q4, s4, z4)


def group_partials(xq: np.ndarray, L: QuantizedLayer) -> np.ndarray:
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    M, K = xq.shape
    assert K == L.K
    P = np.empty((M, L.N, K // L.G), np.int32)
    lib().oracle_group_partials(_p(xq), _p(L.q8), _p(L.q4), _p(L.z4), _p(L.perm),
                                _i64(M), _i64(K), _i64(L.N), _i64(L.n8), _i64(L.G), _p(P))
    return P


def mixed_linear(xq: np.ndarray, xs: np.ndarray, L: QuantizedLayer, want_f64: bool = False):
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    xsb = _h(xs)
    M, K = xq.shape
    assert K == L.K and xsb.shape[0] == M
    act_group = K // xsb.shape[1]
    y = np.empty((M, L.N), np.uint16)
    y64 = np.empty((M, L.N), np.float64) if want_f64 else None
    lib().oracle_mixed_linear(_p(xq), _p(xsb), _i64(act_group),
                              _p(L.q8), _p(_h(L.s8)), _i64(L.w8_group),
                              _p(L.q4), _p(_h(L.s4)), _p(L.z4), _p(L.perm),
                              _i64(M), _i64(K), _i64(L.N), _i64(L.n8), _i64(L.G),
                              _p(y), _p(y64) if want_f64 else None)
    y = y.view(np.float16)
    return (y, y64) if want_f64 else y


def channel_salience(W: np.ndarray, grads, G: int = 128):
    """Salience of every output channel of one layer (Sec. 3.2, Eq. 4): the mean over the
    gradient samples in `grads` (a list of fp16 [N, K] arrays, or one array) of
    |S1 + S1^2 / 2| with S1 = sum_k g (Qdq(W) - W).  Returns (salience float64 [N],
    S1 of the last sample float64 [N])."""
    wb = _h(W)
    N, K = wb.shape
    grads = [grads] if isinstance(grads, np.ndarray) else list(grads)
    sal = np.zeros(N, np.float64)
    s1 = np.zeros(N, np.float64)
    for i, g in enumerate(grads):
        gb = _h(g)
        assert gb.shape == (N, K)
        lib().oracle_channel_salience(_p(wb), _p(gb), _i64(N), _i64(K), _i64(G), C.c_double(1.0 / len(grads)),
                                      C.c_int(1 if i else 0), _p(sal), _p(s1))
    return sal, s1


def select_salient(saliences, T: int):
    """Alg. 1, last two lines: `saliences` is a list of float32 arrays, one per layer; the T
    channels with the largest salience over all layers are chosen (equal values: the earlier
    channel first).  Returns one ascending int32 index array per layer."""
    flat = np.ascontiguousarray(np.concatenate([np.asarray(s, np.float32).ravel() for s in saliences]) if saliences
                                else np.zeros(0, np.float32))
    chosen = np.zeros(flat.size, np.uint8)
    lib().oracle_select_salient.restype = C.c_int
    rc = lib().oracle_select_salient(_p(flat), _i64(flat.size), _i64(T), _p(chosen))
    if rc != 0:
        raise ValueError("T must lie in [0, total number of channels]")
    out, o = [], 0
    for s in saliences:
        n = np.asarray(s).size
        out.append(np.nonzero(chosen[o:o + n])[0].astype(np.int32))
        o += n
    return out
