"""ctypes binding of libmixllm_hip.so: argument marshalling only.

PyTorch supplies device memory (tensors) and the current HIP stream; every step of the
quantized linear runs in the library's own kernels.  There is no fallback: if the shared
library is missing the import of `lib()` raises."""
import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# the in-tree build; MIXLLM_LIB names another build of the same sources (say one made with other launch
# constants through MIXLLM_EXTRA_FLAGS / MIXLLM_LIB_OUT of the build script, to be measured with bench.py)
LIB_PATH = os.environ.get("MIXLLM_LIB") or os.path.join(HERE, "libmixllm_hip.so")
GROUP = 128

PATH_AUTO, PATH_GENERIC, PATH_DECODE, PATH_PREFILL = 0, 1, 2, 3
PATH_DECODE_STREAM, PATH_DECODE_RESIDENT, PATH_DECODE_SPLIT, PATH_MID = 4, 5, 6, 7
PATH_PREFILL_32, PATH_PREFILL_64, PATH_PREFILL_128 = 8, 9, 10


class MixllmError(RuntimeError):
    """A call into the library returned a status other than MIXLLM_OK (kept in .status)."""

    def __init__(self, message: str, status: int = 0):
        super().__init__(message)
        self.status = status


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("M", "K", "N", "n8", "group", "act_group", "w8_group")]


class _Sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("w8_bytes", "w4_bytes", "scales8_bytes", "scales4_bytes",
                                          "zeros4_bytes", "perm_bytes", "xq_bytes", "xscale_bytes",
                                          "y_bytes", "workspace_bytes", "linear_workspace_bytes")]


_lib = None
_VP = C.c_void_p


def lib():
    """Load the shared library (built in-tree by paper_2412_14590_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MixllmError(f"{LIB_PATH} is missing: build it with `python -m paper_2412_14590_amd.build` "
                              "(there is no CPU or PyTorch fallback)")
        L = C.CDLL(LIB_PATH)
        L.mixllm_status_string.restype = C.c_char_p
        L.mixllm_status_string.argtypes = [C.c_int]
        L.mixllm_abi_version.restype = C.c_int
        L.mixllm_query_sizes.argtypes = [C.POINTER(_Desc), C.POINTER(_Sizes)]
        L.mixllm_build_feature_perm.argtypes = [C.c_int32, C.c_int32, _VP, _VP]
        L.mixllm_quantize_weights.argtypes = [C.POINTER(_Desc)] + [_VP] * 9
        L.mixllm_pack_weights.argtypes = [C.POINTER(_Desc)] + [_VP] * 13
        L.mixllm_unpack_weights.argtypes = [C.POINTER(_Desc)] + [_VP] * 13
        L.mixllm_quantize_activations.argtypes = [C.POINTER(_Desc)] + [_VP] * 4
        L.mixllm_mixed_linear.argtypes = [C.POINTER(_Desc)] + [_VP] * 10 + [C.c_size_t, _VP]
        L.mixllm_mixed_linear_path.argtypes = [C.POINTER(_Desc)] + [_VP] * 10 + [C.c_size_t, C.c_int, _VP]
        L.mixllm_debug_group_partials.argtypes = [C.POINTER(_Desc)] + [_VP] * 6 + [C.c_int, _VP]
        L.mixllm_debug_channel_sums.argtypes = [C.POINTER(_Desc)] + [_VP] * 9 + [C.c_int, _VP]
        L.mixllm_mixed_linear_fp16.argtypes = [C.POINTER(_Desc)] + [_VP] * 9 + [C.c_size_t, _VP]
        L.mixllm_mixed_linear_fp16_static.argtypes = [C.POINTER(_Desc)] + [_VP] * 9
        L.mixllm_channel_salience.argtypes = [C.POINTER(_Desc), _VP, _VP, C.c_float, C.c_int, _VP, _VP]
        L.mixllm_select_salient_workspace.argtypes = [C.c_int32]
        L.mixllm_select_salient_workspace.restype = C.c_size_t
        L.mixllm_select_salient.argtypes = [_VP, _VP, C.c_int32, C.c_int64, _VP, _VP, _VP, C.c_size_t, _VP]
        L.mixllm_debug_check_fast_division.argtypes = [_VP, _VP]
        L.mixllm_debug_check_fast_division.restype = C.c_int
        L.mixllm_debug_work_split.argtypes = [C.POINTER(_Desc), C.c_int, _VP]
        L.mixllm_debug_work_split.restype = C.c_int
        L.mixllm_channel_salience.restype = C.c_int
        L.mixllm_select_salient.restype = C.c_int
        for name in ("mixllm_query_sizes", "mixllm_build_feature_perm", "mixllm_quantize_weights",
                     "mixllm_pack_weights", "mixllm_unpack_weights", "mixllm_quantize_activations",
                     "mixllm_mixed_linear", "mixllm_mixed_linear_path", "mixllm_debug_group_partials",
                     "mixllm_mixed_linear_fp16", "mixllm_mixed_linear_fp16_static", "mixllm_debug_channel_sums"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise MixllmError(f"{what}: {lib().mixllm_status_string(rc).decode()} ({rc})", rc)


def abi_version() -> int:
    return int(lib().mixllm_abi_version())


def _desc(M, K, N, n8, act_group=None, w8_group=None) -> _Desc:
    return _Desc(int(M), int(K), int(N), int(n8), GROUP,
                 int(K if act_group is None else act_group), int(K if w8_group is None else w8_group))


def query_sizes(M, K, N, n8, act_group=None, w8_group=None) -> dict:
    d, s = _desc(M, K, N, n8, act_group, w8_group), _Sizes()
    _check(lib().mixllm_query_sizes(C.byref(d), C.byref(s)), "mixllm_query_sizes")
    return {n: int(getattr(s, n)) for n, _ in _Sizes._fields_}


def build_feature_perm(N: int, salient_idx) -> np.ndarray:
    sal = np.ascontiguousarray(salient_idx, dtype=np.int32)
    perm = np.empty(N, np.int32)
    _check(lib().mixllm_build_feature_perm(N, sal.size, sal.ctypes.data, perm.ctypes.data),
           "mixllm_build_feature_perm")
    return perm


def _ptr(t: Optional[torch.Tensor]):
    if t is None or t.numel() == 0:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


@dataclass
class PackedLayer:
    """Packed, quantized weights of one linear layer, resident in HBM."""
    K: int
    N: int
    n8: int
    w8_group: int
    w8: torch.Tensor        # uint8 buffers in the library's packed layouts
    w4: torch.Tensor
    s8: torch.Tensor
    s4: torch.Tensor
    z4: torch.Tensor
    perm: torch.Tensor      # int32 [N]

    def desc(self, M=0, act_group=None):
        return _desc(M, self.K, self.N, self.n8, act_group, self.w8_group)

    def weight_bytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.w8, self.w4, self.s8, self.s4, self.z4, self.perm))

    def clone(self) -> "PackedLayer":
        return PackedLayer(self.K, self.N, self.n8, self.w8_group, self.w8.clone(), self.w4.clone(),
                           self.s8.clone(), self.s4.clone(), self.z4.clone(), self.perm.clone())


def _alloc_layer(K, N, n8, w8_group, device) -> PackedLayer:
    w8_group = K if w8_group is None else w8_group
    sz = query_sizes(0, K, N, n8, None, w8_group)
    u8 = lambda n: torch.empty(n, dtype=torch.uint8, device=device)
    return PackedLayer(K, N, n8, w8_group, u8(sz["w8_bytes"]), u8(sz["w4_bytes"]), u8(sz["scales8_bytes"]),
                       u8(sz["scales4_bytes"]), u8(sz["zeros4_bytes"]),
                       torch.empty(N, dtype=torch.int32, device=device))


def quantize_weights(W: torch.Tensor, salient_idx, w8_group=None) -> PackedLayer:
    """Offline: fp16 W [N,K] on the device + the list of 8-bit channels -> packed layer.  The list is
    an int32 device tensor (say a slice of select_salient's result: nothing crosses to the host), or a
    host sequence / numpy array, which is checked (range, duplicates) and copied to the device here."""
    assert W.dtype == torch.float16 and W.dim() == 2
    N, K = W.shape
    if isinstance(salient_idx, torch.Tensor):
        sal = salient_idx.to(device=W.device, dtype=torch.int32).contiguous()
    else:
        host = np.ascontiguousarray(salient_idx, dtype=np.int32)
        build_feature_perm(N, host)          # raises on an index out of range or a duplicate
        sal = torch.from_numpy(host).to(W.device)
    L = _alloc_layer(K, N, int(sal.numel()), w8_group, W.device)
    d = L.desc()
    _check(lib().mixllm_quantize_weights(C.byref(d), _ptr(W), _ptr(sal), _ptr(L.w8), _ptr(L.w4), _ptr(L.s8),
                                         _ptr(L.s4), _ptr(L.z4), _ptr(L.perm), _stream()), "mixllm_quantize_weights")
    return L


def pack_weights(q8, s8, q4, s4, z4, perm, K: int, w8_group=None) -> PackedLayer:
    """Canonical device tensors (q8 int8 [n8,K], s8 fp16, q4 uint8 [n4,K], s4 fp16 [n4,K/128],
    z4 uint8 [n4,K/128], perm int32 [N]) -> packed layer."""
    N = perm.numel()
    n8 = 0 if q8 is None else q8.shape[0]
    L = _alloc_layer(K, N, n8, w8_group, perm.device)
    d = L.desc()
    _check(lib().mixllm_pack_weights(C.byref(d), _ptr(q8), _ptr(s8), _ptr(q4), _ptr(s4), _ptr(z4), _ptr(perm),
                                     _ptr(L.w8), _ptr(L.w4), _ptr(L.s8), _ptr(L.s4), _ptr(L.z4), _ptr(L.perm),
                                     _stream()), "mixllm_pack_weights")
    return L


def unpack_weights(L: PackedLayer) -> dict:
    """Packed layer -> canonical device tensors (inverse of pack_weights)."""
    dev = L.perm.device
    n4, ng = L.N - L.n8, L.K // GROUP
    ng8 = L.K // L.w8_group
    out = {
        "q8": torch.empty((L.n8, L.K), dtype=torch.int8, device=dev),
        "s8": torch.empty((L.n8, ng8), dtype=torch.float16, device=dev),
        "q4": torch.empty((n4, L.K), dtype=torch.uint8, device=dev),
        "s4": torch.empty((n4, ng), dtype=torch.float16, device=dev),
        "z4": torch.empty((n4, ng), dtype=torch.uint8, device=dev),
        "perm": torch.empty(L.N, dtype=torch.int32, device=dev),
    }
    d = L.desc()
    _check(lib().mixllm_unpack_weights(C.byref(d), _ptr(L.w8), _ptr(L.w4), _ptr(L.s8), _ptr(L.s4), _ptr(L.z4),
                                       _ptr(L.perm), _ptr(out["q8"]), _ptr(out["s8"]), _ptr(out["q4"]),
                                       _ptr(out["s4"]), _ptr(out["z4"]), _ptr(out["perm"]), _stream()),
           "mixllm_unpack_weights")
    return out


def quantize_activations(x: torch.Tensor, act_group=None, out=None):
    """fp16 x [M,K] -> (xq int8 [M,K], xscale fp16 [M, K/act_group])."""
    assert x.dtype == torch.float16 and x.dim() == 2
    M, K = x.shape
    act_group = K if act_group is None else act_group
    if out is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
        xs = torch.empty((M, K // act_group), dtype=torch.float16, device=x.device)
    else:
        xq, xs = out
    d = _desc(M, K, 1, 0, act_group, None)
    _check(lib().mixllm_quantize_activations(C.byref(d), _ptr(x), _ptr(xq), _ptr(xs), _stream()),
           "mixllm_quantize_activations")
    return xq, xs


def mixed_linear(xq: torch.Tensor, xs: torch.Tensor, L: PackedLayer, path: int = PATH_AUTO, out=None, workspace=None):
    """The quantized linear: (xq, xscale, packed layer) -> y fp16 [M,N] in original channel order.
    `workspace` (optional uint8 tensor, query_sizes()['linear_workspace_bytes']) lets the tiled path split K."""
    M, K = xq.shape
    assert K == L.K and xs.shape[0] == M
    act_group = K // xs.shape[1]
    y = torch.empty((M, L.N), dtype=torch.float16, device=xq.device) if out is None else out
    d = L.desc(M, act_group)
    wb = 0 if workspace is None else workspace.numel()
    _check(lib().mixllm_mixed_linear_path(C.byref(d), _ptr(xq), _ptr(xs), _ptr(L.w4), _ptr(L.w8), _ptr(L.s4),
                                          _ptr(L.s8), _ptr(L.z4), _ptr(L.perm), _ptr(y), _ptr(workspace), wb, path,
                                          _stream()), "mixllm_mixed_linear")
    return y


def debug_group_partials(xq: torch.Tensor, L: PackedLayer, path: int = PATH_AUTO) -> torch.Tensor:
    """Exact int32 partial sums P [M,N,K/128] (original channel order) from the chosen path."""
    M, K = xq.shape
    P = torch.empty((M, L.N, K // GROUP), dtype=torch.int32, device=xq.device)
    d = L.desc(M)
    _check(lib().mixllm_debug_group_partials(C.byref(d), _ptr(xq), _ptr(L.w4), _ptr(L.w8), _ptr(L.z4),
                                             _ptr(L.perm), _ptr(P), path, _stream()),
           "mixllm_debug_group_partials")
    return P


def debug_channel_sums(xq: torch.Tensor, xs: torch.Tensor, L: PackedLayer, path: int = PATH_PREFILL) -> torch.Tensor:
    """S [M,N] int32 = the per-group partial sums added up over the groups, from the kernels the
    linear launches for this shape (generic or tiled path)."""
    M, K = xq.shape
    S = torch.empty((M, L.N), dtype=torch.int32, device=xq.device)
    d = L.desc(M, K // xs.shape[1])
    _check(lib().mixllm_debug_channel_sums(C.byref(d), _ptr(xq), _ptr(xs), _ptr(L.w4), _ptr(L.w8), _ptr(L.s4),
                                           _ptr(L.s8), _ptr(L.z4), _ptr(L.perm), _ptr(S), path, _stream()),
           "mixllm_debug_channel_sums")
    return S


def linear(x: torch.Tensor, L: PackedLayer, act_group=None, path: int = PATH_AUTO) -> torch.Tensor:
    """fp16 x [M,K] -> fp16 y [M,N]: activation quantizer followed by the quantized linear."""
    xq, xs = quantize_activations(x, act_group)
    return mixed_linear(xq, xs, L, path)


def linear_fp16(x: torch.Tensor, L: PackedLayer, act_group=None, out=None, workspace=None) -> torch.Tensor:
    """fp16 x [M,K] -> fp16 y [M,N] through mixllm_mixed_linear_fp16: one kernel for a single token
    where the decode kernel can quantize its own activations, otherwise quantizer + linear with
    xq / xscale in `workspace` (a uint8 tensor of query_sizes()['workspace_bytes'], allocated here
    when not given)."""
    assert x.dtype == torch.float16 and x.dim() == 2
    M, K = x.shape
    assert K == L.K
    d = L.desc(M, act_group)
    y = torch.empty((M, L.N), dtype=torch.float16, device=x.device) if out is None else out
    need = query_sizes(M, K, L.N, L.n8, act_group, L.w8_group)["workspace_bytes"]
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    wb = 0 if workspace is None else workspace.numel()
    _check(lib().mixllm_mixed_linear_fp16(C.byref(d), _ptr(x), _ptr(L.w4), _ptr(L.w8), _ptr(L.s4), _ptr(L.s8),
                                          _ptr(L.z4), _ptr(L.perm), _ptr(y), _ptr(workspace), wb, _stream()),
           "mixllm_mixed_linear_fp16")
    return y


def linear_fp16_static(x: torch.Tensor, L: PackedLayer, out: torch.Tensor, act_group=None) -> torch.Tensor:
    """mixllm_mixed_linear_fp16_static: the same as linear_fp16 with the scratch inside the library; the
    caller brings the output tensor, and nothing is allocated on the way."""
    assert x.dtype == torch.float16 and x.dim() == 2 and out.dtype == torch.float16 and out.shape == (x.shape[0], L.N)
    d = L.desc(x.shape[0], act_group)
    _check(lib().mixllm_mixed_linear_fp16_static(C.byref(d), _ptr(x), _ptr(L.w4), _ptr(L.w8), _ptr(L.s4), _ptr(L.s8),
                                                 _ptr(L.z4), _ptr(L.perm), _ptr(out), _stream()),
           "mixllm_mixed_linear_fp16_static")
    return out


def channel_salience(W: torch.Tensor, G: torch.Tensor, out=None, weight: float = 1.0, accumulate: bool = False) -> torch.Tensor:
    """Salience of every output channel of one layer for one gradient sample (fp16 W, G [N,K] ->
    fp32 [N]); with `out`, weight and accumulate the mean over several samples is built call by call."""
    assert W.dtype == torch.float16 and G.dtype == torch.float16 and W.shape == G.shape and W.dim() == 2
    N, K = W.shape
    W, G = W.contiguous(), G.contiguous()
    sal = torch.empty(N, dtype=torch.float32, device=W.device) if out is None else out
    assert sal.dtype == torch.float32 and sal.numel() == N
    d = _desc(0, K, N, 0, None, None)
    _check(lib().mixllm_channel_salience(C.byref(d), _ptr(W), _ptr(G), C.c_float(weight), int(bool(accumulate)),
                                         _ptr(sal), _stream()), "mixllm_channel_salience")
    return sal


def select_salient(saliences, T: int):
    """The T most salient channels over all layers: `saliences` is a list of fp32 device tensors (one
    per layer); returns one ascending int32 index tensor per layer (on the device) - the salient_idx
    of quantize_weights for that layer."""
    sizes = [int(s.numel()) for s in saliences]
    flat = torch.cat([s.reshape(-1).to(torch.float32) for s in saliences]) if len(saliences) > 1 else \
        saliences[0].reshape(-1).to(torch.float32).contiguous()
    L = len(sizes)
    offsets = (C.c_int64 * (L + 1))(*np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64).tolist())
    selected = torch.empty(max(int(T), 1), dtype=torch.int32, device=flat.device)
    counts = torch.empty(L, dtype=torch.int32, device=flat.device)
    need = int(lib().mixllm_select_salient_workspace(L))
    ws = torch.empty(need, dtype=torch.uint8, device=flat.device)
    _check(lib().mixllm_select_salient(_ptr(flat), C.cast(offsets, _VP), L, int(T), _ptr(selected), _ptr(counts),
                                       _ptr(ws), need, _stream()), "mixllm_select_salient")
    cnt = counts.cpu().tolist()
    out, o = [], 0
    for c in cnt:
        out.append(selected[o:o + c])
        o += c
    return out
