"""Measured ceilings of the GPU the benchmark runs on (register-resident int8 MFMA loop,
streaming HBM read, plain copy).  Used by bench.py only."""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(os.path.join(HERE, "libmixllm_probe.so"))
        _lib.mixllm_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _lib.mixllm_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p]
        _lib.mixllm_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
    return _lib


def _time(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) * 1e-3)
    return best


def mfma_int8_tops(blocks_per_cu=2, iters=4000, n_cu=256) -> float:
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    blocks = blocks_per_cu * n_cu
    t = _time(lambda: lib().mixllm_probe_mfma(blocks, iters, out.data_ptr(), st))
    ops = blocks * 4 * iters * 8 * 2.0 * 32 * 32 * 32
    return ops / t / 1e12


def hbm_read_gbs(nbytes=4 << 30, blocks=256 * 16) -> float:
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    t = _time(lambda: lib().mixllm_probe_read(src.data_ptr(), nbytes, blocks, out.data_ptr(), st))
    return nbytes / t / 1e9


def copy(src: torch.Tensor, dst: torch.Tensor, blocks=256 * 16):
    lib().mixllm_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), blocks,
                            torch.cuda.current_stream().cuda_stream)


def kernel_floor_us(reps=200, blocks=256, nbytes=1 << 20) -> float:
    """Time per launch of a kernel that does next to nothing (every block reads 4 KB and writes
    nothing), launched `reps` times back to back on one stream and replayed from a HIP graph:
    the share of a short kernel's duration that no kernel design removes (dispatch, the cache
    write-back and invalidate between dependent launches)."""
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    launch = lambda st: lib().mixllm_probe_read(src.data_ptr(), nbytes, blocks, out.data_ptr(), st)
    launch(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for _ in range(reps):
                launch(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    return _time(g.replay) / reps * 1e6
