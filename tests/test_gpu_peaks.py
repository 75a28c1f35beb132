"""GPU: the bench-only micro-benchmarks of libffpeaks.so do what bench.py assumes: the streaming copy copies,
the product loops run and report the number of operations they perform."""
import ctypes as C
import os

import pytest
import torch

pytestmark = pytest.mark.gpu

LIB = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2301_08739_amd", "libffpeaks.so")


def test_stream_copy_and_mfma_loops():
    lib = C.CDLL(LIB)
    lib.ffpeak_stream_copy.restype, lib.ffpeak_stream_copy.argtypes = C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.ffpeak_mfma_bf16.restype = C.c_int
    lib.ffpeak_mfma_bf16.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for nbytes in (16, 4096 * 16 + 16, 3 << 20):
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda")
        dst = torch.zeros(nbytes + 16, dtype=torch.uint8, device="cuda")
        assert lib.ffpeak_stream_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(dst[:nbytes], src) and int(dst[nbytes:].sum().item()) == 0
    assert lib.ffpeak_stream_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), 24, stream) == -1   # not a multiple of 16
    for shape, per in ((0, 2.0 * 16 * 16 * 32), (1, 2.0 * 32 * 32 * 16)):
        blocks, iters = 8, 10
        sink = torch.zeros(blocks * 256, dtype=torch.float32, device="cuda")
        ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
        flops = C.c_double(0.0)
        assert lib.ffpeak_mfma_bf16(C.c_void_p(sink.data_ptr()), blocks, iters, shape, C.c_void_p(ticks.data_ptr()),
                                    C.byref(flops), stream) == 0
        torch.cuda.synchronize()
        assert flops.value == blocks * 4 * iters * 8 * per
        assert int(ticks[0].item()) > 0 and int(ticks[1].item()) >= 0
        assert torch.isfinite(sink).all()
    assert lib.ffpeak_mfma_bf16(C.c_void_p(sink.data_ptr()), 1, 1, 2, None, None, stream) == -1
