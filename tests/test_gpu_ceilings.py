"""The benchmark's ceiling probes compute what their FLOP and byte accounting says (GPU)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
P, I, Z = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t


@pytest.fixture(scope="module")
def lib():
    from paper_2505_11432_amd import build
    build.ensure_built()
    lib = ctypes.CDLL(build.CEILINGS_LIB_PATH)
    lib.moe_ceiling_mfma_loop.argtypes = [I, P, I, I, P, P]
    lib.moe_ceiling_mfma_lds_loop.argtypes = [P, I, I, P, P]
    lib.moe_ceiling_mfma_lds_dma_loop.argtypes = [P, P, Z, I, I, I, P, P]
    lib.moe_ceiling_copy.argtypes = [P, P, Z, P]
    lib.moe_ceiling_read.argtypes = [P, Z, P, P]
    return lib


def test_mfma_loop_counts_every_mfma(lib):
    """All-ones bf16 operands: every MFMA adds K = 16 to each accumulator element, so a lane's sum over its 8
    accumulators of 16 elements after `iters` MFMAs per accumulator is 8 * 16 * iters * 16 (exact in fp32 here)."""
    stream = torch.cuda.current_stream().cuda_stream
    ops = torch.zeros((2 * 6 * 64, 16), dtype=torch.bfloat16)
    ops[:, :8] = 1.0
    ops = ops.cuda()
    wgs, iters = 3, 64
    sink = torch.zeros((wgs * 512,), device="cuda")
    assert lib.moe_ceiling_mfma_loop(0, ops.data_ptr(), iters, wgs, sink.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    assert torch.all(sink == 8 * 16 * iters * 16)
    # e4m3: code 0x38 is 1.0; K = 64
    ops8 = torch.full((2 * 6 * 64, 32), 0x38, dtype=torch.uint8, device="cuda")
    assert lib.moe_ceiling_mfma_loop(1, ops8.data_ptr(), iters, wgs, sink.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    assert torch.all(sink == 8 * 16 * iters * 64)
    # LDS-fed loop on an all-ones image: the same count as the register loop
    image = torch.ones((65536,), dtype=torch.bfloat16, device="cuda")
    assert lib.moe_ceiling_mfma_lds_loop(image.data_ptr(), iters, wgs, sink.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    assert torch.all(sink == 8 * 16 * iters * 16)
    # the same with the direct-to-LDS loads beside it, in every combination of loads / waits / barriers: the loads
    # bring in ones as well, so whatever a fragment read sees, the count stays
    src = torch.ones((3 * 32768,), dtype=torch.bfloat16, device="cuda")                       # three 64 KiB slices
    for flags in range(8):
        sink.zero_()
        assert lib.moe_ceiling_mfma_lds_dma_loop(image.data_ptr(), src.data_ptr(), src.numel() * 2, iters, flags, wgs,
                                                 sink.data_ptr(), stream) == 0
        torch.cuda.synchronize()
        assert torch.all(sink == 8 * 16 * iters * 16), flags


def test_copy_kernel_copies(lib):
    stream = torch.cuda.current_stream().cuda_stream
    n = (1 << 22) + 16 * 7
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    assert lib.moe_ceiling_copy(src.data_ptr(), dst.data_ptr(), n, stream) == 0
    sink = torch.zeros((4096,), device="cuda")
    assert lib.moe_ceiling_read(src.data_ptr(), n, sink.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
