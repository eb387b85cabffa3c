"""GPU test of nvfp4_gemm_noalloc, the entry point for callers that cannot allocate: it must give
the bytes of nvfp4_gemm_ws (same kernels, the partial sums in the library's static scratch array
instead of a caller-owned workspace), on two calls in a row, the second with a smaller input, and
those bytes must meet the oracle.  Called through the C ABI (ctypes), outputs preallocated."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import _lib

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_scalar, dev_u8, host_bits

pytestmark = pytest.mark.gpu


def _case(M, N, K, seed):
    rng = np.random.default_rng([M, N, K, seed])
    ac = rng.integers(0, 256, size=(M, K // 2)).astype(np.uint8)
    asc = rng.integers(0x28, 0x48, size=(M, K // 16)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    bsc = rng.integers(0x28, 0x48, size=(N, K // 16)).astype(np.uint8)
    a = oracle.dequantize(ac, asc, np.float32(0.5))
    b = oracle.dequantize(bc, bsc, np.float32(3.0))
    ref = (oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b))
    dev = [dev_u8(t) for t in oracle.to_ktile(ac, asc) + oracle.to_ktile(bc, bsc)]
    return dev, dev_scalar(0.5), dev_scalar(3.0), ref


def test_noalloc_matches_workspace_entry_point_on_two_calls_in_a_row():
    lib = _lib.load()
    assert lib.mq_init() == _lib.MQ_OK
    stream = torch.cuda.current_stream().cuda_stream
    # first a problem that is cut into several slabs, then a smaller one (fewer rows and columns, shorter K)
    # that leaves most of the scratch array holding the first call's partial sums
    shapes = [(128, 4096, 14336), (40, 264, 8192)]
    for out, dtype in ((mq.MQ_OUT_BF16, torch.bfloat16), (mq.MQ_OUT_FP32, torch.float32)):
        for M, N, K in shapes:
            print(f"\n[case] nvfp4_gemm_noalloc out={out} M={M} N={N} K={K}", flush=True)
            d, a_al, b_al, (ref, na, nb) = _case(M, N, K, 0)
            need = lib.mq_gemm_workspace_bytes(M, N, K)
            assert 2 * M * N * 4 <= need <= mq.NOALLOC_SCRATCH_BYTES       # slabs are really used
            ws = torch.empty(mq.NOALLOC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
            y_ws = torch.empty((M, N), dtype=dtype, device="cuda")
            y_na = torch.full((M, N), -5.0, dtype=dtype, device="cuda")
            args = [d[0].data_ptr(), d[1].data_ptr(), a_al.data_ptr(), d[2].data_ptr(), d[3].data_ptr(),
                    b_al.data_ptr(), M, N, K]
            tail = [N, out, mq.MQ_LAYOUT_KTILE]
            assert lib.nvfp4_gemm_ws(*args, y_ws.data_ptr(), *tail, ws.data_ptr(), ws.numel(), stream) == _lib.MQ_OK
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
            assert lib.nvfp4_gemm_noalloc(*args, y_na.data_ptr(), *tail, stream) == _lib.MQ_OK
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free_before              # nothing was allocated
            assert torch.equal(y_na, y_ws)
            if out == mq.MQ_OUT_BF16:
                check_gemm_bf16(host_bits(y_na), ref, na, nb)
            else:
                check_gemm_fp32(y_na.cpu().numpy(), ref, na, nb)


def test_noalloc_argument_errors():
    lib = _lib.load()
    y = torch.empty((4, 8), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((4, 32), dtype=torch.uint8, device="cuda")
    s = torch.zeros((4, 4), dtype=torch.uint8, device="cuda")
    a = dev_scalar(1.0)
    p = lambda t: t.data_ptr()
    assert lib.nvfp4_gemm_noalloc(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 24, p(y), 8, 0, 0, None) == 2
    assert lib.nvfp4_gemm_noalloc(None, p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 8, 0, 0, None) == 1
    assert lib.nvfp4_gemm_noalloc(p(c), p(s), p(a), p(c), p(s), p(a), 4, 4, 64, p(y), 8, 0, 0, None) == 0
    torch.cuda.synchronize()
    assert lib.mq_status_string(6).decode().startswith("MQ_ERR_SCRATCH")
