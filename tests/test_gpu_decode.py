"""GPU parity of the BF16 product on decode batches of 17 .. 64 tokens (the high-precision path
that the decode phase keeps), with and without a caller-owned workspace: the weight-streaming
kernel whose waves split N and share the activations through LDS, and its K slabs across
workgroups.  Every output is compared with the oracle's FP64 product of the BF16 inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import _lib, workloads as wl

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_bf16, host_bits

pytestmark = pytest.mark.gpu

# (M, N, K).  A wide N (at least 128 row groups of 128) takes the kernel without slabs, with or
# without a workspace; a narrow N takes it above 32 tokens with K >= 8192 and a workspace, slabs =
# min(512 / row groups, K / 512, K / (8 M)); everything else the K-split kernel.
# (64, 4096, 14336): 16 slabs of 7 super-steps; (33, 6152, 8192): ragged N, 10 slabs of 7 or 6;
# (40, 4096, 8320): 65 super-steps in 16 slabs (5 + 15 x 4); (48, 1000, 8192): N % 128 != 0;
# (64, 24640, 384): wide N, three super-steps; (32, 16392, 1024), (17, 28672, 512): wide ragged N,
# two token tiles; (20, 520, 1024), (24, 4096, 8192): narrow N below 33 tokens; (64, 4096, 4096):
# narrow N, short K; (64, 4098, 8192): N % 4 != 0, no slabs; (40, 4096, 320): K % 128 != 0.
SHAPES = [(64, 4096, 14336), (33, 6152, 8192), (40, 4096, 8320), (48, 1000, 8192),
          (64, 24640, 384), (32, 16392, 1024), (17, 28672, 512), (20, 520, 1024), (24, 4096, 8192),
          (64, 4096, 4096), (64, 4098, 8192), (40, 4096, 320)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_decode_batches_with_and_without_workspace(M, N, K):
    print(f"\n[case] bf16 decode M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng([M, N, K])
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
    a, b = oracle.bf16_to_f64(x), oracle.bf16_to_f64(w)
    ref, na, nb = oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b)
    xd, wd = dev_bf16(x), dev_bf16(w)
    need = mq.mq_bf16_gemm_workspace_bytes(M, N, K)
    assert need % (M * N * 4) == 0
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    ld = (N + 7) // 8 * 8 + 8
    for workspace in (None, ws):
        b32 = torch.full((M + 1, ld), -7.0, dtype=torch.float32, device="cuda")
        b16 = torch.full((M + 1, ld), -7.0, dtype=torch.bfloat16, device="cuda")
        y32 = mq.bf16_gemm_ws(xd, wd, workspace, mq.MQ_OUT_FP32, b32[:M, :N])
        y16 = mq.bf16_gemm_ws(xd, wd, workspace, mq.MQ_OUT_BF16, b16[:M, :N])
        again = torch.empty((M, ld), dtype=torch.bfloat16, device="cuda")
        mq.bf16_gemm_ws(xd, wd, workspace, mq.MQ_OUT_BF16, again[:, :N])
        torch.cuda.synchronize()
        check_gemm_fp32(y32.cpu().numpy(), ref, na, nb)
        check_gemm_bf16(host_bits(y16), ref, na, nb)
        assert torch.equal(y32.to(torch.bfloat16), y16)
        assert torch.equal(again[:, :N], y16)
        for buf in (b32, b16):
            assert bool((buf[M:] == -7.0).all()) and bool((buf[:, N:] == -7.0).all())
    # the plain entry point is the workspace variant without a workspace
    y_plain = torch.empty((M, ld), dtype=torch.bfloat16, device="cuda")
    mq.bf16_gemm(xd, wd, mq.MQ_OUT_BF16, y_plain[:, :N])
    y_none = torch.empty((M, ld), dtype=torch.bfloat16, device="cuda")
    mq.bf16_gemm_ws(xd, wd, None, mq.MQ_OUT_BF16, y_none[:, :N])
    torch.cuda.synchronize()
    assert torch.equal(y_plain[:, :N], y_none[:, :N])


def test_workspace_query_and_small_workspaces():
    q = mq.mq_bf16_gemm_workspace_bytes
    assert q(64, 4096, 8192) == 16 * 64 * 4096 * 4
    assert q(64, 4096, 14336) == 16 * 64 * 4096 * 4
    assert q(48, 6144, 14336) == 10 * 48 * 6144 * 4
    assert q(16, 4096, 8192) == 0 and q(65, 4096, 8192) == 0          # other kernels serve these
    assert q(64, 4098, 8192) == 0 and q(64, 4096, 8256) == 0 and q(64, 4096, 4096) == 0
    assert q(64, 28672, 8192) == 0 and q(32, 4096, 8192) == 0      # wide N: no slabs; up to 32 tokens: none
    M, N, K = 64, 4096, 8192
    rng = np.random.default_rng(3)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
    a, b = oracle.bf16_to_f64(x), oracle.bf16_to_f64(w)
    ref, na, nb = oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b)
    xd, wd = dev_bf16(x), dev_bf16(w)
    # room for five slabs, for one (= none), for a fraction of one, and an unaligned size
    for nbytes in (5 * M * N * 4, M * N * 4, 100, q(M, N, K) - 4):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        y = mq.bf16_gemm_ws(xd, wd, ws, mq.MQ_OUT_FP32)
        torch.cuda.synchronize()
        check_gemm_fp32(y.cpu().numpy(), ref, na, nb)
    lib = _lib.load()
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    args = [xd.data_ptr(), K, wd.data_ptr(), K, M, N, K, y.data_ptr(), N, mq.MQ_OUT_BF16]
    assert lib.bf16_gemm_ws(*args, ws.data_ptr() + 4, 1 << 19, 0) == 3      # MQ_ERR_ALIGN
    assert lib.bf16_gemm_ws(*args, ws.data_ptr(), -1, 0) == 2              # MQ_ERR_SHAPE
    assert lib.bf16_gemm_ws(*args, None, 1 << 20, 0) == _lib.MQ_OK         # NULL with a size: treated as none
    torch.cuda.synchronize()
    check_gemm_bf16(host_bits(y), ref, na, nb)
