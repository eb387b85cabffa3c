"""GPU parity of the NVFP4 product on prefill chunks of a few hundred tokens, where K is cut
into slabs across workgroups and the partial sums pass through a caller-owned workspace
(nvfp4_gemm_ws), and of the same shapes without a workspace (four-way split inside a workgroup).
Every output is compared with the oracle; shapes cover one and several slabs, slabs whose last
workgroup has waves without any K step, ragged M and N, N % 4 != 0 (no slabs possible) and a
workspace that is too small for the preferred number of slabs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import _lib

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_scalar, dev_u8, host_bits, to_ktile

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed):
    rng = np.random.default_rng([M, N, K, seed])
    ac = rng.integers(0, 256, size=(M, K // 2)).astype(np.uint8)
    asc = rng.integers(0x28, 0x48, size=(M, K // 16)).astype(np.uint8)
    bc = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    bsc = rng.integers(0x28, 0x48, size=(N, K // 16)).astype(np.uint8)
    return ac, asc, np.float32(0.5), bc, bsc, np.float32(3.0)


def _reference(ac, asc, aa, bc, bsc, ba):
    a = oracle.dequantize(ac, asc, aa)
    b = oracle.dequantize(bc, bsc, ba)
    return oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b)


# (M, N, K, slabs expected with a full workspace).  Slabs of K across workgroups need at most 128
# tiles of 64x64 and a K long enough to pay for the second pass; the launcher picks up to
# min(256 / tiles, K / 2048) of them.  (100, 520, 8192): 18 tiles, 4 slabs; (128, 4096, 14336): 128
# tiles, 2 slabs, 224 K steps; (300, 264, 8192): 25 tiles; (64, 1032, 12288): 6 slabs of 32 K steps,
# odd N tail; (17, 136, 8192): 3 tiles; (130, 2048, 8256): 96 tiles, 129 K steps: too short for two
# slabs to pay; (1, 8, 8192): one tile.  A shorter K takes the one-launch kernel with or without a
# workspace.
SHAPES = [(100, 520, 8192, True), (128, 4096, 14336, True), (300, 264, 8192, True), (64, 1032, 12288, True),
          (17, 136, 8192, True), (130, 2048, 8256, False), (1, 8, 8192, True), (100, 520, 4096, False),
          (300, 264, 1024, False), (64, 1032, 1536, False), (1, 8, 1024, False), (64, 264, 20544, True)]


@pytest.mark.parametrize("M,N,K,slabs", SHAPES)
@pytest.mark.parametrize("layout", [mq.MQ_LAYOUT_KTILE, mq.MQ_LAYOUT_LINEAR])
def test_small_m_with_and_without_workspace(M, N, K, slabs, layout):
    ops = _operands(M, N, K, 0)
    ref, na, nb = _reference(*ops)
    ac, asc, aa, bc, bsc, ba = ops
    arrs = (to_ktile(ac, asc) + to_ktile(bc, bsc)) if layout == mq.MQ_LAYOUT_KTILE else (ac, asc, bc, bsc)
    d = [dev_u8(t) for t in arrs]
    a_al, b_al = dev_scalar(aa), dev_scalar(ba)
    need = mq.mq_gemm_workspace_bytes(M, N, K)
    assert 0 <= need <= 16 << 20
    assert (need > 0) == slabs
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    got = {}
    for out in (mq.MQ_OUT_BF16, mq.MQ_OUT_FP32):
        ys = [mq.nvfp4_gemm(d[0], d[1], a_al, d[2], d[3], b_al, out, layout=layout),
              mq.nvfp4_gemm_ws(d[0], d[1], a_al, d[2], d[3], b_al, ws, out, layout=layout),
              mq.nvfp4_gemm_ws(d[0], d[1], a_al, d[2], d[3], b_al, ws, out, layout=layout)]
        torch.cuda.synchronize()
        assert torch.equal(ys[1], ys[2])  # bit-identical from run to run
        for y in ys[:2]:
            if out == mq.MQ_OUT_BF16:
                check_gemm_bf16(host_bits(y), ref, na, nb)
            else:
                check_gemm_fp32(y.cpu().numpy(), ref, na, nb)
        got[out] = ys[:2]
    # the BF16 output is the nearest-even rounding of the scaled FP32 sums, with and without slabs
    for y16, y32 in zip(got[mq.MQ_OUT_BF16], got[mq.MQ_OUT_FP32]):
        assert torch.equal(y32.to(torch.bfloat16), y16)


def test_workspace_size_limits_the_slabs_and_odd_n_uses_none():
    M, N, K = 96, 1024, 8192
    ops = _operands(M, N, K, 1)
    ref, na, nb = _reference(*ops)
    ac, asc, aa, bc, bsc, ba = ops
    d = [dev_u8(t) for t in to_ktile(ac, asc) + to_ktile(bc, bsc)]
    a_al, b_al = dev_scalar(aa), dev_scalar(ba)
    need = mq.mq_gemm_workspace_bytes(M, N, K)
    assert need >= 2 * M * N * 4
    # room for exactly two slabs, for one (= none are used), for a fraction of one, and an unaligned size
    for nbytes in (2 * M * N * 4, M * N * 4, 100, need - 4):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        y = mq.nvfp4_gemm_ws(d[0], d[1], a_al, d[2], d[3], b_al, ws, mq.MQ_OUT_FP32, layout=mq.MQ_LAYOUT_KTILE)
        torch.cuda.synchronize()
        check_gemm_fp32(y.cpu().numpy(), ref, na, nb)
    # N % 4 != 0: the second pass works on groups of four columns, so no slabs; the result must be right
    M, N, K = 40, 1030, 8192
    assert mq.mq_gemm_workspace_bytes(M, N, K) == 0 and mq.mq_gemm_workspace_bytes(M, N + 2, K) > 0
    ops = _operands(M, N, K, 2)
    ref, na, nb = _reference(*ops)
    ac, asc, aa, bc, bsc, ba = ops
    d = [dev_u8(t) for t in to_ktile(ac, asc) + to_ktile(bc, bsc)]
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    ld = 1032
    buf = torch.full((M, ld), -3.0, dtype=torch.bfloat16, device="cuda")
    mq.nvfp4_gemm_ws(d[0], d[1], dev_scalar(aa), d[2], d[3], dev_scalar(ba), ws, mq.MQ_OUT_BF16, buf[:, :N],
                     mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    check_gemm_bf16(host_bits(buf[:, :N]), ref, na, nb)
    assert bool((buf[:, N:] == -3.0).all())


def test_slabs_into_a_column_slice_and_workspace_argument_checks():
    M, N, K = 120, 520, 8192
    ops = _operands(M, N, K, 3)
    ref, na, nb = _reference(*ops)
    ac, asc, aa, bc, bsc, ba = ops
    d = [dev_u8(t) for t in to_ktile(ac, asc) + to_ktile(bc, bsc)]
    a_al, b_al = dev_scalar(aa), dev_scalar(ba)
    ws = torch.empty(mq.mq_gemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
    buf = torch.full((M + 1, N + 32), 5.0, dtype=torch.bfloat16, device="cuda")
    view = buf[:M, 16:16 + N]
    mq.nvfp4_gemm_ws(d[0], d[1], a_al, d[2], d[3], b_al, ws, mq.MQ_OUT_BF16, view, mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    check_gemm_bf16(host_bits(view), ref, na, nb)
    rest = buf.clone()
    rest[:M, 16:16 + N] = 5.0
    assert bool((rest == 5.0).all())

    lib = _lib.load()
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    args = [d[0].data_ptr(), d[1].data_ptr(), a_al.data_ptr(), d[2].data_ptr(), d[3].data_ptr(), b_al.data_ptr(),
            M, N, K, y.data_ptr(), N, mq.MQ_OUT_BF16, mq.MQ_LAYOUT_KTILE]
    assert lib.nvfp4_gemm_ws(*args, ws.data_ptr() + 4, 1 << 20, 0) == 3      # MQ_ERR_ALIGN
    assert lib.nvfp4_gemm_ws(*args, ws.data_ptr(), -1, 0) == 2           # MQ_ERR_SHAPE
    assert lib.nvfp4_gemm_ws(*args, None, 0, 0) == _lib.MQ_OK       # no workspace: same as nvfp4_gemm
    assert lib.nvfp4_gemm_ws(*args, None, 1 << 20, 0) == _lib.MQ_OK  # NULL with a size: treated as none
    torch.cuda.synchronize()
    check_gemm_bf16(host_bits(y), ref, na, nb)


def test_slab_split_chain_replays_from_a_hip_graph():
    """nvfp4_gemm_ws launches two kernels and nothing else (no allocation, no memset, no
    synchronisation), so amax -> quantize -> slab-split GEMM can be captured once and replayed on
    new inputs; every replay must equal the eager result on the same input."""
    from paper_2605_20315_amd import workloads as wl
    from _gpu_util import dev_bf16
    rng = np.random.default_rng(79)
    M, K, N = 96, 8192, 2048
    mk = lambda: dev_bf16(wl.f32_to_bf16_bits((rng.standard_normal((M, K)) * rng.uniform(0.5, 4.0)).astype(np.float32)))
    w = dev_bf16(wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32)))
    aw = mq.nvfp4_global_scale(w)
    wc, wsc = mq.nvfp4_quantize(w, aw, layout=mq.MQ_LAYOUT_KTILE)
    need = mq.mq_gemm_workspace_bytes(M, N, K)
    assert need > 0
    work = torch.empty(need, dtype=torch.uint8, device="cuda")
    x = mk()
    ax = torch.empty(1, dtype=torch.float32, device="cuda")
    xc = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    xs = torch.empty((M, K // 16), dtype=torch.uint8, device="cuda")
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")

    def chain():
        mq.nvfp4_global_scale(x, ax)
        mq.nvfp4_quantize(x, ax, xc, xs, mq.MQ_LAYOUT_KTILE)
        mq.nvfp4_gemm_ws(xc, xs, ax, wc, wsc, aw, work, mq.MQ_OUT_BF16, y, mq.MQ_LAYOUT_KTILE)
    mq.mq_init()                           # one-time set-up of the device; no eager warm-up of the chain is needed
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for _ in range(3):
        x.copy_(mk())
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        work.fill_(0xFF)                   # the workspace carries nothing from call to call
        chain()                            # eager, same input
        torch.cuda.synchronize()
        assert torch.equal(got, y)
    # and the eager result is the oracle's
    xb = x.view(torch.int16).cpu().numpy().view(np.uint16)
    wb = w.view(torch.int16).cpu().numpy().view(np.uint16)
    axr, awr = oracle.global_scale(xb), oracle.global_scale(wb)
    a = oracle.dequantize(*oracle.quantize(xb, axr), axr)
    b = oracle.dequantize(*oracle.quantize(wb, awr), awr)
    check_gemm_bf16(host_bits(y), oracle.gemm_f64(a, b), oracle.row_norms(a), oracle.row_norms(b))
