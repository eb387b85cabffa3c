"""GPU parity at the full sizes of the five workload configurations, in the launch configuration
the benchmark times: quantizer output compared bit for bit in full (the oracle is O(M*K)),
GEMM output compared on sampled rows (all N, full K) that include tile edges and the ragged
tail, because the FP64 oracle cannot finish whole products of this size in seconds."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20315_amd as mq
from paper_2605_20315_amd import workloads as wl

from _gpu_util import check_gemm_bf16, check_gemm_fp32, dev_bf16, host_bits, to_ktile

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

CASES = [(c.cfg_id, li) for c in wl.configs() for li in range(len(c.layers))]


def _sample_rows(M: int, rng) -> np.ndarray:
    """At least 64 random rows, the rows within 1 of every multiple of 256 (the tallest workgroup
    tile; its multiples include those of the 128- and 32-row sub-tiles' seams that matter most),
    a few sub-tile seams at both ends, the middle and the last rows."""
    seams = np.arange(256, M + 1, 256)
    edges = np.concatenate([seams - 1, seams, seams + 1,
                            [0, 1, 31, 32, 33, 63, 64, 127, 128, 129, M // 2, M - 129, M - 128, M - 65, M - 64,
                             M - 33, M - 32, M - 17, M - 16, M - 2, M - 1]])
    rows = np.concatenate([edges[(edges >= 0) & (edges < M)], rng.integers(0, M, 64)])
    return np.unique(rows)


@pytest.mark.parametrize("cfg_id,layer_idx", CASES)
def test_config_layer(cfg_id, layer_idx):
    cfg = wl.configs()[cfg_id]
    layer = cfg.layers[layer_idx]
    print(f"\n[case] cfg={cfg.name} layer={layer.name} M={cfg.M} K={layer.K} N={layer.N}", flush=True)
    x, w = wl.activation(cfg, layer_idx), wl.weight(cfg, layer_idx)
    xd, wd = dev_bf16(x), dev_bf16(w)

    # tensor-level scales
    ax_ref, aw_ref = oracle.global_scale(x), oracle.global_scale(w)
    ax, aw = mq.nvfp4_global_scale(xd), mq.nvfp4_global_scale(wd)
    assert np.float32(ax.item()) == ax_ref and np.float32(aw.item()) == aw_ref

    # quantizer: bit-exact, whole tensors
    xc, xs = mq.nvfp4_quantize(xd, ax)
    wc, ws = mq.nvfp4_quantize(wd, aw)
    torch.cuda.synchronize()
    xc_ref, xs_ref = oracle.quantize(x, ax_ref)
    wc_ref, ws_ref = oracle.quantize(w, aw_ref)
    assert np.array_equal(xs.cpu().numpy(), xs_ref)
    assert np.array_equal(xc.cpu().numpy(), xc_ref)
    assert np.array_equal(ws.cpu().numpy(), ws_ref)
    assert np.array_equal(wc.cpu().numpy(), wc_ref)
    # the K-step-major layout the benchmark uses: same bytes, documented permutation
    xck, xsk = mq.nvfp4_quantize(xd, ax, layout=mq.MQ_LAYOUT_KTILE)
    wck, wsk = mq.nvfp4_quantize(wd, aw, layout=mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    ck_ref, sk_ref = to_ktile(xc_ref, xs_ref)
    assert np.array_equal(xsk.cpu().numpy(), sk_ref) and np.array_equal(xck.cpu().numpy(), ck_ref)
    ck_ref, sk_ref = to_ktile(wc_ref, ws_ref)
    assert np.array_equal(wsk.cpu().numpy(), sk_ref) and np.array_equal(wck.cpu().numpy(), ck_ref)
    del ck_ref, sk_ref
    # clipping invariant on the real workload: a normal, unsaturated scale puts the block's
    # largest element on +-6
    normal = (xs_ref >= 0x08) & (xs_ref < 0x7E)
    xa = np.abs(wl.bf16_bits_to_f32(x[:4096])).reshape(min(cfg.M, 4096), -1, 16)
    cc = (np.stack([xc_ref[:4096] & 15, xc_ref[:4096] >> 4], axis=-1).reshape(xa.shape) & 7)
    top = np.take_along_axis(cc, xa.argmax(axis=2)[..., None], axis=2)[..., 0]
    assert (top[normal[:4096]] == 7).all()
    del x, w, xd, wd

    # GEMM: full launch, sampled rows against the FP64 oracle
    rng = np.random.default_rng([cfg_id, layer_idx, 99])
    rows = _sample_rows(cfg.M, rng)
    a = oracle.dequantize(xc_ref[rows], xs_ref[rows], ax_ref)
    b = oracle.dequantize(wc_ref, ws_ref, aw_ref)
    ref = oracle.gemm_f64(a, b)
    na, nb = oracle.row_norms(a), oracle.row_norms(b)
    ridx = torch.from_numpy(rows).cuda()
    y16 = mq.nvfp4_gemm(xck, xsk, ax, wck, wsk, aw, mq.MQ_OUT_BF16, layout=mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    strict = check_gemm_bf16(host_bits(y16[ridx]), ref, na, nb)
    # same launch configuration with the scaled FP32 accumulators as output: the BF16 output must
    # be exactly their nearest-even rounding, on every element of the full problem
    y32 = mq.nvfp4_gemm(xck, xsk, ax, wck, wsk, aw, mq.MQ_OUT_FP32, layout=mq.MQ_LAYOUT_KTILE)
    torch.cuda.synchronize()
    worst = check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
    assert torch.equal(y32.to(torch.bfloat16), y16)
    del y16, y32
    # the canonical byte order feeds the same kernels through other strides
    y32 = mq.nvfp4_gemm(xc, xs, ax, wc, ws, aw, mq.MQ_OUT_FP32)
    torch.cuda.synchronize()
    check_gemm_fp32(y32[ridx].cpu().numpy(), ref, na, nb)
    del y32
    print(f"[case] ok: {len(rows)} rows, worst |err|/(|row||col|) = {worst:.2e}, "
          f"within 1 ulp of RNE(Y*): {strict:.6f}", flush=True)
    assert strict >= 0.9999
    torch.cuda.empty_cache()
