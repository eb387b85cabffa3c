"""MI355X-native NVFP4 W4A4 prefill linear path of Mix-Quant (Section 3.3): HIP kernels behind
the C ABI of include/mixquant.h, with a thin torch-tensor binding in ``ops``."""
from .ops import (  # noqa: F401
    MQ_LAYOUT_KTILE,
    MQ_LAYOUT_LINEAR,
    MQ_OUT_BF16,
    MQ_OUT_FP32,
    NOALLOC_SCRATCH_BYTES,
    MixQuantError,
    bf16_gemm,
    mfma_probe,
    mq_gemm_workspace_bytes,
    mq_init,
    nvfp4_gemm,
    nvfp4_gemm_noalloc,
    nvfp4_gemm_ws,
    nvfp4_global_scale,
    nvfp4_linear,
    nvfp4_quantize,
    nvfp4_quantize_rmsnorm,
    nvfp4_quantize_silu_mul,
    nvfp4_relayout,
)
