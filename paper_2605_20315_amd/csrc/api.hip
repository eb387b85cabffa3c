// extern "C" entry points of libmixquant: argument validation on the host, then one or a
// few kernel launches on the caller's stream.  Nothing here allocates or synchronises.
#include <atomic>

#include "mq_common.h"

namespace mq {

static thread_local int g_last_hip_error = 0;

int note_launch(hipError_t e)
{
    if (e == hipSuccess) return MQ_OK;
    g_last_hip_error = (int)e;
    return MQ_ERR_HIP;
}

static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// One-time set-up per device: kernel attributes (dynamic LDS limits) and, for the entry point
// that may not allocate, the address of this device's copy of the static scratch array.
constexpr int kMaxDevices = 64;
static std::atomic<int> g_device_ready[kMaxDevices];
static void *g_scratch_ptr[kMaxDevices];

}  // namespace mq

// Scratch memory of nvfp4_gemm_noalloc: FP32 partial sums of the slab-split product.  Every GPU
// the library runs on holds its own copy until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress; kernels receive the per-device address kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[MQ_NOALLOC_SCRATCH_BYTES];

namespace mq {

// Current device's slot, set up on first use.  Returns MQ_OK or MQ_ERR_HIP.
static int ensure_device(int *slot_out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_launch(e);
    if (dev < 0 || dev >= kMaxDevices) return note_launch(hipErrorInvalidDevice);
    if (slot_out) *slot_out = dev;
    if (g_device_ready[dev].load(std::memory_order_acquire)) return MQ_OK;
    if (int rc = configure_gemm_kernels()) return rc;
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr) return note_launch(e != hipSuccess ? e : hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = ptr;  // two racing threads store the same address
    g_device_ready[dev].store(1, std::memory_order_release);
    return MQ_OK;
}

}  // namespace mq

using namespace mq;

extern "C" {

size_t mq_codes_bytes(int64_t rows, int64_t K)
{
    if (rows < 0 || K <= 0 || K % kBlock != 0) return 0;
    return (size_t)rows * (size_t)(K / 2);
}

size_t mq_scales_bytes(int64_t rows, int64_t K)
{
    if (rows < 0 || K <= 0 || K % kBlock != 0) return 0;
    return (size_t)rows * (size_t)(K / kBlock);
}

int nvfp4_global_scale(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, float *alpha_dev,
                       void *stream)
{
    if (!alpha_dev || (!x_bf16 && rows > 0)) return MQ_ERR_NULL;
    if (rows < 0 || K <= 0 || K % kBlock != 0 || ldx < K) return MQ_ERR_SHAPE;
    if (!aligned(x_bf16, 16) || ldx % 8 != 0 || !aligned(alpha_dev, 4)) return MQ_ERR_ALIGN;
    return launch_global_scale(static_cast<const uint16_t *>(x_bf16), rows, K, ldx, alpha_dev,
                               static_cast<hipStream_t>(stream));
}

int nvfp4_quantize(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, const float *alpha_dev,
                   uint8_t *codes, uint8_t *scales, int layout, void *stream)
{
    if (layout != MQ_LAYOUT_LINEAR && layout != MQ_LAYOUT_KTILE) return MQ_ERR_ARG;
    if (rows < 0 || K <= 0 || K % kBlock != 0 || ldx < K) return MQ_ERR_SHAPE;
    if (layout == MQ_LAYOUT_KTILE && K % 64 != 0) return MQ_ERR_SHAPE;
    if (rows == 0) return MQ_OK;
    if (!x_bf16 || !alpha_dev || !codes || !scales) return MQ_ERR_NULL;
    if (!aligned(x_bf16, 16) || ldx % 8 != 0 || !aligned(codes, 16) || !aligned(alpha_dev, 4))
        return MQ_ERR_ALIGN;
    if (layout == MQ_LAYOUT_KTILE && !aligned(scales, 4)) return MQ_ERR_ALIGN;
    return launch_quantize(static_cast<const uint16_t *>(x_bf16), rows, K, ldx, alpha_dev, codes, scales, layout,
                           static_cast<hipStream_t>(stream));
}

static int check_quant_out(int64_t rows, int64_t K, const float *alpha_dev, const uint8_t *codes,
                           const uint8_t *scales, int layout, const void *dbg, int64_t ldd)
{
    if (layout != MQ_LAYOUT_LINEAR && layout != MQ_LAYOUT_KTILE) return MQ_ERR_ARG;
    if (rows < 0 || K <= 0 || K % kBlock != 0) return MQ_ERR_SHAPE;
    if (layout == MQ_LAYOUT_KTILE && K % 64 != 0) return MQ_ERR_SHAPE;
    if (dbg && ldd < K) return MQ_ERR_SHAPE;
    if (rows == 0) return MQ_OK;
    if (!alpha_dev || !codes || !scales) return MQ_ERR_NULL;
    if (!aligned(codes, 16) || !aligned(alpha_dev, 4)) return MQ_ERR_ALIGN;
    if (layout == MQ_LAYOUT_KTILE && !aligned(scales, 4)) return MQ_ERR_ALIGN;
    if (dbg && (!aligned(dbg, 16) || ldd % 8 != 0)) return MQ_ERR_ALIGN;
    return MQ_OK;
}

int nvfp4_quantize_silu_mul(const void *gate_up_bf16, int64_t rows, int64_t K, int64_t ld, const float *alpha_dev,
                            uint8_t *codes, uint8_t *scales, int layout, void *p_bf16, int64_t ldp, void *stream)
{
    if (K > 0 && ld < 2 * K) return MQ_ERR_SHAPE;
    if (int rc = check_quant_out(rows, K, alpha_dev, codes, scales, layout, p_bf16, ldp)) return rc;
    if (rows == 0) return MQ_OK;
    if (!gate_up_bf16) return MQ_ERR_NULL;
    if (!aligned(gate_up_bf16, 16) || ld % 8 != 0) return MQ_ERR_ALIGN;
    return launch_quantize_silu_mul(static_cast<const uint16_t *>(gate_up_bf16), rows, K, ld, alpha_dev, codes,
                                    scales, layout, static_cast<uint16_t *>(p_bf16), ldp,
                                    static_cast<hipStream_t>(stream));
}

int nvfp4_quantize_rmsnorm(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, const void *w_bf16, float eps,
                           const float *alpha_dev, uint8_t *codes, uint8_t *scales, int layout, void *y_bf16,
                           int64_t ldy, void *stream)
{
    if (K > 0 && K % 64 != 0) return MQ_ERR_SHAPE;
    if (!(eps >= 0.0f) || eps > 3.0e38f) return MQ_ERR_ARG;
    if (int rc = check_quant_out(rows, K, alpha_dev, codes, scales, layout, y_bf16, ldy)) return rc;
    if (ldx < K) return MQ_ERR_SHAPE;
    if (rows == 0) return MQ_OK;
    if (!x_bf16 || !w_bf16) return MQ_ERR_NULL;
    if (!aligned(x_bf16, 16) || !aligned(w_bf16, 16) || ldx % 8 != 0) return MQ_ERR_ALIGN;
    return launch_quantize_rmsnorm(static_cast<const uint16_t *>(x_bf16), rows, K, ldx,
                                   static_cast<const uint16_t *>(w_bf16), eps, alpha_dev, codes, scales, layout,
                                   static_cast<uint16_t *>(y_bf16), ldy, static_cast<hipStream_t>(stream));
}

int nvfp4_relayout(const uint8_t *src_codes, const uint8_t *src_scales, uint8_t *dst_codes, uint8_t *dst_scales,
                   int64_t rows, int64_t K, int from_layout, int to_layout, void *stream)
{
    if ((from_layout != MQ_LAYOUT_LINEAR && from_layout != MQ_LAYOUT_KTILE) ||
        (to_layout != MQ_LAYOUT_LINEAR && to_layout != MQ_LAYOUT_KTILE) || from_layout == to_layout)
        return MQ_ERR_ARG;
    if (rows < 0 || K <= 0 || K % 64 != 0) return MQ_ERR_SHAPE;
    if (rows == 0) return MQ_OK;
    if (!src_codes || !src_scales || !dst_codes || !dst_scales) return MQ_ERR_NULL;
    if (!aligned(src_codes, 16) || !aligned(dst_codes, 16) || !aligned(src_scales, 4) || !aligned(dst_scales, 4))
        return MQ_ERR_ALIGN;
    return launch_relayout(src_codes, src_scales, dst_codes, dst_scales, rows, K, to_layout == MQ_LAYOUT_KTILE,
                           static_cast<hipStream_t>(stream));
}

static int check_out(const void *y, int64_t N, int64_t ldy, int out)
{
    if (out != MQ_OUT_BF16 && out != MQ_OUT_FP32) return MQ_ERR_ARG;
    if (ldy < N) return MQ_ERR_SHAPE;
    if (!aligned(y, 16)) return MQ_ERR_ALIGN;
    if (ldy % (out == MQ_OUT_BF16 ? 8 : 4) != 0) return MQ_ERR_ALIGN;
    return MQ_OK;
}

// gfx950 parts have at most 256 compute units; the launcher uses what the device reports and
// at most one 64x64 FP32 tile of partial sums per compute unit.
static constexpr int kMaxComputeUnits = 256;

int64_t mq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const SmallPlan plan = gemm_fp4_small_plan(M, N, K, INT64_MAX, kMaxComputeUnits);
    return plan.waves > 0 && plan.slabs >= 2 ? (int64_t)plan.slabs * M * N * 4 : 0;
}

int mq_init(void) { return ensure_device(nullptr); }

int nvfp4_gemm(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
               const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev, int64_t M,
               int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout, void *stream)
{
    return nvfp4_gemm_ws(a_codes, a_scales, a_alpha_dev, b_codes, b_scales, b_alpha_dev, M, N, K, y, ldy, out,
                         layout, nullptr, 0, stream);
}

// Shared body of the three NVFP4 product entry points.  use_static: the workspace is this
// device's copy of the static scratch array (looked up after the arguments have been validated).
static int gemm_fp4_entry(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
                          const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev, int64_t M,
                          int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout, void *workspace,
                          int64_t workspace_bytes, bool use_static, void *stream);

int nvfp4_gemm_noalloc(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
                       const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev, int64_t M,
                       int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout, void *stream)
{
    return gemm_fp4_entry(a_codes, a_scales, a_alpha_dev, b_codes, b_scales, b_alpha_dev, M, N, K, y, ldy, out,
                          layout, nullptr, 0, true, stream);
}

int nvfp4_gemm_ws(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
                  const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev, int64_t M,
                  int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout, void *workspace,
                  int64_t workspace_bytes, void *stream)
{
    return gemm_fp4_entry(a_codes, a_scales, a_alpha_dev, b_codes, b_scales, b_alpha_dev, M, N, K, y, ldy, out,
                          layout, workspace, workspace_bytes, false, stream);
}

static int gemm_fp4_entry(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
                          const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev, int64_t M,
                          int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout, void *workspace,
                          int64_t workspace_bytes, bool use_static, void *stream)
{
    if (M < 0 || N < 0 || K <= 0 || K % kBlock != 0 || workspace_bytes < 0) return MQ_ERR_SHAPE;
    if (out != MQ_OUT_BF16 && out != MQ_OUT_FP32) return MQ_ERR_ARG;
    if (layout != MQ_LAYOUT_LINEAR && layout != MQ_LAYOUT_KTILE) return MQ_ERR_ARG;
    if (layout == MQ_LAYOUT_KTILE && K % 64 != 0) return MQ_ERR_SHAPE;
    if (M == 0 || N == 0) return MQ_OK;
    if (!a_codes || !a_scales || !a_alpha_dev || !b_codes || !b_scales || !b_alpha_dev || !y)
        return MQ_ERR_NULL;
    int rc = check_out(y, N, ldy, out);
    if (rc != MQ_OK) return rc;
    if (!aligned(a_codes, 16) || !aligned(b_codes, 16) || !aligned(a_alpha_dev, 4) ||
        !aligned(b_alpha_dev, 4))
        return MQ_ERR_ALIGN;
    if (K % 64 == 0 && (!aligned(a_scales, 4) || !aligned(b_scales, 4))) return MQ_ERR_ALIGN;
    if (workspace && !aligned(workspace, 16)) return MQ_ERR_ALIGN;
    // lane offsets are relative to a wave tile of 128 rows and must fit 32 bits
    if (128 * (K / 2) + 64 >= ((int64_t)1 << 32)) return MQ_ERR_SHAPE;
    if (use_static && mq_gemm_workspace_bytes(M, N, K) > (int64_t)MQ_NOALLOC_SCRATCH_BYTES) return MQ_ERR_SCRATCH;
    int dev = 0;
    if (int rc2 = ensure_device(&dev)) return rc2;
    if (use_static) {
        workspace = g_scratch_ptr[dev];
        workspace_bytes = (int64_t)MQ_NOALLOC_SCRATCH_BYTES;
    }
    GemmArgs g{};
    g.ws = workspace_bytes > 0 ? static_cast<float *>(workspace) : nullptr;
    g.ws_bytes = g.ws ? workspace_bytes : 0;
    g.ksplit = 1;
    g.a = a_codes;
    g.b = b_codes;
    g.a_scales = a_scales;
    g.b_scales = b_scales;
    g.a_alpha = a_alpha_dev;
    g.b_alpha = b_alpha_dev;
    g.lda = g.ldb = K;
    if (layout == MQ_LAYOUT_LINEAR) {
        g.a_c_row = g.b_c_row = K / 2;
        g.a_c_step = g.b_c_step = 32;
        g.a_s_row = g.b_s_row = K / kBlock;
        g.a_s_step = g.b_s_step = 4;
    } else {
        g.a_c_row = g.b_c_row = 32;
        g.a_c_step = M * 32;
        g.b_c_step = N * 32;
        g.a_s_row = g.b_s_row = 4;
        g.a_s_step = M * 4;
        g.b_s_step = N * 4;
    }
    g.M = M;
    g.N = N;
    g.K = K;
    g.y = y;
    g.ldy = ldy;
    g.out = out;
    return launch_gemm_fp4(g, static_cast<hipStream_t>(stream));
}

int64_t mq_bf16_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const int ks = gemm_bf16_decode_slabs(M, N, K, INT64_MAX, kMaxComputeUnits);
    return ks >= 2 ? (int64_t)ks * M * N * 4 : 0;
}

int bf16_gemm(const void *x_bf16, int64_t ldx, const void *w_bf16, int64_t ldw, int64_t M, int64_t N,
              int64_t K, void *y, int64_t ldy, int out, void *stream)
{
    return bf16_gemm_ws(x_bf16, ldx, w_bf16, ldw, M, N, K, y, ldy, out, nullptr, 0, stream);
}

int bf16_gemm_ws(const void *x_bf16, int64_t ldx, const void *w_bf16, int64_t ldw, int64_t M, int64_t N,
                 int64_t K, void *y, int64_t ldy, int out, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (M < 0 || N < 0 || K <= 0 || K % 8 != 0 || ldx < K || ldw < K || workspace_bytes < 0) return MQ_ERR_SHAPE;
    if (out != MQ_OUT_BF16 && out != MQ_OUT_FP32) return MQ_ERR_ARG;
    if (M == 0 || N == 0) return MQ_OK;
    if (!x_bf16 || !w_bf16 || !y) return MQ_ERR_NULL;
    int rc = check_out(y, N, ldy, out);
    if (rc != MQ_OK) return rc;
    if (!aligned(x_bf16, 16) || !aligned(w_bf16, 16) || ldx % 8 != 0 || ldw % 8 != 0) return MQ_ERR_ALIGN;
    if (workspace && !aligned(workspace, 16)) return MQ_ERR_ALIGN;
    GemmArgs g{};
    g.ws = workspace_bytes > 0 ? static_cast<float *>(workspace) : nullptr;
    g.ws_bytes = g.ws ? workspace_bytes : 0;
    g.ksplit = 1;
    g.a = x_bf16;
    g.b = w_bf16;
    g.lda = ldx;
    g.ldb = ldw;
    // thread offsets are relative to a tile of 256 rows and must fit 32 bits
    if (256 * (ldx > ldw ? ldx : ldw) * 2 + 256 >= ((int64_t)1 << 32)) return MQ_ERR_SHAPE;
    if (int rc = ensure_device(nullptr)) return rc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.y = y;
    g.ldy = ldy;
    g.out = out;
    return launch_gemm_bf16(g, static_cast<hipStream_t>(stream));
}

int mq_mfma_probe(float *scratch_dev, int iters, void *stream, double *flop_out)
{
    if (!scratch_dev) return MQ_ERR_NULL;
    if (iters < 1 || iters > (1 << 20)) return MQ_ERR_SHAPE;
    const int blocks = 256;  // one workgroup of four waves per compute unit: one wave per SIMD
    if (flop_out) *flop_out = (double)blocks * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
    return launch_mfma_probe(scratch_dev, iters, blocks, static_cast<hipStream_t>(stream));
}

const char *mq_status_string(int status)
{
    switch (status) {
    case MQ_OK: return "MQ_OK";
    case MQ_ERR_NULL: return "MQ_ERR_NULL: a required pointer is NULL";
    case MQ_ERR_SHAPE: return "MQ_ERR_SHAPE: bad extent (K must be a positive multiple of 16, ld >= extent)";
    case MQ_ERR_ALIGN: return "MQ_ERR_ALIGN: pointer or leading dimension breaks the required alignment";
    case MQ_ERR_ARG: return "MQ_ERR_ARG: unknown enum value";
    case MQ_ERR_HIP: return "MQ_ERR_HIP: kernel launch failed (see mq_last_hip_error)";
    case MQ_ERR_SCRATCH:
        return "MQ_ERR_SCRATCH: the problem wants more scratch memory than the static array of "
               "nvfp4_gemm_noalloc holds (use nvfp4_gemm_ws with a workspace)";
    default: return "unknown mq_status";
    }
}

int mq_last_hip_error(void) { return g_last_hip_error; }

const char *mq_version(void) { return "0.2"; }

}  // extern "C"
