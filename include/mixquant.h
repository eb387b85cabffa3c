/*
 * mixquant.h -- C ABI of the MI355X (gfx950) library for the prefill linear layer of
 * Mix-Quant run as NVFP4 W4A4 (Section 3.3, the paragraph on NVFP4 quantization of the
 * prefill phase): on-the-fly activation quantization (Eq. 2 then Eq. 1) followed by a
 * block-scaled FP4 GEMM against offline-quantized weights, plus a plain BF16 GEMM that
 * stands for the high-precision decode path the paper compares against.
 *
 * Conventions shared by every entry point
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *    allocates, frees or keeps a pointer, and never synchronises: each call enqueues its
 *    kernels on `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *    returns.  Calls on one stream execute in order.
 *  - Tensor-level scales (alpha in Eq. 1) are read from device memory, so a scale computed
 *    on the device needs no host round trip.
 *  - Return value: MQ_OK, or an mq_status error.  Arguments are validated on the host before
 *    anything is launched: with any status but MQ_ERR_HIP nothing has been enqueued.
 *    MQ_ERR_HIP means the HIP runtime refused a launch (mq_last_hip_error() returns its
 *    hipError_t); an entry point that launches several kernels (nvfp4_global_scale, a product
 *    cut into K slabs or into two column ranges) may then have enqueued the earlier ones, and
 *    its outputs are undefined.
 *  - One-time set-up per device (kernel attributes, the address of the static scratch array):
 *    done by mq_init(), or else by the first product on that device.  A caller that captures
 *    streams into HIP graphs calls mq_init() once per device beforehand; after that no entry
 *    point does anything but enqueue kernels.
 *  - Outputs must not overlap inputs.
 *
 * NVFP4 tensor (Section 3.3): a [rows, K] matrix whose contraction index K is contiguous
 * (the scale blocks run along the GEMM's contraction dimension, Section 3.3, last sentence),
 * K % 16 == 0, stored as
 *    codes  : uint8 [rows, K/2]   element k of a row in byte k/2, even k in the low nibble;
 *                                 a code is E2M1: bit3 sign, bits2..1 exponent (bias 1),
 *                                 bit0 mantissa -> {0, .5, 1, 1.5, 2, 3, 4, 6}
 *    scales : uint8 [rows, K/16]  one FP8 E4M3 (OCP, max 448, no infinity) byte per block of
 *                                 g = 16 consecutive K elements
 *    alpha  : one float           the tensor-level scale
 * with value x_hat[r, k] = alpha * E4M3(scales[r, k/16]) * E2M1(code[r, k])   (Eq. 1, right).
 * Scale bytes are what Eq. 2 produces: non-negative and finite, 0x00 .. 0x7E.  The quantizers
 * emit nothing else; nvfp4_gemm given a byte with the sign bit set or the NaN pattern 0x7F
 * returns unspecified values for the outputs that the block touches (never a fault).
 */
#ifndef MIXQUANT_H
#define MIXQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MQ_OK = 0,
    MQ_ERR_NULL = 1,   /* a required pointer is NULL */
    MQ_ERR_SHAPE = 2,  /* rows/M/N < 0, K <= 0, K % 16 != 0 (K % 64 != 0 for MQ_LAYOUT_KTILE), ld too small */
    MQ_ERR_ALIGN = 3,  /* a pointer or leading dimension breaks the stated alignment */
    MQ_ERR_ARG = 4,    /* unknown enum value */
    MQ_ERR_HIP = 5,    /* kernel launch failed; see mq_last_hip_error() */
    MQ_ERR_SCRATCH = 6 /* nvfp4_gemm_noalloc: the problem wants more scratch than its static array holds */
} mq_status;

typedef enum {
    MQ_OUT_BF16 = 0,   /* product path: FP32 accumulator rounded to BF16 (nearest even) */
    MQ_OUT_FP32 = 1    /* test path: the scaled FP32 accumulator itself */
} mq_out;

/*
 * Byte order of the two arrays of an NVFP4 tensor.
 * MQ_LAYOUT_LINEAR is the canonical order described at the top of this file.
 * MQ_LAYOUT_KTILE (needs K % 64 == 0) stores the same bytes K-step-major, so that the 64-wide
 * K step the GEMM consumes is contiguous over rows (one way to lay the blocks out along the
 * contraction dimension, which is all that Section 3.3 asks of the layout):
 *    codes_ktile [(t * rows + r) * 32 + j] = codes_linear [r * (K/2)  + t * 32 + j],  j < 32
 *    scales_ktile[(t * rows + r) * 4  + j] = scales_linear[r * (K/16) + t * 4  + j],  j < 4
 * for K step t = 0 .. K/64 - 1.  Sizes are the same in both layouts.
 */
typedef enum {
    MQ_LAYOUT_LINEAR = 0,
    MQ_LAYOUT_KTILE = 1
} mq_layout;

/*
 * One-time set-up of the current device (hipGetDevice): raises the dynamic-LDS limits of the
 * tiled kernels and looks up this device's copy of the static scratch array.  Idempotent,
 * thread-safe, launches nothing.  Optional except before stream capture (see above).
 */
int mq_init(void);

/* Sizes, in bytes, of the two byte arrays of an NVFP4 tensor (0 when K % 16 != 0). */
size_t mq_codes_bytes(int64_t rows, int64_t K);
size_t mq_scales_bytes(int64_t rows, int64_t K);

/*
 * Tensor-level scale (Section 3.3 gives it the role of setting the tensor's overall range and
 * no formula; the workloads use alpha = max|x| / (6 * 448)).
 * Writes alpha = max|x| / 2688 to *alpha_dev (1.0f when the tensor is all zero), all in
 * binary32.  x_bf16: [rows, K] BF16, row stride ldx elements (ldx >= K).  K % 16 == 0,
 * x_bf16 16-byte aligned, ldx % 8 == 0.  rows == 0 writes 1.0f.
 */
int nvfp4_global_scale(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx,
                       float *alpha_dev, void *stream);

/*
 * NVFP4 quantizer for activations (per prefill batch) or weights (once, offline):
 * Eq. 2 gives each block's E4M3 scale from its largest magnitude, Eq. 1 the E2M1 codes.
 * Arithmetic, every step IEEE binary32, nearest-even, unfused, per block b of 16 elements:
 *    s = amax_b / (6 * alpha);  sigma_b = Pi_E4M3(s)   (ties to even, saturating at 448)
 *    r = 1 / (alpha * sigma_b); q_i = Pi_FP4(x_i * r)  (ties to even, clipped to +-6);
 *    sigma_b == 0 gives signed-zero codes.
 * x_bf16: [rows, K] BF16, row stride ldx elements; *alpha_dev finite and > 0, read on the
 * device.  codes: [rows, K/2], scales: [rows, K/16], dense.  Inputs must be finite (Inf
 * saturates, NaN gives unspecified codes; never a fault).
 * layout: mq_layout of the two output arrays.
 * K % 16 == 0; x_bf16 and codes 16-byte aligned (scales 4-byte aligned for MQ_LAYOUT_KTILE);
 * ldx % 8 == 0.  rows == 0 is a no-op.
 */
int nvfp4_quantize(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx,
                   const float *alpha_dev, uint8_t *codes, uint8_t *scales, int layout,
                   void *stream);

/*
 * Quantizer fused with the operation that produces the activation (Section 3.3, last sentence:
 * the layout is chosen so that a backend can fuse quantization with its neighbours).  The paper
 * does not define the producers;
 * these are the two that feed the linear layers of the decoder blocks of the models it
 * evaluates (Section 4.1), by their textbook definitions.  In both, the producer's value is
 * computed in binary32, rounded once to BF16 (nearest even), and that BF16 tensor is quantized
 * exactly as nvfp4_quantize would: the BF16 activations never travel through memory.
 * p_bf16 / y_bf16 (may be NULL): if given, also receives the BF16 tensor that was quantized,
 * [rows, K] with row stride ldp / ldy elements (multiple of 8, 16-byte aligned base); the codes
 * and scales are then bit-identical to nvfp4_quantize applied to it.
 *
 * nvfp4_quantize_silu_mul: gated-MLP activation, the input of the down projection.
 *    p[r, k] = silu(g) * u,  g = gate_up[r, k],  u = gate_up[r, K + k],  silu(g) = g / (1 + exp(-g))
 * gate_up_bf16: [rows, 2K] BF16, row stride ld elements (ld >= 2K, ld % 8 == 0).  Gates below
 * about -88 (exp(-g) overflows binary32) give -0, as any binary32 evaluation does.
 * nvfp4_quantize_rmsnorm: root-mean-square normalisation, the input of the qkv and gate_up
 * projections.
 *    y[r, k] = x[r, k] / sqrt(mean_k(x[r, :]^2) + eps) * w[k]
 * x_bf16: [rows, K] BF16, row stride ldx; w_bf16: [K] BF16; eps >= 0; K % 64 == 0.
 * Other arguments, alignment and errors as in nvfp4_quantize.
 */
int nvfp4_quantize_silu_mul(const void *gate_up_bf16, int64_t rows, int64_t K, int64_t ld,
                            const float *alpha_dev, uint8_t *codes, uint8_t *scales, int layout,
                            void *p_bf16, int64_t ldp, void *stream);
int nvfp4_quantize_rmsnorm(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, const void *w_bf16,
                           float eps, const float *alpha_dev, uint8_t *codes, uint8_t *scales,
                           int layout, void *y_bf16, int64_t ldy, void *stream);

/*
 * Offline weight pre-pack (weights are static across requests: Section 3.3, the paragraph on
 * the disaggregated deployment): copy an NVFP4 tensor from one mq_layout to the other.  Pure byte
 * permutation by the index map given at mq_layout; src and dst must not overlap.
 * K % 64 == 0; code arrays 16-byte aligned, scale arrays 4-byte aligned; from_layout != to_layout.
 */
int nvfp4_relayout(const uint8_t *src_codes, const uint8_t *src_scales, uint8_t *dst_codes,
                   uint8_t *dst_scales, int64_t rows, int64_t K, int from_layout, int to_layout,
                   void *stream);

/*
 * Block-scaled FP4 GEMM (Section 3.3; the W4A4 linear layer of the prefill path):
 *    Y[m, n] = alpha_a * alpha_b * sum_k  sa[m, k/16] * qa[m, k] * sb[n, k/16] * qb[n, k]
 * A = quantized activations [M, K], B = quantized weights [N, K], both NVFP4 tensors as
 * described above.  Every product is formed exactly, sums are accumulated in FP32, the two
 * tensor-level scales are applied once to the accumulator, and the result is written as
 * BF16 (nearest even) or FP32.  y: [M, N], row stride ldy elements (ldy >= N).
 * K % 16 == 0; code arrays 16-byte aligned, scale arrays 4-byte aligned when K % 64 == 0;
 * y 16-byte aligned and ldy % 8 == 0 for BF16 (ldy % 4 == 0 for FP32).  M, N >= 0 arbitrary
 * (ragged batches); M == 0 or N == 0 is a no-op.  Results are bit-identical from run to run.
 * layout: mq_layout of all four operand arrays (both operands use the same one).
 */
int nvfp4_gemm(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
               const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev,
               int64_t M, int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout,
               void *stream);

/*
 * The same product (Section 3.3) with a caller-owned workspace.  A prefill chunk of a few
 * hundred tokens against a layer with a long K and a narrow N has fewer output tiles than the GPU
 * has compute units; with a workspace the K dimension is then cut into slabs across workgroups,
 * each writes FP32 partial sums to the workspace, and a second kernel adds the slabs in ascending
 * order, applies alpha_a * alpha_b and rounds.  Same arguments, requirements, tolerance and
 * run-to-run bit-identity as nvfp4_gemm; the summation order (and so the last bits) may differ
 * from nvfp4_gemm's where slabs are used.
 * workspace: device memory, 16-byte aligned, workspace_bytes >= 0 bytes, or NULL with 0; its
 * contents are undefined afterwards and it must not be used by other work on another stream
 * until this call's kernels have finished.  mq_gemm_workspace_bytes(M, N, K) (host function, no
 * GPU access) returns the size that lets the library choose freely: slabs * M * N * 4 bytes,
 * never more than 4 MiB, and 0 where slabs are never used (N % 4 != 0, K % 64 != 0, more than 128
 * output tiles of 64x64, or a K too short for the second pass to pay: below about 8192).  A
 * smaller workspace is legal and only limits the number of slabs.
 */
int64_t mq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int nvfp4_gemm_ws(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
                  const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev,
                  int64_t M, int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout,
                  void *workspace, int64_t workspace_bytes, void *stream);

/*
 * The same product for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments,
 * requirements, results (bit-identical) and tolerance as nvfp4_gemm_ws given a workspace of
 * MQ_NOALLOC_SCRATCH_BYTES; the partial sums of the slab-split product go to a static device
 * array of that size inside the library, one copy per GPU, held until the process ends.  The
 * call allocates nothing and frees nothing.  A problem for which mq_gemm_workspace_bytes(M, N, K)
 * exceeds MQ_NOALLOC_SCRATCH_BYTES is rejected with MQ_ERR_SCRATCH before anything is enqueued.
 * Every call on a GPU uses that GPU's one array (nothing in it needs to start at zero: each
 * slab is written before it is read): calls that overlap in time on one GPU, from different
 * streams or threads, race on it; calls on one stream are ordered and safe.
 */
#define MQ_NOALLOC_SCRATCH_BYTES (4u << 20)
int nvfp4_gemm_noalloc(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_alpha_dev,
                       const uint8_t *b_codes, const uint8_t *b_scales, const float *b_alpha_dev,
                       int64_t M, int64_t N, int64_t K, void *y, int64_t ldy, int out, int layout,
                       void *stream);

/*
 * High-precision baseline (the BF16 path that decoding keeps and that the paper's prefill
 * speed-up is measured against): Y = X . W^T, X [M, K] and W [N, K] BF16 with row strides
 * ldx, ldw elements, FP32 accumulation, output as in nvfp4_gemm.
 * K % 8 == 0; x, w 16-byte aligned; ldx % 8 == 0, ldw % 8 == 0; y as in nvfp4_gemm.
 */
int bf16_gemm(const void *x_bf16, int64_t ldx, const void *w_bf16, int64_t ldw,
              int64_t M, int64_t N, int64_t K, void *y, int64_t ldy, int out, void *stream);

/*
 * The same product with a caller-owned workspace, for decode batches (the precision that the
 * decode phase keeps, Section 3.3): 33 to 64 tokens against a weight matrix with a narrow N leave
 * most compute units without a row group of W, and the time is the weights' one trip from HBM;
 * with a workspace K is cut into slabs across workgroups (FP32 partial sums, added in ascending
 * order by a second kernel: bit-identical from run to run; the last bits may differ from
 * bf16_gemm's).  Arguments and requirements as bf16_gemm; workspace as in nvfp4_gemm_ws.
 * mq_bf16_gemm_workspace_bytes(M, N, K) (host function) returns the size that lets the library
 * choose freely: slabs * M * N * 4 bytes (at most 16 MiB), 0 where slabs are never used
 * (M <= 32, M > 64, N % 4 != 0, K % 128 != 0, K < 8192, N > 16256, or so few rows of W that even
 * with slabs half of the compute units would stay empty).
 */
int64_t mq_bf16_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int bf16_gemm_ws(const void *x_bf16, int64_t ldx, const void *w_bf16, int64_t ldw,
                 int64_t M, int64_t N, int64_t K, void *y, int64_t ldy, int out,
                 void *workspace, int64_t workspace_bytes, void *stream);

/* Human-readable name of an mq_status value (static storage). */
const char *mq_status_string(int status);

/* hipError_t of the most recent failed launch on the calling thread (0 if none). */
int mq_last_hip_error(void);

/* Library version, "major.minor". */
const char *mq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MIXQUANT_H */
