// Shared declarations of the HIP library (gfx950 only).  Internal; the public C ABI is
// include/mixquant.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mixquant.h"
#include "../../include/mixquant_diag.h"

namespace mq {

constexpr int kBlock = 16;  // g: elements per NVFP4 scale block (Section 3.3)

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// Records a failed launch for mq_last_hip_error() and maps it to MQ_ERR_HIP.
int note_launch(hipError_t e);

// quantize.hip
int launch_global_scale(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, float *alpha,
                        hipStream_t s);
int launch_quantize(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, const float *alpha,
                    uint8_t *codes, uint8_t *scales, int layout, hipStream_t s);

// producer-fused quantizers (p / y: optional BF16 output of the producer, may be null)
int launch_quantize_silu_mul(const uint16_t *gate_up, int64_t rows, int64_t K, int64_t ld, const float *alpha,
                             uint8_t *codes, uint8_t *scales, int layout, uint16_t *p, int64_t ldp, hipStream_t s);
int launch_quantize_rmsnorm(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, const uint16_t *w, float eps,
                            const float *alpha, uint8_t *codes, uint8_t *scales, int layout, uint16_t *y,
                            int64_t ldy, hipStream_t s);

int launch_relayout(const uint8_t *src_c, const uint8_t *src_s, uint8_t *dst_c, uint8_t *dst_s, int64_t rows,
                    int64_t K, bool to_ktile, hipStream_t s);

// gemm.hip
struct GemmArgs {
    // NVFP4 operands (fp4 == true) or BF16 operands (fp4 == false, *_codes hold the BF16 data)
    const void *a;            // [M, K] codes or BF16
    const void *b;            // [N, K] codes or BF16
    const uint8_t *a_scales;  // [M, K/16]
    const uint8_t *b_scales;  // [N, K/16]
    const float *a_alpha;     // device scalars (NVFP4 only)
    const float *b_alpha;
    int64_t lda, ldb;         // BF16 row strides in elements (NVFP4 operands are dense)
    // NVFP4 addressing in bytes, for either layout: the 32 code bytes of (row r, K step t) start at
    // r * c_row + t * c_step, the 4 scale bytes at r * s_row + t * s_step (a K step is 64 elements)
    int64_t a_c_row, a_c_step, a_s_row, a_s_step;
    int64_t b_c_row, b_c_step, b_s_row, b_s_step;
    int64_t M, N, K;
    void *y;
    int64_t ldy;
    int out;                  // mq_out
    // optional workspace for partial sums (NVFP4, a long K with very few output tiles): ws_bytes of
    // device memory, 16-byte aligned, or NULL / 0.  ksplit (K slabs across workgroups, >= 1) is
    // filled in by the launcher.
    float *ws;
    int64_t ws_bytes;
    int ksplit;
};
// Plan of the small-tile NVFP4 kernel for a problem, given this much workspace: waves per 64x64
// tile (0: another kernel serves the problem) and K slabs across workgroups (1: none).
struct SmallPlan {
    int waves;
    int slabs;
};
SmallPlan gemm_fp4_small_plan(int64_t M, int64_t N, int64_t K, int64_t ws_bytes, int cus);
// K slabs of the decode-batch BF16 kernel (17 .. 64 tokens) given this much workspace; 0: not served by it
int gemm_bf16_decode_slabs(int64_t M, int64_t N, int64_t K, int64_t ws_bytes, int cus);
// sets the dynamic-LDS limit of every tiled kernel on the current device (idempotent)
int configure_gemm_kernels();
int launch_gemm_fp4(const GemmArgs &g, hipStream_t s);
int launch_gemm_bf16(const GemmArgs &g, hipStream_t s);
int launch_mfma_probe(float *out, int iters, int blocks, hipStream_t s);

}  // namespace mq
