/*
 * CPU oracle for the NVFP4 prefill linear path of Mix-Quant (Section 3.3, the paragraph on
 * NVFP4 quantization of the prefill phase, Eq. 1 and Eq. 2).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar statement of what the path
 * computes, used only by the tests, the smoke check and the benchmark's cpu_baseline leg.
 * It shares no code, table or helper with the HIP library and the HIP library never calls
 * it.  Nothing here is tuned.
 *
 * What is fixed by the paper: element format E2M1, block size g = 16, block scale in FP8
 * E4M3 chosen from the block's largest magnitude (Eq. 2), one tensor-level scale alpha,
 * projection to the nearest representable value with clipping (Eq. 1), blocks running along
 * the GEMM contraction dimension.
 * What is a reading (the paper states Eq. 1-2 over the reals): every arithmetic step of the
 * quantizer is IEEE binary32, round-to-nearest-even, unfused, subnormals honoured, in the
 * order written in nvfp4_ref_quantize(); ties on both grids go to the even code; E4M3 is
 * the OCP "FN" flavour (no infinities, largest finite 448) and the projection saturates.
 *
 * Parity pins live in tests/ (format enumeration, exact-rational brute force, hand-worked
 * blocks, round-trip identity, closed-form GEMMs; for the two activation producers near the
 * end of this file: identities, invariants, closed forms and library routines).  NaN inputs
 * are outside the contract: "parity unpinned" for NaN only.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC nvfp4_ref.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define NVFP4_BLOCK 16 /* g in Section 3.3 */

/* ---------- formats, by closed form ------------------------------------------------ */

/* E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit; exponent field 0 is subnormal. */
double nvfp4_ref_e2m1_value(int code)
{
    int s = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
    double mag = (e == 0) ? 0.5 * m : ldexp(1.0 + 0.5 * m, e - 1);
    return s ? -mag : mag;
}

/* E4M3 (OCP FN): 1 sign, 4 exponent (bias 7), 3 mantissa bits; S.1111.111 is NaN. */
double nvfp4_ref_e4m3_value(int byte)
{
    int s = (byte >> 7) & 1, e = (byte >> 3) & 15, m = byte & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    mag = (e == 0) ? ldexp(m / 8.0, -6) : ldexp(1.0 + m / 8.0, e - 7);
    return s ? -mag : mag;
}

static float bf16_bits_to_float(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

double nvfp4_ref_bf16_value(uint16_t h) { return (double)bf16_bits_to_float(h); }

/* Pi_E4M3 of Eq. 2 for a non-negative binary32 argument: the nearest of the 127 finite
 * non-negative E4M3 values, ties to the even byte, everything at or above 448 saturates to
 * 0x7E.  Written as a search over the grid with exact midpoint comparisons (2v against
 * lo+hi, both exact in binary64). */
uint8_t nvfp4_ref_e4m3_round(float s)
{
    double v = (double)s;
    int b;
    if (!(v > 0.0)) return 0; /* +0, -0, negatives, NaN */
    if (v >= 448.0) return 0x7E;
    for (b = 0; b < 0x7E; ++b) {
        double lo = nvfp4_ref_e4m3_value(b), hi = nvfp4_ref_e4m3_value(b + 1);
        if (v >= hi) continue;
        if (2.0 * v < lo + hi) return (uint8_t)b;
        if (2.0 * v > lo + hi) return (uint8_t)(b + 1);
        return (uint8_t)((b & 1) ? b + 1 : b);
    }
    return 0x7E;
}

/* Pi_FP4 of Eq. 1: nearest E2M1 magnitude, ties to the code with mantissa bit 0, clipping
 * beyond 6, sign bit copied from the argument (so -0 and tiny negatives give 0x8). */
uint8_t nvfp4_ref_fp4_round(float y)
{
    double v = fabs((double)y);
    int sign = signbit(y) ? 8 : 0, c;
    if (v >= 6.0) return (uint8_t)(sign | 7); /* clipping; +inf lands here too */
    if (!(v > 0.0)) return (uint8_t)sign;
    for (c = 0; c < 7; ++c) {
        double lo = nvfp4_ref_e2m1_value(c), hi = nvfp4_ref_e2m1_value(c + 1);
        if (v >= hi) continue;
        if (2.0 * v < lo + hi) return (uint8_t)(sign | c);
        if (2.0 * v > lo + hi) return (uint8_t)(sign | (c + 1));
        return (uint8_t)(sign | ((c & 1) ? c + 1 : c));
    }
    return (uint8_t)(sign | 7);
}

/* Round a binary64 value to BF16 (8 significand bits, binary32 exponent range), nearest
 * even, in one rounding (not through binary32). */
uint16_t nvfp4_ref_bf16_round(double v)
{
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v), ulp, n;
    int e;
    float f;
    uint32_t u;
    if (isnan(v)) return 0x7FC0;
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80);
    (void)frexp(a, &e);            /* a = m * 2^e, m in [0.5, 1) : top bit has weight 2^(e-1) */
    if (e - 8 < -133) e = -133 + 8; /* subnormal spacing 2^-133 */
    ulp = ldexp(1.0, e - 8);
    n = rint(a / ulp);              /* exact scaling, then nearest-even to an integer */
    a = n * ulp;
    if (a >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80);
    f = (float)a;                   /* exact: at most 8 significant bits */
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (u >> 16));
}

/* ---------- tensor-level scale ------------------------------------------------------ */

/* alpha = amax / (6 * 448), the choice that makes the largest block scale land on 448;
 * 1.0 for an all-zero tensor.  (The paper describes alpha's role only; this formula is the
 * workload definition's.) */
float nvfp4_ref_global_scale(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx)
{
    float amax = 0.0f;
    int64_t r, k;
    for (r = 0; r < rows; ++r)
        for (k = 0; k < K; ++k) {
            float a = fabsf(bf16_bits_to_float(x[r * ldx + k]));
            if (a > amax) amax = a;
        }
    if (amax == 0.0f) return 1.0f;
    return amax / 2688.0f;
}

/* ---------- quantizer (Eq. 2 then Eq. 1) -------------------------------------------- */

/* x: [rows, K] BF16 bits, row stride ldx elements.  codes: [rows, K/2], element k of a row
 * in byte k/2, even k in the low nibble.  scales: [rows, K/16].  Returns 0, or -1 when K is
 * not a multiple of 16. */
int nvfp4_ref_quantize(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, float alpha,
                       uint8_t *codes, uint8_t *scales)
{
    int64_t nblk = K / NVFP4_BLOCK, r;
    volatile float six_alpha = 6.0f * alpha; /* alpha * q_max, one binary32 product */
    const float d6 = six_alpha;
    if (K % NVFP4_BLOCK != 0 || rows < 0) return -1;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t b;
        for (b = 0; b < nblk; ++b) {
            const uint16_t *xb = x + r * ldx + b * NVFP4_BLOCK;
            uint8_t c[NVFP4_BLOCK];
            float amax = 0.0f, s, sigma;
            uint8_t sb;
            int i;
            for (i = 0; i < NVFP4_BLOCK; ++i) {
                float a = fabsf(bf16_bits_to_float(xb[i]));
                if (a > amax) amax = a;
            }
            s = amax / d6;                      /* Eq. 2 argument, one binary32 division */
            sb = nvfp4_ref_e4m3_round(s);       /* Pi_E4M3 */
            sigma = (float)nvfp4_ref_e4m3_value(sb);
            if (sigma == 0.0f) {
                for (i = 0; i < NVFP4_BLOCK; ++i) c[i] = (uint8_t)((xb[i] >> 15) << 3);
            } else {
                volatile float t = alpha * sigma;   /* alpha_x * sigma_b */
                volatile float rcp = 1.0f / t;      /* one binary32 division per block */
                for (i = 0; i < NVFP4_BLOCK; ++i) {
                    volatile float y = bf16_bits_to_float(xb[i]) * rcp; /* Eq. 1 argument */
                    c[i] = nvfp4_ref_fp4_round(y);  /* Pi_FP4 */
                }
            }
            for (i = 0; i < NVFP4_BLOCK / 2; ++i)
                codes[r * (K / 2) + b * (NVFP4_BLOCK / 2) + i] =
                    (uint8_t)(c[2 * i] | (c[2 * i + 1] << 4));
            scales[r * nblk + b] = sb;
        }
    }
    return 0;
}

/* ---------- K-step-major byte order of an NVFP4 tensor --------------------------------- */

/* Section 3.3 (last sentence) places the blocks along the GEMM's contraction dimension and
 * leaves the byte order in memory open.  Besides the canonical row-major order written by
 * nvfp4_ref_quantize(), the library defines a second one in which the bytes of one 64-wide K
 * step are contiguous over rows: for K step t, row r, the 32 code bytes and the 4 scale bytes
 * of that (row, step) pair sit at
 *     codes_ktile [(t * rows + r) * 32 + j] = codes_linear [r * (K/2)  + t * 32 + j],  j < 32
 *     scales_ktile[(t * rows + r) * 4  + j] = scales_linear[r * (K/16) + t * 4  + j],  j < 4.
 * Pure permutation, stated here as the three loops of that sentence.  to_ktile != 0 converts
 * canonical -> K-step-major, 0 the other way.  Returns 0, or -1 when K is not a multiple of 64. */
int nvfp4_ref_relayout(const uint8_t *src_codes, const uint8_t *src_scales, uint8_t *dst_codes,
                       uint8_t *dst_scales, int64_t rows, int64_t K, int to_ktile)
{
    int64_t steps = K / 64, t, r, j;
    if (K % 64 != 0 || rows < 0) return -1;
    for (t = 0; t < steps; ++t)
        for (r = 0; r < rows; ++r) {
            for (j = 0; j < 32; ++j) {
                int64_t kt = (t * rows + r) * 32 + j, lin = r * (K / 2) + t * 32 + j;
                if (to_ktile) dst_codes[kt] = src_codes[lin];
                else dst_codes[lin] = src_codes[kt];
            }
            for (j = 0; j < 4; ++j) {
                int64_t kt = (t * rows + r) * 4 + j, lin = r * (K / 16) + t * 4 + j;
                if (to_ktile) dst_scales[kt] = src_scales[lin];
                else dst_scales[lin] = src_scales[kt];
            }
        }
    return 0;
}

/* x_hat = alpha * sigma * q (Eq. 1, right), evaluated in binary64: exact, the three factors
 * carry 24 + 4 + 2 significant bits.  out: [rows, K]. */
int nvfp4_ref_dequantize(const uint8_t *codes, const uint8_t *scales, float alpha,
                         int64_t rows, int64_t K, double *out)
{
    int64_t nblk = K / NVFP4_BLOCK, r;
    if (K % NVFP4_BLOCK != 0 || rows < 0) return -1;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t k;
        for (k = 0; k < K; ++k) {
            uint8_t byte = codes[r * (K / 2) + k / 2];
            int code = (k & 1) ? (byte >> 4) : (byte & 15);
            double sigma = nvfp4_ref_e4m3_value(scales[r * nblk + k / NVFP4_BLOCK]);
            out[r * K + k] = ((double)alpha * sigma) * nvfp4_ref_e2m1_value(code);
        }
    }
    return 0;
}

/* BF16 bits -> binary64, [rows, K] with row stride ldx. */
void nvfp4_ref_bf16_to_f64(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, double *out)
{
    int64_t r, k;
#pragma omp parallel for schedule(static) private(k)
    for (r = 0; r < rows; ++r)
        for (k = 0; k < K; ++k) out[r * K + k] = (double)bf16_bits_to_float(x[r * ldx + k]);
}

/* ---------- producers of the quantizer's input --------------------------------------- */

/* The paper quantizes "activations" (Section 3.3) and lets the backend fuse the quantizer
 * with its neighbours; it does not define the operations that produce those activations.
 * In the decoder blocks of the models it evaluates (Section 4.1) the inputs of the four
 * linear layers come from two of them, stated here by their textbook definitions in
 * binary64.  A fused "producer -> quantize" kernel is checked against
 * nvfp4_ref_quantize(BF16(producer)): the producer's value rounded once to BF16, which is the
 * tensor an unfused pipeline would have stored. */

/* Gated-MLP activation feeding the down projection: out[r, k] = silu(g) * u with
 * g = gate_up[r, k], u = gate_up[r, K + k], silu(g) = g / (1 + exp(-g)).
 * gate_up: [rows, 2K] BF16, row stride ld; out: [rows, K] binary64, dense. */
void nvfp4_ref_silu_mul_f64(const uint16_t *gate_up, int64_t rows, int64_t K, int64_t ld, double *out)
{
    int64_t r, k;
#pragma omp parallel for schedule(static) private(k)
    for (r = 0; r < rows; ++r)
        for (k = 0; k < K; ++k) {
            double g = (double)bf16_bits_to_float(gate_up[r * ld + k]);
            double u = (double)bf16_bits_to_float(gate_up[r * ld + K + k]);
            out[r * K + k] = g / (1.0 + exp(-g)) * u;
        }
}

/* Root-mean-square normalisation feeding the qkv and gate_up projections:
 * out[r, k] = x[r, k] / sqrt(mean_k(x[r, :]^2) + eps) * w[k].
 * x: [rows, K] BF16, row stride ldx; w: [K] BF16; out: [rows, K] binary64, dense. */
void nvfp4_ref_rmsnorm_f64(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, const uint16_t *w,
                           double eps, double *out)
{
    int64_t r, k;
#pragma omp parallel for schedule(static) private(k)
    for (r = 0; r < rows; ++r) {
        double ss = 0.0, d;
        for (k = 0; k < K; ++k) {
            double v = (double)bf16_bits_to_float(x[r * ldx + k]);
            ss += v * v;
        }
        d = sqrt(ss / (double)K + eps);
        for (k = 0; k < K; ++k)
            out[r * K + k] = (double)bf16_bits_to_float(x[r * ldx + k]) / d * (double)bf16_bits_to_float(w[k]);
    }
}

/* ---------- GEMM: the plain definition ---------------------------------------------- */

/* y[m, n] = sum_{k ascending} a[m, k] * b[n, k] in binary64; a: [M, K], b: [N, K],
 * y: [M, N], all dense row-major.  Both operands have the contraction index contiguous:
 * the blocks of Section 3.3 run along it. */
void nvfp4_ref_gemm_f64(const double *a, const double *b, int64_t M, int64_t N, int64_t K,
                        double *y)
{
    int64_t m;
#pragma omp parallel for schedule(dynamic, 1)
    for (m = 0; m < M; ++m) {
        int64_t n, k;
        for (n = 0; n < N; ++n) {
            double acc = 0.0;
            for (k = 0; k < K; ++k) acc += a[m * K + k] * b[n * K + k];
            y[m * N + n] = acc;
        }
    }
}

/* Euclidean norm of each row of a [rows, K] binary64 matrix (the tolerance of the GEMM
 * comparison is stated relative to ||row|| * ||col||). */
void nvfp4_ref_row_norms(const double *a, int64_t rows, int64_t K, double *out)
{
    int64_t r, k;
#pragma omp parallel for schedule(static) private(k)
    for (r = 0; r < rows; ++r) {
        double s = 0.0;
        for (k = 0; k < K; ++k) s += a[r * K + k] * a[r * K + k];
        out[r] = sqrt(s);
    }
}

/* Element-wise BF16 rounding of a binary64 array. */
void nvfp4_ref_bf16_round_array(const double *v, int64_t n, uint16_t *out)
{
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; ++i) out[i] = nvfp4_ref_bf16_round(v[i]);
}

int nvfp4_ref_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
