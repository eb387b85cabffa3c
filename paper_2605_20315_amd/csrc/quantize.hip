// NVFP4 quantizer kernels for gfx950: Eq. 2 (block scale) then Eq. 1 (element codes) of
// Section 3.3, plus the amax-based tensor-level scale.
//
// The quantizer is HBM-bound: per element it reads 2 bytes (BF16) and writes 0.5 byte of
// codes and 1/16 byte of scale.  One lane owns one 16-element block: two 128-bit loads, a
// packed 16-bit integer max for the block amax (|x| of a BF16 is its low 15 bits, and for
// non-NaN values integer order equals magnitude order), two IEEE binary32 divisions per
// block, then one multiply per element and one hardware FP32->FP4 pack per element pair.
//
// Hardware conversions used, with the behaviour measured on gfx950:
//   v_cvt_pk_fp8_f32           OCP E4M3, nearest-even, gradual underflow; overflow gives the
//                              NaN byte, so the argument is clamped to 448 first (exact).
//   v_cvt_pk_f32_fp8           exact decode of all 256 bytes.
//   v_cvt_scalef32_pk_fp4_f32  nearest-even onto the E2M1 grid, clips to +-6, keeps the sign
//                              of zero; first source -> low nibble, second -> high nibble of
//                              the selected byte; only the exponent of its scale operand is
//                              used, so the scale is passed as 1.0 and the multiply by
//                              1/(alpha*sigma) is done beforehand in FP32.
#include "mq_common.h"

namespace mq {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ uint32_t amax16_bits(uint4 v0, uint4 v1)
{
    const uint32_t m = 0x7FFF7FFFu;
    u16x2 a = __builtin_bit_cast(u16x2, v0.x & m);
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v0.y & m));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v0.z & m));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v0.w & m));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v1.x & m));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v1.y & m));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v1.z & m));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v1.w & m));
    uint32_t lo = a[0], hi = a[1];
    return lo > hi ? lo : hi;
}

// Two BF16 in one dword (element 2i low, 2i+1 high) -> one byte of two E2M1 codes written
// into byte `SEL` of `packed`.
template <int SEL>
__device__ __forceinline__ uint32_t pack_pair(uint32_t packed, uint32_t w, float r)
{
    float y0 = __uint_as_float(w << 16) * r;          // Eq. 1 argument, element 2i
    float y1 = __uint_as_float(w & 0xFFFF0000u) * r;  // element 2i+1
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, y0, y1, 1.0f, SEL);
}

// Eq. 2 then Eq. 1 for one block of 16 BF16 values (v0: elements 0..7, v1: 8..15, two per dword):
// scale byte and two dwords of packed codes.  Every step IEEE binary32, nearest-even, unfused.
__device__ __forceinline__ void quantize_block16(uint4 v0, uint4 v1, float alpha, float d6, uint32_t &c0,
                                                 uint32_t &c1, int &sb)
{
    const float amax = __uint_as_float(amax16_bits(v0, v1) << 16);
    float s = amax / d6;                                     // Eq. 2 argument (IEEE division)
    s = fminf(s, 448.0f);                                    // saturation of Pi_E4M3
    sb = __builtin_amdgcn_cvt_pk_fp8_f32(s, 0.0f, 0, false) & 0xFF;  // Pi_E4M3
    const float sigma = __builtin_amdgcn_cvt_pk_f32_fp8(sb, false)[0];
    const float t = alpha * sigma;
    const float r = (sigma == 0.0f) ? 0.0f : 1.0f / t;       // IEEE division
    c0 = c1 = 0;
    c0 = pack_pair<0>(c0, v0.x, r);
    c0 = pack_pair<1>(c0, v0.y, r);
    c0 = pack_pair<2>(c0, v0.z, r);
    c0 = pack_pair<3>(c0, v0.w, r);
    c1 = pack_pair<0>(c1, v1.x, r);
    c1 = pack_pair<1>(c1, v1.y, r);
    c1 = pack_pair<2>(c1, v1.z, r);
    c1 = pack_pair<3>(c1, v1.w, r);
}

// ---- where a block's 16 BF16 values come from ---------------------------------------------------

// The tensor itself.
struct PlainSrc {
    const uint16_t *x;
    int64_t ldx;
    __device__ __forceinline__ void load(int64_t row, int64_t col, uint4 &v0, uint4 &v1) const
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(x + row * ldx + col);
        v0 = src[0];
        v1 = src[1];
    }
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)  // nearest-even, element 2i in the low half
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// The gated-MLP activation silu(gate) * up of a [rows, 2K] tensor (gate = columns [0, K), up =
// columns [K, 2K)), computed in binary32 and rounded once to BF16: the tensor an unfused
// pipeline would have stored and read back.  silu(g) = g / (1 + exp(-g)) with the hardware
// exponential (about 1 ulp: far inside half a BF16 ulp except within 1e-4 of a rounding
// boundary) and an IEEE division, which keeps the tiny quotients of strongly negative gates
// (the approximate reciprocal flushes them to zero).  Below about -88 exp(-g) overflows and the
// result is -0.  p, when not null, receives the BF16 values (checking aid).
struct SiluMulSrc {
    const uint16_t *gu;
    int64_t ld, K;
    uint16_t *p;
    int64_t ldp;
    static __device__ __forceinline__ uint32_t pair(uint32_t g, uint32_t u)
    {
        const float g0 = __uint_as_float(g << 16), g1 = __uint_as_float(g & 0xFFFF0000u);
        const float u0 = __uint_as_float(u << 16), u1 = __uint_as_float(u & 0xFFFF0000u);
        const float s0 = g0 / (1.0f + __expf(-g0));
        const float s1 = g1 / (1.0f + __expf(-g1));
        return pack_bf16(s0 * u0, s1 * u1);
    }
    __device__ __forceinline__ void load(int64_t row, int64_t col, uint4 &v0, uint4 &v1) const
    {
        const uint4 *gs = reinterpret_cast<const uint4 *>(gu + row * ld + col);
        const uint4 *us = reinterpret_cast<const uint4 *>(gu + row * ld + K + col);
        const uint4 g0 = gs[0], g1 = gs[1], u0 = us[0], u1 = us[1];
        v0 = make_uint4(pair(g0.x, u0.x), pair(g0.y, u0.y), pair(g0.z, u0.z), pair(g0.w, u0.w));
        v1 = make_uint4(pair(g1.x, u1.x), pair(g1.y, u1.y), pair(g1.z, u1.z), pair(g1.w, u1.w));
        if (p) {
            uint4 *dst = reinterpret_cast<uint4 *>(p + row * ldp + col);
            dst[0] = v0;
            dst[1] = v1;
        }
    }
};

// One lane per 16-element block, canonical (linear) output.
template <class Src>
__global__ __launch_bounds__(kThreads) void quantize_kernel(Src src, int64_t total_blocks, int blocks_per_row,
                                                            const float *__restrict__ alpha_p,
                                                            uint8_t *__restrict__ codes,
                                                            uint8_t *__restrict__ scales)
{
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (g >= total_blocks) return;
    const float alpha = *alpha_p;
    const float d6 = 6.0f * alpha;  // alpha * q_max
    const int64_t row = g / blocks_per_row;
    const int64_t b = g - row * blocks_per_row;
    uint4 v0, v1;
    src.load(row, b * kBlock, v0, v1);
    uint32_t c0, c1;
    int sb;
    quantize_block16(v0, v1, alpha, d6, c0, c1, sb);
    reinterpret_cast<uint2 *>(codes)[g] = make_uint2(c0, c1);  // dense [rows, K/2]: 8 bytes per block
    scales[g] = (uint8_t)sb;                                   // dense [rows, K/16]
}

// K-step-major output: the code and scale bytes of one 64-wide K step are contiguous over rows.
// A workgroup covers 16 rows x 16 K steps.  Reading: each wave takes four of the rows in turn,
// 2 KB contiguous per row (lane l: K step l/4, block l%4).  The codes and scale bytes go through
// LDS so that writing is contiguous too: per K step 16 rows x 32 code bytes = 512 bytes and
// 16 x 4 scale bytes = 64 bytes.
constexpr int T_STRIDE = 16 * 4 + 4;  // uint2 units per K step in LDS, padded against bank conflicts

// Second half of the transposition: thread (K step ot, row orow) writes one unit of 32 + 4 bytes.
__device__ __forceinline__ void write_ktile_unit(const uint2 *lc, const uint8_t (*ls)[16][4], int t0, int64_t r0,
                                                 int ksteps, int64_t rows, uint8_t *codes, uint8_t *scales)
{
    const int ot = (threadIdx.x >> 4) & 15, orow = threadIdx.x & 15;  // 256 consecutive threads: one unit each
    if (t0 + ot < ksteps && r0 + orow < rows) {
        const int64_t slot = (int64_t)(t0 + ot) * rows + r0 + orow;
        const uint2 *p = &lc[ot * T_STRIDE + orow * 4];
        reinterpret_cast<uint4 *>(codes)[slot * 2] = make_uint4(p[0].x, p[0].y, p[1].x, p[1].y);
        reinterpret_cast<uint4 *>(codes)[slot * 2 + 1] = make_uint4(p[2].x, p[2].y, p[3].x, p[3].y);
        reinterpret_cast<uint32_t *>(scales)[slot] = *reinterpret_cast<const uint32_t *>(&ls[ot][orow][0]);
    }
}

template <class Src>
__global__ __launch_bounds__(kThreads) void quantize_ktile_kernel(Src src, int64_t rows, int64_t row_base,
                                                                  int ksteps, const float *__restrict__ alpha_p,
                                                                  uint8_t *__restrict__ codes,
                                                                  uint8_t *__restrict__ scales)
{
    __shared__ uint2 lc[16 * T_STRIDE];  // [K step][row][block]
    __shared__ uint8_t ls[16][16][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * 16;
    const int64_t r0 = row_base + (int64_t)blockIdx.y * 16;
    const float alpha = *alpha_p;
    const float d6 = 6.0f * alpha;
    const int tl = lane >> 2, blk = lane & 3;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int rl = wave * 4 + it;
        const int64_t row = r0 + rl;
        if (row < rows && t0 + tl < ksteps) {
            uint4 v0, v1;
            src.load(row, (int64_t)(t0 + tl) * 64 + blk * kBlock, v0, v1);
            uint32_t c0, c1;
            int sb;
            quantize_block16(v0, v1, alpha, d6, c0, c1, sb);
            lc[tl * T_STRIDE + rl * 4 + blk] = make_uint2(c0, c1);
            ls[tl][rl][blk] = (uint8_t)sb;
        }
    }
    __syncthreads();
    write_ktile_unit(lc, ls, t0, r0, ksteps, rows, codes, scales);
}

// ---- RMS normalisation fused with the quantizer ----------------------------------------------

// y[r, k] = x[r, k] / sqrt(mean_k x[r, :]^2 + eps) * w[k] in binary32 (sum of squares: each lane
// adds its elements in ascending k, then a butterfly over the wave), rounded once to BF16, then
// quantized as above.  A workgroup of 16 waves owns 16 rows and all of K, one wave per row, so a
// row's sum is a reduction over one wave.  Lane l takes K step c*16 + l/4, block l%4 of chunk c
// (16 K steps = 1024 columns), as in the K-step-major quantizer.
// NC > 0: the row (NC chunks: 8 registers each) stays in registers between the two passes, so x
// is read once; NC == 0: any K, x is read again in the second pass (from cache).
// y_out, when not null, receives the BF16 values (checking aid).
constexpr int kRmsThreads = 1024;

template <int NC, bool KTILE_OUT>
__global__ __launch_bounds__(kRmsThreads) void rmsnorm_quantize_kernel(const uint16_t *__restrict__ x, int64_t rows,
                                                                       int ksteps, int64_t ldx,
                                                                       const uint16_t *__restrict__ w, float eps,
                                                                       float inv_k,
                                                                       const float *__restrict__ alpha_p,
                                                                       uint8_t *__restrict__ codes,
                                                                       uint8_t *__restrict__ scales,
                                                                       uint16_t *__restrict__ y_out, int64_t ldy)
{
    constexpr int NCR = NC > 0 ? NC : 1;
    // K-step-major output: NC > 0 stages all chunks and synchronises once, NC == 0 chunk by chunk
    __shared__ uint2 lc[NCR][16 * T_STRIDE];
    __shared__ uint8_t ls[NCR][16][16][4];
    const int lane = threadIdx.x & 63, rl = threadIdx.x >> 6;  // rl: row within the group = wave
    const int64_t r0 = (int64_t)blockIdx.x * 16, row = r0 + rl;
    const bool row_ok = row < rows;
    const float alpha = *alpha_p;
    const float d6 = 6.0f * alpha;
    const int tl = lane >> 2, blk = lane & 3;
    const int chunks = (ksteps + 15) / 16;
    const PlainSrc src{x, ldx};

    auto sumsq = [](uint4 v0, uint4 v1) {
        const uint32_t d[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float a = __uint_as_float(d[i] << 16), b = __uint_as_float(d[i] & 0xFFFF0000u);
            s += a * a;
            s += b * b;
        }
        return s;
    };
    uint4 keep[NCR][2];
    float ss = 0.0f;
    if constexpr (NC > 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int t = c * 16 + tl;
            uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
            if (row_ok && t < ksteps) src.load(row, (int64_t)t * 64 + blk * kBlock, v0, v1);
            keep[c][0] = v0;
            keep[c][1] = v1;
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) ss += sumsq(keep[c][0], keep[c][1]);
    } else {
        for (int c = 0; c < chunks; ++c) {
            const int t = c * 16 + tl;
            if (row_ok && t < ksteps) {
                uint4 v0, v1;
                src.load(row, (int64_t)t * 64 + blk * kBlock, v0, v1);
                ss += sumsq(v0, v1);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    // IEEE square root and division, once per row (the approximate reciprocal square root moved
    // two orders of magnitude more elements across a BF16 rounding boundary than these do)
    const float iv = 1.0f / __fsqrt_rn(ss * inv_k + eps);

    auto norm_pair = [](uint32_t xv, uint32_t wv, float inv) {
        const float a = __uint_as_float(xv << 16) * inv, b = __uint_as_float(xv & 0xFFFF0000u) * inv;
        return pack_bf16(a * __uint_as_float(wv << 16), b * __uint_as_float(wv & 0xFFFF0000u));
    };
    auto chunk = [&](int c, uint4 x0, uint4 x1) {
        const int t = c * 16 + tl;
        if (row_ok && t < ksteps) {
            const uint4 *ws = reinterpret_cast<const uint4 *>(w + (int64_t)t * 64 + blk * kBlock);
            const uint4 w0 = ws[0], w1 = ws[1];
            const uint4 v0 = make_uint4(norm_pair(x0.x, w0.x, iv), norm_pair(x0.y, w0.y, iv),
                                        norm_pair(x0.z, w0.z, iv), norm_pair(x0.w, w0.w, iv));
            const uint4 v1 = make_uint4(norm_pair(x1.x, w1.x, iv), norm_pair(x1.y, w1.y, iv),
                                        norm_pair(x1.z, w1.z, iv), norm_pair(x1.w, w1.w, iv));
            if (y_out) {
                uint4 *dst = reinterpret_cast<uint4 *>(y_out + row * ldy + (int64_t)t * 64 + blk * kBlock);
                dst[0] = v0;
                dst[1] = v1;
            }
            uint32_t c0, c1;
            int sb;
            quantize_block16(v0, v1, alpha, d6, c0, c1, sb);
            if constexpr (KTILE_OUT) {
                const int slot = NC > 0 ? c : 0;
                lc[slot][tl * T_STRIDE + rl * 4 + blk] = make_uint2(c0, c1);
                ls[slot][tl][rl][blk] = (uint8_t)sb;
            } else {
                const int64_t g = row * ((int64_t)ksteps * 4) + (int64_t)t * 4 + blk;
                reinterpret_cast<uint2 *>(codes)[g] = make_uint2(c0, c1);
                scales[g] = (uint8_t)sb;
            }
        }
        if constexpr (KTILE_OUT && NC == 0) {
            __syncthreads();
            if (threadIdx.x < 256) write_ktile_unit(lc[0], ls[0], c * 16, r0, ksteps, rows, codes, scales);
            __syncthreads();
        }
    };
    if constexpr (NC > 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (c < chunks) chunk(c, keep[c][0], keep[c][1]);  // uniform
        if constexpr (KTILE_OUT) {
            __syncthreads();
#pragma unroll
            for (int c = (int)(threadIdx.x >> 8); c < NC; c += kRmsThreads / 256)
                if (c < chunks) write_ktile_unit(lc[c], ls[c], c * 16, r0, ksteps, rows, codes, scales);
        }
    } else {
        for (int c = 0; c < chunks; ++c) {
            const int t = c * 16 + tl;
            uint4 x0 = make_uint4(0, 0, 0, 0), x1 = x0;
            if (row_ok && t < ksteps) src.load(row, (int64_t)t * 64 + blk * kBlock, x0, x1);
            chunk(c, x0, x1);
        }
    }
}

// Byte permutation between the two layouts of an NVFP4 tensor (offline weight pre-pack).
// One thread moves one (row, K step) unit: 32 code bytes and 4 scale bytes.
__global__ __launch_bounds__(kThreads) void relayout_kernel(const uint8_t *__restrict__ src_c,
                                                            const uint8_t *__restrict__ src_s,
                                                            uint8_t *__restrict__ dst_c, uint8_t *__restrict__ dst_s,
                                                            int64_t rows, int64_t ksteps, bool to_ktile)
{
    const int64_t u = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // K-step-major unit index
    if (u >= rows * ksteps) return;
    const int64_t t = u / rows, r = u - t * rows;
    const int64_t lin = r * ksteps + t;                              // row-major unit index
    const int64_t from = to_ktile ? lin : u, to = to_ktile ? u : lin;
    const uint4 c0 = reinterpret_cast<const uint4 *>(src_c)[from * 2];
    const uint4 c1 = reinterpret_cast<const uint4 *>(src_c)[from * 2 + 1];
    const uint32_t sc = reinterpret_cast<const uint32_t *>(src_s)[from];
    reinterpret_cast<uint4 *>(dst_c)[to * 2] = c0;
    reinterpret_cast<uint4 *>(dst_c)[to * 2 + 1] = c1;
    reinterpret_cast<uint32_t *>(dst_s)[to] = sc;
}

// ---- tensor-level scale ------------------------------------------------------------------

__global__ void amax_init_kernel(uint32_t *acc) { *acc = 0u; }

__device__ __forceinline__ uint32_t amax8_bits(uint4 v)
{
    const uint32_t k = 0x7FFF7FFFu;
    u16x2 a = __builtin_bit_cast(u16x2, v.x & k);
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v.y & k));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v.z & k));
    a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, v.w & k));
    uint32_t lo = a[0], hi = a[1];
    return lo > hi ? lo : hi;
}

// Largest |x| of the tensor as BF16 bits, folded into *acc with one atomic per workgroup.  At
// most one workgroup of 1024 threads per compute unit, each reading one contiguous share of the
// tensor with four 16-byte loads in flight per thread: atomics on a single address serialise in
// L2, and with 2048 workgroups they cost more than the read itself (measured on [8192, 4096]:
// 30.7 us with 2048 atomics, 13.4 us for the same reads without any, 14.5 us with 256).
// CONTIG: ldx == K.
constexpr int kAmaxThreads = 1024;

template <bool CONTIG>
__global__ __launch_bounds__(kAmaxThreads) void amax_kernel(const uint16_t *__restrict__ x, int64_t total_chunks,
                                                            int chunks_per_row, int64_t ldx, uint32_t *acc)
{
    const int64_t per = (total_chunks + gridDim.x - 1) / gridDim.x;
    const int64_t b0 = (int64_t)blockIdx.x * per, b1 = b0 + per < total_chunks ? b0 + per : total_chunks;
    uint32_t m = 0;
    auto addr = [&](int64_t c) -> const uint4 * {
        if (CONTIG) return reinterpret_cast<const uint4 *>(x) + c;
        const int64_t row = c / chunks_per_row;
        return reinterpret_cast<const uint4 *>(x + row * ldx) + (c - row * chunks_per_row);
    };
    constexpr int64_t T = kAmaxThreads;
    int64_t c = b0 + threadIdx.x;
    for (; c + 3 * T < b1; c += 4 * T) {
        const uint4 v0 = *addr(c), v1 = *addr(c + T), v2 = *addr(c + 2 * T), v3 = *addr(c + 3 * T);
        uint32_t t0 = amax8_bits(v0), t1 = amax8_bits(v1), t2 = amax8_bits(v2), t3 = amax8_bits(v3);
        t0 = t0 > t1 ? t0 : t1;
        t2 = t2 > t3 ? t2 : t3;
        t0 = t0 > t2 ? t0 : t2;
        m = m > t0 ? m : t0;
    }
    for (; c < b1; c += T) {
        const uint32_t t = amax8_bits(*addr(c));
        m = m > t ? m : t;
    }
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = __shfl_xor(m, off);
        m = o > m ? o : m;
    }
    __shared__ uint32_t wave_max[kAmaxThreads / 64];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kAmaxThreads / 64; ++w) m = wave_max[w] > m ? wave_max[w] : m;
        if (m != 0) atomicMax(acc, m);
    }
}

// *acc holds the largest |x| as BF16 bits; overwrite it with alpha = amax / (6 * 448).
__global__ void amax_final_kernel(uint32_t *acc)
{
    const float amax = __uint_as_float(*acc << 16);
    const float alpha = (amax == 0.0f) ? 1.0f : amax / 2688.0f;
    *reinterpret_cast<float *>(acc) = alpha;
}

}  // namespace

namespace {

template <class Src>
int launch_quantize_from(const Src &src, int64_t rows, int64_t K, const float *alpha, uint8_t *codes,
                         uint8_t *scales, int layout, hipStream_t s)
{
    const int64_t bpr = K / kBlock;
    const int64_t total = rows * bpr;
    if (total == 0) return MQ_OK;
    if (layout == MQ_LAYOUT_KTILE) {
        const int64_t ksteps = K / 64, gy = (rows + 15) / 16;
        // grid.y is limited to 65535: fold the excess row groups into extra launches
        for (int64_t y0 = 0; y0 < gy; y0 += 65535) {
            const int64_t ny = gy - y0 < 65535 ? gy - y0 : 65535;
            quantize_ktile_kernel<Src><<<dim3((unsigned)((ksteps + 15) / 16), (unsigned)ny), dim3(kThreads), 0, s>>>(
                src, rows, y0 * 16, (int)ksteps, alpha, codes, scales);
            int rc = note_launch(hipGetLastError());
            if (rc != MQ_OK) return rc;
        }
        return MQ_OK;
    }
    const int64_t grid = (total + kThreads - 1) / kThreads;
    if (grid > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    quantize_kernel<Src><<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(src, total, (int)bpr, alpha, codes, scales);
    return note_launch(hipGetLastError());
}

}  // namespace

int launch_quantize(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, const float *alpha,
                    uint8_t *codes, uint8_t *scales, int layout, hipStream_t s)
{
    return launch_quantize_from(PlainSrc{x, ldx}, rows, K, alpha, codes, scales, layout, s);
}

int launch_quantize_silu_mul(const uint16_t *gate_up, int64_t rows, int64_t K, int64_t ld, const float *alpha,
                             uint8_t *codes, uint8_t *scales, int layout, uint16_t *p, int64_t ldp, hipStream_t s)
{
    return launch_quantize_from(SiluMulSrc{gate_up, ld, K, p, ldp}, rows, K, alpha, codes, scales, layout, s);
}

int launch_quantize_rmsnorm(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, const uint16_t *w, float eps,
                            const float *alpha, uint8_t *codes, uint8_t *scales, int layout, uint16_t *y,
                            int64_t ldy, hipStream_t s)
{
    if (rows == 0) return MQ_OK;
    const int64_t groups = (rows + 15) / 16;
    if (groups > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    const int ksteps = (int)(K / 64);
    const float inv_k = 1.0f / (float)K;
    const dim3 grid((unsigned)groups), block(kRmsThreads);
    const bool kt = layout == MQ_LAYOUT_KTILE;
#define MQ_RMS(NC_)                                                                                              \
    (kt ? rmsnorm_quantize_kernel<NC_, true><<<grid, block, 0, s>>>(x, rows, ksteps, ldx, w, eps, inv_k, alpha,  \
                                                                    codes, scales, y, ldy)                      \
        : rmsnorm_quantize_kernel<NC_, false><<<grid, block, 0, s>>>(x, rows, ksteps, ldx, w, eps, inv_k, alpha, \
                                                                     codes, scales, y, ldy))
    if (ksteps <= 64)
        MQ_RMS(4);  // K <= 4096: the row stays in registers (32 per lane)
    else
        MQ_RMS(0);  // (8 chunks in registers spill at 1024 threads per workgroup: measured 2x slower)
#undef MQ_RMS
    return note_launch(hipGetLastError());
}

int launch_relayout(const uint8_t *src_c, const uint8_t *src_s, uint8_t *dst_c, uint8_t *dst_s, int64_t rows,
                    int64_t K, bool to_ktile, hipStream_t s)
{
    const int64_t ksteps = K / 64, units = rows * ksteps;
    if (units == 0) return MQ_OK;
    const int64_t grid = (units + kThreads - 1) / kThreads;
    if (grid > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    relayout_kernel<<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(src_c, src_s, dst_c, dst_s, rows, ksteps, to_ktile);
    return note_launch(hipGetLastError());
}

int launch_global_scale(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, float *alpha,
                        hipStream_t s)
{
    uint32_t *acc = reinterpret_cast<uint32_t *>(alpha);
    amax_init_kernel<<<1, 1, 0, s>>>(acc);
    int rc = note_launch(hipGetLastError());
    if (rc != MQ_OK) return rc;
    if (rows > 0) {
        const int64_t total = rows * (K / 8);
        int64_t grid = (total + kAmaxThreads * 4 - 1) / (kAmaxThreads * 4);
        grid = grid < 1 ? 1 : (grid > 256 ? 256 : grid);   // one workgroup per compute unit
        if (ldx == K)
            amax_kernel<true><<<dim3((unsigned)grid), dim3(kAmaxThreads), 0, s>>>(x, total, (int)(K / 8), ldx, acc);
        else
            amax_kernel<false><<<dim3((unsigned)grid), dim3(kAmaxThreads), 0, s>>>(x, total, (int)(K / 8), ldx, acc);
        rc = note_launch(hipGetLastError());
        if (rc != MQ_OK) return rc;
    }
    amax_final_kernel<<<1, 1, 0, s>>>(acc);
    return note_launch(hipGetLastError());
}

}  // namespace mq
