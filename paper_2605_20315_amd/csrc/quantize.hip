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

// One lane per 16-element block.  CONTIG: ldx == K, so block g starts at element 16*g.
template <bool CONTIG>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const uint16_t *__restrict__ x,
                                                            int64_t total_blocks, int blocks_per_row,
                                                            int64_t ldx,
                                                            const float *__restrict__ alpha_p,
                                                            uint8_t *__restrict__ codes,
                                                            uint8_t *__restrict__ scales)
{
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (g >= total_blocks) return;
    const float alpha = *alpha_p;
    const float d6 = 6.0f * alpha;  // alpha * q_max
    const uint16_t *src;
    if (CONTIG) {
        src = x + g * kBlock;
    } else {
        const int64_t row = g / blocks_per_row;
        const int64_t b = g - row * blocks_per_row;
        src = x + row * ldx + b * kBlock;
    }
    const uint4 v0 = reinterpret_cast<const uint4 *>(src)[0];
    const uint4 v1 = reinterpret_cast<const uint4 *>(src)[1];

    const float amax = __uint_as_float(amax16_bits(v0, v1) << 16);
    float s = amax / d6;                                     // Eq. 2 argument (IEEE division)
    s = fminf(s, 448.0f);                                    // saturation of Pi_E4M3
    const int sb = __builtin_amdgcn_cvt_pk_fp8_f32(s, 0.0f, 0, false) & 0xFF;  // Pi_E4M3
    const float sigma = __builtin_amdgcn_cvt_pk_f32_fp8(sb, false)[0];
    const float t = alpha * sigma;
    const float r = (sigma == 0.0f) ? 0.0f : 1.0f / t;       // IEEE division

    uint32_t c0 = 0, c1 = 0;
    c0 = pack_pair<0>(c0, v0.x, r);
    c0 = pack_pair<1>(c0, v0.y, r);
    c0 = pack_pair<2>(c0, v0.z, r);
    c0 = pack_pair<3>(c0, v0.w, r);
    c1 = pack_pair<0>(c1, v1.x, r);
    c1 = pack_pair<1>(c1, v1.y, r);
    c1 = pack_pair<2>(c1, v1.z, r);
    c1 = pack_pair<3>(c1, v1.w, r);

    reinterpret_cast<uint2 *>(codes)[g] = make_uint2(c0, c1);  // dense [rows, K/2]: 8 bytes per block
    scales[g] = (uint8_t)sb;                                   // dense [rows, K/16]
}

// K-step-major output: the code and scale bytes of one 64-wide K step are contiguous over rows.
// A workgroup covers 16 rows x 16 K steps.  Reading: each wave takes four of the rows in turn,
// 2 KB contiguous per row (lane l: K step l/4, block l%4).  The codes and scale bytes go through
// LDS so that writing is contiguous too: per K step 16 rows x 32 code bytes = 512 bytes and
// 16 x 4 scale bytes = 64 bytes.
__global__ __launch_bounds__(kThreads) void quantize_ktile_kernel(const uint16_t *__restrict__ x, int64_t rows,
                                                                  int64_t row_base, int ksteps, int64_t ldx,
                                                                  const float *__restrict__ alpha_p,
                                                                  uint8_t *__restrict__ codes,
                                                                  uint8_t *__restrict__ scales)
{
    constexpr int T_STRIDE = 16 * 4 + 4;        // uint2 units per K step in LDS, padded against bank conflicts
    __shared__ uint2 lc[16 * T_STRIDE];         // [K step][row][block]
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
            const uint16_t *src = x + row * ldx + (int64_t)(t0 + tl) * 64 + blk * kBlock;
            const uint4 v0 = reinterpret_cast<const uint4 *>(src)[0];
            const uint4 v1 = reinterpret_cast<const uint4 *>(src)[1];
            const float amax = __uint_as_float(amax16_bits(v0, v1) << 16);
            float s = amax / d6;
            s = fminf(s, 448.0f);
            const int sb = __builtin_amdgcn_cvt_pk_fp8_f32(s, 0.0f, 0, false) & 0xFF;
            const float sigma = __builtin_amdgcn_cvt_pk_f32_fp8(sb, false)[0];
            const float tt = alpha * sigma;
            const float r = (sigma == 0.0f) ? 0.0f : 1.0f / tt;
            uint32_t c0 = 0, c1 = 0;
            c0 = pack_pair<0>(c0, v0.x, r);
            c0 = pack_pair<1>(c0, v0.y, r);
            c0 = pack_pair<2>(c0, v0.z, r);
            c0 = pack_pair<3>(c0, v0.w, r);
            c1 = pack_pair<0>(c1, v1.x, r);
            c1 = pack_pair<1>(c1, v1.y, r);
            c1 = pack_pair<2>(c1, v1.z, r);
            c1 = pack_pair<3>(c1, v1.w, r);
            lc[tl * T_STRIDE + rl * 4 + blk] = make_uint2(c0, c1);
            ls[tl][rl][blk] = (uint8_t)sb;
        }
    }
    __syncthreads();
    const int ot = threadIdx.x >> 4, orow = threadIdx.x & 15;   // output unit: (K step, row)
    if (t0 + ot < ksteps && r0 + orow < rows) {
        const int64_t slot = (int64_t)(t0 + ot) * rows + r0 + orow;
        const uint2 *p = &lc[ot * T_STRIDE + orow * 4];
        reinterpret_cast<uint4 *>(codes)[slot * 2] = make_uint4(p[0].x, p[0].y, p[1].x, p[1].y);
        reinterpret_cast<uint4 *>(codes)[slot * 2 + 1] = make_uint4(p[2].x, p[2].y, p[3].x, p[3].y);
        reinterpret_cast<uint32_t *>(scales)[slot] = *reinterpret_cast<const uint32_t *>(&ls[ot][orow][0]);
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

// Largest |x| of the tensor as BF16 bits, folded into *acc with one atomic per wave.  Grid-stride
// over 16-byte chunks, four independent loads in flight per thread.  CONTIG: ldx == K.
template <bool CONTIG>
__global__ __launch_bounds__(kThreads) void amax_kernel(const uint16_t *__restrict__ x, int64_t total_chunks,
                                                        int chunks_per_row, int64_t ldx, uint32_t *acc)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    uint32_t m = 0;
    auto addr = [&](int64_t c) -> const uint4 * {
        if (CONTIG) return reinterpret_cast<const uint4 *>(x) + c;
        const int64_t row = c / chunks_per_row;
        return reinterpret_cast<const uint4 *>(x + row * ldx) + (c - row * chunks_per_row);
    };
    int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    for (; c + 3 * stride < total_chunks; c += 4 * stride) {
        const uint4 v0 = *addr(c), v1 = *addr(c + stride), v2 = *addr(c + 2 * stride), v3 = *addr(c + 3 * stride);
        uint32_t t0 = amax8_bits(v0), t1 = amax8_bits(v1), t2 = amax8_bits(v2), t3 = amax8_bits(v3);
        t0 = t0 > t1 ? t0 : t1;
        t2 = t2 > t3 ? t2 : t3;
        t0 = t0 > t2 ? t0 : t2;
        m = m > t0 ? m : t0;
    }
    for (; c < total_chunks; c += stride) {
        const uint32_t t = amax8_bits(*addr(c));
        m = m > t ? m : t;
    }
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = __shfl_xor(m, off);
        m = o > m ? o : m;
    }
    // one atomic per workgroup: atomics on a single address serialise in L2
    __shared__ uint32_t wave_max[kThreads / 64];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) m = wave_max[w] > m ? wave_max[w] : m;
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

int launch_quantize(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, const float *alpha,
                    uint8_t *codes, uint8_t *scales, int layout, hipStream_t s)
{
    const int64_t bpr = K / kBlock;
    const int64_t total = rows * bpr;
    if (total == 0) return MQ_OK;
    if (layout == MQ_LAYOUT_KTILE) {
        const int64_t ksteps = K / 64, gy = (rows + 15) / 16;
        // grid.y is limited to 65535: fold the excess row groups into extra launches
        for (int64_t y0 = 0; y0 < gy; y0 += 65535) {
            const int64_t ny = gy - y0 < 65535 ? gy - y0 : 65535;
            quantize_ktile_kernel<<<dim3((unsigned)((ksteps + 15) / 16), (unsigned)ny), dim3(kThreads), 0, s>>>(
                x, rows, y0 * 16, (int)ksteps, ldx, alpha, codes, scales);
            int rc = note_launch(hipGetLastError());
            if (rc != MQ_OK) return rc;
        }
        return MQ_OK;
    }
    const int64_t grid = (total + kThreads - 1) / kThreads;
    if (grid > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    if (ldx == K)
        quantize_kernel<true><<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(x, total, (int)bpr, ldx, alpha,
                                                                             codes, scales);
    else
        quantize_kernel<false><<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(x, total, (int)bpr, ldx, alpha,
                                                                              codes, scales);
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
        int64_t grid = (total + kThreads * 4 - 1) / (kThreads * 4);
        grid = grid < 1 ? 1 : (grid > 2048 ? 2048 : grid);   // 8 workgroups per compute unit
        if (ldx == K)
            amax_kernel<true><<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(x, total, (int)(K / 8), ldx, acc);
        else
            amax_kernel<false><<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(x, total, (int)(K / 8), ldx, acc);
        rc = note_launch(hipGetLastError());
        if (rc != MQ_OK) return rc;
    }
    amax_final_kernel<<<1, 1, 0, s>>>(acc);
    return note_launch(hipGetLastError());
}

}  // namespace mq
