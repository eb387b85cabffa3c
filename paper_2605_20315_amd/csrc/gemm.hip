// GEMM kernels for gfx950 (CDNA4): the block-scaled NVFP4 W4A4 product of Section 3.3 and the
// BF16 baseline, Y[M,N] = A[M,K] . B[N,K]^T with FP32 accumulation.
//
// Why the NVFP4 product runs on the 16-bit MFMA: an NVFP4 element is sigma*q with sigma an
// E4M3 value (4 significant bits) and q an E2M1 value (2 significant bits), and sigma changes
// every 16 elements along K with a non-power-of-two mantissa.  CDNA4's scaled FP4/FP8 MFMA
// applies one power-of-two (E8M0) scale per 32 elements, and FP8 operands hold only 4
// significant bits, so neither can carry sigma*q exactly.  sigma*q needs 6 significant bits
// and lies in [2^-10, 2688]: it is exactly representable as a normal FP16 number.  The kernel
// therefore expands each operand tile to FP16 once per workgroup while staging it into LDS
// (v_cvt_scalef32_pk_f16_fp4 gives q*2^8, one packed FP16 multiply by sigma*2^-8 gives
// sigma*q, both exact) and runs v_mfma_f32_32x32x16_f16 on it: every product is exact and the
// only rounding is the FP32 accumulation.  alpha_a*alpha_b is applied once in the epilogue.
//
// Structure shared by both products: 256 threads (4 waves, 2x2), block tile BM x BN x 64,
// two LDS stages (global loads for tile k+1 are issued before the MFMAs of tile k and written
// to the other stage afterwards: one barrier per K step), LDS rows of 128 bytes with the
// 16-byte chunk index XOR-swizzled by (row & 7) so that both the staging writes and the
// 128-bit fragment reads are bank-conflict free, and an XCD-aware, grouped tile order so that
// workgroups running on one XCD share operand tiles in that XCD's L2.
#include <type_traits>

#include "mq_common.h"

namespace mq {

namespace {

constexpr int BK = 64;       // K elements per LDS stage: 64 * 2 bytes = one 128-byte LDS row
constexpr int NT = 256;      // threads per workgroup
constexpr int NUM_XCD = 8;

template <int BM_, int BN_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_;
    static constexpr int WM = BM / 2, WN = BN / 2;  // per-wave tile (waves in a 2x2 grid)
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int STAGE_CHUNKS = (BM + BN) * 8;  // 16-byte chunks per stage
    static constexpr size_t LDS_BYTES = 2ull * STAGE_CHUNKS * 16;
};

__device__ __forceinline__ int swz(int row, int chunk) { return row * 8 + (chunk ^ (row & 7)); }

// ---- operand stagers: global -> registers -> LDS --------------------------------------------

// BF16 operand: R rows x 64 elements per stage; a thread moves 16-byte chunks.
template <int R>
struct Bf16Stager {
    static constexpr int PASSES = R * 8 / NT;
    uint4 regs[PASSES];
    const uint16_t *base;  // first row of this tile
    int64_t ld;
    int rows_left;         // rows of the tile that exist (tail predication)

    __device__ __forceinline__ void init(const void *p, int64_t ld_, int64_t row0, int64_t rows_total)
    {
        ld = ld_;
        base = static_cast<const uint16_t *>(p) + row0 * ld_;
        int64_t left = rows_total - row0;
        rows_left = left > R ? R : (int)left;
    }
    __device__ __forceinline__ void load(int64_t k0)
    {
        const int chunk = threadIdx.x & 7;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = (threadIdx.x >> 3) + p * (NT / 8);
            if (row < rows_left)
                regs[p] = *reinterpret_cast<const uint4 *>(base + row * ld + k0 + chunk * 8);
            else
                regs[p] = make_uint4(0, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void store(uint4 *tile) const
    {
        const int chunk = threadIdx.x & 7;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = (threadIdx.x >> 3) + p * (NT / 8);
            tile[swz(row, chunk)] = regs[p];
        }
    }
};

// NVFP4 operand: R rows x 64 elements per stage = 32 bytes of codes + 4 scale bytes per row.
// A thread takes half a row: 16 bytes of codes (32 elements, two scale blocks) and expands
// them to four 16-byte chunks of FP16.
template <int R>
struct Fp4Stager {
    static constexpr int PASSES = R * 2 / NT;
    uint4 c[PASSES];
    uint32_t sc[PASSES];
    const uint8_t *codes;   // first row of this tile
    const uint8_t *scales;
    int64_t ldc, lds_;      // row strides in bytes: K/2 and K/16
    int rows_left;

    __device__ __forceinline__ void init(const void *pc, const uint8_t *ps, int64_t K, int64_t row0,
                                         int64_t rows_total)
    {
        ldc = K / 2;
        lds_ = K / 16;
        codes = static_cast<const uint8_t *>(pc) + row0 * ldc;
        scales = ps + row0 * lds_;
        int64_t left = rows_total - row0;
        rows_left = left > R ? R : (int)left;
    }
    __device__ __forceinline__ void load(int64_t k0)
    {
        const int half = threadIdx.x & 1;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = (threadIdx.x >> 1) + p * (NT / 2);
            if (row < rows_left) {
                c[p] = *reinterpret_cast<const uint4 *>(codes + row * ldc + k0 / 2 + half * 16);
                sc[p] = *reinterpret_cast<const uint16_t *>(scales + row * lds_ + k0 / 16 + half * 2);
            } else {
                c[p] = make_uint4(0, 0, 0, 0);
                sc[p] = 0;
            }
        }
    }
    // 8 codes (one dword) times one block scale -> 8 FP16 values sigma*q (exact).
    // sigma2 holds sigma*2^-8 twice: an E4M3 byte shifted left by 7 is that FP16 number,
    // subnormal scales included.
    static __device__ __forceinline__ uint4 expand(uint32_t w, uint32_t sigma2)
    {
        const f16x2 s = __builtin_bit_cast(f16x2, sigma2);
        f16x2 h0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 0) * s;
        f16x2 h1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 1) * s;
        f16x2 h2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 2) * s;
        f16x2 h3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 3) * s;
        return make_uint4(__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                          __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3));
    }
    __device__ __forceinline__ void store(uint4 *tile) const
    {
        const int half = threadIdx.x & 1;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = (threadIdx.x >> 1) + p * (NT / 2);
            const uint32_t b0 = (sc[p] & 0xFFu) << 7, b1 = (sc[p] & 0xFF00u) >> 1;
            const uint32_t s0 = b0 | (b0 << 16), s1 = b1 | (b1 << 16);
            tile[swz(row, half * 4 + 0)] = expand(c[p].x, s0);
            tile[swz(row, half * 4 + 1)] = expand(c[p].y, s0);
            tile[swz(row, half * 4 + 2)] = expand(c[p].z, s1);
            tile[swz(row, half * 4 + 3)] = expand(c[p].w, s1);
        }
    }
};

// ---- tile order -----------------------------------------------------------------------------

// Workgroup ids are dealt round-robin to the 8 XCDs.  Give each XCD a contiguous range of
// logical tile ids, then walk tiles in groups of GROUP_M tile rows, column by column, so that
// the tiles resident on one XCD at a time share A row-panels and B column-panels in its L2.
__device__ __forceinline__ void tile_of(int wg, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int xcd = wg % NUM_XCD, idx = wg / NUM_XCD;
    const int per = total / NUM_XCD, rem = total % NUM_XCD;
    const int t = xcd * per + (xcd < rem ? xcd : rem) + idx;
    constexpr int GROUP_M = 8;
    const int group_size = GROUP_M * tiles_n;
    const int g = t / group_size;
    const int first_m = g * GROUP_M;
    const int gm = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    const int in_g = t - g * group_size;
    tm = first_m + in_g % gm;
    tn = in_g / gm;
}

// ---- the kernel -----------------------------------------------------------------------------

template <class C, bool FP4, bool OUT_BF16>
__global__ __launch_bounds__(NT) void gemm_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    extern __shared__ uint4 lds[];
    int tm, tn;
    tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;

    typename std::conditional<FP4, Fp4Stager<C::BM>, Bf16Stager<C::BM>>::type sa;
    typename std::conditional<FP4, Fp4Stager<C::BN>, Bf16Stager<C::BN>>::type sb;
    if constexpr (FP4) {
        sa.init(g.a, g.a_scales, g.K, m0, g.M);
        sb.init(g.b, g.b_scales, g.K, n0, g.N);
    } else {
        sa.init(g.a, g.lda, m0, g.M);
        sb.init(g.b, g.ldb, n0, g.N);
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave >> 1) * C::WM, wn0 = (wave & 1) * C::WN;
    const int frow = lane & 31, fhalf = lane >> 5;

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int KT = (int)(g.K / BK);
    sa.load(0);
    sb.load(0);
    sa.store(lds);
    sb.store(lds + C::BM * 8);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const uint4 *A = lds + (kt & 1) * C::STAGE_CHUNKS;
        const uint4 *B = A + C::BM * 8;
        const bool more = kt + 1 < KT;
        if (more) {
            sa.load((int64_t)(kt + 1) * BK);
            sb.load((int64_t)(kt + 1) * BK);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            uint4 af[C::TM], bf[C::TN];
#pragma unroll
            for (int i = 0; i < C::TM; ++i) af[i] = A[swz(wm0 + i * 32 + frow, ks * 2 + fhalf)];
#pragma unroll
            for (int j = 0; j < C::TN; ++j) bf[j] = B[swz(wn0 + j * 32 + frow, ks * 2 + fhalf)];
#pragma unroll
            for (int i = 0; i < C::TM; ++i)
#pragma unroll
                for (int j = 0; j < C::TN; ++j) {
                    if constexpr (FP4)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            __builtin_bit_cast(f16x8, af[i]), __builtin_bit_cast(f16x8, bf[j]), acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf[j]), acc[i][j], 0, 0, 0);
                }
        }
        if (more) {
            uint4 *An = lds + ((kt + 1) & 1) * C::STAGE_CHUNKS;
            sa.store(An);
            sb.store(An + C::BM * 8);
        }
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4,
    // column lane%32.
    float scale = 1.0f;
    if constexpr (FP4) scale = (*g.a_alpha) * (*g.b_alpha);
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j) {
            const int64_t n = n0 + wn0 + j * 32 + frow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm0 + i * 32 + 8 * (r / 4) + 4 * fhalf + (r % 4);
                if (m < g.M && n < g.N) {
                    const float v = acc[i][j][r] * scale;
                    if constexpr (OUT_BF16)
                        static_cast<__bf16 *>(g.y)[m * g.ldy + n] = (__bf16)v;
                    else
                        static_cast<float *>(g.y)[m * g.ldy + n] = v;
                }
            }
        }
}

// ---- fallback for K not a multiple of 64: one thread per output, exact products ---------------

__device__ __forceinline__ float e2m1_f32(uint32_t c)
{
    const uint32_t m = c & 7u;
    float v = (m >= 2u) ? __uint_as_float((((m >> 1) + 126u) << 23) | ((m & 1u) << 22)) : 0.5f * (float)m;
    return (c & 8u) ? -v : v;
}

template <bool FP4, bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmArgs g)
{
    const int64_t n = (int64_t)blockIdx.x * 16 + (threadIdx.x & 15);
    const int64_t m = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4);
    if (m >= g.M || n >= g.N) return;
    float acc = 0.0f;
    if constexpr (FP4) {
        const uint8_t *ac = static_cast<const uint8_t *>(g.a) + m * (g.K / 2);
        const uint8_t *bc = static_cast<const uint8_t *>(g.b) + n * (g.K / 2);
        const uint8_t *as = g.a_scales + m * (g.K / 16), *bs = g.b_scales + n * (g.K / 16);
        for (int64_t b = 0; b < g.K / 16; ++b) {
            float dot = 0.0f;  // sum of 16 products q*q: multiples of 1/4 up to 576, exact
            for (int i = 0; i < 8; ++i) {
                const uint32_t x = ac[b * 8 + i], w = bc[b * 8 + i];
                dot += e2m1_f32(x & 15u) * e2m1_f32(w & 15u);
                dot += e2m1_f32(x >> 4) * e2m1_f32(w >> 4);
            }
            const float sx = __builtin_amdgcn_cvt_pk_f32_fp8((int)as[b], false)[0];
            const float sw = __builtin_amdgcn_cvt_pk_f32_fp8((int)bs[b], false)[0];
            acc += (sx * sw) * dot;
        }
        acc *= (*g.a_alpha) * (*g.b_alpha);
    } else {
        const uint16_t *a = static_cast<const uint16_t *>(g.a) + m * g.lda;
        const uint16_t *b = static_cast<const uint16_t *>(g.b) + n * g.ldb;
        for (int64_t k = 0; k < g.K; ++k)
            acc += __uint_as_float((uint32_t)a[k] << 16) * __uint_as_float((uint32_t)b[k] << 16);
    }
    if constexpr (OUT_BF16)
        static_cast<__bf16 *>(g.y)[m * g.ldy + n] = (__bf16)acc;
    else
        static_cast<float *>(g.y)[m * g.ldy + n] = acc;
}

template <class C, bool FP4, bool OUT_BF16>
int launch_tiled(const GemmArgs &g, hipStream_t s)
{
    static bool configured = false;
    auto kern = gemm_kernel<C, FP4, OUT_BF16>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        if (e != hipSuccess) return note_launch(e);
        configured = true;
    }
    const int64_t tiles_m = (g.M + C::BM - 1) / C::BM, tiles_n = (g.N + C::BN - 1) / C::BN;
    if (tiles_m * tiles_n > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(NT), C::LDS_BYTES, s>>>(g, (int)tiles_m, (int)tiles_n);
    return note_launch(hipGetLastError());
}

template <bool FP4, bool OUT_BF16>
int launch_any(const GemmArgs &g, hipStream_t s)
{
    if (g.M == 0 || g.N == 0) return MQ_OK;
    if (g.K % BK != 0) {
        dim3 grid((unsigned)((g.N + 15) / 16), (unsigned)((g.M + 15) / 16));
        if ((g.M + 15) / 16 > 65535) return MQ_ERR_SHAPE;
        gemm_simple_kernel<FP4, OUT_BF16><<<grid, dim3(256), 0, s>>>(g);
        return note_launch(hipGetLastError());
    }
    // Large tiles once they fill the 256 CUs at least twice; smaller tiles below that.
    const int64_t big_tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big_tiles >= 512) return launch_tiled<Cfg<256, 256>, FP4, OUT_BF16>(g, s);
    return launch_tiled<Cfg<128, 128>, FP4, OUT_BF16>(g, s);
}

}  // namespace

int launch_gemm_fp4(const GemmArgs &g, hipStream_t s)
{
    return g.out == MQ_OUT_BF16 ? launch_any<true, true>(g, s) : launch_any<true, false>(g, s);
}

int launch_gemm_bf16(const GemmArgs &g, hipStream_t s)
{
    return g.out == MQ_OUT_BF16 ? launch_any<false, true>(g, s) : launch_any<false, false>(g, s);
}

}  // namespace mq
