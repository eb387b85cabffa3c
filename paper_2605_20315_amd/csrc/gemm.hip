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

// LDS rows are 128 bytes = 8 chunks of 16 bytes.  The LDS serves 128-bit reads 16 lanes at a
// time over 64 four-byte banks (256 bytes per clock), i.e. over two consecutive rows, so the
// chunk index is XOR-ed with bits 1..3 of the row: 16 consecutive rows reading the same logical
// chunk then touch 16 different bank groups.
__device__ __forceinline__ int swz_key(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz(int row, int chunk) { return row * 8 + (chunk ^ swz_key(row)); }

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

// ---- software-pipelined NVFP4 kernel --------------------------------------------------------
//
// Same tiling and LDS layout as gemm_kernel, but with every latency covered inside one wave, since
// a 256x256 tile leaves room for only one wave per SIMD:
//   * a K step of 64 is four MFMA phases of 16; the fragments of phase p+1 are read from LDS
//     into a second register set while the 16 MFMAs of phase p run;
//   * the packed codes of a tile are fetched from global memory two K steps ahead into one of two
//     register sets, and expanded to FP16 and written to the free LDS stage one quarter per
//     phase, between the MFMAs, so the VALU work and the LDS writes hide under the matrix pipe;
//   * one barrier per K step, at the start of phase 3: before it every wave has finished writing
//     tile t+1 and reading tile t; after it tile t's stage is free and receives tile t+2.
// Rows beyond M or N are clamped to the last valid row instead of being zero-filled: they only
// feed outputs that the epilogue does not store.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct PCfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int PA = BM * 2 / THREADS, PB = BN * 2 / THREADS, NP = PA + PB;
    static constexpr int STAGE_CHUNKS = (BM + BN) * 8;
    static constexpr size_t LDS_BYTES = 2ull * STAGE_CHUNKS * 16;
    static_assert(NP == 1 || NP == 2 || NP == 4, "staging parts must divide the four phases");
};

struct Fp4Part {
    uint4 c;       // 32 codes of this thread's half row
    uint32_t sc;   // the row's four E4M3 scale bytes for this K step (both halves)
};

// Scheduling hint: interleave, per MFMA, one LDS read (while any remain), a few VALU
// instructions, and now and then an LDS write / a global load.
template <int MFMAS, int READS, int VALU_PER, int WRITES, int VMEMS>
__device__ __forceinline__ void sched_phase()
{
#pragma unroll
    for (int i = 0; i < MFMAS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                     // MFMA
        if (i < READS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // DS read
        if (VALU_PER > 0) __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);
        if (WRITES > 0 && (i % (MFMAS / WRITES)) == (MFMAS / WRITES) - 1)
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                 // DS write
        if (VMEMS > 0 && i < VMEMS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
    }
    // Nothing moves across a phase boundary: in particular no consumer of a global load is
    // hoisted towards the load, which would turn the prefetch distance into a stall.
    __builtin_amdgcn_sched_barrier(0);
}

template <class C, bool OUT_BF16>
__global__ __launch_bounds__(C::THREADS) void gemm_fp4_pipelined(GemmArgs g, int tiles_m, int tiles_n)
{
    extern __shared__ uint4 lds[];
    int tm, tn;
    tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / C::WAVES_N) * C::WM, wn0 = (wave % C::WAVES_N) * C::WN;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int half = tid & 1;
    const int KT = (int)(g.K / BK);

    // staging: part q of a tile is half a row (32 codes) of operand A (q < PA) or B
    const uint8_t *pc[C::NP];
    const uint8_t *ps[C::NP];
    int wrow[C::NP];  // LDS row (in 16-byte chunks: row * 8) incl. the operand's offset in the stage
    int wx[C::NP];    // the row's swizzle key
#pragma unroll
    for (int q = 0; q < C::NP; ++q) {
        const bool isA = q < C::PA;
        const int r = (tid >> 1) + (isA ? q : q - C::PA) * (C::THREADS / 2);
        const int64_t total = isA ? g.M : g.N, row0 = isA ? m0 : n0;
        int64_t grow = row0 + r;
        grow = grow < total ? grow : total - 1;
        pc[q] = static_cast<const uint8_t *>(isA ? g.a : g.b) + grow * (g.K / 2) + half * 16;
        ps[q] = (isA ? g.a_scales : g.b_scales) + grow * (g.K / 16);
        wrow[q] = (isA ? 0 : C::BM * 8) + r * 8;
        wx[q] = swz_key(r);
    }
    Fp4Part st[2][C::NP];
    auto load_tile = [&](int t, Fp4Part(&s)[C::NP]) {
        t = t < KT ? t : KT - 1;
#pragma unroll
        for (int q = 0; q < C::NP; ++q) {
            s[q].c = *reinterpret_cast<const uint4 *>(pc[q] + (int64_t)t * (BK / 2));
            s[q].sc = *reinterpret_cast<const uint32_t *>(ps[q] + (int64_t)t * (BK / 16));
        }
    };
    auto store_part = [&](int q, Fp4Part p, uint4 *stage) {
        // Pin the first use of the prefetched registers to this point of the program: without
        // it the compiler sinks cheap consumers of the loads to the loop header, right behind
        // the loads themselves, and the wait for them lands two phases too early.
        asm volatile("" : "+v"(p.c.x), "+v"(p.c.y), "+v"(p.c.z), "+v"(p.c.w), "+v"(p.sc));
        const uint32_t two = p.sc >> (half * 16);
        const uint32_t b0 = (two & 0xFFu) << 7, b1 = (two & 0xFF00u) >> 1;
        const uint32_t s0 = b0 | (b0 << 16), s1 = b1 | (b1 << 16);
        uint4 *row = stage + wrow[q];
        row[(half * 4 + 0) ^ wx[q]] = Fp4Stager<256>::expand(p.c.x, s0);
        row[(half * 4 + 1) ^ wx[q]] = Fp4Stager<256>::expand(p.c.y, s0);
        row[(half * 4 + 2) ^ wx[q]] = Fp4Stager<256>::expand(p.c.z, s1);
        row[(half * 4 + 3) ^ wx[q]] = Fp4Stager<256>::expand(p.c.w, s1);
    };
    // parts handled in rotating slot `slot` (0: phase 3 of the previous K step, 1..3: phases 0..2)
    auto store_slot = [&](int slot, const Fp4Part(&s)[C::NP], uint4 *stage) {
#pragma unroll
        for (int q = 0; q < C::NP; ++q)
            if (q * 4 / C::NP == slot && (q * 4) % C::NP == 0) store_part(q, s[q], stage);
    };

    // fragment addresses: one per phase, the 32-row tiles of a wave are 4096 bytes apart
    int fa[4], fb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        fa[ks] = (wm0 + frow) * 8 + ((ks * 2 + fhalf) ^ swz_key(frow));
        fb[ks] = (C::BM + wn0 + frow) * 8 + ((ks * 2 + fhalf) ^ swz_key(frow));
    }
    uint4 fra[2][C::TM], frb[2][C::TN];
    auto read_frags = [&](const uint4 *stage, int ks, uint4(&a)[C::TM], uint4(&b)[C::TN]) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i) a[i] = stage[fa[ks] + i * 256];
#pragma unroll
        for (int j = 0; j < C::TN; ++j) b[j] = stage[fb[ks] + j * 256];
    };

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    auto mfmas = [&](const uint4(&a)[C::TM], const uint4(&b)[C::TN]) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(f16x8, a[i]), __builtin_bit_cast(f16x8, b[j]), acc[i][j], 0, 0, 0);
    };

    constexpr int NMFMA = C::TM * C::TN, NREAD = C::TM + C::TN;
    constexpr int SLOT_WRITES = C::NP >= 4 ? 4 : 0;  // LDS writes per phase when every phase stores a part
    uint4 *stage0 = lds, *stage1 = lds + C::STAGE_CHUNKS;

    // prologue
    load_tile(0, st[0]);
    load_tile(1, st[1]);
#pragma unroll
    for (int q = 0; q < C::NP; ++q) store_part(q, st[0][q], stage0);
    store_slot(0, st[1], stage1);
    load_tile(2, st[0]);
    __syncthreads();
    read_frags(stage0, 0, fra[0], frb[0]);

    // one K step; PAR = parity of kt (stage and register-set indices must be compile-time)
    auto kstep = [&](int kt, auto par) {
        constexpr int PAR = decltype(par)::value;
        uint4 *cur = PAR ? stage1 : stage0, *nxt = PAR ? stage0 : stage1;
        Fp4Part(&s_next)[C::NP] = st[PAR ^ 1];  // tile kt+1, later refilled with tile kt+3
        Fp4Part(&s_cur)[C::NP] = st[PAR];       // tile kt+2
        // phase 0
        read_frags(cur, 1, fra[1], frb[1]);
        store_slot(1, s_next, nxt);
        mfmas(fra[0], frb[0]);
        sched_phase<NMFMA, NREAD, 3, SLOT_WRITES, 0>();
        // phase 1
        read_frags(cur, 2, fra[0], frb[0]);
        store_slot(2, s_next, nxt);
        mfmas(fra[1], frb[1]);
        sched_phase<NMFMA, NREAD, 3, (C::NP >= 2 ? 4 : 0), 0>();
        // phase 2
        read_frags(cur, 3, fra[1], frb[1]);
        store_slot(3, s_next, nxt);
        mfmas(fra[0], frb[0]);
        sched_phase<NMFMA, NREAD, 3, SLOT_WRITES, 0>();
        // phase 3
        __syncthreads();
        read_frags(nxt, 0, fra[0], frb[0]);
        store_slot(0, s_cur, cur);
        load_tile(kt + 3, s_next);
        mfmas(fra[1], frb[1]);
        sched_phase<NMFMA, NREAD, 3, 4, 2 * C::NP>();
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
        kstep(kt, std::integral_constant<int, 0>{});
        kstep(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) kstep(kt, std::integral_constant<int, 0>{});

    const float scale = (*g.a_alpha) * (*g.b_alpha);
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

template <class C, bool OUT_BF16>
int launch_pipelined(const GemmArgs &g, hipStream_t s)
{
    static bool configured = false;
    auto kern = gemm_fp4_pipelined<C, OUT_BF16>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        if (e != hipSuccess) return note_launch(e);
        configured = true;
    }
    const int64_t tiles_m = (g.M + C::BM - 1) / C::BM, tiles_n = (g.N + C::BN - 1) / C::BN;
    if (tiles_m * tiles_n > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(C::THREADS), C::LDS_BYTES, s>>>(g, (int)tiles_m, (int)tiles_n);
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
    if constexpr (FP4) {
        if (big_tiles >= 512) return launch_pipelined<PCfg<256, 256, 2, 2>, OUT_BF16>(g, s);
        return launch_pipelined<PCfg<128, 128, 2, 2>, OUT_BF16>(g, s);
    }
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
