// GEMM kernels for gfx950 (CDNA4): the block-scaled NVFP4 W4A4 product of Section 3.3 and the
// BF16 baseline, Y[M,N] = A[M,K] . B[N,K]^T with FP32 accumulation.
//
// Why the NVFP4 product runs on the 16-bit MFMA: an NVFP4 element is sigma*q with sigma an
// E4M3 value (4 significant bits) and q an E2M1 value (2 significant bits), and sigma changes
// every 16 elements along K with a non-power-of-two mantissa.  CDNA4's scaled FP4/FP8 MFMA
// applies one power-of-two (E8M0) scale per 32 elements, and FP8 operands hold only 4
// significant bits, so neither can carry sigma*q exactly.  sigma*q needs 6 significant bits
// and lies in [2^-10, 2688]: it is exactly representable as a normal FP16 number.  The kernel
// therefore expands the codes to FP16 (v_cvt_scalef32_pk_f16_fp4 gives q*2^8, one packed FP16
// multiply by sigma*2^-8 gives sigma*q, both exact) and runs v_mfma_f32_32x32x16_f16 on them:
// every product is exact and the only rounding is the FP32 accumulation.  alpha_a*alpha_b is
// applied once in the epilogue.
//
// Kernels in this file
//   gemm_fp4_direct     every NVFP4 problem with K % 64 == 0.  Four waves of 128x128 per
//                       workgroup, persistent workgroups, no LDS and no barriers in the K loop:
//                       each wave loads its own operand rows in MFMA order and expands them in
//                       registers (described at the kernel).  A 256x256 tile, a 256x128 tile
//                       with K split over wave pairs, or a 128x128 tile with K split over all
//                       four waves.
//   gemm_fp4_small      NVFP4 problems of up to 2 x CUs tiles of 64x64 (a few hundred tokens): one
//                       workgroup per tile, K split over its waves; for a long K with very few
//                       tiles also over workgroups (splitk_reduce_kernel then adds the slabs).
//   gemm_bf16_d2l       the BF16 baseline on large problems: 256x256 tile, four waves of 128x128,
//                       tiles loaded from global memory straight into LDS.
//   gemm_bf16_pipelined the BF16 baseline on smaller problems, same LDS pipeline, tiles staged
//                       through registers.
//   bf16_skinny_kernel  BF16 with M <= 64 (decode shapes), weight streaming, K split over the waves.
//   bf16_decode_kernel  BF16 with 17 <= M <= 64, weight streaming, N split over the waves, the
//                       activations shared through LDS, K slabs across workgroups with a workspace.
//   gemm_simple_kernel  any K % 16 == 0 / K % 8 == 0 that the tiled kernels do not take.
//
// The LDS pipeline (the BF16 kernels): block tile BM x BN x 64, two LDS stages, and the
// latencies covered inside each wave:
//   * a K step of 64 is four MFMA phases of 16; the fragments of phase p+1 are read from LDS
//     into a second register set while the MFMAs of phase p run;
//   * tiles are fetched two K steps ahead straight into the free LDS stage (gemm_bf16_d2l), or
//     one K step ahead into registers and written to the free stage over two phases
//     (gemm_bf16_pipelined);
//   * one barrier per K step, at the start of phase 3: before it every wave has finished writing
//     tile t+1 and reading tile t; after it tile t's stage is free and receives tile t+2.
// (An NVFP4 kernel of the same structure, operands expanded once per workgroup on their way
// into LDS, measured 6 % slower than the register-direct kernel on large problems and 1.4-1.8x
// slower on small ones, and is gone.)
// LDS rows are 128 bytes with a bank swizzle (below); tiles are walked in an XCD-aware grouped
// order.  Rows beyond M or N are clamped to the last valid row instead of being zero-filled:
// they only feed outputs that the epilogue does not store.
#include <atomic>
#include <type_traits>

#include "mq_common.h"

namespace mq {

namespace {

constexpr int BK = 64;       // K elements per LDS stage: 64 * 2 bytes = one 128-byte LDS row
constexpr int NUM_XCD = 8;

// LDS rows are 128 bytes = 8 chunks of 16 bytes.  The LDS serves 128-bit reads 16 lanes at a
// time over 64 four-byte banks (256 bytes per clock), i.e. over two consecutive rows, so the
// chunk index is XOR-ed with bits 1..3 of the row: 16 consecutive rows reading the same logical
// chunk then touch 16 different bank groups (measured: XOR with bits 0..2 gives 2-way conflicts).
__device__ __forceinline__ int swz_key(int row) { return (row >> 1) & 7; }

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct PCfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // per-wave tile
    static constexpr int TM = WM / 32, TN = WN / 32;      // 32x32 MFMA tiles per wave
    static constexpr int LA = BM * 8 / THREADS, LB = BN * 8 / THREADS;                // BF16 direct loads
    // LDS map in bytes: A stage 0, A stage 1, B stage 0, B stage 1 (stage strides fit the
    // 16-bit immediate offset of the LDS instructions)
    static constexpr int A_STAGE = BM * 128, B_STAGE = BN * 128, B_BASE = 2 * A_STAGE;
    static constexpr size_t LDS_BYTES = 2ull * (A_STAGE + B_STAGE);
    static_assert(TM >= 1 && TN >= 1 && LA >= 1 && LB >= 1, "tile too small for this wave grid");
};

// ---- tile order -----------------------------------------------------------------------------

// Workgroup ids are dealt round-robin to the 8 XCDs.  Give each XCD a contiguous range of
// logical tile ids, then walk tiles in groups of GROUP_M tile rows, column by column, so that
// the tiles resident on one XCD at a time share A row-panels and B column-panels in its L2.
__device__ __forceinline__ int logical_id(int wg, int total)
{
    const int xcd = wg % NUM_XCD, idx = wg / NUM_XCD;
    const int per = total / NUM_XCD, rem = total % NUM_XCD;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ void tile_of_logical(int t, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int GROUP_M = 8;
    const int group_size = GROUP_M * tiles_n;
    const int g = t / group_size;
    const int first_m = g * GROUP_M;
    const int gm = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    const int in_g = t - g * group_size;
    tm = first_m + in_g % gm;
    tn = in_g / gm;
}

__device__ __forceinline__ void tile_of(int wg, int tiles_m, int tiles_n, int &tm, int &tn)
{
    tile_of_logical(logical_id(wg, tiles_m * tiles_n), tiles_m, tiles_n, tm, tn);
}

// Scheduling hint for one phase: per MFMA one LDS read (while any remain), a few VALU
// instructions, and now and then an LDS write / a global load.  Nothing moves across a phase
// boundary: in particular no consumer of a global load is hoisted towards the load, which would
// turn the prefetch distance into a stall.
template <int MFMAS, int READS, int VALU_PER, int WRITES, int VMEMS, int SALUS = 0>
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
        if (SALUS > 0 && i < SALUS) __builtin_amdgcn_sched_group_barrier(0x004, 1, 0);  // SALU
    }
    __builtin_amdgcn_sched_barrier(0);
}

// Accumulator register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
// A wave tile that lies wholly inside the output takes the first path: one uniform row pointer
// per output row (scalar arithmetic) plus a constant 32-bit lane offset, no guards.  Tiles that
// cross the M or N edge take the guarded element-by-element path.
// I0, NI: the wave stores only its 32-row tiles I0 .. I0+NI-1.
template <class C, bool OUT_BF16, int I0 = 0, int NI = C::TM>
__device__ __forceinline__ void epilogue(const GemmArgs &g, f32x16 (&acc)[C::TM][C::TN], float scale,
                                         int64_t m0, int64_t n0, int wm0, int wn0, int frow, int fhalf)
{
    using T = std::conditional_t<OUT_BF16, __bf16, float>;
    const int64_t mw = m0 + wm0, nw = n0 + wn0;  // uniform over the wave
    if (mw + (I0 + NI) * 32 <= g.M && nw + C::WN <= g.N && g.ldy * (int64_t)(4 * sizeof(T)) < (1ll << 31)) {
        char *const base = static_cast<char *>(g.y) + (mw * g.ldy + nw) * (int64_t)sizeof(T);
        const uint32_t lane_off = (uint32_t)((4 * fhalf) * g.ldy + frow) * (uint32_t)sizeof(T);
        const int64_t row_bytes = g.ldy * (int64_t)sizeof(T);
        // A wave alone on its SIMD executes a chain of dependent instructions at about 8 cycles
        // each, so the values of two output rows go through scaling, rounding and the stores
        // stage by stage (the empty asm statements keep the stages apart), not value by value:
        // measured 5.1 us per 128x128 tile for the value-by-value order.  BF16: one conversion
        // packs the values of rows r and r + 1, stored as the low and the high half.
#pragma unroll
        for (int i = I0; i < I0 + NI; ++i)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                char *const rowp = base + (int64_t)(i * 32 + 8 * (r / 4) + (r % 4)) * row_bytes;
                float v[2][C::TN];
                // (read as AGPRs where they are: copies made through plain assignments let the
                // compiler move the whole accumulator set to VGPRs and scratch at the loop exit)
#pragma unroll
                for (int j = 0; j < C::TN; ++j) {
                    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[0][j]) : "a"(acc[i][j][r]));
                    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[1][j]) : "a"(acc[i][j][r + 1]));
                }
#pragma unroll
                for (int j = 0; j < C::TN; ++j) v[0][j] *= scale, v[1][j] *= scale;
#pragma unroll
                for (int j = 0; j < C::TN; ++j) asm volatile("" : "+v"(v[0][j]), "+v"(v[1][j]));
                if constexpr (OUT_BF16) {
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                    uint32_t ob[C::TN];
#pragma unroll
                    for (int j = 0; j < C::TN; ++j)
                        ob[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{v[0][j], v[1][j]}, bf16x2));
#pragma unroll
                    for (int j = 0; j < C::TN; ++j) asm volatile("" : "+v"(ob[j]));
#pragma unroll
                    for (int j = 0; j < C::TN; ++j) {
                        char *const pj = rowp + (uint64_t)lane_off + j * 32 * sizeof(T);
                        *reinterpret_cast<uint16_t *>(pj) = (uint16_t)ob[j];
                        *reinterpret_cast<uint16_t *>(pj + row_bytes) = (uint16_t)(ob[j] >> 16);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < C::TN; ++j) {
                        char *const pj = rowp + (uint64_t)lane_off + j * 32 * sizeof(T);
                        *reinterpret_cast<float *>(pj) = v[0][j];
                        *reinterpret_cast<float *>(pj + row_bytes) = v[1][j];
                    }
                }
            }
        return;
    }
#pragma unroll
    for (int i = I0; i < I0 + NI; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j) {
            const int64_t n = nw + j * 32 + frow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = mw + i * 32 + 8 * (r / 4) + 4 * fhalf + (r % 4);
                float v;
                asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][r]));
                if (m < g.M && n < g.N) static_cast<T *>(g.y)[m * g.ldy + n] = (T)(v * scale);
            }
        }
}

// ---- NVFP4, register-direct ------------------------------------------------------------------

// The same product without LDS and without barriers.  A wave owns a 128x128 output tile (four
// waves, one per SIMD, cover 256x256) and loads the packed codes of its own 128 A rows and 128 B
// rows straight from global memory in MFMA operand order: lane (r = lane%32, h = lane/32) takes
// the 16 bytes h of row r's 32-byte K step, dword p of which feeds phase p.  Within a K step the
// K index a lane supplies to the MFMA is therefore 32h + 8p + j instead of 16p + 8h + j; A and B
// use the same map, so each MFMA still sums 16 matching products and a K step covers all 64.
// Codes are expanded to FP16 in registers, one phase ahead of the MFMAs that use them; every
// operand row is expanded by the two waves that share it (twice the conversion work of the LDS
// pipeline, but no LDS traffic at all: measured 6 % faster on the 8192-token shapes).  Global
// loads run two K steps ahead, and the first loads of a workgroup's next tile are issued before
// the stores of the finished one.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
struct RawTile {
    uint4 c[8];      // 4 A tiles, 4 B tiles: this lane's 32 codes of each
    uint32_t s[8];   // the rows' four E4M3 scale bytes
};

// SPLIT = 2 (problems that fill the chip only with finer tiles): the workgroup tile is 256x128,
// its four waves are two 128x128 wave tiles times two halves of K; after the K loop each wave
// hands the half of its accumulators that its partner will store to the partner through LDS.
// SPLIT = 4: the workgroup tile is one 128x128 wave tile, its four waves take a quarter of K
// each, and two such exchanges leave every wave with 32 fully summed rows to store.
template <bool OUT_BF16, int SPLIT>
__global__ __launch_bounds__(256) void gemm_fp4_direct(GemmArgs g, int tiles_m, int tiles_n)
{
    using C = PCfg<256, 256, 2, 2>;  // wave-level constants: 128x128 wave tile, 4x4 MFMA tiles
    static_assert(SPLIT == 1 || SPLIT == 2 || SPLIT == 4, "K is split over 1, 2 or 4 waves");
    constexpr int BM = SPLIT == 4 ? 128 : 256, BN = SPLIT == 1 ? 256 : 128;
    constexpr int NSETS = 2;  // register sets of prefetched codes (3, i.e. two K steps of lookahead: no faster)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: the K range depends on it
    const int wm0 = SPLIT == 1 ? (wave >> 1) * 128 : SPLIT == 2 ? (wave & 1) * 128 : 0;
    const int wn0 = SPLIT == 1 ? (wave & 1) * 128 : 0;
    const int kpart = SPLIT == 1 ? 0 : SPLIT == 2 ? wave >> 1 : wave;  // which part of K this wave sums
    // SPLIT > 1: a wave holds its 32-row A tiles in the order i ^ aswap.  The tiles it will store
    // then sit in accumulator rows 0.. and the ones it hands to its partner(s) behind them, the
    // same in every wave (no divergent code): SPLIT = 2 keeps rows 0..1; SPLIT = 4 sends rows
    // 2..3 to wave w^2 first, then row 1 to wave w^1, and keeps row 0 = output tile w.
    const int aswap = SPLIT == 2 ? kpart << 1 : kpart;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int KT = (int)(g.K / BK);
    // this wave's K steps [k0, k1); every part but the last is a whole number of NSETS groups
    const int parts = SPLIT;
    const int KH = SPLIT == 1 ? KT : ((KT + parts - 1) / parts + NSETS - 1) / NSETS * NSETS;
    int k0 = kpart * KH, k1 = (k0 + KH < KT) ? k0 + KH : KT;
    const int total_tiles = tiles_m * tiles_n;
    auto item_of = [&](int item, int &tm, int &tn) { tile_of(item, tiles_m, tiles_n, tm, tn); };

    // Buffer loads: per K step a uniform resource whose 64-bit base is the start of that K step
    // (scalar arithmetic only), plus the lane's row and half as a 32-bit vector offset.  Rows
    // are clamped below, so every access is in bounds by construction and the resources carry
    // the maximal size.
    // The lane offsets are relative to the first row of the wave tile (whose 64-bit address is
    // scalar), so they fit 32 bits for any operand size.
    uint32_t vc[8], vs[8];
    // Running pointers to the K step that the next load_tile reads, for the first A / B row of
    // this wave's tile (codes, scales); advance() moves them on by one K step and stops at the
    // last step of K, so the loads issued past the end of a tile re-read that step.  (Advancing
    // costs some twenty scalar instructions per K step, placed under the MFMAs of the phase in
    // front of the loads; recomputing base + t * step cost thirty, in one block at the loads.)
    const char *pa_c, *pb_c, *pa_s, *pb_s;
    int t_next;
    auto set_tile = [&](int64_t m0, int64_t n0) {
        int64_t ra = m0 + wm0, rb = n0 + wn0;
        ra = ra < g.M ? ra : g.M - 1;
        rb = rb < g.N ? rb : g.N - 1;
        t_next = k0 < KT ? k0 : KT - 1;
        pa_c = static_cast<const char *>(g.a) + ra * g.a_c_row + t_next * g.a_c_step;
        pb_c = static_cast<const char *>(g.b) + rb * g.b_c_row + t_next * g.b_c_step;
        pa_s = reinterpret_cast<const char *>(g.a_scales) + ra * g.a_s_row + t_next * g.a_s_step;
        pb_s = reinterpret_cast<const char *>(g.b_scales) + rb * g.b_s_row + t_next * g.b_s_step;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const bool isA = q < 4;
            const int64_t total = isA ? g.M : g.N;
            int64_t grow = (isA ? m0 + wm0 + ((q & 3) ^ aswap) * 32 : n0 + wn0 + (q & 3) * 32) + frow;
            grow = grow < total ? grow : total - 1;
            const int64_t rel = grow - (isA ? ra : rb);  // 0 .. 127
            vc[q] = (uint32_t)(rel * (isA ? g.a_c_row : g.b_c_row) + fhalf * 16);
            vs[q] = (uint32_t)(rel * (isA ? g.a_s_row : g.b_s_row));
        }
    };
    RawTile st[NSETS];
    auto load_tile = [&](RawTile &r) {
        auto rsrc = [](const char *p) {
            return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(p), 0, -1, 0x00020000);
        };
        const __amdgpu_buffer_rsrc_t rac = rsrc(pa_c), rbc = rsrc(pb_c), ras = rsrc(pa_s), rbs = rsrc(pb_s);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const u32x4 c = __builtin_amdgcn_raw_buffer_load_b128(q < 4 ? rac : rbc, (int)vc[q], 0, 0);
            r.c[q] = make_uint4(c[0], c[1], c[2], c[3]);
            r.s[q] = __builtin_amdgcn_raw_buffer_load_b32(q < 4 ? ras : rbs, (int)vs[q], 0, 0);
        }
    };
    auto advance = [&]() {
        const int64_t adv = -(int64_t)(t_next + 1 < KT);  // all ones while a next K step exists (no branch)
        t_next -= (int)adv;
        pa_c += g.a_c_step & adv;
        pb_c += g.b_c_step & adv;
        pa_s += g.a_s_step & adv;
        pb_s += g.b_s_step & adv;
    };
    // Scale register of the K step being expanded: sigma*2^-8 as FP16 for block 2h in the low
    // half and for block 2h+1 in the high half (an E4M3 byte shifted left by 7 is that number).
    // One byte permute picks the lane's two scale bytes, or zeros for a K step past the end.
    uint32_t sg[8];
    const uint32_t sel_valid = 0x0C000C00u | (uint32_t)(2 * fhalf) | ((uint32_t)(2 * fhalf + 1) << 16);
    auto prep_scales = [&](const RawTile &r, bool valid) {
        const uint32_t sel = valid ? sel_valid : 0x0C0C0C0Cu;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint32_t sc = r.s[q];
            asm("" : "+v"(sc));  // first use of the prefetched register stays here
            sg[q] = __builtin_amdgcn_perm(0u, sc, sel) << 7;
        }
    };
    uint4 fr[2][8];
    // q0 .. q1-1: the operand tiles to expand (0..3 = A row tiles, 4..7 = B row tiles)
    auto expand_phase = [&](const RawTile &r, int p, uint4(&f)[8], int q0 = 0, int q1 = 8) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (q < q0 || q >= q1) continue;
            uint32_t w = p == 0 ? r.c[q].x : p == 1 ? r.c[q].y : p == 2 ? r.c[q].z : r.c[q].w;
            asm("" : "+v"(w));
            const _Float16 sig = __builtin_bit_cast(_Float16, (uint16_t)(p < 2 ? sg[q] : sg[q] >> 16));
            const f16x2 s = {sig, sig};
            // four conversions, then four multiplies: a multiply issued right behind the
            // conversion it consumes stalls the wave (measured 36 instead of 33 cycles per MFMA).
            // The empty asm statements order through their operands only; they must not be
            // volatile: a volatile asm counts as a side effect that no memory operation may
            // cross, which pinned the loads of a K step behind all conversions of their phase
            // and cost 4 to 6 % of the kernel.
            f16x2 c0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 0);
            f16x2 c1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 1);
            f16x2 c2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 2);
            f16x2 c3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 3);
            asm("" : "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3));
            c0 *= s, c1 *= s, c2 *= s, c3 *= s;
            f[q] = make_uint4(__builtin_bit_cast(uint32_t, c0), __builtin_bit_cast(uint32_t, c1),
                              __builtin_bit_cast(uint32_t, c2), __builtin_bit_cast(uint32_t, c3));
        }
    };
    f32x16 acc[4][4];
    auto mfmas = [&](const uint4(&f)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(f16x8, f[i]), __builtin_bit_cast(f16x8, f[4 + j]), acc[i][j], 0, 0, 0);
    };
    // one K step; R = kt % NSETS is the register set that holds tile kt
    auto kstep = [&](int kt, auto rr) {
        constexpr int R = decltype(rr)::value;
        RawTile &cur = st[R], &nxt = st[(R + 1) % NSETS];
        // The last two A row tiles of this step's first phase are expanded here, right before
        // the MFMAs that use them (the ninth onwards), not in the load phase of the previous K
        // step, which is the one phase that fills the wave's issue slots (+0.5-1 %; three tiles
        // deferred: no better).
        expand_phase(cur, 0, fr[0], 2, 4);
        expand_phase(cur, 1, fr[1]);
        mfmas(fr[0]);
        sched_phase<16, 0, 5, 0, 0>();
        expand_phase(cur, 2, fr[0]);
        mfmas(fr[1]);
        sched_phase<16, 0, 4, 0, 0>();
        // the scalar pointer arithmetic of the loads below, spread under this phase's MFMAs
        advance();
        expand_phase(cur, 3, fr[1]);
        mfmas(fr[0]);
        sched_phase<16, 0, 4, 0, 0, 16>();
        // The only loads in flight here are the 16 of the next K step, a whole step old: one wait
        // for all of them instead of one in front of each first use (this phase is the one that
        // fills the wave's issue slots, and a wait is an instruction like any other: +0.5-0.8 %).
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        prep_scales(nxt, kt + 1 < k1);
        expand_phase(nxt, 0, fr[0], 0, 2);
        expand_phase(nxt, 0, fr[0], 4, 8);
        load_tile(cur);
        mfmas(fr[1]);
        sched_phase<16, 0, 5, 0, 16>();
    };

    // Persistent workgroups: tile ids blockIdx.x, blockIdx.x + gridDim.x, ...  The first loads of
    // the next tile are issued before the stores of the finished one.
    const float scale = (*g.a_alpha) * (*g.b_alpha);
    int tile = blockIdx.x;
    int tm, tn;
    item_of(tile, tm, tn);
    set_tile((int64_t)tm * BM, (int64_t)tn * BN);
#pragma unroll
    for (int u = 0; u < NSETS; ++u) {
        if (u) advance();
        load_tile(st[u]);
    }
    while (true) {
        const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        prep_scales(st[0], k0 < k1);
        expand_phase(st[0], 0, fr[0], 0, 2);
        expand_phase(st[0], 0, fr[0], 4, 8);
        // No separate tail: the loop runs whole groups of NSETS K steps, and a step past the end
        // multiplies by zero scales.  (Peeled tail steps make the compiler shuffle all 256
        // accumulator registers at the control-flow joins.)
        for (int kt = k0; kt < k1; kt += NSETS) {
            kstep(kt, std::integral_constant<int, 0>{});
            if constexpr (NSETS > 1) kstep(kt + 1, std::integral_constant<int, 1>{});
            if constexpr (NSETS > 2) kstep(kt + 2, std::integral_constant<int, 2>{});
        }
        tile += gridDim.x;
        const bool more = tile < total_tiles;
        if (more) {
            item_of(tile, tm, tn);
            set_tile((int64_t)tm * BM, (int64_t)tn * BN);
#pragma unroll
            for (int u = 0; u < NSETS; ++u) {
        if (u) advance();
        load_tile(st[u]);
    }
        }
        if constexpr (SPLIT == 1) {
            epilogue<C, OUT_BF16>(g, acc, scale, m0, n0, wm0, wn0, frow, fhalf);
        } else {
            // Waves that hold different parts of K for the same 128x128 tile exchange through LDS:
            // a wave sends the accumulator rows [first, first + count) to `partner` and adds what
            // the partner sent to its rows [0, count) (a + b in both, so the result does not
            // depend on which wave adds).  1 KB per (32x32 tile, register quad) and wave.
            extern __shared__ uint4 lds[];
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            f32x4 *const X = reinterpret_cast<f32x4 *>(lds);
            auto exchange = [&](auto firstc, auto countc, int partner) {
                constexpr int first = decltype(firstc)::value, count = decltype(countc)::value;
#pragma unroll
                for (int i = 0; i < count; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const f32x16 &t = acc[first + i][j];
                            X[((wave * 8 + i * 4 + j) * 4 + c) * 64 + lane] =
                                f32x4{t[4 * c], t[4 * c + 1], t[4 * c + 2], t[4 * c + 3]};
                        }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < count; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const f32x4 v = X[((partner * 8 + i * 4 + j) * 4 + c) * 64 + lane];
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[i][j][4 * c + e] += v[e];
                        }
                __syncthreads();  // the next sends must not overtake these reads
            };
            exchange(std::integral_constant<int, 2>{}, std::integral_constant<int, 2>{}, wave ^ 2);
            if constexpr (SPLIT == 2) {
                epilogue<C, OUT_BF16, 0, 2>(g, acc, scale, m0, n0, wm0 + kpart * 64, wn0, frow, fhalf);
            } else {
                exchange(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, wave ^ 1);
                epilogue<C, OUT_BF16, 0, 1>(g, acc, scale, m0, n0, wm0 + wave * 32, wn0, frow, fhalf);
            }
        }
        if (!more) break;
    }
}

// ---- NVFP4, register-direct, small tiles: prefill chunks of 64 .. 1024 tokens -------------------

// With a few hundred tokens the 128x128 wave tiles above are too few to occupy the chip, and the
// time of a layer is launch latency plus one trip of the weights from HBM.  Here a workgroup owns
// one (32 TM) x (32 TN) output tile; its S waves (S chosen at launch, S <= MAXS) take consecutive
// parts of K and each runs the same register-direct K loop as above (operands loaded in MFMA
// order, expanded in registers, no LDS and no barrier in the loop) with NSETS K steps of codes in
// flight per wave.  The S partial tiles are then added through LDS in a fixed order (wave 0, 1,
// ...: bit-identical from run to run), each wave summing, scaling, rounding and storing 1/S of the
// tile.  No workspace and no second kernel: one launch per layer.  Only a long K with very few
// tiles is also cut into g.ksplit slabs across workgroups when the caller passes a workspace: a
// work item is then (slab, tile), its workgroup writes unscaled FP32 partial sums to
// g.ws[slab][M][N], and splitk_reduce_kernel adds the slabs in ascending order.  Smaller wave tiles raise the
// conversion work per MFMA (TM + TN operand tiles expanded for TM x TN MFMAs: 8 VALU instructions
// per MFMA for 64x64, 6 for 128x64) but multiply the number of waves that pull on memory.
template <int TM_, int TN_>
struct SmallCfg {
    static constexpr int TM = TM_, TN = TN_, WN = 32 * TN_;
};

// End of the small-tile kernels: the S waves of a workgroup hold partial sums of one
// (32 TM) x (32 TN) tile over their parts of K.  S == 1: plain epilogue.  Otherwise the partial
// tiles are added through LDS, four 32x32 tiles (16 KB per wave) per pass.  A pass holds 16 chunks
// of four accumulator registers per wave; wave w adds the S copies of chunks w, w + S, ... in
// wave order (bit-identical from run to run), scales, rounds and stores them: chunk c of a tile =
// rows 8c + 4 (lane / 32) .. + 3, column lane % 32.
template <int TM, int TN, bool OUT_BF16>
__device__ __forceinline__ void small_tile_finish(const GemmArgs &g, f32x16 (&acc)[TM][TN], float scale, int64_t m0,
                                                  int64_t n0, int S, int wave, int lane)
{
    constexpr int NM = TM * TN;
    const int frow = lane & 31, fhalf = lane >> 5;
    if (S == 1) {
        epilogue<SmallCfg<TM, TN>, OUT_BF16>(g, acc, scale, m0, n0, 0, 0, frow, fhalf);
        return;
    }
    extern __shared__ uint4 lds[];
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4 *const X = reinterpret_cast<f32x4 *>(lds);
    using T = std::conditional_t<OUT_BF16, __bf16, float>;
    constexpr int PASS = NM < 4 ? NM : 4;  // tiles per pass
#pragma unroll
    for (int p0 = 0; p0 < NM; p0 += PASS) {
        if (p0 > 0) __syncthreads();  // the previous pass has been read
#pragma unroll
        for (int u = 0; u < PASS; ++u) {
            const f32x16 &tl = acc[(p0 + u) / TN][(p0 + u) % TN];
#pragma unroll
            for (int c = 0; c < 4; ++c)
                X[((wave * PASS + u) * 4 + c) * 64 + lane] = f32x4{tl[4 * c], tl[4 * c + 1], tl[4 * c + 2], tl[4 * c + 3]};
        }
        __syncthreads();
        for (int ch = wave; ch < PASS * 4; ch += S) {
            f32x4 sum = X[ch * 64 + lane];
            for (int w = 1; w < S; ++w) sum += X[(w * PASS * 4 + ch) * 64 + lane];
            const int tile = p0 + (ch >> 2), c = ch & 3;
            const int64_t n = n0 + (tile % TN) * 32 + frow;
            const int64_t mrow = m0 + (tile / TN) * 32 + 8 * c + 4 * fhalf;
            if (n < g.N) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (mrow + e < g.M) static_cast<T *>(g.y)[(mrow + e) * g.ldy + n] = (T)(sum[e] * scale);
            }
        }
    }
}

template <int TM, int TN, int MAXS, int NSETS, bool OUT_BF16>
__global__ __launch_bounds__(64 * MAXS) void gemm_fp4_small(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int NT = TM + TN;
    static_assert((TM * TN) % 4 == 0 || TM * TN < 4, "the LDS reduction moves four 32x32 tiles per pass");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = (int)(blockDim.x >> 6);  // waves that share this tile's K range
    const int frow = lane & 31, fhalf = lane >> 5;
    const int KT = (int)(g.K / BK);
    // work item = (K slab, tile), slab-major; tiles that share a column panel of B are neighbours
    // in that order and run on one XCD.  g.ksplit == 1: the tile's whole K.
    const int tiles = tiles_m * tiles_n;
    const int item = logical_id(blockIdx.x, tiles * g.ksplit);
    const int slab = item / tiles, t = item - slab * tiles;
    const int tm = t % tiles_m, tn = t / tiles_m;
    const int64_t m0 = (int64_t)tm * (32 * TM), n0 = (int64_t)tn * (32 * TN);  // m0 < M, n0 < N
    // K steps of the slab, then of this wave within it
    const int SL = (KT + g.ksplit - 1) / g.ksplit;
    const int s0 = slab * SL < KT ? slab * SL : KT, s1 = s0 + SL < KT ? s0 + SL : KT;
    const int KH = (s1 - s0 + S - 1) / S;
    const int k0 = s0 + wave * KH < s1 ? s0 + wave * KH : s1;
    const int k1 = k0 + KH < s1 ? k0 + KH : s1;

    // operand q: A row tile q (q < TM), else B row tile q - TM.  Lane offsets relative to the tile.
    const char *const ta_c = static_cast<const char *>(g.a) + m0 * g.a_c_row;
    const char *const tb_c = static_cast<const char *>(g.b) + n0 * g.b_c_row;
    const char *const ta_s = reinterpret_cast<const char *>(g.a_scales) + m0 * g.a_s_row;
    const char *const tb_s = reinterpret_cast<const char *>(g.b_scales) + n0 * g.b_s_row;
    uint32_t vc[NT], vs[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        const bool isA = q < TM;
        const int64_t total = isA ? g.M : g.N, first = isA ? m0 : n0;
        int64_t grow = first + (isA ? q : q - TM) * 32 + frow;
        grow = grow < total ? grow : total - 1;
        vc[q] = (uint32_t)((grow - first) * (isA ? g.a_c_row : g.b_c_row) + fhalf * 16);
        vs[q] = (uint32_t)((grow - first) * (isA ? g.a_s_row : g.b_s_row));
    }
    uint4 rc[NSETS][NT];     // this lane's 32 codes of each operand tile, NSETS K steps
    uint32_t rs[NSETS][NT];  // the rows' four E4M3 scale bytes
    // K steps are loaded in ascending order, so the four K-step bases advance by their strides
    // (scalar additions) instead of being recomputed by 64-bit multiplications; a step past the
    // end of K re-reads the last one (its products are multiplied by zero scales).
    int next_t = k0 < KT ? k0 : KT - 1;
    const char *pa_c = ta_c + (int64_t)next_t * g.a_c_step, *pb_c = tb_c + (int64_t)next_t * g.b_c_step;
    const char *pa_s = ta_s + (int64_t)next_t * g.a_s_step, *pb_s = tb_s + (int64_t)next_t * g.b_s_step;
    auto load_step = [&](auto setc) {
        constexpr int R = decltype(setc)::value;
        auto rsrc = [](const char *base) {
            return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, -1, 0x00020000);
        };
        const __amdgpu_buffer_rsrc_t rac = rsrc(pa_c), rbc = rsrc(pb_c), ras = rsrc(pa_s), rbs = rsrc(pb_s);
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            const u32x4 c = __builtin_amdgcn_raw_buffer_load_b128(q < TM ? rac : rbc, (int)vc[q], 0, 0);
            rc[R][q] = make_uint4(c[0], c[1], c[2], c[3]);
            rs[R][q] = __builtin_amdgcn_raw_buffer_load_b32(q < TM ? ras : rbs, (int)vs[q], 0, 0);
        }
        const int64_t adv = next_t + 1 < KT ? -1 : 0;  // all ones while K steps remain (no branch in the loop)
        next_t -= (int)adv;
        pa_c += g.a_c_step & adv, pb_c += g.b_c_step & adv, pa_s += g.a_s_step & adv, pb_s += g.b_s_step & adv;
    };
    // scales, expansion and MFMAs exactly as in gemm_fp4_direct (K index of a lane: 32h + 8p + j)
    uint32_t sg[NT];
    const uint32_t sel_valid = 0x0C000C00u | (uint32_t)(2 * fhalf) | ((uint32_t)(2 * fhalf + 1) << 16);
    auto prep_scales = [&](auto setc, bool valid) {
        constexpr int R = decltype(setc)::value;
        const uint32_t sel = valid ? sel_valid : 0x0C0C0C0Cu;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            uint32_t sc = rs[R][q];
            asm("" : "+v"(sc));
            sg[q] = __builtin_amdgcn_perm(0u, sc, sel) << 7;
        }
    };
    uint4 fr[2][NT];
    auto expand_phase = [&](auto setc, int p, uint4(&f)[NT]) {
        constexpr int R = decltype(setc)::value;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            uint32_t w = p == 0 ? rc[R][q].x : p == 1 ? rc[R][q].y : p == 2 ? rc[R][q].z : rc[R][q].w;
            asm("" : "+v"(w));
            const _Float16 sig = __builtin_bit_cast(_Float16, (uint16_t)(p < 2 ? sg[q] : sg[q] >> 16));
            const f16x2 sv = {sig, sig};
            f16x2 c0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 0);
            f16x2 c1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 1);
            f16x2 c2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 2);
            f16x2 c3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 3);
            asm("" : "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3));
            c0 *= sv, c1 *= sv, c2 *= sv, c3 *= sv;
            f[q] = make_uint4(__builtin_bit_cast(uint32_t, c0), __builtin_bit_cast(uint32_t, c1),
                              __builtin_bit_cast(uint32_t, c2), __builtin_bit_cast(uint32_t, c3));
        }
    };
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    auto mfmas = [&](const uint4(&f)[NT]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(f16x8, f[i]), __builtin_bit_cast(f16x8, f[TM + j]), acc[i][j], 0, 0, 0);
    };
    constexpr int NM = TM * TN, VPER = (NT * 8 + NM - 1) / NM;
    auto kstep = [&](int kt, auto setc) {
        constexpr int R = decltype(setc)::value;
        using Next = std::integral_constant<int, (R + 1) % NSETS>;
        expand_phase(setc, 1, fr[1]);
        mfmas(fr[0]);
        sched_phase<NM, 0, VPER, 0, 0>();
        expand_phase(setc, 2, fr[0]);
        mfmas(fr[1]);
        sched_phase<NM, 0, VPER, 0, 0>();
        expand_phase(setc, 3, fr[1]);
        mfmas(fr[0]);
        sched_phase<NM, 0, VPER, 0, 0>();
        prep_scales(Next{}, kt + 1 < k1);
        expand_phase(Next{}, 0, fr[0]);
        load_step(setc);  // K step kt + NSETS
        mfmas(fr[1]);
        sched_phase<NM, 0, VPER + 2, 0, (2 * NT + NM - 1) / NM>();
    };
    auto for_sets = [&](auto &&fn) {  // fn(set index as a constant), sets 0 .. NSETS-1
        fn(std::integral_constant<int, 0>{});
        if constexpr (NSETS > 1) fn(std::integral_constant<int, 1>{});
        if constexpr (NSETS > 2) fn(std::integral_constant<int, 2>{});
        if constexpr (NSETS > 3) fn(std::integral_constant<int, 3>{});
    };
    static_assert(NSETS >= 1 && NSETS <= 4, "one to four K steps in flight");
    // The first NSETS K steps, issued set by set.  (Left to the scheduler, the B loads of all sets
    // went last, and the counter the compiler waits on in the loop then demanded that nearly
    // everything in flight had landed before each K step: a prefetch distance of one step, not three.)
    for_sets([&](auto u) {
        load_step(u);
        __builtin_amdgcn_sched_barrier(0);
    });
    const float scale = (*g.a_alpha) * (*g.b_alpha);
    prep_scales(std::integral_constant<int, 0>{}, k0 < k1);
    expand_phase(std::integral_constant<int, 0>{}, 0, fr[0]);
    // whole groups of NSETS K steps; a step past the end multiplies by zero scales
    for (int kt = k0; kt < k1; kt += NSETS) for_sets([&](auto u) { kstep(kt + decltype(u)::value, u); });

    if (g.ksplit > 1) {
        GemmArgs part = g;  // the slab's [M, N] FP32 matrix of partial sums; splitk_reduce_kernel scales and rounds
        part.y = g.ws + (int64_t)slab * g.M * g.N;
        part.ldy = g.N;
        small_tile_finish<TM, TN, false>(part, acc, 1.0f, m0, n0, S, wave, lane);
    } else {
        small_tile_finish<TM, TN, OUT_BF16>(g, acc, scale, m0, n0, S, wave, lane);
    }
}

// Second pass of the slab-split product: y[m][n] = round(scale * (ws[0][m][n] + ws[1][m][n] + ...)),
// slabs added in ascending order.  One thread per four consecutive columns (N % 4 == 0 here).
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs g)
{
    const int64_t quads_per_row = g.N / 4, total = g.M * quads_per_row;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int64_t m = i / quads_per_row, n = (i - m * quads_per_row) * 4;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 *p = reinterpret_cast<const f32x4 *>(g.ws + m * g.N + n);
    const int64_t slab_quads = g.M * g.N / 4;
    f32x4 sum = p[0];
    for (int sl = 1; sl < g.ksplit; ++sl) sum += p[sl * slab_quads];
    if (g.a_alpha) sum *= (*g.a_alpha) * (*g.b_alpha);  // NVFP4: the two tensor-level scales; BF16: none
    if constexpr (OUT_BF16) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        const bf16x4 o = {(__bf16)sum[0], (__bf16)sum[1], (__bf16)sum[2], (__bf16)sum[3]};
        *reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(g.y) + m * g.ldy + n) = o;
    } else {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(g.y) + m * g.ldy + n) = sum;
    }
}

// ---- BF16 -----------------------------------------------------------------------------------

// Same phases as the NVFP4 LDS pipeline.  A tile is fetched into registers right after the
// barrier of K step t (16 x 128 bits per thread), and written to the free LDS stage during
// phases 1 and 2 of K step t+1.  Used for the 256x128 and 128x128 tile configurations.
template <class C, bool OUT_BF16>
__global__ __launch_bounds__(C::THREADS) void gemm_bf16_pipelined(GemmArgs g, int tiles_m, int tiles_n)
{
    extern __shared__ uint4 lds[];
    char *const L = reinterpret_cast<char *>(lds);
    int tm, tn;
    tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / C::WAVES_N) * C::WM, wn0 = (wave % C::WAVES_N) * C::WN;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int KT = (int)(g.K / BK);

    // chunk j of this thread: row (tid>>3) + j*(THREADS/8) of the tile, 16-byte chunk tid&7 of its 128 bytes
    constexpr int NL = C::LA + C::LB;
    uint32_t vo[NL];  // global byte offsets from the tile's first row (K step 0): 32 bits for any operand size
    int wad[NL];      // LDS byte addresses (stage 0)
    const char *const ta = static_cast<const char *>(g.a) + m0 * g.lda * 2;  // m0 < M, n0 < N
    const char *const tb = static_cast<const char *>(g.b) + n0 * g.ldb * 2;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const bool isA = j < C::LA;
        const int r = (tid >> 3) + (isA ? j : j - C::LA) * (C::THREADS / 8);
        int64_t grow = (isA ? m0 : n0) + r;
        const int64_t total = isA ? g.M : g.N;
        grow = grow < total ? grow : total - 1;
        vo[j] = (uint32_t)((grow - (isA ? m0 : n0)) * (isA ? g.lda : g.ldb) * 2 + (tid & 7) * 16);
        wad[j] = (isA ? 0 : C::B_BASE) + (r * 8 + ((tid & 7) ^ swz_key(r))) * 16;
    }
    uint4 regs[NL];
    auto load_tile = [&](int t) {
        t = t < KT ? t : KT - 1;
        const char *a = ta + (int64_t)t * (BK * 2);
        const char *b = tb + (int64_t)t * (BK * 2);
#pragma unroll
        for (int j = 0; j < NL; ++j) regs[j] = *reinterpret_cast<const uint4 *>((j < C::LA ? a : b) + vo[j]);
    };
    auto store_range = [&](int j0, int j1, int stage) {
#pragma unroll
        for (int j = j0; j < j1; ++j) {
            uint4 v = regs[j];
            asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));  // first use stays in this phase
            *reinterpret_cast<uint4 *>(L + wad[j] + stage * (j < C::LA ? C::A_STAGE : C::B_STAGE)) = v;
        }
    };

    int fa[4], fb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        fa[ks] = ((wm0 + frow) * 8 + ((ks * 2 + fhalf) ^ swz_key(frow))) * 16;
        fb[ks] = C::B_BASE + ((wn0 + frow) * 8 + ((ks * 2 + fhalf) ^ swz_key(frow))) * 16;
    }
    uint4 fra[2][C::TM], frb[2][C::TN];
    auto read_frags = [&](int stage, int ks, uint4(&a)[C::TM], uint4(&b)[C::TN]) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
            a[i] = *reinterpret_cast<const uint4 *>(L + fa[ks] + i * 4096 + stage * C::A_STAGE);
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
            b[j] = *reinterpret_cast<const uint4 *>(L + fb[ks] + j * 4096 + stage * C::B_STAGE);
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
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]), acc[i][j], 0, 0, 0);
    };
    constexpr int NMFMA = C::TM * C::TN, NREAD = C::TM + C::TN;

    load_tile(0);
    store_range(0, NL, 0);
    load_tile(1);
    __syncthreads();
    read_frags(0, 0, fra[0], frb[0]);

    auto kstep = [&](int kt, auto par) {
        constexpr int PAR = decltype(par)::value;
        constexpr int cur = PAR, nxt = PAR ^ 1;
        // phase 0
        read_frags(cur, 1, fra[1], frb[1]);
        mfmas(fra[0], frb[0]);
        sched_phase<NMFMA, NREAD, 0, 0, 0>();
        // phase 1: first half of tile kt+1 -> LDS
        read_frags(cur, 2, fra[0], frb[0]);
        store_range(0, NL / 2, nxt);
        mfmas(fra[1], frb[1]);
        sched_phase<NMFMA, NREAD, 0, (NL / 2 < NMFMA ? NL / 2 : NMFMA), 0>();
        // phase 2: second half
        read_frags(cur, 3, fra[1], frb[1]);
        store_range(NL / 2, NL, nxt);
        mfmas(fra[0], frb[0]);
        sched_phase<NMFMA, NREAD, 0, (NL / 2 < NMFMA ? NL / 2 : NMFMA), 0>();
        // phase 3
        __syncthreads();
        read_frags(nxt, 0, fra[0], frb[0]);
        load_tile(kt + 2);
        mfmas(fra[1], frb[1]);
        sched_phase<NMFMA, NREAD, 0, 0, NL>();
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
        kstep(kt, std::integral_constant<int, 0>{});
        kstep(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) kstep(kt, std::integral_constant<int, 0>{});

    epilogue<C, OUT_BF16>(g, acc, 1.0f, m0, n0, wm0, wn0, frow, fhalf);
}

// ---- BF16, direct global-to-LDS loads ----------------------------------------------------------

// 256x256x64 tile with four waves of 128x128 (one per SIMD), or 256x128x64 with four waves of
// 128x64; same LDS layout, phases and barrier as gemm_bf16_pipelined, but the tiles never pass
// through registers: every wave issues 16 (12) global_load_lds_dwordx4 per K step (1 KB each:
// 8 rows of one operand tile), which write LDS at
// M0 + 16 * lane.  The bank swizzle is applied on the global side: the lane that fills chunk c' of
// row r fetches chunk c' ^ key(r).  The loads are written in inline assembly because the compiler
// orders every LDS read behind all outstanding LDS-writing loads (s_waitcnt vmcnt(0) right after
// the load), which serialises the pipeline; here the only wait is the one before the barrier.
// The loads of tile t+2 are issued one per two MFMAs: the first half in the phase behind the
// barrier that frees their stage, the second half in the first phase of the next K step.  All
// 16 in the one phase measured 3 to 8 % slower (the texture path is shared by the four waves and
// the same instants see everybody's loads), in one burst 5 % slower again; three phases no better.
template <class C, bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_bf16_d2l(GemmArgs g, int tiles_m, int tiles_n)
{
    static_assert(C::THREADS == 256, "four waves");
    constexpr int GA = C::BM / 32, GB = C::BN / 32, NL = GA + GB;  // 8-row groups per wave and operand
    extern __shared__ uint4 lds[];
    char *const L = reinterpret_cast<char *>(lds);
    int tm, tn;
    tile_of(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave / C::WAVES_N) * C::WM, wn0 = (wave % C::WAVES_N) * C::WN;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int KT = (int)(g.K / BK);

    // load u of this wave: rows 8 * (wave * GA + u) .. + 7 of the A tile (u < GA), else of the B tile
    // byte offsets from the tile's first row: 32 bits for any operand size
    uint32_t vo[NL];
    const char *const ta = static_cast<const char *>(g.a) + m0 * g.lda * 2;  // m0 < M, n0 < N
    const char *const tb = static_cast<const char *>(g.b) + n0 * g.ldb * 2;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
        const bool isA = u < GA;
        const int r = 8 * (isA ? wave * GA + u : wave * GB + (u - GA)) + (lane >> 3);
        int64_t grow = (isA ? m0 : n0) + r;
        const int64_t total = isA ? g.M : g.N;
        grow = grow < total ? grow : total - 1;
        vo[u] = (uint32_t)((grow - (isA ? m0 : n0)) * (isA ? g.lda : g.ldb) * 2 + (((lane & 7) ^ swz_key(r)) * 16));
    }
    // LDS byte address of the dynamic segment
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)L;
    // load u of tile t into LDS stage `stage`
    auto load_group = [&](int t, int stage, int u) {
        t = t < KT ? t : KT - 1;
        const bool isA = u < GA;
        const char *base = (isA ? ta : tb) + (int64_t)t * (BK * 2);
        const uint32_t dst = lds0 + (isA ? stage * C::A_STAGE + (wave * GA + u) * 1024
                                         : C::B_BASE + stage * C::B_STAGE + (wave * GB + (u - GA)) * 1024);
        // m0 is named as clobbered so that the compiler never keeps a value of its own in it across
        // this statement (it calls m0 "reserved" and warns about any clobber of it: silenced here)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(dst), "v"(vo[u]), "s"(base)
                     : "memory", "m0");
#pragma clang diagnostic pop
    };
    auto load_tile = [&](int t, int stage) {
#pragma unroll
        for (int u = 0; u < NL; ++u) load_group(t, stage, u);
    };

    int fa[4], fb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        fa[ks] = ((wm0 + frow) * 8 + ((ks * 2 + fhalf) ^ swz_key(frow))) * 16;
        fb[ks] = C::B_BASE + ((wn0 + frow) * 8 + ((ks * 2 + fhalf) ^ swz_key(frow))) * 16;
    }
    uint4 fra[2][C::TM], frb[2][C::TN];
    auto read_frags = [&](int stage, int ks, uint4(&a)[C::TM], uint4(&b)[C::TN]) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
            a[i] = *reinterpret_cast<const uint4 *>(L + fa[ks] + i * 4096 + stage * C::A_STAGE);
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
            b[j] = *reinterpret_cast<const uint4 *>(L + fb[ks] + j * 4096 + stage * C::B_STAGE);
    };
    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    constexpr int NMFMA = C::TM * C::TN;

    load_tile(0, 0);
    load_tile(1, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    read_frags(0, 0, fra[0], frb[0]);

    // One phase: the MFMAs of one 16-wide K sub-step on fragments (ca, cb); meanwhile the
    // fragments of sub-step ks of stage rs are read into (na, nb), one per MFMA while any remain,
    // and loads [U0, U1) of tile t go to stage ls, spread evenly over the MFMAs.
    auto phase = [&](const uint4(&ca)[C::TM], const uint4(&cb)[C::TN], uint4(&na)[C::TM], uint4(&nb)[C::TN], int ks,
                     int rs, int t, int ls, auto u0c, auto u1c) {
        constexpr int U0 = decltype(u0c)::value, U1 = decltype(u1c)::value;
#pragma unroll
        for (int n = 0; n < NMFMA; ++n) {
            const int i = n / C::TN, j = n % C::TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, ca[i]), __builtin_bit_cast(bf16x8, cb[j]), acc[i][j], 0, 0, 0);
            if (n < C::TM)
                na[n] = *reinterpret_cast<const uint4 *>(L + fa[ks] + n * 4096 + rs * C::A_STAGE);
            else if (n < C::TM + C::TN)
                nb[n - C::TM] = *reinterpret_cast<const uint4 *>(L + fb[ks] + (n - C::TM) * 4096 + rs * C::B_STAGE);
#pragma unroll
            for (int u = U0 + n * (U1 - U0) / NMFMA; u < U0 + (n + 1) * (U1 - U0) / NMFMA; ++u) load_group(t, ls, u);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using U_0 = std::integral_constant<int, 0>;
    using U_H = std::integral_constant<int, NL / 2>;
    using U_N = std::integral_constant<int, NL>;
    auto kstep = [&](int kt, auto par) {
        constexpr int cur = decltype(par)::value, nxt = cur ^ 1;
        // second half of tile kt+1 (the first K step of a tile fetches it a second time: harmless)
        phase(fra[0], frb[0], fra[1], frb[1], 1, cur, kt + 1, nxt, U_H{}, U_N{});
        phase(fra[1], frb[1], fra[0], frb[0], 2, cur, 0, 0, U_N{}, U_N{});
        phase(fra[0], frb[0], fra[1], frb[1], 3, cur, 0, 0, U_N{}, U_N{});
        // tile kt+1 has landed in this wave's share of stage nxt; after the barrier in everyone's,
        // and nobody reads stage cur any more (this wave's last fragment reads of it have
        // returned: lgkmcnt, which the MFMAs behind the barrier would wait for anyway): it
        // receives tile kt+2
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        phase(fra[1], frb[1], fra[0], frb[0], 0, nxt, kt + 2, cur, U_0{}, U_H{});
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
        kstep(kt, std::integral_constant<int, 0>{});
        kstep(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) kstep(kt, std::integral_constant<int, 0>{});
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the clamped loads past the end still target LDS

    epilogue<C, OUT_BF16>(g, acc, 1.0f, m0, n0, wm0, wn0, frow, fhalf);
}

// ---- decode-shape BF16 product (M <= 64): weight streaming, HBM-bound ---------------------------

// The high-precision decode path multiplies a handful of tokens by the whole weight matrix, so
// the time is the time to stream W once from HBM.  A workgroup of 8 waves owns 16*RT rows of W;
// wave w takes the 128-wide K super-steps w, w+8, ... (together 2 KB contiguous per row and round),
// so 8 x (N / (16*RT)) waves keep enough bytes in flight without splitting K across workgroups.
// A lane (row r = lane%16, group g = lane/16) loads 64 contiguous bytes of W rows r, r+16, ... and
// of X rows r, r+16, ...; four v_mfma_f32_16x16x32_bf16 per super-step and (row tile, token tile)
// pair accumulate D[W row][token]; the 8 partial sums are added pairwise, in a fixed order,
// through LDS.  Every workgroup re-reads the activations from L2, which delivers about 6 TB/s to
// the CUs in total: with MT token tiles and RT row tiles per wave the weights stream at
// 6 / (1 + MT/RT) TB/s at best, so RT grows with N as far as the grid still covers half the chip.
// DB: two super-steps of loads in flight per wave (when the registers allow), else one.
template <int MT, int RT, bool DB, bool OUT_BF16>
__global__ __launch_bounds__(512) void bf16_skinny_kernel(GemmArgs g)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int NT = RT * MT;
    __shared__ f32x4 red[4][NT][64];  // 4 * NT KB: at most 64 KB
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = lane & 15, grp = lane >> 4;
    const int64_t n0 = (int64_t)blockIdx.x * (16 * RT);
    const uint4 *wp[RT], *xp[MT];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        int64_t wr = n0 + r * 16 + row;
        wr = wr < g.N ? wr : g.N - 1;
        wp[r] = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(g.b) + wr * g.ldb + grp * 32);
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int64_t xr = t * 16 + row;
        xr = xr < g.M ? xr : g.M - 1;
        xp[t] = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(g.a) + xr * g.lda + grp * 32);
    }
    f32x4 acc[RT][MT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[r][t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int S = (int)(g.K / 128);  // super-steps; 16 uint4 per row each
    auto load = [&](int s, uint4(&w)[RT][4], uint4(&x)[MT][4]) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j) w[r][j] = wp[r][s * 16 + j];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) x[t][j] = xp[t][s * 16 + j];
    };
    auto step = [&](const uint4(&w)[RT][4], const uint4(&x)[MT][4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int t = 0; t < MT; ++t)
                    acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, w[r][j]), __builtin_bit_cast(bf16x8, x[t][j]), acc[r][t], 0, 0, 0);
    };
    int s = wave;
    if constexpr (DB) {
        for (; s + 8 < S; s += 16) {  // two super-steps of loads in flight
            uint4 w0[RT][4], w1[RT][4], x0[MT][4], x1[MT][4];
            load(s, w0, x0);
            load(s + 8, w1, x1);
            __builtin_amdgcn_sched_barrier(0);  // every load is issued before the first MFMA waits
            step(w0, x0);
            step(w1, x1);
        }
    }
    for (; s < S; s += 8) {
        uint4 w0[RT][4], x0[MT][4];
        load(s, w0, x0);
        __builtin_amdgcn_sched_barrier(0);
        step(w0, x0);
    }

    // waves 4..7 hand their sums to waves 0..3, then 2..3 to 0..1, then 1 to 0
#pragma unroll
    for (int h = 4; h >= 1; h >>= 1) {
        if (wave >= h && wave < 2 * h) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int t = 0; t < MT; ++t) red[wave - h][r * MT + t][lane] = acc[r][t];
        }
        __syncthreads();
        if (wave < h) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int t = 0; t < MT; ++t) acc[r][t] += red[wave][r * MT + t][lane];
        }
        __syncthreads();
    }
    if (wave != 0) return;
    // accumulator i of a 16x16 tile: W row 4*(lane/16) + i, token lane%16
    using T = std::conditional_t<OUT_BF16, __bf16, float>;
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int64_t m = t * 16 + row, n = n0 + r * 16 + 4 * grp;
            if (m >= g.M) continue;
            T *dst = static_cast<T *>(g.y) + m * g.ldy + n;
            if (n + 3 < g.N) {
                if constexpr (OUT_BF16) {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    *reinterpret_cast<bf16x4 *>(dst) = bf16x4{(__bf16)acc[r][t][0], (__bf16)acc[r][t][1],
                                                              (__bf16)acc[r][t][2], (__bf16)acc[r][t][3]};
                } else {
                    *reinterpret_cast<f32x4 *>(dst) = acc[r][t];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (n + i < g.N) dst[i] = (T)acc[r][t][i];
            }
        }
}

// ---- decode batches of 17 .. 64 tokens: weight streaming with the activations shared through LDS ---

// Above 16 tokens the kernel above is bound by its own re-reads of the activations: every
// workgroup (16 RT rows of W) fetches all of X from L2, which for 64 tokens is four times the
// weight traffic at RT = 1.  Here the eight waves of a workgroup split N instead of K (16 rows of
// W each, 128 per workgroup) and share one copy of X: per 128-wide K super-step the workgroup
// loads the [16 MT, 128] slice of X once, through registers into a double-buffered LDS tile (rows
// padded by 16 bytes: the 16 rows a quarter-wave reads then fall on different banks), and every
// wave reads its MFMA fragments from there; W goes from global memory to registers, 64 contiguous
// bytes per lane and super-step, four super-steps ahead.  X then costs 1/8 of the weight traffic
// per token tile.  A narrow N (N = 4096: 32 workgroups) is made up for by K slabs across
// workgroups when the caller passes a workspace: a work item is (slab, row group), partial sums go
// to ws[slab][M][N] and splitk_reduce_kernel adds them in ascending order.  Lane roles as above:
// row r = lane % 16 of the wave's 16 W rows (or of a token tile), group g = lane / 16 holds the
// 32 k values [32 g, 32 g + 32) of a super-step; accumulator i: W row 4 g + i, token lane % 16.
template <int MT, bool OUT_BF16>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void bf16_decode_kernel(GemmArgs g,
                                                                                                  int row_groups)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int XROW = 256 + 16;                 // bytes per X row in LDS (128 BF16 + padding)
    constexpr int XBUF = MT * 16 * XROW;           // one buffer
    constexpr int XCH = MT * 16 * 16 / 512;        // 16-byte chunks of the X slice per thread: MT / 2 (MT even)
    static_assert(MT == 2 || MT == 4, "token tiles in pairs: the X slice is loaded by 512 threads");
    static_assert(XCH == 1 || XCH == 2, "one or two 16-byte chunks of X per thread and super-step");
    __shared__ __attribute__((aligned(16))) char xl[2 * XBUF];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = lane & 15, grp = lane >> 4;
    const int rg = (int)(blockIdx.x % row_groups), slab = (int)(blockIdx.x / row_groups);
    const int64_t n0 = (int64_t)rg * 128 + wave * 16;
    const int S = (int)(g.K / 128);
    const int SL = (S + g.ksplit - 1) / g.ksplit;
    const int s0 = slab * SL < S ? slab * SL : S, s1 = s0 + SL < S ? s0 + SL : S;

    int64_t wr = n0 + row;
    wr = wr < g.N ? wr : g.N - 1;
    const uint4 *wp = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(g.b) + wr * g.ldb + grp * 32);
    // this thread's chunks of the X slice: chunk c = tid + 512 u -> token c / 16, bytes 16 (c % 16) of the 256
    const uint4 *xg[XCH];
    int xdst[XCH];
#pragma unroll
    for (int u = 0; u < XCH; ++u) {
        const int c = tid + 512 * u;
        int64_t tok = c >> 4;
        xdst[u] = (int)tok * XROW + (c & 15) * 16;
        tok = tok < g.M ? tok : g.M - 1;
        xg[u] = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(g.a) + tok * g.lda) + (c & 15);
    }
    // Register rings, four super-steps deep: slot of X(st) and of W(st) = (st - s0) % 4.  The X ring
    // is a set of named registers (as an array the compiler moved it to LDS and waited for every
    // load right after issuing it); the W ring is indexed by compile-time constants only.
    uint4 xa0, xa1, xa2, xa3, xb0, xb1, xb2, xb3, wq[4][4];
    xb0 = xb1 = xb2 = xb3 = make_uint4(0, 0, 0, 0);
    auto load_x = [&](int st, uint4 &ra, uint4 &rb) __attribute__((always_inline)) {
        st = st < S ? st : S - 1;
        ra = xg[0][st * 16];
        if constexpr (XCH > 1) rb = xg[XCH - 1][st * 16];
    };
    auto store_x = [&](auto bufc, const uint4 &ra, const uint4 &rb) __attribute__((always_inline)) {
        constexpr int B = decltype(bufc)::value;
        *reinterpret_cast<uint4 *>(xl + B * XBUF + xdst[0]) = ra;
        if constexpr (XCH > 1) *reinterpret_cast<uint4 *>(xl + B * XBUF + xdst[XCH - 1]) = rb;
    };
    auto load_w = [&](int st, auto slot) __attribute__((always_inline)) {
        constexpr int Q = decltype(slot)::value;
        st = st < S ? st : S - 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) wq[Q][j] = wp[st * 16 + j];
    };
    f32x4 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    // all fragment reads of a super-step are issued before its first MFMA (one LDS round trip per
    // step instead of one per MFMA), and the MT accumulation chains are interleaved
    auto compute = [&](auto bufc, auto slot) __attribute__((always_inline)) {
        constexpr int B = decltype(bufc)::value, Q = decltype(slot)::value;
        uint4 xf[MT][4];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const char *xrow = xl + B * XBUF + (t * 16 + row) * XROW + grp * 64;
#pragma unroll
            for (int j = 0; j < 4; ++j) xf[t][j] = *reinterpret_cast<const uint4 *>(xrow + j * 16);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wq[Q][j]),
                                                                 __builtin_bit_cast(bf16x8, xf[t][j]), acc[t], 0, 0, 0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // prologue: X(s0) into buffer 0; X(s0 + 1 .. s0 + 4) and W(s0 .. s0 + 3) in registers
    // (issue order pinned: the load counter is in order, and what the loop may leave in flight
    // follows from the order here)
    load_x(s0, xa0, xb0);
    load_w(s0, I0{});
    __builtin_amdgcn_sched_barrier(0);
    load_x(s0 + 1, xa1, xb1);
    load_w(s0 + 1, I1{});
    __builtin_amdgcn_sched_barrier(0);
    load_x(s0 + 2, xa2, xb2);
    load_w(s0 + 2, I2{});
    __builtin_amdgcn_sched_barrier(0);
    load_x(s0 + 3, xa3, xb3);
    load_w(s0 + 3, I3{});
    __builtin_amdgcn_sched_barrier(0);
    store_x(I0{}, xa0, xb0);
    load_x(s0 + 4, xa0, xb0);
    __builtin_amdgcn_sched_barrier(0);
    // __syncthreads() would also wait for every global load in flight (it drains the vector-memory
    // counter), i.e. expose the full HBM latency once per super-step; the barrier here only waits
    // for this wave's LDS traffic.  The loads return into registers that the compiler tracks itself.
    auto lds_barrier = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    lds_barrier();
    // Super-step st computes from buffer (st - s0) % 2; meanwhile X(st + 1) goes from registers into
    // the other buffer (everybody left it before the barrier that ended step st - 1), and the
    // registers just used are refilled four super-steps ahead, X(st + 5) and W(st + 4).  The
    // hardware counts returning loads in issue order, so a value is only waited for together
    // with everything issued before it: X, which comes from L2, is therefore fetched as far ahead
    // as W, or every step would wait for all of the weights in flight.  One barrier per step.
#define MQ_DECODE_STEP(ST, U, BUF, XA, XB)                                       \
    if ((ST) < s1) compute(std::integral_constant<int, BUF>{}, U{}); /* uniform */ \
    store_x(std::integral_constant<int, (BUF) ^ 1>{}, XA, XB);       /* X(st + 1) */ \
    load_x((ST) + 5, XA, XB);                                                    \
    load_w((ST) + 4, U{});                                                       \
    lds_barrier();                                                               \
    __builtin_amdgcn_sched_barrier(0);
    for (int st = s0; st < s1; st += 4) {
        MQ_DECODE_STEP(st, I0, 0, xa1, xb1)
        MQ_DECODE_STEP(st + 1, I1, 1, xa2, xb2)
        MQ_DECODE_STEP(st + 2, I2, 0, xa3, xb3)
        MQ_DECODE_STEP(st + 3, I3, 1, xa0, xb0)
    }
#undef MQ_DECODE_STEP

    // accumulator i: W row 4 * grp + i, token lane % 16
    const int64_t n = n0 + 4 * grp;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int64_t m = t * 16 + row;
        if (m >= g.M || n >= g.N) continue;
        if (g.ksplit > 1) {  // unscaled partial sums of this slab (N % 4 == 0 here)
            *reinterpret_cast<f32x4 *>(g.ws + ((int64_t)slab * g.M + m) * g.N + n) = acc[t];
            continue;
        }
        using T = std::conditional_t<OUT_BF16, __bf16, float>;
        T *dst = static_cast<T *>(g.y) + m * g.ldy + n;
        if (n + 3 < g.N) {
            if constexpr (OUT_BF16) {
                typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                *reinterpret_cast<bf16x4 *>(dst) =
                    bf16x4{(__bf16)acc[t][0], (__bf16)acc[t][1], (__bf16)acc[t][2], (__bf16)acc[t][3]};
            } else {
                *reinterpret_cast<f32x4 *>(dst) = acc[t];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (n + i < g.N) dst[i] = (T)acc[t][i];
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
        const uint8_t *ac = static_cast<const uint8_t *>(g.a) + m * g.a_c_row;
        const uint8_t *bc = static_cast<const uint8_t *>(g.b) + n * g.b_c_row;
        const uint8_t *as = g.a_scales + m * g.a_s_row, *bs = g.b_scales + n * g.b_s_row;
        for (int64_t b = 0; b < g.K / 16; ++b) {
            // block b of a row: K step b/4 (stride *_step), 8 code bytes and 1 scale byte at b%4
            const uint8_t *xa = ac + (b >> 2) * g.a_c_step + (b & 3) * 8;
            const uint8_t *xb = bc + (b >> 2) * g.b_c_step + (b & 3) * 8;
            float dot = 0.0f;  // sum of 16 products q*q: multiples of 1/4 up to 576, exact
            for (int i = 0; i < 8; ++i) {
                const uint32_t x = xa[i], w = xb[i];
                dot += e2m1_f32(x & 15u) * e2m1_f32(w & 15u);
                dot += e2m1_f32(x >> 4) * e2m1_f32(w >> 4);
            }
            const float sx = __builtin_amdgcn_cvt_pk_f32_fp8((int)as[(b >> 2) * g.a_s_step + (b & 3)], false)[0];
            const float sw = __builtin_amdgcn_cvt_pk_f32_fp8((int)bs[(b >> 2) * g.b_s_step + (b & 3)], false)[0];
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

// ---- matrix-pipe rate probe -------------------------------------------------------------------

// A loop of independent v_mfma_f32_32x32x16_f16 on pseudo-random operands, one wave per SIMD,
// nothing else: what the matrix pipe sustains on this chip at the clock its power management
// allows for realistic operand toggling.  Used by the benchmark as the measured roof next to the
// published peak.
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *out, int iters)
{
    f16x8 a[4], b[4];
    f32x16 c0, c1, c2, c3;
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int q = 0; q < 4; ++q)
        for (int j = 0; j < 8; ++j) {
            h = h * 1664525u + 1013904223u;
            a[q][j] = (_Float16)(((int)(h >> 20) - 2048) * (1.0f / 512.0f));
            h = h * 1664525u + 1013904223u;
            b[q][j] = (_Float16)(((int)(h >> 20) - 2048) * (1.0f / 512.0f));
        }
    for (int r = 0; r < 16; ++r) c0[r] = c1[r] = c2[r] = c3[r] = 0.0f;
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0], b[0], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1], b[1], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[2], b[2], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[3], b[3], c3, 0, 0, 0);
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1], b[2], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[2], b[3], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[3], b[0], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0], b[1], c3, 0, 0, 0);
    }
    float s = 0.0f;
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    if (s == 123.456f) out[0] = s;  // keeps the loop alive; practically never true
}

// ---- launchers ------------------------------------------------------------------------------

template <class Kern>
int launch_tiles(Kern kern, size_t lds_bytes, int bm, int bn, int threads, const GemmArgs &g, hipStream_t s)
{
    const int64_t tiles_m = (g.M + bm - 1) / bm, tiles_n = (g.N + bn - 1) / bn;
    if (tiles_m * tiles_n > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(threads), lds_bytes, s>>>(g, (int)tiles_m, (int)tiles_n);
    return note_launch(hipGetLastError());
}

// Persistent register-direct kernels: one workgroup per compute unit (a wave of 512 registers
// fills its SIMD), each walking tile ids wg, wg + grid, ...
inline int compute_units(int &n)
{
    static std::atomic<int> cus{0};
    n = cus.load(std::memory_order_acquire);
    if (n == 0) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return note_launch(e);
        n = n >= NUM_XCD ? n / NUM_XCD * NUM_XCD : NUM_XCD;  // a multiple of the XCD count keeps wg % 8 = XCD
        cus.store(n, std::memory_order_release);
    }
    return MQ_OK;
}

template <class Kern>
int launch_persistent(Kern kern, int bm, int bn, size_t lds_bytes, const GemmArgs &g, hipStream_t s, int cus,
                      int items_per_tile = 1)
{
    const int64_t tiles_m = (g.M + bm - 1) / bm, tiles_n = (g.N + bn - 1) / bn;
    if (tiles_m * tiles_n > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    const int64_t items = tiles_m * tiles_n * items_per_tile;
    if (items > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    const int64_t grid = items < cus ? items : cus;
    kern<<<dim3((unsigned)grid), dim3(256), lds_bytes, s>>>(g, (int)tiles_m, (int)tiles_n);
    return note_launch(hipGetLastError());
}

// One workgroup of S waves per (32 TM) x (32 TN) tile.
template <int TM, int TN, int MAXS, int NSETS, bool OUT_BF16>
int launch_small(const GemmArgs &g0, hipStream_t s, SmallPlan plan)
{
    const int S = plan.waves;
    GemmArgs g = g0;
    g.ksplit = plan.slabs;
    const int64_t tiles_m = (g.M + 32 * TM - 1) / (32 * TM), tiles_n = (g.N + 32 * TN - 1) / (32 * TN);
    if (tiles_m * tiles_n * g.ksplit > 0x7FFFFFFF || S < 1 || S > MAXS || g.ksplit < 1) return MQ_ERR_SHAPE;
    constexpr int PASS = TM * TN < 4 ? TM * TN : 4;
    const size_t lds = S > 1 ? (size_t)S * PASS * 4096 : 0;
    gemm_fp4_small<TM, TN, MAXS, NSETS, OUT_BF16>
        <<<dim3((unsigned)(tiles_m * tiles_n * g.ksplit)), dim3(64 * S), lds, s>>>(g, (int)tiles_m, (int)tiles_n);
    int rc = note_launch(hipGetLastError());
    if (rc != MQ_OK || g.ksplit == 1) return rc;
    const int64_t quads = g.M * (g.N / 4);
    splitk_reduce_kernel<OUT_BF16><<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s>>>(g);
    return note_launch(hipGetLastError());
}

template <bool FP4, bool OUT_BF16>
int launch_simple(const GemmArgs &g, hipStream_t s)
{
    dim3 grid((unsigned)((g.N + 15) / 16), (unsigned)((g.M + 15) / 16));
    if ((g.M + 15) / 16 > 65535) return MQ_ERR_SHAPE;
    gemm_simple_kernel<FP4, OUT_BF16><<<grid, dim3(256), 0, s>>>(g);
    return note_launch(hipGetLastError());
}

// Token tiles by M.  Row tiles per wave, measured on N = 4096 .. 28672: more than one pays only
// while the grid keeps every CU busy several times over, and not for a single token (whose
// activations come from L1 anyway).
template <bool OUT_BF16>
int launch_skinny(const GemmArgs &g, hipStream_t s)
{
    const int mt = (int)((g.M + 15) / 16);
    const int rt = g.M <= 4 ? 1 : g.N >= 24576 ? 4 : g.N >= 6144 ? 2 : 1;
    const dim3 grid((unsigned)((g.N + 16 * rt - 1) / (16 * rt))), block(512);
#define MQ_SKINNY(MT_, RT_) bf16_skinny_kernel<MT_, RT_, (MT_ + RT_ <= 5), OUT_BF16><<<grid, block, 0, s>>>(g)
#define MQ_SKINNY_RT(MT_) (rt == 4 ? MQ_SKINNY(MT_, 4) : rt == 2 ? MQ_SKINNY(MT_, 2) : MQ_SKINNY(MT_, 1))
    if (mt == 1)
        MQ_SKINNY_RT(1);
    else if (mt == 2)
        MQ_SKINNY_RT(2);
    else if (mt == 3)
        MQ_SKINNY_RT(3);
    else
        MQ_SKINNY_RT(4);
#undef MQ_SKINNY_RT
#undef MQ_SKINNY
    return note_launch(hipGetLastError());
}

// 17 .. 64 tokens with K % 128 == 0 and the row stride rules of the decode kernel.
template <bool OUT_BF16>
int launch_decode(const GemmArgs &g0, hipStream_t s, int slabs)
{
    GemmArgs g = g0;
    g.ksplit = slabs;
    const int64_t row_groups = (g.N + 127) / 128;
    if (row_groups * slabs > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    const dim3 grid((unsigned)(row_groups * slabs)), block(512);
    if (g.M <= 32)
        bf16_decode_kernel<2, OUT_BF16><<<grid, block, 0, s>>>(g, (int)row_groups);
    else
        bf16_decode_kernel<4, OUT_BF16><<<grid, block, 0, s>>>(g, (int)row_groups);
    int rc = note_launch(hipGetLastError());
    if (rc != MQ_OK || slabs == 1) return rc;
    const int64_t quads = g.M * (g.N / 4);
    splitk_reduce_kernel<OUT_BF16><<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s>>>(g);
    return note_launch(hipGetLastError());
}

template <bool FP4, bool OUT_BF16>
int launch_any(const GemmArgs &g, hipStream_t s)
{
    if (g.M == 0 || g.N == 0) return MQ_OK;
    if constexpr (!FP4) {
        // decode shapes: a few tokens against the whole weight matrix
        if (g.M > 16 && g.M <= 64 && g.K % 128 == 0) {
            int cus = 0;
            if (int rc = compute_units(cus)) return rc;
            const int slabs = gemm_bf16_decode_slabs(g.M, g.N, g.K, g.ws ? g.ws_bytes : 0, cus);
            if (slabs > 0) return launch_decode<OUT_BF16>(g, s, slabs);
        }
        if (g.M <= 64 && g.K % 128 == 0 && (g.N + 15) / 16 <= 0x7FFFFFFF) return launch_skinny<OUT_BF16>(g, s);
    }
    // The tiled kernels step K by 64.
    if (g.K % BK != 0) return launch_simple<FP4, OUT_BF16>(g, s);
    const int64_t big_tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    using Mid = PCfg<256, 128, 2, 2>;   // BF16 only: 4 waves of 128x64
    using Small = PCfg<128, 128, 2, 2>;  // BF16 only: 4 waves of 64x64
    const int64_t mid_tiles = ((g.M + 255) / 256) * ((g.N + 127) / 128);
    if constexpr (FP4) {
        // Three workgroup shapes: 256x256 (whole K per wave), 256x128 with K split over wave
        // pairs, 128x128 with K split over the four waves; once the 128x128 tiles fill at least
        // half of the chip, the one whose rounds of workgroups cost least wins, a split workgroup
        // being charged 55 / 34 percent of a whole one (measured on M = 512 .. 8192).
        int cus = 0;
        if (int rc = compute_units(cus)) return rc;
        // A few hundred tokens (at most 2 x CUs tiles of 64x64): the small-tile kernel, one launch
        // (plus, for a long K with very few tiles and a workspace, slabs of K across workgroups).
        const SmallPlan plan = gemm_fp4_small_plan(g.M, g.N, g.K, g.ws ? g.ws_bytes : 0, cus);
        if (plan.waves > 0) return launch_small<2, 2, 8, 4, OUT_BF16>(g, s, plan);
        // From here on the 128x128 wave tiles fill at least half of the chip.
        const int64_t small_tiles = ((g.M + 127) / 128) * ((g.N + 127) / 128);
        const int64_t r1 = (big_tiles + cus - 1) / cus, r2 = (mid_tiles + cus - 1) / cus,
                      r4 = (small_tiles + cus - 1) / cus;
        const int64_t c1 = 100 * r1, c2 = 55 * r2, c4 = 34 * r4;
        auto launch_variant = [&](int variant, const GemmArgs &ga) {
            if (variant == 4) return launch_persistent(gemm_fp4_direct<OUT_BF16, 4>, 128, 128, 128 * 1024, ga, s, cus);
            if (variant == 2) return launch_persistent(gemm_fp4_direct<OUT_BF16, 2>, 256, 128, 128 * 1024, ga, s, cus);
            return launch_persistent(gemm_fp4_direct<OUT_BF16, 1>, 256, 256, 0, ga, s, cus);
        };
        const int one = (2 * mid_tiles < cus || (c4 < c1 && c4 < c2)) ? 4 : c2 < c1 ? 2 : 1;
        const int64_t one_cost = one == 4 ? c4 : one == 2 ? c2 : c1;
        // Two launches instead of one when the tiles leave a ragged last round: the first columns
        // of N in one shape, the remaining columns in another (M = 2048, N = 28672: 3 rounds of
        // whole tiles + 16 tile columns as 256x128 tiles cost 3.55 tile times instead of 3.85;
        // M = 2048, N = 6144: 256x128 tiles on 4096 columns + 128x128 tiles on 2048 cost 0.89
        // instead of 1).  Rounds are charged as above, the second launch four microseconds in
        // units of a hundredth of a whole tile's time (0.022 us per K element + 6).
        auto cost_of = [&](int variant, int64_t n) {
            const int64_t bm = variant == 4 ? 128 : 256, bn = variant == 1 ? 256 : 128;
            const int64_t tiles = ((g.M + bm - 1) / bm) * ((n + bn - 1) / bn);
            return (variant == 1 ? 100 : variant == 2 ? 55 : 34) * ((tiles + cus - 1) / cus);
        };
        const int64_t second = (int64_t)(400.0 / (0.022 * (double)g.K + 6.0)) + 1;
        int64_t best = one_cost, best_n = 0;
        int best_a = 0, best_b = 0;
        static const int variants[3] = {1, 2, 4};
        for (int64_t n = 256; n < g.N; n += 256)
            for (int va : variants)
                for (int vb : variants) {
                    if (va == vb) continue;
                    const int64_t c = cost_of(va, n) + cost_of(vb, g.N - n) + second;
                    if (c < best) best = c, best_n = n, best_a = va, best_b = vb;
                }
        if (best_n > 0) {
            GemmArgs ga = g, gb = g;
            ga.N = best_n;
            gb.N = g.N - best_n;
            gb.b = static_cast<const char *>(g.b) + best_n * g.b_c_row;
            gb.b_scales = g.b_scales + best_n * g.b_s_row;
            gb.y = static_cast<char *>(g.y) + best_n * (int64_t)(OUT_BF16 ? 2 : 4);
            if (int rc = launch_variant(best_a, ga)) return rc;
            return launch_variant(best_b, gb);
        }
        return launch_variant(one, g);
    } else {
        // Same choice by rounds of workgroups as above: 256x256 tiles, or 256x128 tiles (half the
        // work per workgroup, somewhat less efficient) when they waste less of the last round;
        // 128x128 register-staged tiles for small problems.
        int cus = 0;
        if (int rc = compute_units(cus)) return rc;
        const int64_t r1 = (big_tiles + cus - 1) / cus, r2 = (mid_tiles + cus - 1) / cus;
        using D = PCfg<256, 256, 2, 2>;
        if (2 * mid_tiles >= cus && 100 * r1 > 58 * r2)
            return launch_tiles(gemm_bf16_d2l<Mid, OUT_BF16>, Mid::LDS_BYTES, 256, 128, Mid::THREADS, g, s);
        if (2 * mid_tiles >= cus)
            return launch_tiles(gemm_bf16_d2l<D, OUT_BF16>, D::LDS_BYTES, 256, 256, D::THREADS, g, s);
        return launch_tiles(gemm_bf16_pipelined<Small, OUT_BF16>, Small::LDS_BYTES, 128, 128, Small::THREADS, g, s);
    }
}

}  // namespace

// Raises the dynamic-LDS limit of every kernel that asks for more than the default.  Done once
// per device before the first launch (mq_init, or the first product on a device), so that no
// launch path has one-time work left that a stream capture could trip over.
int configure_gemm_kernels()
{
    auto set = [](auto kern, size_t bytes) {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)bytes);
    };
    using D = PCfg<256, 256, 2, 2>;
    using Mid = PCfg<256, 128, 2, 2>;
    using Small = PCfg<128, 128, 2, 2>;
    constexpr size_t X = 128 * 1024;  // accumulator exchange of the K-split variants
    hipError_t e = hipSuccess;
    auto both = [&](auto k_bf16, auto k_fp32, size_t bytes) {
        if (e == hipSuccess) e = set(k_bf16, bytes);
        if (e == hipSuccess) e = set(k_fp32, bytes);
    };
    both(gemm_fp4_direct<true, 2>, gemm_fp4_direct<false, 2>, X);
    both(gemm_fp4_direct<true, 4>, gemm_fp4_direct<false, 4>, X);
    both(gemm_fp4_small<2, 2, 8, 4, true>, gemm_fp4_small<2, 2, 8, 4, false>, X);
    both(gemm_bf16_d2l<D, true>, gemm_bf16_d2l<D, false>, D::LDS_BYTES);
    both(gemm_bf16_d2l<Mid, true>, gemm_bf16_d2l<Mid, false>, Mid::LDS_BYTES);
    both(gemm_bf16_pipelined<Small, true>, gemm_bf16_pipelined<Small, false>, Small::LDS_BYTES);
    return note_launch(e);
}

// Does the small-tile kernel serve this problem, with how many waves per 64x64 tile and how
// many K slabs across workgroups?  Measured on the Llama-3-8B layer set at 64 .. 1024 tokens (one
// GPU, one launch inside a HIP graph): up to 2 x CUs tiles of 64x64 it beats the 128x128 wave tiles
// (M = 128, N = 4096, K = 4096: 10.9 us against 19.2 with slabs of 128x128 tiles and 27 without),
// beyond that the larger tiles' lower conversion work per MFMA wins.  Eight waves per tile (two
// per SIMD) while every tile gets a compute unit of its own, four beyond.  A launch costs about
// 6.5 us plus 0.5 us per K step of a wave; slabs add a second launch and the partial sums' way
// through the workspace, about 4.5 us: they are used when at most half of the compute units
// would otherwise hold a tile and the K steps they take off each wave are worth more than that.
SmallPlan gemm_fp4_small_plan(int64_t M, int64_t N, int64_t K, int64_t ws_bytes, int cus)
{
    SmallPlan plan{0, 1};
    if (M <= 0 || N <= 0 || K <= 0 || K % BK != 0) return plan;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64), kt = K / BK;
    if (tiles > 2 * (int64_t)cus) return plan;
    int64_t waves = tiles <= cus ? 8 : 4;
    if (waves > kt / 2) waves = kt / 2 > 0 ? kt / 2 : 1;  // at least two K steps per wave
    plan.waves = (int)waves;
    if (ws_bytes > 0 && N % 4 == 0 && 2 * tiles <= cus) {
        int64_t ks = cus / tiles;                                  // one round of work items
        if (ks > kt / (waves * 4)) ks = kt / (waves * 4);          // at least four K steps per wave
        if (ks > ws_bytes / (M * N * 4)) ks = ws_bytes / (M * N * 4);
        // K-loop time saved, (kt / waves) * (1 - 1 / ks) * 0.5 us, against 4.5 us for the second pass
        if (ks >= 2 && kt * (ks - 1) > 9 * waves * ks) plan.slabs = (int)ks;
    }
    return plan;
}

// K slabs for the decode-batch BF16 kernel (17 .. 64 tokens), given this much workspace; 0: the
// kernel does not serve the problem, 1: no slabs.  Measured on N = 4096 .. 28672 (us per launch,
// this kernel / the K-split kernel above): a wide N (at least CUs/2 row groups of 128) needs no
// slabs: gate_up 41.5 / 69.5 at 64 tokens, 38.3 / 51.1 at 32.  A narrow N needs slabs, i.e. a
// workspace and a second pass of about 5 us, which pays above 32 tokens with a long K (down,
// K = 14336: 42.6 / 63.4 at 64 tokens, 40.7 / 51.6 at 48) and not otherwise (K = 4096 at 48 tokens:
// o 16.1 / 17.0 but qkv 26.1 / 21.6; o at 32 tokens 14.5 / 13.3).  Slabs fill about two workgroups
// per compute unit, keep at least four 128-wide super-steps each, and keep the partial sums'
// traffic (8 bytes per output and slab) below half of the weights'.
int gemm_bf16_decode_slabs(int64_t M, int64_t N, int64_t K, int64_t ws_bytes, int cus)
{
    if (M <= 16 || M > 64 || N <= 0 || K <= 0 || K % 128 != 0) return 0;
    const int64_t groups = (N + 127) / 128, steps = K / 128;
    if (2 * groups >= cus) return 1;
    if (M <= 32 || K < 8192 || ws_bytes <= 0 || N % 4 != 0) return 0;
    int64_t ks = 2 * cus / groups;
    if (ks > steps / 4) ks = steps / 4;
    if (ks > K / (8 * M)) ks = K / (8 * M);
    if (ks > ws_bytes / (M * N * 4)) ks = ws_bytes / (M * N * 4);
    if (ks < 2 || 2 * groups * ks < cus) return 0;  // too few workgroups even so
    return (int)ks;
}

int launch_mfma_probe(float *out, int iters, int blocks, hipStream_t s)
{
    mfma_probe_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(out, iters);
    return note_launch(hipGetLastError());
}

int launch_gemm_fp4(const GemmArgs &g, hipStream_t s)
{
    return g.out == MQ_OUT_BF16 ? launch_any<true, true>(g, s) : launch_any<true, false>(g, s);
}

int launch_gemm_bf16(const GemmArgs &g, hipStream_t s)
{
    return g.out == MQ_OUT_BF16 ? launch_any<false, true>(g, s) : launch_any<false, false>(g, s);
}

}  // namespace mq
