// Fast path for large token counts: every product of the layer as a plain bf16 GEMM
//
//   C[M x N] = alpha * sum_seg  A_seg[M x K_seg] * B_seg[K_seg x N]        (fp32 accumulate)
//
// with both operands bf16, each stored either rows x K (K contiguous) or K x rows (rows contiguous).
// NF4 operands are dequantised to bf16 once per call (nf4_dequantize_kernel, or the fold epilogue
// below) instead of once per output tile; at thousands of tokens that costs a few per cent of the
// GEMM and keeps every VALU and LDS cycle of the inner loop for feeding the matrix cores.
//
// Work-group: 256 threads = 4 waves (2 x 2), tile BM x BN x 64; v_mfma_f32_16x16x32_bf16 for the plain bf16
// products and the fp32 slices on 256-row tiles (most of a training step), v_mfma_f32_32x32x16_bf16 for everything
// else (fold, merge, compensation, 128x128 tiles).
//  * operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, no registers, no
//    ds_write) into two stages.  The loads of a tile are issued one by one between the MFMAs, spread over
//    the slots, never in a burst (the memory pipeline of a compute unit limits the requests in flight, and a
//    stalled load holds back the MFMAs behind it in the in-order wave).  The 16x16x32 loop has two barriers per
//    k-tile -- one as soon as the tile's last fragments are in registers, which frees its stage for the tile after
//    next, one that publishes the next tile -- so a load has 1.25 to 2 k-tiles to land; the 32x32x16 loop has one
//    barrier and issues half a tile after it and half in the next k-step.  Loads past the end of the range are
//    switched off through EXEC (or, in the kernel variants for contractions of whole k-tiles, fetch the last tile
//    once more into a stage nobody reads), and a k-tile that is not full (the last one of a K segment that is not a
//    multiple of 64) is staged through registers with zero fill instead;
//  * 16-byte chunks of an LDS row are XOR-swizzled so that fragment reads are free of bank conflicts (the
//    pattern depends on the MFMA shape); the swizzle is applied on the global side (which chunk a lane
//    fetches), the LDS side of a direct load is lane-linear;
//  * K-contiguous tiles are read back with one 16-byte read per fragment, row-contiguous tiles
//    with two transposing reads (ds_read_b64_tr_b16): no operand is ever transposed in memory;
//  * MFMA fragments are double-buffered in registers one k-step ahead; the instruction order of the loop
//    is fixed by hand (a scheduling fence after every MFMA slot): fragment reads after the first MFMAs of
//    a step, direct loads after the last ones;
//  * the accumulators are kept transposed (lane = row m, registers = 4 consecutive n) so the
//    epilogues can pack along n: bf16 results are staged through LDS and leave as whole
//    16-byte-per-lane row segments; the fold epilogue adds the dequantised NF4 weight on the way;
//    the merge epilogue requantises 64-blocks in registers (paper sec. 5.1, Alg. 1 line 5);
//  * tiles are dealt to the 8 XCDs in contiguous ranges and walked in groups of 4 or 8 tile rows so that the
//    work-groups sharing an L2 also share operand panels.
// The 256x256 kernels use every vector register; tests/test_isa_guard.py checks their generated loop.
#include <string.h>

#include <type_traits>

#include "loqt_internal.h"

namespace loqt {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BK = 64;
constexpr int ROWB = 128;  // bytes of one LDS row (64 bf16)

#define LOQT_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define LOQT_GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ uint32_t nib4(uint32_t word, int e) {
    // element e (0..3) of a 2-byte group: byte e/2, even e in the high nibble
    return (word >> (8 * (e >> 1) + ((e & 1) ? 0 : 4))) & 15u;
}

template <int BM, int BN, int NS = 2>
struct NtCfg {
    static constexpr int TM = BM / 64, TN = BN / 64;   // 32x32 tiles per wave
    static constexpr int WTM = BM / 2, WTN = BN / 2;   // wave tile
    static constexpr int STAGE = (BM + BN) * ROWB;
    static constexpr int NCH = (BM + BN) / 32;         // 16-byte chunks per thread per stage
    static constexpr int NCHA = BM / 32;               // of which belong to A
    static constexpr int NCHB = BN / 32;               // and to B
    static constexpr int EPITCH = WTN * 2 + 8;         // staging pitch of the bf16 epilogue
    static constexpr int SMEM_MAIN = NS * STAGE;       // NS stages: tiles kt .. kt+NS-1 are in LDS or in flight
    static constexpr int SMEM_EPI = 4 * WTM * EPITCH;
    static constexpr int SMEM = (SMEM_MAIN > SMEM_EPI ? SMEM_MAIN : SMEM_EPI) + 64;
};

// One output tile.  L: index of the tile in the walk order described above (tiles past the end return at once);
// split: slice of the contraction (EPI_F32_SPLITK), else 0.
// NOTAIL (16x16x32 form only): every K segment is a whole number of k-tiles, so no tile ever takes the register path
// and the loads need no mask -- see hot_load_live.
template <int BM, int BN, int EPI, bool ARC, bool BRC, int NS = 2, bool NOTAIL = false>
__device__ __forceinline__ void nt_gemm_tile(const GemmParams& p, const int L, const int split) {
    using Cfg = NtCfg<BM, BN, NS>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, STAGE = Cfg::STAGE;
    constexpr int NM = TM * TN;  // MFMAs per k16 step
    constexpr int NL = Cfg::NCH / 2;                    // direct loads of half a k-tile
    constexpr int LPS = (NL + NM - 1) / NM, NSL = NL / LPS;  // LPS loads after each of the last NSL MFMAs of a k16 step
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);

    // ---- tile of this work-group: contiguous range per XCD, groups of GM tile rows inside
    const int tiles_m = (p.M + BM - 1) / BM;
    const int tiles_n0 = (p.N + BN - 1) / BN, tiles_n = tiles_n0 + (p.Nx + BN - 1) / BN;
    if (L >= tiles_m * tiles_n) return;
    constexpr int GM = (EPI == EPI_BF16 && !ARC && !BRC) ? 4 : 8;  // measured per operand layout
    const int gid = L / (GM * tiles_n);
    const int first_m = gid * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int rem = L - gid * GM * tiles_n;
    const int tm = first_m + rem % gsz;
    int tn = rem / gsz;
    const bool part1 = tn >= tiles_n0;  // second column range
    if (part1) tn -= tiles_n0;
    const int m0 = tm * BM, n0 = tn * BN;
    const int N = part1 ? p.Nx : p.N;
    const float alpha = part1 ? p.alphax : p.alpha;

    const int nkt0 = (p.A[0].K + BK - 1) / BK;
    const int nkt1 = (p.A[1].K + BK - 1) / BK;
    int kt_begin = 0, kt_end = nkt0 + nkt1;
    if (EPI == EPI_F32_SPLITK) {
        const int per = (kt_end + p.splits - 1) / p.splits;
        kt_begin = split * per;
        kt_end = min(kt_end, kt_begin + per);
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    // The plain bf16 products on 256x256 tiles (y, dx: most of a training step) use v_mfma_f32_16x16x32_bf16
    // instead: the same flops per cycle and the same LDS bytes, but a quarter of the accumulator registers read and
    // written per instruction, which on this power-limited part is worth a few per cent of clock (measured: 5 %
    // with both operands K-contiguous, 1 % with B stored K x rows; on 128x128 tiles nothing, or a loss).  Their accumulators:
    // 16x16 tiles (ti, tj) of the wave tile, lane = row ti*16 + (lane & 15), register r = column tj*16 + 4*(lane >> 4) + r.
    constexpr bool MF16 = NS == 2 && BM == 256 &&
                          ((EPI == EPI_BF16 && (BN == 256 || BN == 128)) || (EPI == EPI_F32_SPLITK && BN == 128));
    constexpr int TM2 = MF16 ? 2 * TM : 1, TN2 = MF16 ? 2 * TN : 1;
    f32x4 acc16[TM2][TN2];
#pragma unroll
    for (int i = 0; i < TM2; ++i)
#pragma unroll
        for (int j = 0; j < TN2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc16[i][j][e] = 0.f;

    // merge with 128x128 tiles: the old codes and scales of this lane's 64-blocks are fetched here, ahead of the
    // product, so that the epilogue does not start with a round trip to memory (18 registers; the 256-wide tiles
    // have none to spare).  Row m = m0 + wm*WTM + ti*32 + (lane & 31), block b of the wave's columns.
    constexpr bool MERGE_PREFETCH = EPI == EPI_MERGE && BM == 128 && BN == 128;
    constexpr int NPB = MERGE_PREFETCH ? TM * (TN / 2) : 1;
    uint4 pre_cw[NPB][2];
    float pre_am[NPB];
    if constexpr (MERGE_PREFETCH) {
        const int64_t ldb = p.w_ld >> 1, lda = p.w_ld >> 6;
#pragma unroll
        for (int ti = 0; ti < TM; ++ti)
#pragma unroll
            for (int b = 0; b < TN / 2; ++b) {
                const int m = m0 + wm * Cfg::WTM + ti * 32 + (lane & 31);
                const int nb = n0 + wn * Cfg::WTN + b * 64;
                const int k = ti * (TN / 2) + b;
                pre_cw[k][0] = pre_cw[k][1] = make_uint4(0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u);
                pre_am[k] = 0.f;
                if (m < p.M && nb < p.w_ld) {
                    pre_am[k] = p.w_absmax[m * lda + (nb >> 6)];
                    pre_cw[k][0] = *reinterpret_cast<const uint4*>(p.w_codes + m * ldb + (nb >> 1));
                    pre_cw[k][1] = *reinterpret_cast<const uint4*>(p.w_codes + m * ldb + (nb >> 1) + 16);
                }
            }
    }

    // ---- staging.  Chunk i of this thread is LDS slot (i*256 + tid) of the operand tile (the LDS side
    // of a direct load is lane-linear); which 16 bytes of global memory go there carries the swizzle.
    //  K-contiguous operand (rows x K): tile [row][64 k], slot -> row slot>>3, physical chunk slot&7,
    //    logical chunk (slot&7) ^ swz(row); rows are i*32 apart, so the chunk column is the same for all i.
    //  row-contiguous operand (K x rows): tile [64 k][BR rows], slot -> k = slot / (BR/8), physical chunk
    //    slot % (BR/8), logical chunk physical ^ 4*(k&3); read back transposed by ds_read_b64_tr_b16.  Half a
    //    wave of such a read touches 4 k rows x 4 chunks; a row is a multiple of 256 bytes (all 64 banks), so
    //    the XOR has to move the four k rows to four different 64-byte groups of chunks.
    // Addresses are a wave-uniform 64-bit base (operand pointer + tile origin + K offset, scalar
    // registers) plus a 32-bit per-lane byte offset inside the tile's rows, so the loads use the
    // scalar-base form and no 64-bit address arithmetic runs on the vector unit.
    // A k-tile that is not full (the last one of a K segment whose extent is not a multiple of 64) takes the
    // path below instead: through registers, elements past K zeroed, ordinary LDS stores.
    // XOR of the chunk index of k row kk of a row-contiguous tile.  The 16x16x32 form reads k rows kk and kk + 8 in
    // the same half-wave (lanes 0-15 and 16-31), so there bit 3 of kk moves the row by a further 32 bytes.
    // XOR of the chunk index of row `row` of a K-contiguous tile.  A 16-byte LDS read is served in sets of
    // 16 lanes, {0-3, 12-15, 20-23, 24-27} and {4-7, 8-11, 16-19, 28-31} of each half-wave (measured), and a row is
    // half the banks.  In the 32x32x16 form a set holds 16 different rows of one chunk column pair; in the
    // 16x16x32 form it holds rows 0-3 and 12-15 of one column and rows 4-11 of the next, which needs another map.
    auto kc_swz = [](int row) {
        if constexpr (MF16) {
            const int e = (row >> 1) & 7;
            return (e & 1) | ((e & 2) << 1) | ((e & 4) >> 1);
        } else {
            return swz(row);
        }
    };
    auto rc_swz = [](int kk) { return (4 * (kk & 3)) ^ (MF16 ? 2 * ((kk >> 3) & 1) : 0); };
    auto tail_operand = [&](auto rc_tag, auto br_tag, const void* optr, int64_t old, int orows, int oK, int row0, int k0,
                            char* tile) {
        constexpr bool RC = decltype(rc_tag)::value;
        constexpr int BR = decltype(br_tag)::value;
        constexpr int NC = BR / 32;  // chunks per thread
        // a tile that lies wholly past the operand's last row (the merge walks the padding columns of the
        // code matrix, which can exceed `in` by more than a tile) reads the operand's first rows instead:
        // its products are never used, and the clamps below then never go negative
        if (row0 >= orows) row0 = 0;
        const int kleft = oK - k0;
        const uint32_t ld2 = (uint32_t)old * 2u;  // row pitch in bytes (a tile spans < 2^32 bytes)
        if constexpr (!RC) {
            const int r0 = tid >> 3;
            const int kc = (tid & 7) ^ kc_swz(r0);
            const int rlast = orows - 1 - row0;  // rows past the end: any valid row
            const char* sbase = reinterpret_cast<const char*>(optr) + ((int64_t)row0 * old + k0) * 2;
            const int nv = kleft - kc * 8;  // valid elements of this thread's chunk column
#pragma unroll 1
            for (int i = 0; i < NC; ++i) {
                const uint32_t off = (uint32_t)min(i * 32 + r0, rlast) * ld2 + (uint32_t)kc * 16u;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (nv > 0) {
                    v = *reinterpret_cast<const uint4*>(sbase + off);
                    uint32_t* w = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        if (2 * d >= nv) w[d] = 0;
                        else if (2 * d + 1 >= nv) w[d] &= 0xffffu;
                    }
                }
                *reinterpret_cast<uint4*>(tile + i * 4096 + tid * 16) = v;
            }
        } else {
            constexpr int CPR = BR / 8;       // chunks per k row
            constexpr int KPI = 256 / CPR;    // k rows covered by one pass of the 256 threads
            const int kq = tid / CPR;         // k of chunk i is i*KPI + kq  (KPI is a multiple of 4)
            const int clast = (((orows - 1) >> 3) << 3) - row0;  // columns past the end: any valid chunk
            const char* sbase = reinterpret_cast<const char*>(optr) + ((int64_t)k0 * old + row0) * 2;
#pragma unroll 1
            for (int i = 0; i < NC; ++i) {
                const int logical = (tid % CPR) ^ rc_swz(i * KPI + kq);
                const uint32_t off = (uint32_t)(i * KPI + kq) * ld2 + (uint32_t)min(logical * 8, clast) * 2u;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (i * KPI + kq < kleft) v = *reinterpret_cast<const uint4*>(sbase + off);
                *reinterpret_cast<uint4*>(tile + i * 4096 + tid * 16) = v;
            }
        }
    };
    // the operand of K segment `seg`, field by field (selects on scalars: a run-time index into the by-value
    // parameter block, or a copy of an Operand, would go through scratch memory)
    auto a_ptr = [&](bool seg) { return seg ? p.A[1].ptr : p.A[0].ptr; };
    auto a_ld = [&](bool seg) { return seg ? p.A[1].ld : p.A[0].ld; };
    auto a_rows = [&](bool seg) { return seg ? p.A[1].rows : p.A[0].rows; };
    auto b_ptr = [&](bool seg) { return part1 ? p.Bx.ptr : (seg ? p.B[1].ptr : p.B[0].ptr); };
    auto b_ld = [&](bool seg) { return part1 ? p.Bx.ld : (seg ? p.B[1].ld : p.B[0].ld); };
    auto b_rows = [&](bool seg) { return part1 ? p.Bx.rows : (seg ? p.B[1].rows : p.B[0].rows); };
    auto tail_tile = [&](int kt, char* stage) {
        const bool seg = kt >= nkt0;
        const int k0 = (kt - (seg ? nkt0 : 0)) * BK;
        const int segK = seg ? p.A[1].K : p.A[0].K;
        tail_operand(std::integral_constant<bool, ARC>{}, std::integral_constant<int, BM>{}, a_ptr(seg), a_ld(seg), a_rows(seg),
                     segK, m0, k0, stage);
        tail_operand(std::integral_constant<bool, BRC>{}, std::integral_constant<int, BN>{}, b_ptr(seg), b_ld(seg), b_rows(seg),
                     segK, n0, k0, stage + BM * ROWB);
    };
    // index of the tail tile of each segment, or -1
    const int tail0 = (p.A[0].K % BK) ? nkt0 - 1 : -1, tail1 = (p.A[1].K % BK) ? nkt0 + nkt1 - 1 : -1;

    // ---- fragments.  A lane holds row (lane & 31) of a 32-row fragment and the 8 k-values
    // 16*ks + 8*(lane >> 5) .. +7.  K-contiguous tiles: one 16-byte read of logical chunk 2*ks + (lane>>5).
    // Row-contiguous tiles: two transposing 8-byte reads; within a group of 16 lanes, lane 4*j + q supplies
    // the address of k row j, columns 4q..4q+3 and receives the four k of column (lane & 15).
    const int frow = lane & 31;
    const int h = lane >> 5;
    const int fsw = h ^ swz(frow);
    const int a_off = (wm * Cfg::WTM + frow) * ROWB;
    const int b_off = BM * ROWB + (wn * Cfg::WTN + frow) * ROWB;
    int a_rc[TM], b_rc[TN];
    {
        const int jj = (lane >> 2) & 3, q = lane & 3, cb = ((lane >> 4) & 1) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int chunk = ((wm * Cfg::WTM + i * 32 + cb) >> 3) + (q >> 1);
            a_rc[i] = (8 * h + jj) * (BM * 2) + ((chunk ^ (4 * jj)) << 4) + (q & 1) * 8;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int chunk = ((wn * Cfg::WTN + j * 32 + cb) >> 3) + (q >> 1);
            b_rc[j] = BM * ROWB + (8 * h + jj) * (BN * 2) + ((chunk ^ (4 * jj)) << 4) + (q & 1) * 8;
        }
    }
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    auto read_tr = [&](const char* ptr, int pitch) -> bf16x8 {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(ptr));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(ptr + 4 * pitch));
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    };
    bf16x8 fa[2][TM], fb[2][TN];
    auto load_frags = [&](const char* stage, int ks, int buf) {
        const int coff = ((2 * ks) ^ fsw) << 4;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (ARC) fa[buf][i] = read_tr(stage + a_rc[i] + 16 * ks * (BM * 2), BM * 2);
            else fa[buf][i] = *reinterpret_cast<const bf16x8*>(stage + a_off + i * 32 * ROWB + coff);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (BRC) fb[buf][j] = read_tr(stage + b_rc[j] + 16 * ks * (BN * 2), BN * 2);
            else fb[buf][j] = *reinterpret_cast<const bf16x8*>(stage + b_off + j * 32 * ROWB + coff);
        }
    };
    {
        // ---- main loop.  The lane offsets of a thread's chunks are loop-invariant registers (per K segment) and
        // the tile origin is a scalar pointer that advances by a constant, so a load is one instruction plus
        // scalar bookkeeping and can sit between the MFMAs.  A k-tile is issued in two halves: the first during
        // the last k16 step of the tile two before it (right after the barrier that frees its stage), the second
        // during the first k16 step of the tile before it; the two k16 steps in between carry no loads, so
        // every load has at least half a k-tile of MFMAs to land before the barrier that publishes it.
        uint32_t offA[Cfg::NCHA], offB[Cfg::NCHB];
        const char *hotA = nullptr, *hotB = nullptr;  // operand bytes of the tile whose first half was issued last
        int64_t stepA = 0, stepB = 0;
        auto hot_operand = [&](auto rc_tag, auto br_tag, const void* optr, int64_t old, int orows, int row0, int k0,
                               uint32_t* off, const char*& base, int64_t& step) {
            constexpr bool RC = decltype(rc_tag)::value;
            constexpr int BR = decltype(br_tag)::value;
            constexpr int NC = BR / 32;
            if (row0 >= orows) row0 = 0;  // as in tail_operand
            const uint32_t ld2 = (uint32_t)old * 2u;
            if constexpr (!RC) {
                const int r0 = tid >> 3;
                const int kc = (tid & 7) ^ kc_swz(r0);
                const int rlast = orows - 1 - row0;
#pragma unroll
                for (int i = 0; i < NC; ++i) off[i] = (uint32_t)min(i * 32 + r0, rlast) * ld2 + (uint32_t)kc * 16u;
                base = reinterpret_cast<const char*>(optr) + ((int64_t)row0 * old + k0) * 2;
                step = BK * 2;
            } else {
                constexpr int CPR = BR / 8;
                constexpr int KPI = 256 / CPR;
                const int kq = tid / CPR;
                const int clast = (((orows - 1) >> 3) << 3) - row0;
#pragma unroll
                for (int i = 0; i < NC; ++i) {
                    const int logical = (tid % CPR) ^ rc_swz(kq + i * KPI);
                    off[i] = (uint32_t)(kq + i * KPI) * ld2 + (uint32_t)min(logical * 8, clast) * 2u;
                }
                base = reinterpret_cast<const char*>(optr) + ((int64_t)k0 * old + row0) * 2;
                step = (int64_t)BK * old * 2;
            }
        };
        auto hot_setup = [&](int kt) {  // kt: a tile of the range
            const bool seg = kt >= nkt0;
            const int k0 = (kt - (seg ? nkt0 : 0)) * BK;
            hot_operand(std::integral_constant<bool, ARC>{}, std::integral_constant<int, BM>{}, a_ptr(seg), a_ld(seg),
                        a_rows(seg), m0, k0, offA, hotA, stepA);
            hot_operand(std::integral_constant<bool, BRC>{}, std::integral_constant<int, BN>{}, b_ptr(seg), b_ld(seg),
                        b_rows(seg), n0, k0, offB, hotB, stepB);
        };
        auto hot_advance = [&](int kt) {  // move on to tile kt, the successor of the current one (kt < kt_end)
            if (kt == nkt0) hot_setup(kt);
            else hotA += stepA, hotB += stepB;
        };
        const uint32_t lds0 = (uint32_t)(uintptr_t)LOQT_LDS_PTR(smem);
        // Load n of half H (0: first half of the chunks of A then of B, 1: second half, 2: all) into `stage`.
        // The direct load is inline assembly for two reasons.  (1) The compiler cannot tell that the LDS reads of
        // the running tile never touch the stage the loads in flight are writing, and would wait for all of
        // them (vmcnt(0)) before every group of transposing reads; written this way it does not see them, and the
        // loop waits for them itself before each barrier.  (2) `live` (wave-uniform, all ones or zero) goes into
        // both halves of EXEC for the one instruction, so the loads past the end of the range are switched off without a
        // second copy of the loop body.  EXEC is all ones here: the loop is in uniform control flow.
        auto hot_load = [&](auto h_tag, int n, char* stage, uint32_t live) {
            constexpr int H = decltype(h_tag)::value;
            constexpr int A0 = H == 1 ? Cfg::NCHA / 2 : 0, A1 = H == 0 ? Cfg::NCHA / 2 : Cfg::NCHA;
            constexpr int B0 = H == 1 ? Cfg::NCHB / 2 : 0;
            const bool isA = n < A1 - A0;
            const int i = isA ? A0 + n : B0 + n - (A1 - A0);
            const uint32_t o = isA ? offA[i] : offB[i];
            const char* base = isA ? hotA : hotB;
            const uint32_t dst = lds0 + (uint32_t)(stage - smem) + (uint32_t)((isA ? 0 : BM * ROWB) + i * 4096 + wave_s * 1024);
            asm volatile(
                "s_mov_b32 m0, %2\n\t"
                "s_mov_b32 exec_lo, %3\n\t"
                "s_mov_b32 exec_hi, %3\n\t"
                "global_load_lds_dwordx4 %0, %1\n\t"
                "s_mov_b64 exec, -1"
                :
                : "v"(o), "s"(base), "s"(dst), "s"(live)
                : "memory");
            // M0 cannot be named as a clobber (the compiler reserves it and warns that a clobber is not honoured): it
            // never keeps a value in M0 across other code, it writes M0 right in front of each of its own uses.
            // tests/test_isa_guard.py checks that nothing else in the loop touches M0.  EXEC is restored to all
            // ones, the value it has in this uniform control flow.
        };
        // The same load without the mask, for kernels whose tiles are all full (NOTAIL): two scalar instructions
        // less per load.  A wave issues at most one instruction every four cycles, and the six-instruction form
        // between two MFMAs of sixteen cycles each holds the second one back.  Tiles past the end of the contraction
        // are not masked either: the tile pointers stop advancing, so such a load fetches the last tile once more
        // into a stage nobody reads again (the loop's exit waits for them before LDS is reused).
        auto hot_load_live = [&](int n, char* stage) {
            const bool isA = n < Cfg::NCHA;
            const int i = isA ? n : n - Cfg::NCHA;
            const uint32_t o = isA ? offA[i] : offB[i];
            const char* base = isA ? hotA : hotB;
            const uint32_t dst = lds0 + (uint32_t)(stage - smem) + (uint32_t)((isA ? 0 : BM * ROWB) + i * 4096 + wave_s * 1024);
            asm volatile(
                "s_mov_b32 m0, %2\n\t"
                "global_load_lds_dwordx4 %0, %1"
                :
                : "v"(o), "s"(base), "s"(dst)
                : "memory");
        };
        // fragment u (A fragments first) of k16 step ks of the tile at `stage` into buffer nb
        auto read_unit = [&](int ks, int nb, int u, const char* stage) {
            const int coff = ((2 * ks) ^ fsw) << 4;
            if (u < TM) {
                if constexpr (ARC) fa[nb][u] = read_tr(stage + a_rc[u] + 16 * ks * (BM * 2), BM * 2);
                else fa[nb][u] = *reinterpret_cast<const bf16x8*>(stage + a_off + u * 32 * ROWB + coff);
            } else {
                const int j = u - TM;
                if constexpr (BRC) fb[nb][j] = read_tr(stage + b_rc[j] + 16 * ks * (BN * 2), BN * 2);
                else fb[nb][j] = *reinterpret_cast<const bf16x8*>(stage + b_off + j * 32 * ROWB + coff);
            }
        };
        // One k16 step with the instruction order fixed by hand (a scheduling fence after every slot): the NM
        // MFMAs on fragment buffer CB; after MFMA q the fragment reads of slot q (step KS of the tile at
        // `fstage`, into the other buffer) and, when LD is 0 or 1, the loads of slot q (half LD of the tile at
        // hotA / hotB into `lstage`).
        constexpr int NU = TM + TN, UPS = (NU + NM - 1) / NM;  // fragments, fragments per slot
        auto kstep = [&](auto cb_tag, auto ks_tag, auto ld_tag, const char* fstage, char* lstage, uint32_t live) {
            constexpr int CB = decltype(cb_tag)::value, KS = decltype(ks_tag)::value, LD = decltype(ld_tag)::value;
#pragma unroll
            for (int q = 0; q < NM; ++q) {
                const int i = q / TN, j = q % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[CB][j], fa[CB][i], acc[i][j], 0, 0, 0);
#pragma unroll
                for (int u = q * UPS; u < (q + 1) * UPS && u < NU; ++u) read_unit(KS, CB ^ 1, u, fstage);
                if constexpr (LD >= 0) {
                    // the NL loads of the half spread evenly over the NM slots of the step (a burst of loads fills the
                    // memory pipeline's queue and stalls the issue of the MFMAs behind it)
#pragma unroll
                    for (int n = q * NL / NM; n < (q + 1) * NL / NM; ++n) hot_load(ld_tag, n, lstage, live);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // ---- the same loop for the 16x16x32 form: two k32 steps per k-tile, two MFMAs per slot.  Step A: the
        // MFMAs of k32 step 0, the reads of step 1 after the first slots, the second half of tile kt+1 after the last
        // ones.  Step B: the MFMAs of step 1; the barrier sits in its middle, and after it come the reads of the next
        // tile's step 0 and the first half of tile kt+2.
        constexpr int NM2 = TM2 * TN2, NS2 = NM2 / 2, NU2 = TM2 + TN2;
        // the loads of a tile go out one every LSP-th slot over the last three quarters of the previous tile's slots
        // (256x256: 16 loads over 48 slots; 256x128: 12 over 24); LBY of them precede barrier Y
        constexpr int LSP = MF16 ? (3 * NS2 / 2) / Cfg::NCH : 1, LBY = MF16 ? (NS2 + LSP - 1) / LSP : 0;
        constexpr int RPQ = MF16 ? (NU2 + NS2 / 2 - 1) / (NS2 / 2) : 1;  // fragment reads per slot over a quarter of the slots
        const int frow16 = lane & 15, q4 = lane >> 4;
        uint32_t a_ko[2], b_ko[2];  // K-contiguous tiles: byte offset of this lane's fragment row and chunk per k32 step
        int a_rc16[ARC ? TM2 : 1], b_rc16[BRC ? TN2 : 1];
        bf16x8 fa16[2][TM2], fb16[2][TN2];
        if constexpr (MF16) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int coff = ((4 * ks + q4) ^ kc_swz(frow16)) << 4;
                a_ko[ks] = (uint32_t)((wm * Cfg::WTM + frow16) * ROWB + coff);
                b_ko[ks] = (uint32_t)(BM * ROWB + (wn * Cfg::WTN + frow16) * ROWB + coff);
            }
            // row-contiguous tiles: within a group of 16 lanes, lane 4*jj + q supplies the address of k row
            // 8*(lane >> 4) + jj, columns 4q..4q+3, and receives the four k of column (lane & 15)
            const int jj = (lane >> 2) & 3, q = lane & 3;
            if constexpr (ARC) {
#pragma unroll
                for (int u = 0; u < TM2; ++u) {
                    const int chunk = ((wm * Cfg::WTM + u * 16) >> 3) + (q >> 1);
                    a_rc16[u] = (8 * q4 + jj) * (BM * 2) + ((chunk ^ rc_swz(8 * q4 + jj)) << 4) + (q & 1) * 8;
                }
            }
            if constexpr (BRC) {
#pragma unroll
                for (int u = 0; u < TN2; ++u) {
                    const int chunk = ((wn * Cfg::WTN + u * 16) >> 3) + (q >> 1);
                    b_rc16[u] = BM * ROWB + (8 * q4 + jj) * (BN * 2) + ((chunk ^ rc_swz(8 * q4 + jj)) << 4) + (q & 1) * 8;
                }
            }
        }
        // fragment u (A fragments first) of k32 step ks of the tile at `stage` into buffer nb
        auto rd16 = [&](int ks, int nb, int u, const char* stage) {
            if (u < TM2) {
                if constexpr (ARC) fa16[nb][u] = read_tr(stage + a_rc16[u] + 32 * ks * (BM * 2), BM * 2);
                else fa16[nb][u] = *reinterpret_cast<const bf16x8*>(stage + a_ko[ks] + u * 16 * ROWB);
            } else {
                const int j = u - TM2;
                if constexpr (BRC) fb16[nb][j] = read_tr(stage + b_rc16[j] + 32 * ks * (BN * 2), BN * 2);
                else fb16[nb][j] = *reinterpret_cast<const bf16x8*>(stage + b_ko[ks] + j * 16 * ROWB);
            }
        };
        // slots S0..S1-1 (two MFMAs each) of a k32 step on fragment buffer CB.  RD > 0: the fragment reads of k32 step
        // RKS of the tile at `rstage` into the other buffer, RD per slot from the first slot of the range on.  LD (0 / 1:
        // that half of the tile at hotA / hotB, 2: all of it, -1: none): its loads into `lstage`, one per slot on the
        // last slots of the range.
        using I2tag = std::integral_constant<int, 2>;
        auto slots16 = [&](auto cb_tag, auto s0_tag, auto s1_tag, auto rd_tag, auto rks_tag, auto ld_tag, const char* rstage,
                           char* lstage, uint32_t live) {
            constexpr int CB = decltype(cb_tag)::value, S0 = decltype(s0_tag)::value, S1 = decltype(s1_tag)::value;
            constexpr int RPS = decltype(rd_tag)::value;                 // fragment reads per slot
            constexpr int RKS = decltype(rks_tag)::value, LD = decltype(ld_tag)::value;
            constexpr int NSL = S1 - S0;
            constexpr int NLD = LD == 2 ? Cfg::NCH : NL;                 // loads to place ...
            constexpr int LPS16 = (NLD + NSL - 1) / NSL;                 // ... LPS16 per slot ...
            constexpr int LSL = (NLD + LPS16 - 1) / LPS16;               // ... on LSL slots ...
            constexpr int LST = NSL >= 2 * LSL ? 2 : 1;                  // ... every LST-th of the last LST * LSL
#pragma unroll
            for (int sl = S0; sl < S1; ++sl) {
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int m = 2 * sl + e, i = m / TN2, j = m % TN2;
                    acc16[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb16[CB][j], fa16[CB][i], acc16[i][j], 0, 0, 0);
                }
                const int t = sl - S0;
                if constexpr (RPS > 0) {
#pragma unroll
                    for (int u = t * RPS; u < (t + 1) * RPS && u < NU2; ++u) rd16(RKS, CB ^ 1, u, rstage);
                }
                if constexpr (LD >= 100) {
                    // spread form without masks (schedule slot LD - 100 + t)
                    const int g = LD - 100 + t;
                    if (g % LSP == 0 && g / LSP < Cfg::NCH) hot_load_live(g / LSP, lstage);
                } else if constexpr (LD >= 10) {
                    // spread form: the whole tile, one load every third slot from slot LD - 10 of the schedule on
                    // (this range starts at schedule slot LD - 10)
                    const int g = LD - 10 + t;
                    if (g % LSP == 0 && g / LSP < Cfg::NCH) hot_load(I2tag{}, g / LSP, lstage, live);
                } else if constexpr (LD >= 0) {
                    const int tl = t - (NSL - LST * LSL);
                    if (tl >= 0 && tl % LST == 0) {
#pragma unroll
                        for (int n = (tl / LST) * LPS16; n < (tl / LST + 1) * LPS16 && n < NLD; ++n)
                            hot_load(ld_tag, n, lstage, live);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I3 = std::integral_constant<int, 3>;
        using NOLD = std::integral_constant<int, -1>;
        // all ones when tile t exists and is a full tile (its direct loads are live), else zero; computed in
        // assembly so that it is certain to sit in a scalar register (hot_load moves it into EXEC)
        auto live_mask = [&](int t) {
            uint32_t m;
            asm("s_sub_i32 %0, %1, %2\n\t"
                "s_ashr_i32 %0, %0, 31\n\t"
                "s_cmp_lg_u32 %1, %3\n\t"
                "s_cselect_b32 %0, %0, 0\n\t"
                "s_cmp_lg_u32 %1, %4\n\t"
                "s_cselect_b32 %0, %0, 0"
                : "=&s"(m)
                : "s"(t), "s"(kt_end), "s"(tail0), "s"(tail1)
                : "scc");
            return m;
        };
        auto is_tail = [&](int t) { return t == tail0 || t == tail1; };
        // The ring of NS stages: tile t lives in stage (t - kt_begin) % NS.  At the top of iteration kt the tiles
        // kt .. kt+NS-2 are in LDS or on their way, and so is the first half of tile kt+NS-1.
        auto wait_loads = [&](bool later_live) {
            // tile kt+1 must have landed.  Loads return in order, so it is enough that no more are outstanding
            // than were issued after it: the NS-2 whole tiles kt+2 .. kt+NS-1 -- provided all of those went out
            // as direct loads (a masked load may not count, a tail tile is stored through registers)
            if (NS > 2 && later_live) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * Cfg::NCH) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        };
        if constexpr (MF16) {
            // ---- 16x16x32 form (two stages).  A stage is free as soon as the fragments of its second k32 step sit in
            // registers, a quarter of the way into its tile, so its refill does not have to wait for the barrier
            // that publishes the next tile.  Per k-tile kt:
            //   slots  0-15 of k32 step 0: the fragment reads of step 1 (two per slot on the first eight)
            //   barrier X                : every wave has tile kt in registers, its stage is free
            //   slots 16-31 of step 0    : the 16 loads of tile kt+2 into that stage, one per slot
            //   slots  0-15 of step 1    : MFMAs only
            //   barrier Y                : tile kt+1 has landed (loads return in order: all but the 16 of kt+2)
            //   slots 16-31 of step 1    : the fragment reads of step 0 of tile kt+1, one per slot
            // A load so has from slot 16 of its issue tile to barrier Y of the next one, 1.25 to 1.5 k-tiles (about
            // 3000 cycles), to land: measured against a library GEMM of the same tile shape, instruction mix and
            // cache traffic, the loop with one barrier per tile (loads issued 0.25 to 1 tile ahead) spent 27 % of
            // its wave cycles waiting where that kernel spent 6 %.
            using SH = std::integral_constant<int, NS2 / 2>;
            using SE = std::integral_constant<int, NS2>;
            auto whole_tile = [&](int t, char* stage) -> bool {  // all of tile t into `stage`; true if by direct loads
                if (is_tail(t)) {
                    tail_tile(t, stage);
                    return false;
                }
                const uint32_t live = live_mask(t);
#pragma unroll
                for (int n = 0; n < Cfg::NCH; ++n) hot_load(I2{}, n, stage, live);
                return true;
            };
            if (kt_begin < kt_end) {
                hot_setup(kt_begin);
                whole_tile(kt_begin, smem);
                bool second = false;
                if (kt_begin + 1 < kt_end) {
                    hot_advance(kt_begin + 1);
                    second = whole_tile(kt_begin + 1, smem + STAGE);
                }
                if (second) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(Cfg::NCH) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
#pragma unroll
                for (int u = 0; u < NU2; ++u) rd16(0, 0, u, smem);
            }
            if constexpr (NOTAIL) {
                for (int kt = kt_begin; kt < kt_end; ++kt) {
                    char* cur = smem + ((kt - kt_begin) & 1) * STAGE;
                    char* nxt = smem + (((kt - kt_begin) & 1) ^ 1) * STAGE;
                    slots16(I0{}, I0{}, SH{}, I2{}, I1{}, NOLD{}, cur, cur, 0);
                    __syncthreads();  // X
                    if (kt + 2 < kt_end) hot_advance(kt + 2);
                    slots16(I0{}, SH{}, SE{}, I0{}, I0{}, std::integral_constant<int, 100>{}, cur, cur, 0);
                    slots16(I1{}, I0{}, SH{}, I0{}, I0{}, std::integral_constant<int, 100 + NS2 / 2>{}, cur, cur, 0);
                    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LBY) : "memory");
                    __syncthreads();  // Y
                    slots16(I1{}, SH{}, SE{}, std::integral_constant<int, RPQ>{}, I0{}, std::integral_constant<int, 100 + NS2>{}, nxt, cur, 0);
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the loads past the end, before LDS is reused
            } else
            for (int kt = kt_begin; kt < kt_end; ++kt) {
                char* cur = smem + ((kt - kt_begin) & 1) * STAGE;
                char* nxt = smem + (((kt - kt_begin) & 1) ^ 1) * STAGE;
                const uint32_t live2 = live_mask(kt + 2);
                slots16(I0{}, I0{}, SH{}, I2{}, I1{}, NOLD{}, cur, cur, 0);
                __syncthreads();  // X: nobody reads `cur` any more
                if (kt + 2 < kt_end) {
                    hot_advance(kt + 2);
                    if (live2 == 0) tail_tile(kt + 2, cur);  // a tail tile (rare): through registers
                }
                // the 16 loads of tile kt+2 go out one every third slot over the remaining 48 slots of the tile: the
                // memory pipeline limits the requests in flight per compute unit, and a burst of loads stalls the
                // issue of the MFMAs behind it
                slots16(I0{}, SH{}, SE{}, I0{}, I0{}, std::integral_constant<int, 10>{}, cur, cur, live2);
                slots16(I1{}, I0{}, SH{}, I0{}, I0{}, std::integral_constant<int, 10 + NS2 / 2>{}, cur, cur, live2);
                // tile kt+1 must have landed; the loads of tile kt+2 issued so far (schedule slots 0-31: 11 of them)
                // came after it and may stay in flight, provided they went out as direct loads (a masked load may
                // not count)
                if (live2 != 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LBY) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();  // Y
                // harmless stale reads after the last tile
                slots16(I1{}, SH{}, SE{}, std::integral_constant<int, RPQ>{}, I0{}, std::integral_constant<int, 10 + NS2>{}, nxt, cur, live2);
            }
        } else {
        if (kt_begin < kt_end) {
            hot_setup(kt_begin);
#pragma unroll
            for (int t = 0; t < NS - 1; ++t) {
                if (kt_begin + t < kt_end) {
                    if (t > 0) hot_advance(kt_begin + t);
                    if (is_tail(kt_begin + t)) {
                        tail_tile(kt_begin + t, smem + t * STAGE);
                    } else {
                        const uint32_t live = live_mask(kt_begin + t);
#pragma unroll
                        for (int n = 0; n < Cfg::NCH; ++n) hot_load(I2{}, n, smem + t * STAGE, live);
                    }
                }
            }
            wait_loads(false);
            __syncthreads();
            load_frags(smem, 0, 0);
            if (kt_begin + NS - 1 < kt_end) {
                hot_advance(kt_begin + NS - 1);
                if (is_tail(kt_begin + NS - 1)) {
                    tail_tile(kt_begin + NS - 1, smem + (NS - 1) * STAGE);
                } else {
                    const uint32_t live = live_mask(kt_begin + NS - 1);
#pragma unroll
                    for (int n = 0; n < NL; ++n) hot_load(I0{}, n, smem + (NS - 1) * STAGE, live);
                }
            }
        }
        uint32_t live1 = live_mask(kt_begin + NS - 1);  // tile kt+NS-1 at the top of iteration kt
        // all ones while the tiles kt+2 .. kt+NS-1 all went out as direct loads (bit j: tile kt+2+j)
        uint32_t later = 0;
        if constexpr (NS > 2) {
#pragma unroll
            for (int j = 0; j < NS - 2; ++j) later |= (live_mask(kt_begin + 2 + j) & 1u) << j;
        }
        int si = 0;  // stage of tile kt
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            // (with two stages the same expressions as ever: the register allocation of the 256x256 kernels,
            // which use every register, does not survive a change here)
            char* cur = smem + (NS == 2 ? (kt - kt_begin) & 1 : si) * STAGE;
            char* nxt = smem + (NS == 2 ? ((kt - kt_begin) & 1) ^ 1 : (si + 1 == NS ? 0 : si + 1)) * STAGE;  // tile kt+1
            char* prv = NS == 2 ? nxt : smem + (si == 0 ? NS - 1 : si - 1) * STAGE;  // tile kt+NS-1 (the stage tile kt-1 left)
            const uint32_t live2 = live_mask(kt + NS);
            kstep(I0{}, I1{}, I1{}, cur, prv, live1);  // + second half of tile kt+NS-1
            if (kt + NS < kt_end) hot_advance(kt + NS);
            kstep(I1{}, I2{}, NOLD{}, cur, nxt, 0);
            kstep(I0{}, I3{}, NOLD{}, cur, nxt, 0);
            wait_loads(NS > 2 && later == (1u << (NS > 2 ? NS - 2 : 0)) - 1u);
            __syncthreads();         // tile kt+1 has landed; nobody reads `cur` any more
            if (live2 == 0) {        // no tile kt+NS, or a tail tile (rare)
                if (kt + NS < kt_end) tail_tile(kt + NS, cur);
            }
            // + first half of tile kt+NS (harmless stale reads after the last tile)
            kstep(I1{}, I0{}, I0{}, nxt, cur, live2);
            if constexpr (NS > 2) later = (later >> 1) | ((live2 & 1u) << (NS - 3));
            live1 = live2;
            if constexpr (NS > 2) si = si + 1 == NS ? 0 : si + 1;
        }
    }
        }
    __syncthreads();  // LDS is free for the epilogue

    // ------------------------------------------------------------------ epilogues
    // accumulator tile (ti, tj): lane holds row m = ti*32 + (lane & 31); register 4*g + j holds
    // column n = tj*32 + 8*g + 4*(lane >> 5) + j.
    if (EPI == EPI_BF16 || EPI == EPI_FOLD || EPI == EPI_ACC_BF16) {
        constexpr int EPITCH = Cfg::EPITCH, WTM = Cfg::WTM, WTN = Cfg::WTN;
        float* lut = reinterpret_cast<float*>(smem + Cfg::SMEM - 64);
        if (EPI == EPI_FOLD) {
            if (tid < 16) lut[tid] = kNf4Levels[tid];
            __syncthreads();
        }
        // The fold stages 32 rows at a time (the same 32 rows of LDS for every block of rows: the LDS operations of a
        // wave complete in order), which leaves room for the old codes of the whole tile beside them.
        constexpr bool FOLD = EPI == EPI_FOLD;
        constexpr int EROWS = FOLD ? 32 : WTM;
        char* ebuf = smem + wave * (EROWS * EPITCH);
        const int64_t ldb = p.w_ld >> 1, lda = p.w_ld >> 6;
        // Fold: the old codes of the wave's rows (WTN / 2 bytes each) come in as direct-to-LDS loads, all issued at
        // once, and the block scales as ordinary loads into registers: one round trip to memory for the tile instead
        // of one per 32x32 piece (fetched piece by piece, a piece ahead of its use, the epilogue took as long as
        // eleven k-tiles of the product, most of it waiting for these loads).
        constexpr int CROW = WTN / 2;              // code bytes per row of the wave tile
        constexpr int LPR = WTN / 32;              // lanes (16 bytes each) per row
        constexpr int RPI = 64 / LPR;              // rows per load instruction
        constexpr int NCI = FOLD ? WTM / RPI : 1;  // load instructions
        char* cbuf = smem + 4 * EROWS * EPITCH + wave * (WTM * CROW);
        float amr[FOLD ? TM : 1][FOLD ? TN / 2 : 1];
        if constexpr (FOLD) {
            const int wm_s = wave_s >> 1, wn_s = wave_s & 1;
            const int crow = lane / LPR, cch = lane % LPR;
            const int nt = n0 + wn * WTN + cch * 32;
            const uint32_t lds_c = (uint32_t)(uintptr_t)LOQT_LDS_PTR(smem) + (uint32_t)(4 * EROWS * EPITCH) +
                                   (uint32_t)(wave_s * (WTM * CROW));
            const uint32_t off = (uint32_t)crow * (uint32_t)ldb + (uint32_t)cch * 16u;
#pragma unroll
            for (int i = 0; i < NCI; ++i) {
                const int m = m0 + wm * WTM + i * RPI + crow;
                const uint64_t mask = __ballot(m < p.M && nt < p.w_ld);
                const uint8_t* base = p.w_codes + (int64_t)(m0 + wm_s * WTM + i * RPI) * ldb + ((n0 + wn_s * WTN) >> 1);
                asm volatile(
                    "s_mov_b32 m0, %2\n\t"
                    "s_mov_b64 exec, %3\n\t"
                    "global_load_lds_dwordx4 %0, %1\n\t"
                    "s_mov_b64 exec, -1"
                    :
                    : "v"(off), "s"(base), "s"(lds_c + (uint32_t)(i * 1024)), "s"(mask)
                    : "memory");
            }
#pragma unroll
            for (int ti = 0; ti < TM; ++ti)
#pragma unroll
                for (int b = 0; b < TN / 2; ++b) {
                    const int m = m0 + wm * WTM + ti * 32 + frow;
                    const int nb = n0 + wn * WTN + b * 64;
                    amr[ti][b] = (m < p.M && nb < p.w_ld) ? p.w_absmax[m * lda + (nb >> 6)] : 0.f;
                }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // each wave reads back only what it loaded itself
        }
        // A block of rows is staged through the wave's private LDS region and leaves as whole 16-byte row
        // segments right after it has been computed (LDS operations of one wave complete in order, so no
        // barrier), so that the stores of one block are under way while the next one is computed.
        constexpr int CPR = WTN / 8;  // 16-byte chunks per row
        uint16_t* C = reinterpret_cast<uint16_t*>(part1 ? p.Cx : p.C);
        const int64_t ldc = part1 ? p.ldcx : p.ldc;
        // rows row0 .. row0+nrows-1 of the wave tile, staged from row erow0 of the staging region on
        auto store_rows = [&](int row0, int nrows, int erow0) {
#pragma unroll 4
            for (int it = 0; it < nrows * CPR / 64; ++it) {
                const int idx = it * 64 + lane, row = row0 + idx / CPR, ch = idx % CPR;
                const int m = m0 + wm * WTM + row, n = n0 + wn * WTN + ch * 8;
                const uint4 v = *reinterpret_cast<const uint4*>(ebuf + (erow0 + idx / CPR) * EPITCH + ch * 16);
                if (m < p.M) {
                    uint16_t* dst = C + (int64_t)m * ldc + n;
                    if (n + 8 <= N) {
                        typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
                        __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), reinterpret_cast<u32x4_t*>(dst));
                    } else {
                        const uint16_t* sv = reinterpret_cast<const uint16_t*>(&v);
                        for (int e = 0; e < 8; ++e)
                            if (n + e < N) dst[e] = sv[e];
                    }
                }
            }
        };
        if constexpr (MF16) {
            const int frow16 = lane & 15, q4 = lane >> 4;
#pragma unroll
            for (int ti = 0; ti < TM2; ++ti) {
#pragma unroll
                for (int tj = 0; tj < TN2; ++tj) {
                    const uint2 v = make_uint2(pack_bf16(alpha * acc16[ti][tj][0], alpha * acc16[ti][tj][1]),
                                               pack_bf16(alpha * acc16[ti][tj][2], alpha * acc16[ti][tj][3]));
                    *reinterpret_cast<uint2*>(ebuf + (ti * 16 + frow16) * EPITCH + (tj * 16 + 4 * q4) * 2) = v;
                }
                if (ti & 1) store_rows((ti - 1) * 16, 32, (ti - 1) * 16);
            }
        } else {
#pragma unroll
        for (int ti = 0; ti < TM; ++ti) {
#pragma unroll
            for (int tj = 0; tj < TN; ++tj) {
                // folded weight (M = out, N = in): the 16 code bytes of row m, columns nt..nt+31 (both
                // lanes of a pair load them; this lane uses the half-words (lane >> 5) of each dword)
                uint32_t cw4[4] = {0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u};
                float am = 0.f;
                if constexpr (FOLD) {
                    const int m = m0 + wm * WTM + ti * 32 + frow;
                    const int nt = n0 + wn * WTN + tj * 32;
                    if (m < p.M && nt < p.w_ld) {
                        const uint4 c = *reinterpret_cast<const uint4*>(cbuf + (ti * 32 + frow) * CROW + tj * 16);
                        cw4[0] = c.x, cw4[1] = c.y, cw4[2] = c.z, cw4[3] = c.w;
                        am = amr[ti][tj >> 1];
                    }
                }
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v0 = alpha * acc[ti][tj][4 * g + 0], v1 = alpha * acc[ti][tj][4 * g + 1];
                    float v2 = alpha * acc[ti][tj][4 * g + 2], v3 = alpha * acc[ti][tj][4 * g + 3];
                    if (EPI == EPI_ACC_BF16) {
                        // unquantised merge (M = out, N = in): add the old bf16 weight in fp32; the 8 bytes stay
                        // inside the row's pitch (a multiple of 8 elements) even where n + 4 > N
                        const int m = m0 + wm * WTM + ti * 32 + frow;
                        const int n = n0 + wn * WTN + tj * 32 + 8 * g + 4 * h;
                        if (m < p.M && n < N) {
                            const uint2 o = *reinterpret_cast<const uint2*>(p.w_bf16 + (int64_t)m * p.w_bf16_ld + n);
                            v0 += bf16_lo(o.x), v1 += bf16_hi(o.x), v2 += bf16_lo(o.y), v3 += bf16_hi(o.y);
                        }
                    }
                    if (EPI == EPI_FOLD) {
                        const uint32_t cw = (cw4[g] >> (16 * h)) & 0xffffu;
                        v0 += am * lut[nib4(cw, 0)];
                        v1 += am * lut[nib4(cw, 1)];
                        v2 += am * lut[nib4(cw, 2)];
                        v3 += am * lut[nib4(cw, 3)];
                    }
                    const uint2 v = make_uint2(pack_bf16(v0, v1), pack_bf16(v2, v3));
                    *reinterpret_cast<uint2*>(ebuf + ((FOLD ? 0 : ti * 32) + frow) * EPITCH + (tj * 32 + 8 * g + 4 * h) * 2) = v;
                }
            }
            store_rows(ti * 32, 32, FOLD ? 0 : ti * 32);
        }
        }
    } else if (EPI == EPI_F32_SPLITK || EPI == EPI_FOLD_F32) {
        // fp32 results, 16 bytes per lane (row m, 4 consecutive n).  EPI_F32_SPLITK: slice `split` of the
        // contraction.  EPI_FOLD_F32 (M = out, N = in): the dense merged weight of Alg. 1 line 5,
        // fma(alpha, acc, fl32(absmax * q[code])), the same expression the merge epilogue quantises.
        float* C = reinterpret_cast<float*>(p.C);
        if (EPI == EPI_F32_SPLITK) C += (int64_t)split * p.M * p.ldc;
        float* lut = reinterpret_cast<float*>(smem);
        if (EPI == EPI_FOLD_F32) {
            if (tid < 16) lut[tid] = kNf4Levels[tid];
            __syncthreads();
        }
        const int64_t ldb = p.w_ld >> 1, lda = p.w_ld >> 6;
        if constexpr (MF16) {
            // 16x16 accumulator tiles: lane holds row ti*16 + (lane & 15), columns tj*16 + 4*(lane >> 4) .. +3
            const int frow16 = lane & 15, q4 = lane >> 4;
#pragma unroll
            for (int ti = 0; ti < TM2; ++ti) {
                const int m = m0 + wm * Cfg::WTM + ti * 16 + frow16;
#pragma unroll
                for (int tj = 0; tj < TN2; ++tj) {
                    const int n = n0 + wn * Cfg::WTN + tj * 16 + 4 * q4;
                    if (m < p.M) {
                        float* dst = C + (int64_t)m * p.ldc + n;
                        if (n + 4 <= p.N) {
                            *reinterpret_cast<float4*>(dst) =
                                make_float4(p.alpha * acc16[ti][tj][0], p.alpha * acc16[ti][tj][1],
                                            p.alpha * acc16[ti][tj][2], p.alpha * acc16[ti][tj][3]);
                        } else {
                            for (int j = 0; j < 4; ++j)
                                if (n + j < p.N) dst[j] = p.alpha * acc16[ti][tj][j];
                        }
                    }
                }
            }
        } else
#pragma unroll
        for (int ti = 0; ti < TM; ++ti) {
            const int m = m0 + wm * Cfg::WTM + ti * 32 + frow;
#pragma unroll
            for (int tj = 0; tj < TN; ++tj) {
                uint32_t cw4[4] = {0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u};
                float am = 0.f;
                if (EPI == EPI_FOLD_F32) {
                    const int nt = n0 + wn * Cfg::WTN + tj * 32;
                    if (m < p.M && nt < p.w_ld) {
                        const uint4 c = *reinterpret_cast<const uint4*>(p.w_codes + m * ldb + (nt >> 1));
                        cw4[0] = c.x, cw4[1] = c.y, cw4[2] = c.z, cw4[3] = c.w;
                        am = p.w_absmax[m * lda + (nt >> 6)];
                    }
                }
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n0 + wn * Cfg::WTN + tj * 32 + 8 * g + 4 * h;
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (EPI == EPI_FOLD_F32) {
                            const uint32_t cw = (cw4[g] >> (16 * h)) & 0xffffu;
                            v[j] = __builtin_fmaf(p.alpha, acc[ti][tj][4 * g + j], am * lut[nib4(cw, j)]);
                        } else {
                            v[j] = p.alpha * acc[ti][tj][4 * g + j];
                        }
                    }
                    if (m < p.M) {
                        float* dst = C + (int64_t)m * p.ldc + n;
                        if (n + 4 <= p.N) {
                            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                        } else {
                            for (int j = 0; j < 4; ++j)
                                if (n + j < p.N) dst[j] = v[j];
                        }
                    }
                }
            }
        }
    } else {
        // merge (M = out, N = in): W_new = fl32(absmax * q[code]) + alpha * acc, requantised per
        // 64-block along n (Alg. 1 line 5).  A block of row m is 32 values in this lane and 32 in lane ^ 32.
        // compensation step (Alg. 2 lines 8-10): the same with W_hat = w_f32 + alpha * acc; the residual
        // w_f32 - deq(q(W_hat)) leaves as bf16.
        Nf4EncTables* enc = reinterpret_cast<Nf4EncTables*>(smem);
        float* lut = reinterpret_cast<float*>(smem + sizeof(Nf4EncTables));
        if (tid < 64) nf4_enc_tables_fill(enc, tid);
        else if (tid < 80) lut[tid - 64] = kNf4Levels[tid - 64];
        __syncthreads();
        const int64_t ldb = p.w_ld >> 1, lda = p.w_ld >> 6;
#pragma unroll
        for (int ti = 0; ti < TM; ++ti) {
            const int m = m0 + wm * Cfg::WTM + ti * 32 + frow;
            const bool mvalid = m < p.M;
#pragma unroll
            for (int b = 0; b < TN / 2; ++b) {
                const int nb = n0 + wn * Cfg::WTN + b * 64;  // first `in` index of the block
                const bool live = mvalid && nb < p.w_ld;
                float v[32];
                float wsrc[EPI == EPI_COMP ? 32 : 1];
                if constexpr (EPI == EPI_MERGE) {
                    float am_old = 0.f;
                    // the 2 x 16 code bytes of the block (columns nb..nb+63 of row m); both lanes of a pair
                    // load them, this lane owns the half-words (lane >> 5) of each dword
                    uint4 cw4[2];
                    if constexpr (MERGE_PREFETCH) {
                        am_old = pre_am[ti * (TN / 2) + b];
                        cw4[0] = pre_cw[ti * (TN / 2) + b][0];
                        cw4[1] = pre_cw[ti * (TN / 2) + b][1];
                    } else {
                        if (live) am_old = p.w_absmax[m * lda + (nb >> 6)];
                        cw4[0] = cw4[1] = make_uint4(0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u);
                        if (live) {
                            cw4[0] = *reinterpret_cast<const uint4*>(p.w_codes + m * ldb + (nb >> 1));
                            cw4[1] = *reinterpret_cast<const uint4*>(p.w_codes + m * ldb + (nb >> 1) + 16);
                        }
                    }
#pragma unroll
                    for (int q = 0; q < 8; ++q) {  // q = 4*tt + g: tile tt of the pair, column group g
                        const uint32_t cw =
                            (reinterpret_cast<const uint32_t*>(&cw4[q >> 2])[q & 3] >> (16 * h)) & 0xffffu;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            v[4 * q + j] = __builtin_fmaf(p.alpha, acc[ti][2 * b + (q >> 2)][4 * (q & 3) + j],
                                                          am_old * lut[nib4(cw, j)]);
                    }
                } else {
                    const float* wrow = p.w_f32 + (int64_t)m * p.w_f32_ld;
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int nq = nb + (q >> 2) * 32 + 8 * (q & 3) + 4 * h;
                        float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (mvalid && nq < p.w_f32_ld) f = *reinterpret_cast<const float4*>(wrow + nq);
                        wsrc[4 * q + 0] = f.x, wsrc[4 * q + 1] = f.y, wsrc[4 * q + 2] = f.z, wsrc[4 * q + 3] = f.w;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            v[4 * q + j] = __builtin_fmaf(p.alpha, acc[ti][2 * b + (q >> 2)][4 * (q & 3) + j],
                                                          wsrc[4 * q + j]);
                    }
                }
                if (nb + 64 > p.w_cols) {  // ragged last block (wave-uniform): columns past the end count as 0
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int nq = nb + (q >> 2) * 32 + 8 * (q & 3) + 4 * h;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (nq + j >= p.w_cols) {
                                v[4 * q + j] = 0.f;
                                if constexpr (EPI == EPI_COMP) wsrc[4 * q + j] = 0.f;
                            }
                    }
                }
                float amax = 0.f;
#pragma unroll
                for (int e = 0; e < 32; ++e) amax = fmaxf(amax, fabsf(v[e]));
                amax = fmaxf(amax, __shfl_xor(amax, 32));
                Nf4BlockEncoder be;
                be.set(amax);
                // single-precision encoder first; the exact one again for the whole block when any lane of the
                // wave has an element within rounding of a decision point (about one block in 10^4)
                uint32_t code[32];
                uint32_t near = 0;
#pragma unroll
                for (int e = 0; e < 32; ++e) code[e] = be.encode_fast(enc, v[e], near);
                if (__any(near)) {
#pragma unroll
                    for (int e = 0; e < 32; ++e) code[e] = be.encode(enc, v[e]);
                }
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    uint32_t o[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int q = 4 * tt + g;
                        uint32_t c[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) c[j] = code[4 * q + j];
                        if constexpr (EPI == EPI_COMP) {
                            const int nq = nb + tt * 32 + 8 * g + 4 * h;
                            float e[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) e[j] = wsrc[4 * q + j] - amax * lut[c[j]];
                            if (mvalid && nq < p.e_ld)
                                *reinterpret_cast<uint2*>(p.e_out + (int64_t)m * p.e_ld + nq) =
                                    make_uint2(pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3]));
                        }
                        uint32_t word = nf4_pack4(c[0], c[1], c[2], c[3]);
                        word <<= 16 * h;                       // this lane's half of dword g
                        o[g] = word | __shfl_xor(word, 32);    // the partner lane holds the other half
                    }
                    if (live && h == 0)
                        *reinterpret_cast<uint4*>(p.out_codes + m * ldb + (nb >> 1) + tt * 16) =
                            make_uint4(o[0], o[1], o[2], o[3]);
                }
                if (live && h == 0) p.out_absmax[m * lda + (nb >> 6)] = amax;
            }
        }
    }
}

// Work-groups are dealt to the 8 XCDs round-robin by the hardware; each XCD walks a contiguous range of tiles.
template <int BM, int BN, int EPI, bool ARC, bool BRC, int NS = 2, bool NOTAIL = false>
__global__ __launch_bounds__(256) void nt_gemm_kernel(const GemmParams p) {
    const int per_xcd = gridDim.x >> 3;
    nt_gemm_tile<BM, BN, EPI, ARC, BRC, NS, NOTAIL>(p, (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3), blockIdx.y);
}

// The merges of several layers (Alg. 1 line 5, one layer after the other) as ONE launch: the tiles of all layers
// form one grid, so the prologue and epilogue of one layer's tiles overlap with the products of the next layer's
// instead of every layer paying its own ramp-up, tail round and launch gap.  The per-layer descriptors travel in
// the kernel argument block itself (no device-side table to fill, nothing to allocate, capture-safe), which
// bounds a group at MERGE_GROUP_MAX layers.  per_xcd_end: running total of the tiles each XCD has walked when it
// is through with this layer.
struct MergeGroupItem {
    const void* A;      // left operand of s * A B: deq(P) in bf16, out x r, K contiguous
    const void* B;      // right operand: r x in stored K x rows (BRC) or in x r stored rows x K
    int64_t lda, ldb;
    const uint8_t* w_codes;
    const float* w_absmax;
    uint8_t* out_codes;
    float* out_absmax;
    int64_t w_ld;
    int M, N, K, w_cols;
    float alpha;
    int per_xcd_end;
};
struct MergeGroupParams {
    int n;
    MergeGroupItem it[MERGE_GROUP_MAX];
};
static_assert(sizeof(MergeGroupParams) <= 4096, "kernel arguments are limited to 4 KB");

template <bool BRC>
__global__ __launch_bounds__(256) void nt_merge_grouped_kernel(const MergeGroupParams g) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    int li = 0;
    while (li + 1 < g.n && j >= g.it[li].per_xcd_end) ++li;  // wave-uniform
    const int start = li ? g.it[li - 1].per_xcd_end : 0;
    const MergeGroupItem& it = g.it[li];
    GemmParams p;
    p.A[0].ptr = it.A, p.A[0].absmax = nullptr, p.A[0].ld = it.lda, p.A[0].rows = it.M, p.A[0].K = it.K;
    p.B[0].ptr = it.B, p.B[0].absmax = nullptr, p.B[0].ld = it.ldb, p.B[0].rows = it.w_cols, p.B[0].K = it.K;
    p.A[1].ptr = nullptr, p.A[1].absmax = nullptr, p.A[1].ld = 0, p.A[1].rows = 0, p.A[1].K = 0;
    p.B[1] = p.A[1];
    p.Bx = p.A[1];
    p.M = it.M, p.N = it.N, p.alpha = it.alpha;
    p.C = nullptr, p.ldc = 0, p.splits = 1;
    p.Cx = nullptr, p.ldcx = 0, p.Nx = 0, p.alphax = 0.f;
    p.w_codes = it.w_codes, p.w_absmax = it.w_absmax, p.out_codes = it.out_codes, p.out_absmax = it.out_absmax;
    p.w_ld = it.w_ld, p.w_cols = it.w_cols;
    p.w_bf16 = nullptr, p.w_bf16_ld = 0, p.w_f32 = nullptr, p.w_f32_ld = 0, p.e_out = nullptr, p.e_ld = 0;
    const int per_xcd = it.per_xcd_end - start;
    nt_gemm_tile<128, 128, EPI_MERGE, false, BRC>(p, xcd * per_xcd + (j - start), 0);
}

// the kernel's LDS size has to be raised above the default once per process (first launch, or loqt_prepare)
template <int BM, int BN, int EPI, bool ARC, bool BRC, int NS = 2, bool NOTAIL = false>
hipError_t ensure_attr() {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(nt_gemm_kernel<BM, BN, EPI, ARC, BRC, NS, NOTAIL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, NtCfg<BM, BN, NS>::SMEM);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    return hipSuccess;
}
template <bool BRC>
hipError_t ensure_attr_grouped() {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(nt_merge_grouped_kernel<BRC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, NtCfg<128, 128, 2>::SMEM);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    return hipSuccess;
}

template <int BM, int BN, int EPI, bool ARC, bool BRC, int NS = 2, bool NOTAIL = false>
hipError_t launch_nt(const GemmParams& p, hipStream_t st) {
    if constexpr (((EPI == EPI_BF16 && BM == 256 && (BN == 256 || BN == 128)) ||
                   (EPI == EPI_F32_SPLITK && BM == 256 && BN == 128)) && NS == 2 && !NOTAIL) {
        // the plain bf16 products on 256x256 tiles have a variant for contractions that are whole k-tiles
        if (p.A[0].K % BK == 0 && p.A[1].K % BK == 0) return launch_nt<BM, BN, EPI, ARC, BRC, NS, true>(p, st);
    }
    auto kern = nt_gemm_kernel<BM, BN, EPI, ARC, BRC, NS, NOTAIL>;
    constexpr int smem = NtCfg<BM, BN, NS>::SMEM;
    hipError_t e0 = ensure_attr<BM, BN, EPI, ARC, BRC, NS, NOTAIL>();
    if (e0 != hipSuccess) return e0;
    const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN + (p.Nx + BN - 1) / BN);
    dim3 grid((tiles + 7) / 8 * 8, EPI == EPI_F32_SPLITK ? p.splits : 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, p);
    return hipGetLastError();
}

}  // namespace

// Plan of a bf16-output product of M rows and N (+ Nx extra) columns in units of one round of 256x256 tiles
// (256 tiles, one per compute unit).  A round of 128x128 tiles (512, two per compute unit) takes 0.68 of that,
// measured, whether it is full or half full.  n1 > 0: the first n1 columns as 256x256 tiles in whole rounds, the
// rest and the extra columns as 128x128 tiles.
BF16Plan plan_bf16_product(int64_t M, int64_t N, int64_t Nx) {
    auto cdiv = [](int64_t a, int64_t b) { return (a + b - 1) / b; };
    const int64_t tm = cdiv(M, 256), tn = cdiv(N, 256), tnx = cdiv(Nx, 256);
    BF16Plan plan;
    plan.n1 = 0;
    plan.cost = (double)cdiv(tm * (tn + tnx), 256);
    const int64_t whole = tm * tn / 256;
    const int64_t c1 = whole * 256 / tm;  // tile columns of the first launch
    if (whole >= 1 && c1 > 0 && c1 < tn && whole * 256 - c1 * tm < 32) {
        const int64_t n1 = c1 * 256;
        const int64_t tiles_b = cdiv(M, 128) * (cdiv(N - n1, 128) + cdiv(Nx, 128));
        const double cost = (double)whole + 0.68 * (double)cdiv(tiles_b, 512);
        if (cost < plan.cost) plan.cost = cost, plan.n1 = (int)n1;
    }
    return plan;
}

// Scratch (floats) for the column remainder of a bf16-output product of M rows and N columns in two fp32 slices
// of the contraction: when the plan has a remainder and its 256x128 tiles number 64 to 128 (see launch_nt_sized).
int64_t remainder_split_floats(int64_t M, int64_t N) {
    if (M < 512 || M * 2 > (int64_t)1 << 30) return 0;
    if (((M + 255) / 256) * ((N + 255) / 256) < 224) return 0;  // such a product takes no 256x256 tiles at all
    const BF16Plan plan = plan_bf16_product(M, N, 0);
    if (plan.n1 <= 0) return 0;
    const int64_t nb = N - plan.n1;
    const int64_t tiles = ((M + 255) / 256) * ((nb + 127) / 128);
    if (tiles < 64 || tiles > 128) return 0;
    return 2 * M * ((nb + 3) / 4 * 4);
}

namespace {

template <int EPI, bool ARC, bool BRC>
hipError_t launch_nt_sized(const GemmParams& p, hipStream_t st) {
    // largest tile that still gives every compute unit a work-group
    const int64_t z = EPI == EPI_F32_SPLITK ? p.splits : 1;
    auto tiles = [&](int bm, int bn) {
        return z * ((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn + (p.Nx + bn - 1) / bn);
    };
    // 256x256 tiles (one work-group per compute unit) have the best ratio of MFMA work to LDS and
    // global traffic and win on long contractions with a light epilogue.  With short contractions
    // or a heavy epilogue (merge, fp32 slices; measured on real data, the fold is better off with the
    // large tile) two or three resident 128x128 work-groups per
    // compute unit win: the epilogue and prologue of one overlap with the main loop of another.
    if constexpr (EPI == EPI_COMP || EPI == EPI_FOLD_F32) {
        return launch_nt<128, 128, EPI, ARC, BRC>(p, st);  // heavy epilogue: small tiles only
    } else {
    int choice = g_nt_tile_override;
    if (choice == 0) {
        const int K = p.A[0].K + p.A[1].K;
        const bool light = (EPI == EPI_BF16 && K >= 2048) || EPI == EPI_FOLD || EPI == EPI_ACC_BF16;
        choice = (light && tiles(256, 256) >= 224) ? 1 : 3;
        // skinny bf16 products with a long contraction (Z = s dy deq(P) at rank 1024: 8192 x 1024 outputs) fill the
        // chip with 256x128 tiles, one per compute unit, at half the LDS traffic per flop of the 128x128 ones.  With
        // only half as many tiles (4096 x 1024 outputs: half the compute units stay idle) they are still ahead when
        // the contraction is very long (13B gate / up, K = 13824: 180 -> 162 us) and behind at K = 5461.
        if (EPI == EPI_BF16 && choice == 3 && K >= 2048 && p.Nx == 0 && tiles(256, 128) <= 256 &&
            (tiles(256, 128) >= 224 || (tiles(256, 128) >= 128 && K >= 8192)))
            choice = 2;
    }
    if constexpr (EPI == EPI_BF16) {
        // 256x256 tiles run in rounds of one tile per compute unit.  When the last round would be mostly
        // empty, the tile columns that fill whole rounds go out as one launch and the remaining columns
        // (with the extra columns Nx, if any) as a second launch of 128x128 tiles.
        const BF16Plan plan = plan_bf16_product(p.M, p.N, p.Nx);
        if (g_nt_tile_override == 0 && choice == 1 && plan.n1 > 0) {
            const int n1 = plan.n1;
            GemmParams a = p, b = p;
            a.N = n1;
            a.Nx = 0;
            for (int seg = 0; seg < 2; ++seg) {
                if (p.A[seg].K == 0) continue;
                a.B[seg].rows = min(p.B[seg].rows, n1);
                b.B[seg].rows = p.B[seg].rows - n1;
                b.B[seg].ptr = reinterpret_cast<const uint16_t*>(p.B[seg].ptr) + (BRC ? (int64_t)n1 : (int64_t)n1 * p.B[seg].ld);
            }
            b.N = p.N - n1;
            b.C = reinterpret_cast<uint16_t*>(p.C) + n1;
            hipError_t e = launch_nt<256, 256, EPI, ARC, BRC>(a, st);
            if (e != hipSuccess) return e;
            if constexpr (!ARC) {
                // A remainder whose 256x128 tiles would fill no more than half of the compute units (13B block at
                // 4096 tokens: 1024 of 5120 columns, 128 tiles) goes out as two fp32 slices of the contraction,
                // twice the work-groups at half the depth, and the fixed-order sum of the two into bf16 (75 -> 47 us)
                const int64_t need = remainder_split_floats(p.M, p.N);
                if (need > 0 && b.Nx == 0 && p.split_ws != nullptr && p.split_ws_floats >= need &&
                    p.A[0].K + p.A[1].K >= 2048) {
                    GemmParams c = b;
                    c.C = p.split_ws;
                    c.ldc = (b.N + 3) / 4 * 4;
                    c.splits = 2;
                    e = launch_nt<256, 128, EPI_F32_SPLITK, ARC, BRC, 2>(c, st);
                    if (e != hipSuccess) return e;
                    return launch_reduce_db(p.split_ws, 2, b.M, b.N, c.ldc, b.C, LOQT_BF16, b.ldc, 0, st, false);
                }
            }
            {
                // between 129 and 256 tiles of 256x128 (7B gate / up forward: 768 of 11008 columns; 13B gate / up
                // forward: 1536 of 13824): that shape, one work-group per compute unit
                const int64_t t2 = ((int64_t)(b.M + 255) / 256) * ((b.N + 127) / 128);
                if (b.Nx == 0 && t2 > 128 && t2 <= 256 && p.A[0].K + p.A[1].K >= 2048)
                    return launch_nt<256, 128, EPI, ARC, BRC>(b, st);
            }
            return launch_nt<128, 128, EPI, ARC, BRC>(b, st);
        }
    }
    if (choice == 1) return launch_nt<256, 256, EPI, ARC, BRC>(p, st);
    if (choice == 2) return launch_nt<256, 128, EPI, ARC, BRC>(p, st);
    if constexpr (EPI == EPI_F32_SPLITK) {
        // The fp32 slices (dB and its relatives: short rows of 128 outputs, both operands stored K x rows) run on
        // 256x128 tiles, one work-group per compute unit, from 512 output rows (rank 512) up (1B block, rank 512:
        // dB 0.30 -> 0.24 ms against 128x128 tiles).  History of this choice: 128x128 with two stages waited for its
        // loads more than for anything else (dB 0.78 ms on the 7B block); 256x128 with a ring of three stages in the
        // 32x32x16 loop 0.66 ms; the 16x16x32 loop with two stages, whose loads run up to 1.5 k-tiles ahead and are
        // spread over the tile, 0.60 ms (A/B on one machine: 79 -> 73 us for 1024 x 4096 x 8192).
        if (g_nt_tile_override == 0 && p.M >= 512)
            return launch_nt<256, 128, EPI, ARC, BRC, 2>(p, st);
    }
    return launch_nt<128, 128, EPI, ARC, BRC>(p, st);
    }
}

}  // namespace

int g_nt_tile_override = 0;

hipError_t launch_merge_grouped(int slot, bool b_rc, const MergeGroupLayer* layers, int n, hipStream_t st) {
    if (n < 1 || n > MERGE_GROUP_MAX) return hipErrorInvalidValue;
    TimedLaunch tl(slot, st);
    MergeGroupParams g;
    memset(&g, 0, sizeof(g));
    g.n = n;
    int per_xcd_total = 0;
    for (int i = 0; i < n; ++i) {
        const MergeGroupLayer& l = layers[i];
        MergeGroupItem& it = g.it[i];
        it.A = l.A, it.lda = l.lda, it.B = l.B, it.ldb = l.ldb;
        it.w_codes = l.w_codes, it.w_absmax = l.w_absmax, it.out_codes = l.out_codes, it.out_absmax = l.out_absmax;
        it.w_ld = l.w_ld, it.M = l.out, it.N = (int)l.w_ld, it.K = l.r, it.w_cols = l.in, it.alpha = l.s;
        const int tiles = ((l.out + 127) / 128) * (int)((l.w_ld + 127) / 128);
        per_xcd_total += (tiles + 7) / 8;
        it.per_xcd_end = per_xcd_total;
    }
    constexpr int smem = NtCfg<128, 128, 2>::SMEM;
    const dim3 grid((unsigned)per_xcd_total * 8u);
    hipError_t e0 = b_rc ? ensure_attr_grouped<true>() : ensure_attr_grouped<false>();
    if (e0 != hipSuccess) return e0;
    if (b_rc) hipLaunchKernelGGL(nt_merge_grouped_kernel<true>, grid, dim3(256), smem, st, g);
    else hipLaunchKernelGGL(nt_merge_grouped_kernel<false>, grid, dim3(256), smem, st, g);
    return hipGetLastError();
}

// every kernel configuration launch_gemm_nt / launch_merge_grouped can reach
hipError_t prepare_nt_kernels() {
    hipError_t e;
#define LOQT_PREP3(EPI, ARC, BRC)                                                   \
    if ((e = ensure_attr<256, 256, EPI, ARC, BRC>()) != hipSuccess) return e;       \
    if ((e = ensure_attr<256, 128, EPI, ARC, BRC>()) != hipSuccess) return e;       \
    if ((e = ensure_attr<128, 128, EPI, ARC, BRC>()) != hipSuccess) return e
    LOQT_PREP3(EPI_BF16, false, false);
    LOQT_PREP3(EPI_MERGE, false, false);
    LOQT_PREP3(EPI_FOLD, false, false);
    LOQT_PREP3(EPI_BF16, false, true);
    LOQT_PREP3(EPI_MERGE, false, true);
    LOQT_PREP3(EPI_FOLD, false, true);
    LOQT_PREP3(EPI_ACC_BF16, false, true);
    LOQT_PREP3(EPI_F32_SPLITK, true, true);
    LOQT_PREP3(EPI_F32_SPLITK, false, true);
#undef LOQT_PREP3
    if ((e = ensure_attr<256, 128, EPI_F32_SPLITK, true, true, 3>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 256, EPI_BF16, false, false, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 256, EPI_BF16, false, true, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 128, EPI_F32_SPLITK, true, true, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 128, EPI_F32_SPLITK, false, true, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 128, EPI_F32_SPLITK, false, false, 2, false>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 128, EPI_F32_SPLITK, false, false, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 128, EPI_BF16, false, false, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<256, 128, EPI_BF16, false, true, 2, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<128, 128, EPI_COMP, false, true>()) != hipSuccess) return e;
    if ((e = ensure_attr<128, 128, EPI_FOLD_F32, false, true>()) != hipSuccess) return e;
    if ((e = ensure_attr_grouped<true>()) != hipSuccess) return e;
    return ensure_attr_grouped<false>();
}

// a_rc / b_rc: the operand is stored K x rows (rows contiguous) instead of rows x K
hipError_t launch_gemm_nt(int slot, int epi, bool a_rc, bool b_rc, const GemmParams& p, hipStream_t st) {
    TimedLaunch tl(slot, st);
    if (!a_rc && !b_rc) {
        switch (epi) {
            case EPI_BF16: return launch_nt_sized<EPI_BF16, false, false>(p, st);
            case EPI_MERGE: return launch_nt_sized<EPI_MERGE, false, false>(p, st);
            case EPI_FOLD: return launch_nt_sized<EPI_FOLD, false, false>(p, st);
            default: break;
        }
    } else if (!a_rc && b_rc) {
        switch (epi) {
            case EPI_BF16: return launch_nt_sized<EPI_BF16, false, true>(p, st);
            case EPI_MERGE: return launch_nt_sized<EPI_MERGE, false, true>(p, st);
            case EPI_FOLD: return launch_nt_sized<EPI_FOLD, false, true>(p, st);
            case EPI_COMP: return launch_nt_sized<EPI_COMP, false, true>(p, st);
            case EPI_FOLD_F32: return launch_nt_sized<EPI_FOLD_F32, false, true>(p, st);
            case EPI_ACC_BF16: return launch_nt_sized<EPI_ACC_BF16, false, true>(p, st);
            case EPI_F32_SPLITK: return launch_nt_sized<EPI_F32_SPLITK, false, true>(p, st);
            default: break;
        }
    } else if (a_rc && b_rc) {
        switch (epi) {
            case EPI_F32_SPLITK: return launch_nt_sized<EPI_F32_SPLITK, true, true>(p, st);
            default: break;
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace loqt
