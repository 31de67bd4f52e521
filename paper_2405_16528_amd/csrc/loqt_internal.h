// Internal declarations shared by the translation units of libloqt (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/loqt.h"

namespace loqt {

// ---------------------------------------------------------------------------------------
// NF4 level table (the published 4-bit NormalFloat data type; paper sec. 5.1 defers to it).
// ---------------------------------------------------------------------------------------
#define LOQT_NF4_LEVELS                                                                          \
    {-1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,                   \
     -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,                  \
     0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,     \
     0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f}

static __device__ __constant__ const float kNf4Levels[16] = LOQT_NF4_LEVELS;

// Decision thresholds of the quantiser, as doubles: kNf4Mid[j] = (q_j + q_{j+1}) / 2, exact
// (the sum of two fp32 values of nearby exponent fits a double; halving is exact).
static __device__ __constant__ const double kNf4Mid[15] = {
    (-1.0 + -0.6961928009986877) * 0.5,
    (-0.6961928009986877 + -0.5250730514526367) * 0.5,
    (-0.5250730514526367 + -0.39491748809814453) * 0.5,
    (-0.39491748809814453 + -0.28444138169288635) * 0.5,
    (-0.28444138169288635 + -0.18477343022823334) * 0.5,
    (-0.18477343022823334 + -0.09105003625154495) * 0.5,
    (-0.09105003625154495 + 0.0) * 0.5,
    (0.0 + 0.07958029955625534) * 0.5,
    (0.07958029955625534 + 0.16093020141124725) * 0.5,
    (0.16093020141124725 + 0.24611230194568634) * 0.5,
    (0.24611230194568634 + 0.33791524171829224) * 0.5,
    (0.33791524171829224 + 0.44070982933044434) * 0.5,
    (0.44070982933044434 + 0.5626170039176941) * 0.5,
    (0.5626170039176941 + 0.7229568362236023) * 0.5,
    (0.7229568362236023 + 1.0) * 0.5,
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// two floats -> packed bf16 pair (round to nearest even), a in the low half
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// ---------------------------------------------------------------------------------------
// Exact NF4 encoder.
//
// The code of w in a block with scale M > 0 is #{ j : w > mid_j * M } with the comparison in
// real arithmetic.  mid_j * M is exact in fp64 (29 x 24 significant bits).  For an fp32 w,
//     w > t   <=>   w > RD32(t)         (RD32 = round toward -inf to fp32)
// because no fp32 number lies strictly between RD32(t) and t.  So the 15 thresholds are
// rounded down to fp32 once per block and every element then needs fp32 compares only.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float nf4_threshold(double mid, float absmax) {
    const double t = mid * (double)absmax;  // exact
    float f = (float)t;                     // round to nearest
    if ((double)f > t) {                    // went up: step to the next fp32 below
        uint32_t u = __float_as_uint(f);
        u = (f > 0.0f) ? u - 1u : ((f < 0.0f) ? u + 1u : 0x80000001u);
        f = __uint_as_float(u);
    }
    return f;
}

struct Nf4Thresholds {
    float t[15];
    __device__ __forceinline__ void set(float absmax) {
#pragma unroll
        for (int j = 0; j < 15; ++j) t[j] = nf4_threshold(kNf4Mid[j], absmax);
    }
    // binary search over the 15 thresholds (a select tree: registers cannot be indexed)
    __device__ __forceinline__ uint32_t encode(float w) const {
        const bool b3 = w > t[7];
        const float t2 = b3 ? t[11] : t[3];
        const bool b2 = w > t2;
        const float t1a = b2 ? t[5] : t[1];
        const float t1b = b2 ? t[13] : t[9];
        const bool b1 = w > (b3 ? t1b : t1a);
        const float t0a = b1 ? t[2] : t[0];
        const float t0b = b1 ? t[6] : t[4];
        const float t0c = b1 ? t[10] : t[8];
        const float t0d = b1 ? t[14] : t[12];
        const float t0ab = b2 ? t0b : t0a;
        const float t0cd = b2 ? t0d : t0c;
        const bool b0 = w > (b3 ? t0cd : t0ab);
        return (b3 ? 8u : 0u) | (b2 ? 4u : 0u) | (b1 ? 2u : 0u) | (b0 ? 1u : 0u);
    }
};

// ---------------------------------------------------------------------------------------
// kernel timing slots (diagnostics)
// ---------------------------------------------------------------------------------------
enum KernelSlot {
    SLOT_QUANTIZE = 0,
    SLOT_DEQUANTIZE,
    SLOT_GEMM_U,      // U = s x B^T
    SLOT_GEMM_Y,      // y = x W^T + U P^T
    SLOT_GEMM_Z,      // Z = s dy P
    SLOT_GEMM_DX,     // dx = dy W + Z B
    SLOT_GEMM_DB,     // dB partials = Z^T x
    SLOT_REDUCE_DB,   // dB = sum of partials
    SLOT_MERGE,       // fused merge + requantise
    SLOT_PREPASS,     // NF4 -> bf16 (plain or transposed) and bf16 transposes of the large-token path
    SLOT_FOLD,        // W_eff = deq(W) + s deq(P) B in bf16 (folded path)
    SLOT_COUNT
};

struct TimedLaunch {
    hipStream_t stream;
    int slot;
    int idx;
    TimedLaunch(int slot, hipStream_t s);
    ~TimedLaunch();
};

// ---------------------------------------------------------------------------------------
// launchers implemented in codec.hip / gemm.hip
// ---------------------------------------------------------------------------------------
hipError_t launch_quantize(const float* w, int64_t rows, int64_t cols, int64_t ld_w, uint8_t* codes,
                           float* absmax, int64_t ld_q, hipStream_t st);
hipError_t launch_dequantize(const uint8_t* codes, const float* absmax, int64_t rows, int64_t cols,
                             int64_t ld_q, void* out, int out_dtype, int64_t ld_out, hipStream_t st,
                             int slot = SLOT_DEQUANTIZE);

// operand storage kinds of the GEMM
enum OpKind {
    KC_BF16 = 0,  // bf16, rows x K, K contiguous
    RC_BF16 = 1,  // bf16, K x rows, rows contiguous
    KC_NF4 = 2,   // NF4,  rows x K, K contiguous (blocks of 64 along K)
    RC_NF4 = 3,   // NF4,  K x rows, rows contiguous (blocks of 64 along rows)
    OP_NONE = 4
};

struct Operand {
    const void* ptr;      // bf16 elements or packed NF4 codes
    const float* absmax;  // NF4 only
    int64_t ld;           // row pitch of the stored matrix: elements (bf16) or nibbles (NF4)
    int rows;             // extent along M (A operand) or N (B operand)
    int K;                // extent along the contraction
};

enum Epilogue { EPI_BF16 = 0, EPI_F32_SPLITK = 1, EPI_MERGE = 2, EPI_FOLD = 3 };

struct GemmParams {
    Operand A[2], B[2];  // up to two K segments; segment 1 unused when A[1].K == 0
    int M, N;
    float alpha;
    // EPI_BF16: C bf16 M x N pitch ldc.  EPI_F32_SPLITK: C fp32 [split][M][N] dense.
    void* C;
    int64_t ldc;
    int splits;  // EPI_F32_SPLITK: number of K splits (grid.y)
    // optional second column range (NT kernel, EPI_BF16, one K segment): columns N..N+Nx-1 of the
    // product use operand Bx and go to Cx with their own scale; tiles never straddle the ranges
    Operand Bx;
    void* Cx;
    int64_t ldcx;
    int Nx;
    float alphax;
    // EPI_MERGE (M = in, N = out): old weight and destination
    const uint8_t* w_codes;
    const float* w_absmax;
    uint8_t* out_codes;
    float* out_absmax;
    int64_t w_ld;  // pitch in nibbles
    int w_cols;    // logical columns of W (= M)
};

// which GEMM to run
enum GemmId { GEMM_U = 0, GEMM_Y, GEMM_Z, GEMM_DX, GEMM_DB, GEMM_MERGE };
hipError_t launch_gemm(GemmId id, const GemmParams& p, hipStream_t st);
hipError_t launch_reduce_db(const float* partials, int splits, int64_t M, int64_t N, int64_t ldp, void* dB,
                            int dB_dtype, int64_t ld_dB, int accumulate, hipStream_t st);
int gemm_db_splits(int64_t T, int64_t r, int64_t in);

// large-token path (gemm_nt.hip): bf16 operands stored rows x K (K contiguous) or, with the
// a_rc / b_rc flag, K x rows (rows contiguous; Operand::ld is the pitch of that stored matrix)
hipError_t launch_gemm_nt(int slot, int epi, bool a_rc, bool b_rc, const GemmParams& p, hipStream_t st);
// tuning aid for benchmarks: 0 = choose by shape, 1 = 256x256, 2 = 256x128, 3 = 128x128 tiles
extern int g_nt_tile_override;

}  // namespace loqt
