// Internal declarations shared by the translation units of libloqt (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/loqt.h"
#include "../../include/loqt_debug.h"

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
// Exact NF4 encoder (paper sec. 5.1: code = argmin_i |w / M - q_i|, ties to the lower index).
//
// The code of w in a block with scale M > 0 is #{ j : w > mid_j * M } with the comparison in real
// arithmetic, mid_j = (q_j + q_{j+1}) / 2.  Instead of 15 comparisons (or a 4-level select tree over
// 15 per-block thresholds) each element takes about 8 vector operations and two LDS reads:
// with u = w / M in [-1, 1], cut the axis into buckets of width 1/16 whose edges sit at odd
// multiples of 1/32: bucket k = RN(16 u) + 16.  The 15 decision points mid_j are at least 0.0805
// apart and none is closer than 0.004 to a bucket edge, so a bucket holds at most one of them and
// the code of every w that lands in bucket k is
//     c0[k] + [ w > mid[k] * M ],     c0[k] = #{ j : mid_j left of the bucket },
//     mid[k] = mid_{c0[k]}  (+inf when c0[k] = 15; when the bucket holds no decision point the next
//              one to the right is used and the comparison is simply false).
// The bucket index only has to be right up to the guard band (it is computed from an approximate
// reciprocal); the deciding comparison is exact: mid * M is a 29 x 24 bit product, exact in fp64,
// and w converts exactly.  All of it runs in fp64, so every finite fp32 block (denormal or huge
// scale included) takes the same path.  A zero block is encoded against M = 1: every element is 0,
// lands in the bucket around 0 and gets code 7.  The same holds for zero padding inside a live block.
// ---------------------------------------------------------------------------------------
struct Nf4EncTables {
    double mid[64];
    uint32_t c0[64];
    float2 fast[64];  // {fl32(mid[k]), c0[k] as bits}: one 8-byte read for the single-precision path
};

// one entry per calling thread, k = 0..63 (entries above 32 are never addressed by finite data
// but keep every masked index inside the table)
__device__ __forceinline__ void nf4_enc_tables_fill(Nf4EncTables* t, int k) {
    const double left = ((double)k - 16.5) * 0.0625 - 1e-4;  // left edge of bucket k, widened by the guard
    int c = 0;
#pragma unroll
    for (int j = 0; j < 15; ++j) c += (kNf4Mid[j] < left) ? 1 : 0;
    double m = __builtin_inf();
#pragma unroll
    for (int j = 0; j < 15; ++j)
        if (j == c) m = kNf4Mid[j];
    t->mid[k] = m;
    t->c0[k] = (uint32_t)c;
    t->fast[k] = make_float2((float)m, __uint_as_float((uint32_t)c));
}

// Two ways to the same code.  encode(): everything in fp64, exact for every finite block.  encode_fast(): the same
// bucket rule in single precision, with the one comparison that decides taken against th32 = fl32(fl32(mid) * M).
// th32 is within 2^-23 |mid M| < 2^-23 M of the exact threshold and d = w - th32 is computed to within 2^-24 |d|,
// so whenever |d| > 2^-22 M its sign is the sign of the exact difference and the code is the exact one; otherwise
// (about one element in a million) the caller's `near` flag is raised and the block is encoded again with
// encode().  Blocks whose scale is outside [2^-100, 2^100] (where 16 / M, th32 or the guard could leave the normal
// range) raise the flag for every element.  Callers test the flag wave-wide (__any), so the branch is uniform.
struct Nf4BlockEncoder {
    double Md, scd;
    float Mf, scf, guard;
    uint32_t out_of_range;
    __device__ __forceinline__ void set(float absmax) {
        Mf = absmax > 0.f ? absmax : 1.f;
        Md = (double)Mf;
        scd = 16.0 * __builtin_amdgcn_rcp(Md);
        scf = 16.0f * __builtin_amdgcn_rcpf(Mf);
        guard = Mf * 0x1p-22f;
        out_of_range = (Mf >= 0x1p-100f && Mf <= 0x1p100f) ? 0u : 1u;
    }
    __device__ __forceinline__ uint32_t encode(const Nf4EncTables* t, float w) const {
        const double wd = (double)w;
        // 1.5 * 2^52 + 16 + 16 u, rounded to an integer by the addition itself: the low word is k
        const double xd = __builtin_fma(wd, scd, 6755399441055760.0);
        const uint32_t k = (uint32_t)__double2loint(xd) & 63u;
        const double th = t->mid[k] * Md;  // exact
        return t->c0[k] + ((wd > th) ? 1u : 0u);
    }
    __device__ __forceinline__ uint32_t encode_fast(const Nf4EncTables* t, float w, uint32_t& near) const {
        // 1.5 * 2^23 + 16 + 16 u, rounded to an integer by the addition itself: the low bits are k
        const float xf = __builtin_fmaf(w, scf, 12582928.0f);
        const uint32_t k = __float_as_uint(xf) & 63u;
        const float2 e = t->fast[k];
        const float d = w - e.x * Mf;
        near |= (__builtin_fabsf(d) > guard) ? out_of_range : 1u;  // also raised by a NaN (never for finite data)
        return __float_as_uint(e.y) + ((d > 0.f) ? 1u : 0u);
    }
};

// four consecutive codes -> the two code bytes they occupy (even element in the high nibble)
__device__ __forceinline__ uint32_t nf4_pack4(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
    return ((c0 << 4) | c1) | (((c2 << 4) | c3) << 8);
}

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
    SLOT_INIT_Q,      // compensation loop: Q_c = q(W - s P B) and the residual W - deq(Q_c)
    SLOT_INIT_B,      // compensation loop: B = P^T (W - deq(Q_c)) / s (fp32 slices)
    SLOT_MERGE_DENSE, // W = deq(W_q) + s deq(P_q) B in fp32 (Alg. 1 line 5 without requantisation)
    SLOT_ADAM,        // Adam step on B
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
// Adam on a bf16 matrix with fp32 moments (bias corrections bc1 = 1/(1-beta1^t), bc2 = 1/(1-beta2^t) from the host)
hipError_t launch_adam(uint16_t* B, int64_t ld_B, const void* g, int g_dtype, int64_t ld_g, float* m, float* v,
                       int64_t ld_mv, int64_t rows, int64_t cols, float lr, float beta1, float beta2, float eps,
                       float bc1, float bc2, hipStream_t st);
// fp32 rows x cols (pitch ld_in, 16-byte aligned rows) -> bf16 (pitch ld_out, multiple of 8), round to nearest even
hipError_t launch_f32_to_bf16(const float* in, int64_t rows, int64_t cols, int64_t ld_in, uint16_t* out,
                              int64_t ld_out, hipStream_t st);

// double-quantised block scales: codes (1 byte per scale), c1 (one fp32 per 256 scales), mean (one fp32);
// partial: dq_partials(n) doubles of scratch
hipError_t launch_dq_compress(const float* absmax, int64_t n, uint8_t* codes, float* c1, float* mean, double* partial,
                              hipStream_t st);
hipError_t launch_dq_expand(const uint8_t* codes, const float* c1, const float* mean, int64_t n, float* out,
                            hipStream_t st);
int64_t dq_partials(int64_t n);
// allocation-free variant: the partial sums live in a file-scope device array of codec.hip (at most
// dq_static_max_n() scales per call); dq_static_scratch resolves and caches its address on the current device
hipError_t launch_dq_compress_static(const float* absmax, int64_t n, uint8_t* codes, float* c1, float* mean,
                                     hipStream_t st);
hipError_t dq_static_scratch(void** out);
int64_t dq_static_max_n();

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

enum Epilogue { EPI_BF16 = 0, EPI_F32_SPLITK = 1, EPI_MERGE = 2, EPI_FOLD = 3, EPI_COMP = 4, EPI_FOLD_F32 = 5, EPI_ACC_BF16 = 6 };

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
    // EPI_COMP (M = out, N = in): W_hat = w_f32 + alpha * acc is quantised into out_codes / out_absmax
    // (pitch w_ld) and the residual w_f32 - deq(q(W_hat)) goes to e_out (bf16, pitch e_ld >= w_cols
    // rounded up to 64)
    // EPI_ACC_BF16 (M = out, N = in): C = bf16(fp32(w_bf16) + alpha * acc); C may be w_bf16 itself
    const uint16_t* w_bf16;
    int64_t w_bf16_ld;
    const float* w_f32;
    int64_t w_f32_ld;
    uint16_t* e_out;
    int64_t e_ld;
    // EPI_BF16, optional: scratch for the fp32 slices of a column remainder that goes out in two slices of the
    // contraction (remainder_split_floats() floats), or null
    float* split_ws;
    int64_t split_ws_floats;
};
// floats of scratch a bf16-output product of M rows and N columns can use for its column remainder (0: none)
int64_t remainder_split_floats(int64_t M, int64_t N);

// which GEMM to run
enum GemmId { GEMM_U = 0, GEMM_Y, GEMM_Z, GEMM_DX, GEMM_DB, GEMM_MERGE };
hipError_t launch_gemm(GemmId id, const GemmParams& p, hipStream_t st);
hipError_t launch_reduce_db(const float* partials, int splits, int64_t M, int64_t N, int64_t ldp, void* dB,
                            int dB_dtype, int64_t ld_dB, int accumulate, hipStream_t st, bool timed = true);
int gemm_db_splits(int64_t T, int64_t r, int64_t in);

// large-token path (gemm_nt.hip): bf16 operands stored rows x K (K contiguous) or, with the
// a_rc / b_rc flag, K x rows (rows contiguous; Operand::ld is the pitch of that stored matrix)
hipError_t launch_gemm_nt(int slot, int epi, bool a_rc, bool b_rc, const GemmParams& p, hipStream_t st);
// several merges as one launch of 128x128 tiles (EPI_MERGE over the tiles of all layers); at most MERGE_GROUP_MAX
// layers per launch.  A: deq(P) in bf16 (out x r, pitch lda); B: the trainable factor, r x in stored K x rows
// (b_rc) or in x r stored rows x K; the rest as in GemmParams.
constexpr int MERGE_GROUP_MAX = 24;
struct MergeGroupLayer {
    const void* A;
    const void* B;
    int64_t lda, ldb;
    const uint8_t* w_codes;
    const float* w_absmax;
    uint8_t* out_codes;
    float* out_absmax;
    int64_t w_ld;
    int out, in, r;
    float s;
};
// NF4 -> bf16 of up to MERGE_GROUP_MAX matrices in one launch
struct DequantGroupItem {
    const uint8_t* codes;
    const float* absmax;
    uint16_t* out;
    int64_t rows, ld_q, ld_out;
    int cols;
};
hipError_t launch_dequantize_grouped(const DequantGroupItem* items, int n, hipStream_t st, int slot);
hipError_t launch_merge_grouped(int slot, bool b_rc, const MergeGroupLayer* layers, int n, hipStream_t st);
// raise the LDS size of every kernel configuration of gemm_nt.hip / gemm.hip above the default (otherwise done at the
// first launch of each), so that a first call can be recorded into a HIP graph
hipError_t prepare_nt_kernels();
hipError_t prepare_fused_kernels();
// tuning aid for benchmarks: 0 = choose by shape, 1 = 256x256, 2 = 256x128, 3 = 128x128 tiles
extern int g_nt_tile_override;
// how launch_gemm_nt lays out a bf16-output product (EPI_BF16) that is large enough for 256x256 tiles, and its
// estimated duration in rounds of such tiles
struct BF16Plan {
    int n1;       // > 0: columns that go out as 256x256 tiles; the rest (and Nx) follow as 128x128 tiles
    double cost;
};
BF16Plan plan_bf16_product(int64_t M, int64_t N, int64_t Nx);

}  // namespace loqt
