// C ABI of libloqt: argument checking, workspace layout, launch sequences, timing.
#include <math.h>
#include <string.h>

#include <algorithm>

#include "loqt_internal.h"

namespace loqt {

// ---------------------------------------------------------------------------------------
// per-kernel timing (diagnostics): events recorded around every launch while enabled
// ---------------------------------------------------------------------------------------
namespace {
struct TimingState {
    bool on = false;
    int n = 0;
    hipEvent_t* begin = nullptr;
    hipEvent_t* end = nullptr;
    int* slot = nullptr;
    int created = 0;
} g_timing;
const char* kSlotNames[SLOT_COUNT] = {"nf4_quantize", "nf4_dequantize", "gemm_u",   "gemm_y",      "gemm_z",
                                      "gemm_dx",      "gemm_db",        "reduce_db", "merge_requant", "prepass", "fold_weight",
                                      "init_requant", "init_solve_b", "merge_dense", "adam_step"};
}  // namespace

TimedLaunch::TimedLaunch(int slot_, hipStream_t s) : stream(s), slot(slot_), idx(-1) {
    if (slot_ < 0 || !g_timing.on || g_timing.n >= LOQT_TIMING_MAX_EVENTS) return;
    idx = g_timing.n++;
    if (idx >= g_timing.created) {
        (void)hipEventCreate(&g_timing.begin[idx]);
        (void)hipEventCreate(&g_timing.end[idx]);
        g_timing.created = idx + 1;
    }
    g_timing.slot[idx] = slot;
    (void)hipEventRecord(g_timing.begin[idx], stream);
}
TimedLaunch::~TimedLaunch() {
    if (idx >= 0) (void)hipEventRecord(g_timing.end[idx], stream);
}

namespace {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int64_t kMaxDim = (int64_t)1 << 30;  // index arithmetic inside the kernels is 32-bit per axis

loqt_status check_nf4(const loqt_nf4_mat* m) {
    if (!m || !m->codes || !m->absmax) return LOQT_INVALID_ARG;
    if (m->rows < 0 || m->cols < 0 || m->ld < 0) return LOQT_INVALID_ARG;
    if (m->rows == 0 || m->cols == 0 || m->rows > kMaxDim || m->cols > kMaxDim) return LOQT_BAD_SHAPE;
    if (m->ld % 64 != 0 || m->ld < m->cols) return LOQT_BAD_SHAPE;
    if (!aligned(m->codes, 16) || !aligned(m->absmax, 4)) return LOQT_MISALIGNED;
    return LOQT_OK;
}

loqt_status check_bf16(const void* p, int64_t rows, int64_t cols, int64_t ld) {
    if (!p) return LOQT_INVALID_ARG;
    if (rows < 0 || cols < 0 || ld < 0) return LOQT_INVALID_ARG;
    if (rows == 0 || cols == 0 || rows > kMaxDim || cols > kMaxDim) return LOQT_BAD_SHAPE;
    if (ld % 8 != 0 || ld < cols) return LOQT_BAD_SHAPE;
    if (!aligned(p, 16)) return LOQT_MISALIGNED;
    return LOQT_OK;
}

#define LOQT_TRY(expr)                     \
    do {                                   \
        loqt_status st__ = (expr);         \
        if (st__ != LOQT_OK) return st__;  \
    } while (0)
#define LOQT_HIP(expr)                                    \
    do {                                                  \
        if ((expr) != hipSuccess) return LOQT_LAUNCH_FAILED; \
    } while (0)

// shapes of the layer: W out x in, P out x r
loqt_status check_layer(const loqt_nf4_mat* Wq, const loqt_nf4_mat* Pq, const void* B, int64_t ld_B) {
    LOQT_TRY(check_nf4(Wq));
    LOQT_TRY(check_nf4(Pq));
    if (Pq->rows != Wq->rows) return LOQT_BAD_SHAPE;
    LOQT_TRY(check_bf16(B, Pq->cols, Wq->cols, ld_B));
    return LOQT_OK;
}

// ---------------------------------------------------------------------------------------
// Two implementations of every call: "fused" (NF4 expanded inside the GEMM's operand staging,
// no pre-pass; best when few tokens share a weight tile) and "prepass" (NF4 expanded to bf16
// once per call, then plain NT GEMMs; best from about a thousand tokens up).
// ---------------------------------------------------------------------------------------
int g_path = LOQT_PATH_AUTO;

// Forward and backward: measured on 768^2 ... 11008x4096 weights, the pre-pass family is ahead of the fused
// form at every token count from 16 up (the fused GEMM pays the NF4 expansion once per 256-token tile row
// and its main loop is slower), so AUTO never picks the fused form there; it stays selectable.
bool use_prepass(int64_t /*tokens*/) {
    return g_path != LOQT_PATH_FUSED;
}
// Merge: below 1024 columns the pre-pass of P costs as much as it saves.
bool use_prepass_merge(int64_t in) {
    if (g_path == LOQT_PATH_FUSED) return false;
    if (g_path == LOQT_PATH_PREPASS || g_path == LOQT_PATH_FOLDED) return true;
    return in >= 1024;
}

// Within the pre-pass family: carry the rank-r term through every token as a second K segment
// (2 T r (in + out) flop per pass) or fold it into the bf16 copy of the weight once per call
// (W_eff = deq(W) + s deq(P) B, 2 out in r flop).  Folding wins from T = out in / (in + out) up.
bool use_folded(int64_t T, int64_t out, int64_t in) {
    if (g_path == LOQT_PATH_FOLDED) return true;
    if (g_path != LOQT_PATH_AUTO) return false;
    return T * (in + out) >= out * in;  // measured: still ahead at the break-even of the flop counts
}

// Backward pass: Z = s dy deq(P) exists anyway (dB needs it), so carrying the rank-r term as a second K segment of
// the dx product costs only 2 T r in flop at the rate of the large products, against 2 out in r flop at the rate of
// the fold (about half of that: short contraction, heavy epilogue) -- cheaper when the weight has many more rows
// than the step has tokens.  Measured rates put the break-even near out = 0.73 T (7B gate / up at 8192 tokens and
// every projection of the 13B block at 4096 tokens take the second-segment form, the square 7B projections fold).
bool use_folded_bwd(int64_t T, int64_t out, int64_t in) {
    if (!use_folded(T, out, in)) return false;
    if (g_path != LOQT_PATH_AUTO) return true;
    return (double)out <= 0.73 * (double)T;
}

inline size_t bf16_bytes(int64_t rows, int64_t cols) {
    return round_up((size_t)rows * (size_t)round_up(cols, 8) * 2, 256);
}
size_t bwd_z_bytes(int64_t T, int64_t r) { return bf16_bytes(T, r); }

// Workspace layouts of the pre-pass family.  Products take their operands in whichever orientation
// they are stored (rows x K or K x rows), so nothing is ever transposed: the only pre-passes are NF4
// expansions, one per NF4 operand and call.
// Number of slices of the contraction for a product whose result is summed from fp32 slices (dB = Z^T x and its
// relatives: M x N outputs, contraction K).  Estimated duration in k-tile steps: rounds of work-groups (256 tiles
// of 256x128 with one work-group per compute unit from 512 rows up, 512 tiles of 128x128 with two per unit below;
// the launcher makes the same choice) times the k-tiles per slice plus a fixed prologue / epilogue, plus the slices'
// own traffic (each is written once and read once by the reduction: M N 8 bytes against the ~12 MB the chip moves
// in one k-tile step when the slices stay in the Infinity Cache).  A slice is at least 512 deep.
int choose_splits(int64_t M, int64_t N, int64_t K) {
    auto cdiv = [](int64_t a, int64_t b) { return (a + b - 1) / b; };
    const bool wide = M >= 512;
    const int64_t tiles = wide ? cdiv(M, 256) * cdiv(N, 128) : cdiv(M, 128) * cdiv(N, 128);
    const int64_t slots = wide ? 256 : 512;
    const int64_t nkt = cdiv(K, 64);
    const double per_slice = (double)M * (double)N * 8.0 / 12.0e6;
    int best = 1;
    double best_cost = 0.0;
    for (int s = 1; s <= 16; ++s) {
        if (s > 1 && nkt / s < 8) break;
        const double cost = (double)cdiv(tiles * s, slots) * ((double)cdiv(nkt, s) + 6.0) + per_slice * s;
        if (s == 1 || cost < best_cost) best = s, best_cost = cost;
    }
    return best;
}

// Z = s dy deq(P) (T x r outputs, contraction over `out`) in two fp32 slices of the contraction when its 256x128
// tiles would fill no more than half of the compute units (1B block: 8192 x 512; 13B block: 4096 x 1024): twice
// the work-groups at half the depth, then the fixed-order sum of the slices into bf16.  1 = one bf16 product.
int z_splits(int64_t T, int64_t out, int64_t r) {
    if (T < 512 || out < 2048) return 1;
    const int64_t tiles = ((T + 255) / 256) * ((r + 127) / 128);
    return (tiles >= 64 && tiles <= 128) ? 2 : 1;
}

// `saved`: the caller keeps W_eff in a buffer of its own (loqt_linear_fwd_save / loqt_linear_bwd_saved), so the
// workspace holds no copy of the weight (and the forward pass, always folded then, no U)
struct FwdWs {
    size_t U, Wb, Pb, split, total;  // U = s x B^T; Wb = deq(W) or W_eff; Pb = deq(P); slices of y's column remainder
    int64_t split_floats;
    FwdWs(int64_t T, int64_t out, int64_t in, int64_t r, bool saved = false) {
        U = 0;
        Wb = U + (saved ? 0 : bf16_bytes(T, r));
        Pb = Wb + (saved ? 0 : bf16_bytes(out, in));
        split = Pb + bf16_bytes(out, r);
        split_floats = remainder_split_floats(T, out);
        total = split + round_up((size_t)split_floats * 4, 256);
    }
};
struct BwdWs {
    size_t Z, Wb, Pb, partials, total;  // Z = s dy deq(P); Wb = deq(W) or W_eff; Pb = deq(P); fp32 slices
    int splits, zsplits;                // slices of dB; slices of Z (1: none)
    int64_t ldp, ldzp;
    BwdWs(int64_t T, int64_t out, int64_t in, int64_t r, bool saved = false) {
        Z = 0;
        Wb = Z + bf16_bytes(T, r);
        Pb = Wb + (saved ? 0 : bf16_bytes(out, in));
        partials = Pb + bf16_bytes(out, r);
        ldp = (int64_t)round_up(in, 4);
        splits = choose_splits(r, in, T);
        ldzp = (int64_t)round_up(r, 4);
        zsplits = z_splits(T, out, r);
        // the slices of Z are summed into Z before the dB product writes its own: one region serves both
        const size_t db_bytes = (size_t)splits * (size_t)r * (size_t)ldp * 4;
        const size_t z_bytes = zsplits > 1 ? (size_t)zsplits * (size_t)T * (size_t)ldzp * 4 : 0;
        // ... and so can the slices of dx's column remainder, which are summed before dB starts
        const size_t dx_bytes = (size_t)remainder_split_floats(T, in) * 4;
        size_t most = db_bytes > z_bytes ? db_bytes : z_bytes;
        if (dx_bytes > most) most = dx_bytes;
        total = partials + round_up(most, 256);
    }
};
struct MergeWs {
    size_t Pb, total;
    MergeWs(int64_t out, int64_t in, int64_t r) {
        (void)in;
        Pb = 0;
        total = Pb + bf16_bytes(out, r);
    }
};

// compensation loop: Pb = bf16(P) (out x r), E = W - deq(Q_c) (out x round_up(in, 64), bf16),
// fp32 slices of B = P^T E over the contraction along `out`
struct InitWs {
    size_t Pb, E, partials, total;
    int splits;
    int64_t ldp, lde, ldr;
    InitWs(int64_t out, int64_t in, int64_t r) {
        ldr = (int64_t)round_up(r, 8);
        lde = (int64_t)round_up(in, 64);
        ldp = (int64_t)round_up(in, 4);
        Pb = 0;
        E = Pb + round_up((size_t)out * (size_t)ldr * 2, 256);
        partials = E + round_up((size_t)out * (size_t)lde * 2, 256);
        splits = choose_splits(r, in, out);
        total = partials + round_up((size_t)splits * (size_t)r * (size_t)ldp * 4, 256);
    }
};

// right-side variant (W + s Bp Q^T): Qb = deq(Q) (in x r), We = folded weight (out x in), V = s x Qb
// (T x r), fp32 slices of dBp = dy^T V over the contraction along T
struct RightWs {
    size_t Qb, We, V, partials, total;
    int splits;
    int64_t ldr, ldw, ldp;
    RightWs(int op, int64_t T, int64_t out, int64_t in, int64_t r) {
        ldr = (int64_t)round_up(r, 8);
        ldw = (int64_t)round_up(in, 8);
        ldp = (int64_t)round_up(r, 4);
        splits = 1;
        Qb = 0;
        We = Qb + bf16_bytes(in, r);
        V = We + (op == LOQT_OP_MERGE_RIGHT ? 0 : bf16_bytes(out, in));
        partials = V + (op == LOQT_OP_BWD_RIGHT ? bf16_bytes(T, r) : 0);
        total = partials;
        if (op == LOQT_OP_BWD_RIGHT) {
            splits = choose_splits(out, r, T);
            total = partials + round_up((size_t)splits * (size_t)out * (size_t)ldp * 4, 256);
        }
    }
};

// shapes of the right-side layer: W out x in, Q in x r, Bp out x r
loqt_status check_layer_right(const loqt_nf4_mat* Wq, const loqt_nf4_mat* Qq, const void* Bp, int64_t ld_Bp) {
    LOQT_TRY(check_nf4(Wq));
    LOQT_TRY(check_nf4(Qq));
    if (Qq->rows != Wq->cols) return LOQT_BAD_SHAPE;
    LOQT_TRY(check_bf16(Bp, Wq->rows, Qq->cols, ld_Bp));
    return LOQT_OK;
}

Operand nf4_operand(const loqt_nf4_mat* m, int rows, int K) {
    Operand o;
    o.ptr = m->codes;
    o.absmax = m->absmax;
    o.ld = m->ld;
    o.rows = rows;
    o.K = K;
    return o;
}
Operand bf16_operand(const void* p, int64_t ld, int rows, int K) {
    Operand o;
    o.ptr = p;
    o.absmax = nullptr;
    o.ld = ld;
    o.rows = rows;
    o.K = K;
    return o;
}
Operand no_operand() {
    Operand o;
    memset(&o, 0, sizeof(o));
    return o;
}

// W_eff[out x in] (bf16, pitch ldw) = deq(Wq) + s * deq(Pq) B; Pb receives deq(Pq) in bf16
loqt_status fold_weight(const loqt_nf4_mat* Wq, const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s,
                        uint16_t* Pb, uint16_t* We, int64_t ldw, bool dequant_p, hipStream_t st) {
    const int64_t out = Wq->rows, in = Wq->cols, r = Pq->cols;
    const int64_t ldr = (int64_t)round_up(r, 8);
    if (dequant_p)
        LOQT_HIP(launch_dequantize(Pq->codes, Pq->absmax, out, r, Pq->ld, Pb, LOQT_BF16, ldr, st, SLOT_PREPASS));
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(Pb, ldr, (int)out, (int)r);   // out x r, K contiguous
    p.B[0] = bf16_operand(B, ld_B, (int)in, (int)r);    // r x in: K x rows
    p.M = (int)out;
    p.N = (int)in;
    p.alpha = s;
    p.C = We;
    p.ldc = ldw;
    p.w_codes = Wq->codes;
    p.w_absmax = Wq->absmax;
    p.w_ld = Wq->ld;
    p.w_cols = (int)in;
    LOQT_HIP(launch_gemm_nt(SLOT_FOLD, EPI_FOLD, false, true, p, st));
    return LOQT_OK;
}

loqt_status merge_fused(const loqt_nf4_mat* Wq, uint8_t* codes_out, float* absmax_out,
                        const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s, hipStream_t st) {
    const int out = (int)Wq->rows, in = (int)Wq->cols, r = (int)Pq->cols;
    GemmParams p;
    memset(&p, 0, sizeof(p));
    // transposed product: rows of the tile run along `in`; the grid reaches the padding
    // columns cols..ld-1 as well (operand rows past `in` read as zero)
    p.A[0] = bf16_operand(B, ld_B, in, r);  // B is r x in: K x rows
    p.B[0] = nf4_operand(Pq, out, r);       // P is out x r: rows x K
    p.M = (int)Wq->ld;
    p.N = out;
    p.alpha = s;
    p.w_codes = Wq->codes;
    p.w_absmax = Wq->absmax;
    p.out_codes = codes_out;
    p.out_absmax = absmax_out;
    p.w_ld = Wq->ld;
    p.w_cols = in;
    LOQT_HIP(launch_gemm(GEMM_MERGE, p, st));
    return LOQT_OK;
}

loqt_status merge_prepass(const loqt_nf4_mat* Wq, uint8_t* codes_out, float* absmax_out,
                          const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s, void* ws,
                          hipStream_t st) {
    const int64_t out = Wq->rows, in = Wq->cols, r = Pq->cols;
    const MergeWs L(out, in, r);
    uint16_t* Pb = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(ws) + L.Pb);
    const int64_t ldr = (int64_t)round_up(r, 8);
    LOQT_HIP(launch_dequantize(Pq->codes, Pq->absmax, out, r, Pq->ld, Pb, LOQT_BF16, ldr, st, SLOT_PREPASS));
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(Pb, ldr, (int)out, (int)r);  // rows of the tile are rows of W
    p.B[0] = bf16_operand(B, ld_B, (int)in, (int)r);   // r x in: K x rows, columns run along `in`
    p.M = (int)out;
    p.N = (int)Wq->ld;  // reach the padding columns (operand columns past `in` are never used)
    p.alpha = s;
    p.w_codes = Wq->codes;
    p.w_absmax = Wq->absmax;
    p.out_codes = codes_out;
    p.out_absmax = absmax_out;
    p.w_ld = Wq->ld;
    p.w_cols = (int)in;
    LOQT_HIP(launch_gemm_nt(SLOT_MERGE, EPI_MERGE, false, true, p, st));
    return LOQT_OK;
}

size_t merge_ws_bytes(int64_t out, int64_t in, int64_t r) { return MergeWs(out, in, r).total; }

loqt_status merge_checked(const loqt_nf4_mat* Wq, uint8_t* codes_out, float* absmax_out,
                          const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s, void* ws,
                          hipStream_t st) {
    if (use_prepass_merge(Wq->cols)) return merge_prepass(Wq, codes_out, absmax_out, Pq, B, ld_B, s, ws, st);
    return merge_fused(Wq, codes_out, absmax_out, Pq, B, ld_B, s, st);
}

loqt_status check_merge_ws(const loqt_nf4_mat* Wq, const loqt_nf4_mat* Pq, void* ws, size_t ws_bytes) {
    if (!use_prepass_merge(Wq->cols)) return LOQT_OK;
    if (!ws) return LOQT_INVALID_ARG;
    if (!aligned(ws, 256)) return LOQT_MISALIGNED;
    if (ws_bytes < merge_ws_bytes(Wq->rows, Wq->cols, Pq->cols)) return LOQT_WORKSPACE_TOO_SMALL;
    return LOQT_OK;
}

// full aliasing of the merge output with its input is allowed, partial overlap is not
loqt_status check_out_alias(const loqt_nf4_mat* Wq, const uint8_t* codes_out, const float* absmax_out) {
    const size_t cb = (size_t)Wq->rows * (size_t)(Wq->ld / 2), ab = (size_t)Wq->rows * (size_t)(Wq->ld / 64) * 4;
    const uint8_t* ci = Wq->codes;
    const uint8_t* ai = reinterpret_cast<const uint8_t*>(Wq->absmax);
    const uint8_t* ao = reinterpret_cast<const uint8_t*>(absmax_out);
    if (codes_out != ci && codes_out < ci + cb && ci < codes_out + cb) return LOQT_INVALID_ARG;
    if (ao != ai && ao < ai + ab && ai < ao + ab) return LOQT_INVALID_ARG;
    return LOQT_OK;
}

loqt_status check_merge(const loqt_nf4_mat* Wq, uint8_t* codes_out, float* absmax_out,
                        const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B) {
    if (!codes_out || !absmax_out) return LOQT_INVALID_ARG;
    LOQT_TRY(check_layer(Wq, Pq, B, ld_B));
    if (!aligned(codes_out, 16) || !aligned(absmax_out, 4)) return LOQT_MISALIGNED;
    return check_out_alias(Wq, codes_out, absmax_out);
}

}  // namespace
}  // namespace loqt

using namespace loqt;

extern "C" {

const char* loqt_status_string(loqt_status st) {
    switch (st) {
        case LOQT_OK: return "LOQT_OK";
        case LOQT_INVALID_ARG: return "LOQT_INVALID_ARG";
        case LOQT_BAD_SHAPE: return "LOQT_BAD_SHAPE";
        case LOQT_MISALIGNED: return "LOQT_MISALIGNED";
        case LOQT_WORKSPACE_TOO_SMALL: return "LOQT_WORKSPACE_TOO_SMALL";
        case LOQT_LAUNCH_FAILED: return "LOQT_LAUNCH_FAILED";
        case LOQT_STATIC_SCRATCH_TOO_SMALL: return "LOQT_STATIC_SCRATCH_TOO_SMALL";
    }
    return "LOQT_UNKNOWN_STATUS";
}

loqt_status nf4_quantize(const float* w, int64_t rows, int64_t cols, int64_t ld_w, uint8_t* codes,
                         float* absmax, int64_t ld_q, void* hip_stream) {
    if (!w || !codes || !absmax) return LOQT_INVALID_ARG;
    if (rows < 0 || cols < 0 || ld_w < 0 || ld_q < 0) return LOQT_INVALID_ARG;
    if (rows == 0 || cols == 0 || rows > kMaxDim || cols > kMaxDim) return LOQT_BAD_SHAPE;
    if (ld_w % 4 != 0 || ld_w < cols || ld_q % 64 != 0 || ld_q < cols) return LOQT_BAD_SHAPE;
    if (!aligned(w, 16) || !aligned(codes, 16) || !aligned(absmax, 4)) return LOQT_MISALIGNED;
    LOQT_HIP(launch_quantize(w, rows, cols, ld_w, codes, absmax, ld_q, (hipStream_t)hip_stream));
    return LOQT_OK;
}

loqt_status nf4_dequantize(const uint8_t* codes, const float* absmax, int64_t rows, int64_t cols,
                           int64_t ld_q, void* out, int out_dtype, int64_t ld_out, void* hip_stream) {
    if (!codes || !absmax || !out) return LOQT_INVALID_ARG;
    if (out_dtype != LOQT_F32 && out_dtype != LOQT_BF16) return LOQT_INVALID_ARG;
    if (rows < 0 || cols < 0 || ld_q < 0 || ld_out < 0) return LOQT_INVALID_ARG;
    if (rows == 0 || cols == 0 || rows > kMaxDim || cols > kMaxDim) return LOQT_BAD_SHAPE;
    if (ld_q % 64 != 0 || ld_q < cols || ld_out < cols) return LOQT_BAD_SHAPE;
    if (ld_out % (out_dtype == LOQT_BF16 ? 8 : 4) != 0) return LOQT_BAD_SHAPE;
    if (!aligned(codes, 16) || !aligned(absmax, 4) || !aligned(out, 16)) return LOQT_MISALIGNED;
    LOQT_HIP(launch_dequantize(codes, absmax, rows, cols, ld_q, out, out_dtype, ld_out,
                               (hipStream_t)hip_stream));
    return LOQT_OK;
}

size_t loqt_workspace_bytes(int op, int64_t T, int64_t out, int64_t in, int64_t r) {
    if (out <= 0 || in <= 0 || r <= 0) return 0;
    // enough for either implementation, so that the size does not depend on the path option
    switch (op) {
        case LOQT_OP_FWD: {
            if (T <= 0) return 0;
            return FwdWs(T, out, in, r).total;  // the fused path needs only its first part (U)
        }
        case LOQT_OP_BWD: {
            if (T <= 0) return 0;
            const size_t fused = bwd_z_bytes(T, r) + round_up((size_t)gemm_db_splits(T, r, in) * (size_t)r * (size_t)in * 4, 256);
            const size_t pre = BwdWs(T, out, in, r).total;
            return fused > pre ? fused : pre;
        }
        case LOQT_OP_FWD_SAVE: return T <= 0 ? 0 : FwdWs(T, out, in, r, true).total;
        case LOQT_OP_BWD_SAVED: return T <= 0 ? 0 : BwdWs(T, out, in, r, true).total;
        case LOQT_OP_MERGE: return merge_ws_bytes(out, in, r);
        case LOQT_OP_INIT: return InitWs(out, in, r).total;
        case LOQT_OP_FWD_RIGHT:
        case LOQT_OP_BWD_RIGHT:
            if (T <= 0) return 0;
            return RightWs(op, T, out, in, r).total;
        case LOQT_OP_MERGE_RIGHT: return RightWs(op, 0, out, in, r).total;
        // LoQT-nq: U or Z (T x r) first, then the dB slices (backward), then room for the folded weight
        // W_eff (out x in, bf16), whether or not the path option makes this call fold
        case LOQT_OP_FWD_NQ: return T <= 0 ? 0 : bf16_bytes(T, r) + bf16_bytes(out, in);
        case LOQT_OP_BWD_NQ: {
            if (T <= 0) return 0;
            const BwdWs L(T, out, in, r);
            return bf16_bytes(T, r) + (L.total - L.partials) + bf16_bytes(out, in);
        }
        default: return 0;
    }
}

// save_weff != NULL: the folded form is used whatever the path option says and W_eff goes to the caller's
// buffer (pitch ld_save) instead of the workspace
static loqt_status fwd_impl(const loqt_bf16* x, int64_t ld_x, int64_t T, const loqt_nf4_mat* Wq,
                            const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s, loqt_bf16* y,
                            int64_t ld_y, loqt_bf16* save_weff, int64_t ld_save, void* ws, size_t ws_bytes,
                            void* hip_stream) {
    LOQT_TRY(check_layer(Wq, Pq, B, ld_B));
    const int64_t out = Wq->rows, in = Wq->cols, r = Pq->cols;
    LOQT_TRY(check_bf16(x, T, in, ld_x));
    LOQT_TRY(check_bf16(y, T, out, ld_y));
    if (!ws) return LOQT_INVALID_ARG;
    if (!aligned(ws, 256)) return LOQT_MISALIGNED;
    if (ws_bytes < loqt_workspace_bytes(save_weff ? LOQT_OP_FWD_SAVE : LOQT_OP_FWD, T, out, in, r))
        return LOQT_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t ld_u = (int64_t)round_up(r, 8);
    loqt_bf16* U = reinterpret_cast<loqt_bf16*>(ws);
    GemmParams p;

    if (save_weff) LOQT_TRY(check_bf16(save_weff, out, in, ld_save));
    if (save_weff || use_prepass(T)) {
        const FwdWs L(T, out, in, r, save_weff != nullptr);
        char* base = reinterpret_cast<char*>(ws);
        uint16_t* Wb = save_weff ? save_weff : reinterpret_cast<uint16_t*>(base + L.Wb);
        uint16_t* Pb = reinterpret_cast<uint16_t*>(base + L.Pb);
        const int64_t ldw = save_weff ? ld_save : (int64_t)round_up(in, 8);
        const bool folded = save_weff || use_folded(T, out, in);
        if (folded) {
            // y = x W_eff^T with W_eff = deq(W) + s deq(P) B folded once per call
            LOQT_TRY(fold_weight(Wq, Pq, B, ld_B, s, Pb, Wb, ldw, true, st));
        } else {
            LOQT_HIP(launch_dequantize(Wq->codes, Wq->absmax, out, in, Wq->ld, Wb, LOQT_BF16, ldw, st, SLOT_PREPASS));
            LOQT_HIP(launch_dequantize(Pq->codes, Pq->absmax, out, r, Pq->ld, Pb, LOQT_BF16, ld_u, st, SLOT_PREPASS));
            // U = s x B^T
            memset(&p, 0, sizeof(p));
            p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
            p.B[0] = bf16_operand(B, ld_B, (int)r, (int)in);
            p.M = (int)T;
            p.N = (int)r;
            p.alpha = s;
            p.C = U;
            p.ldc = ld_u;
            LOQT_HIP(launch_gemm_nt(SLOT_GEMM_U, EPI_BF16, false, false, p, st));
        }
        // y = x Wb^T (+ U deq(P)^T when the rank-r term is not folded into Wb)
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
        p.B[0] = bf16_operand(Wb, ldw, (int)out, (int)in);
        if (!folded) {
            p.A[1] = bf16_operand(U, ld_u, (int)T, (int)r);
            p.B[1] = bf16_operand(Pb, ld_u, (int)out, (int)r);
        }
        p.M = (int)T;
        p.N = (int)out;
        p.alpha = 1.0f;
        p.C = y;
        p.ldc = ld_y;
        p.split_ws = reinterpret_cast<float*>(base + L.split);
        p.split_ws_floats = L.split_floats;
        LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Y, EPI_BF16, false, false, p, st));
        return LOQT_OK;
    }

    memset(&p, 0, sizeof(p));
    // U = s x B^T
    p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
    p.B[0] = bf16_operand(B, ld_B, (int)r, (int)in);
    p.M = (int)T;
    p.N = (int)r;
    p.alpha = s;
    p.C = U;
    p.ldc = ld_u;
    LOQT_HIP(launch_gemm(GEMM_U, p, st));
    // y = x deq(W)^T + U deq(P)^T
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
    p.B[0] = nf4_operand(Wq, (int)out, (int)in);
    p.A[1] = bf16_operand(U, ld_u, (int)T, (int)r);
    p.B[1] = nf4_operand(Pq, (int)out, (int)r);
    p.M = (int)T;
    p.N = (int)out;
    p.alpha = 1.0f;
    p.C = y;
    p.ldc = ld_y;
    LOQT_HIP(launch_gemm(GEMM_Y, p, st));
    return LOQT_OK;
}

loqt_status loqt_linear_fwd(const loqt_bf16* x, int64_t ld_x, int64_t T, const loqt_nf4_mat* Wq,
                            const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s,
                            loqt_bf16* y, int64_t ld_y, void* ws, size_t ws_bytes, void* hip_stream) {
    return fwd_impl(x, ld_x, T, Wq, Pq, B, ld_B, s, y, ld_y, nullptr, 0, ws, ws_bytes, hip_stream);
}

loqt_status loqt_linear_fwd_save(const loqt_bf16* x, int64_t ld_x, int64_t T, const loqt_nf4_mat* Wq,
                                 const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s, loqt_bf16* y,
                                 int64_t ld_y, loqt_bf16* w_eff, int64_t ld_weff, void* ws, size_t ws_bytes,
                                 void* hip_stream) {
    if (!w_eff) return LOQT_INVALID_ARG;
    return fwd_impl(x, ld_x, T, Wq, Pq, B, ld_B, s, y, ld_y, w_eff, ld_weff, ws, ws_bytes, hip_stream);
}

// saved != NULL: W_eff (out x in_saved, bf16, pitch ld_saved) was produced by loqt_linear_fwd_save with the same
// W_q, P_q, B and s; it replaces the fold, and Wq / B are not looked at
static loqt_status bwd_impl(const loqt_bf16* dy, int64_t ld_dy, const loqt_bf16* x, int64_t ld_x, int64_t T,
                            const loqt_nf4_mat* Wq, const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B,
                            float s, loqt_bf16* dx, int64_t ld_dx, void* dB, int dB_dtype, int64_t ld_dB,
                            int accumulate, const loqt_bf16* saved, int64_t ld_saved, int64_t in_saved, void* ws,
                            size_t ws_bytes, void* hip_stream) {
    if (saved) {
        LOQT_TRY(check_nf4(Pq));
        if (in_saved < 0) return LOQT_INVALID_ARG;
        LOQT_TRY(check_bf16(saved, Pq->rows, in_saved, ld_saved));
    } else {
        LOQT_TRY(check_layer(Wq, Pq, B, ld_B));
    }
    const int64_t out = Pq->rows, in = saved ? in_saved : Wq->cols, r = Pq->cols;
    LOQT_TRY(check_bf16(dy, T, out, ld_dy));
    LOQT_TRY(check_bf16(x, T, in, ld_x));
    if (dx) LOQT_TRY(check_bf16(dx, T, in, ld_dx));
    if (!dB) return LOQT_INVALID_ARG;
    if (dB_dtype != LOQT_F32 && dB_dtype != LOQT_BF16) return LOQT_INVALID_ARG;
    if (ld_dB < in) return LOQT_BAD_SHAPE;
    if (!aligned(dB, dB_dtype == LOQT_BF16 ? 2 : 4)) return LOQT_MISALIGNED;
    if (!ws) return LOQT_INVALID_ARG;
    if (!aligned(ws, 256)) return LOQT_MISALIGNED;
    if (ws_bytes < loqt_workspace_bytes(saved ? LOQT_OP_BWD_SAVED : LOQT_OP_BWD, T, out, in, r))
        return LOQT_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t ld_z = (int64_t)round_up(r, 8);
    loqt_bf16* Z = reinterpret_cast<loqt_bf16*>(ws);
    float* partials = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + bwd_z_bytes(T, r));

    GemmParams p;
    if (saved || use_prepass(T)) {
        const BwdWs L(T, out, in, r, saved != nullptr);
        char* base = reinterpret_cast<char*>(ws);
        const uint16_t* Wb = saved ? saved : reinterpret_cast<const uint16_t*>(base + L.Wb);
        uint16_t* Pb = reinterpret_cast<uint16_t*>(base + L.Pb);
        float* part = reinterpret_cast<float*>(base + L.partials);
        const int64_t ldw = saved ? ld_saved : (int64_t)round_up(in, 8);
        LOQT_HIP(launch_dequantize(Pq->codes, Pq->absmax, out, r, Pq->ld, Pb, LOQT_BF16, ld_z, st, SLOT_PREPASS));
        const bool folded = dx && (saved || use_folded_bwd(T, out, in));
        // Z rides along with dx (one product [dx | Z] over the shared operand dy) when that is estimated to
        // take less time than the two launches: its tiles then fill a partly empty round of the dx product
        bool z_with_dx = false;
        if (folded) {
            const int64_t tm = (T + 255) / 256, tm128 = (T + 127) / 128;
            const int64_t t_dx = tm * ((in + 255) / 256), t_z = tm * ((r + 255) / 256);
            // Z alone: 256x256 tiles when they fill the chip, else 128x128 in rounds of 512
            // (with a long contraction and 224 .. 256 tiles of 256x128 it runs on those: about 0.55 of a round)
            const int64_t t_z2 = tm * ((r + 127) / 128);
            const double z_alone = t_z >= 224 ? plan_bf16_product(T, r, 0).cost
                                   : (out >= 2048 && t_z2 >= 224 && t_z2 <= 256)
                                       ? 0.55
                                       : 0.68 * (double)((tm128 * ((r + 127) / 128) + 511) / 512);
            z_with_dx = t_dx >= 224 && plan_bf16_product(T, in, r).cost < plan_bf16_product(T, in, 0).cost + z_alone;
        }
        if (!z_with_dx) {
            // Z = s dy deq(P): deq(P) is out x r, i.e. K x rows
            memset(&p, 0, sizeof(p));
            p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
            p.B[0] = bf16_operand(Pb, ld_z, (int)r, (int)out);
            p.M = (int)T;
            p.N = (int)r;
            p.alpha = s;
            if (L.zsplits > 1 && g_nt_tile_override == 0) {  // (a forced tile shape keeps the single product)
                p.C = part;
                p.ldc = L.ldzp;
                p.splits = L.zsplits;
                LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Z, EPI_F32_SPLITK, false, true, p, st));
                LOQT_HIP(launch_reduce_db(part, L.zsplits, T, r, L.ldzp, Z, LOQT_BF16, ld_z, 0, st));
            } else {
                p.C = Z;
                p.ldc = ld_z;
                LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Z, EPI_BF16, false, true, p, st));
            }
        }
        if (dx) {
            // dx = dy Wb (+ Z B when the rank-r term is not folded into Wb); Wb is out x in: K x rows
            uint16_t* Wws = reinterpret_cast<uint16_t*>(base + L.Wb);
            if (folded) {
                if (!saved) LOQT_TRY(fold_weight(Wq, Pq, B, ld_B, s, Pb, Wws, ldw, false, st));
            } else {
                LOQT_HIP(launch_dequantize(Wq->codes, Wq->absmax, out, in, Wq->ld, Wws, LOQT_BF16, ldw, st,
                                           SLOT_PREPASS));
            }
            memset(&p, 0, sizeof(p));
            p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
            p.B[0] = bf16_operand(Wb, ldw, (int)in, (int)out);
            if (!folded) {
                p.A[1] = bf16_operand(Z, ld_z, (int)T, (int)r);
                p.B[1] = bf16_operand(B, ld_B, (int)in, (int)r);  // r x in: K x rows
            }
            p.M = (int)T;
            p.N = (int)in;
            p.alpha = 1.0f;
            p.C = dx;
            p.ldc = ld_dx;
            if (z_with_dx) {  // [dx | Z] = dy [W_eff | s deq(P)]
                p.Bx = bf16_operand(Pb, ld_z, (int)r, (int)out);
                p.Nx = (int)r;
                p.alphax = s;
                p.Cx = Z;
                p.ldcx = ld_z;
            }
            p.split_ws = part;  // (the slices of Z, if any, have been summed by now; those of dB come later)
            p.split_ws_floats = remainder_split_floats(T, in);
            LOQT_HIP(launch_gemm_nt(SLOT_GEMM_DX, EPI_BF16, false, true, p, st));
        }
        // dB = Z^T x: Z is T x r and x is T x in, both K x rows; contraction over T in slices
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(Z, ld_z, (int)r, (int)T);
        p.B[0] = bf16_operand(x, ld_x, (int)in, (int)T);
        p.M = (int)r;
        p.N = (int)in;
        p.alpha = 1.0f;
        p.C = part;
        p.ldc = L.ldp;
        p.splits = L.splits;
        LOQT_HIP(launch_gemm_nt(SLOT_GEMM_DB, EPI_F32_SPLITK, true, true, p, st));
        LOQT_HIP(launch_reduce_db(part, L.splits, r, in, L.ldp, dB, dB_dtype, ld_dB, accumulate, st));
        return LOQT_OK;
    }
    memset(&p, 0, sizeof(p));
    // Z = s dy deq(P)
    p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
    p.B[0] = nf4_operand(Pq, (int)r, (int)out);  // P is out x r: K x rows
    p.M = (int)T;
    p.N = (int)r;
    p.alpha = s;
    p.C = Z;
    p.ldc = ld_z;
    LOQT_HIP(launch_gemm(GEMM_Z, p, st));
    if (dx) {
        // dx = dy deq(W) + Z B
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
        p.B[0] = nf4_operand(Wq, (int)in, (int)out);  // W is out x in: K x rows
        p.A[1] = bf16_operand(Z, ld_z, (int)T, (int)r);
        p.B[1] = bf16_operand(B, ld_B, (int)in, (int)r);  // B is r x in: K x rows
        p.M = (int)T;
        p.N = (int)in;
        p.alpha = 1.0f;
        p.C = dx;
        p.ldc = ld_dx;
        LOQT_HIP(launch_gemm(GEMM_DX, p, st));
    }
    // dB = Z^T x, contraction over T split into a fixed number of slices
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(Z, ld_z, (int)r, (int)T);   // Z is T x r: K x rows
    p.B[0] = bf16_operand(x, ld_x, (int)in, (int)T);  // x is T x in: K x rows
    p.M = (int)r;
    p.N = (int)in;
    p.alpha = 1.0f;
    p.C = partials;
    p.splits = gemm_db_splits(T, r, in);
    LOQT_HIP(launch_gemm(GEMM_DB, p, st));
    LOQT_HIP(launch_reduce_db(partials, p.splits, r, in, in, dB, dB_dtype, ld_dB, accumulate, st));
    return LOQT_OK;
}

loqt_status loqt_linear_bwd(const loqt_bf16* dy, int64_t ld_dy, const loqt_bf16* x, int64_t ld_x, int64_t T,
                            const loqt_nf4_mat* Wq, const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B,
                            float s, loqt_bf16* dx, int64_t ld_dx, void* dB, int dB_dtype, int64_t ld_dB,
                            int accumulate, void* ws, size_t ws_bytes, void* hip_stream) {
    return bwd_impl(dy, ld_dy, x, ld_x, T, Wq, Pq, B, ld_B, s, dx, ld_dx, dB, dB_dtype, ld_dB, accumulate, nullptr,
                    0, 0, ws, ws_bytes, hip_stream);
}

loqt_status loqt_linear_bwd_saved(const loqt_bf16* dy, int64_t ld_dy, const loqt_bf16* x, int64_t ld_x, int64_t T,
                                  const loqt_nf4_mat* Pq, int64_t in, float s, const loqt_bf16* w_eff,
                                  int64_t ld_weff, loqt_bf16* dx, int64_t ld_dx, void* dB, int dB_dtype,
                                  int64_t ld_dB, int accumulate, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!w_eff) return LOQT_INVALID_ARG;
    return bwd_impl(dy, ld_dy, x, ld_x, T, nullptr, Pq, nullptr, 0, s, dx, ld_dx, dB, dB_dtype, ld_dB, accumulate,
                    w_eff, ld_weff, in, ws, ws_bytes, hip_stream);
}

loqt_status loqt_merge_requant(const loqt_nf4_mat* Wq, uint8_t* codes_out, float* absmax_out,
                               const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B, float s, void* ws,
                               size_t ws_bytes, void* hip_stream) {
    LOQT_TRY(check_merge(Wq, codes_out, absmax_out, Pq, B, ld_B));
    LOQT_TRY(check_merge_ws(Wq, Pq, ws, ws_bytes));
    return merge_checked(Wq, codes_out, absmax_out, Pq, B, ld_B, s, ws, (hipStream_t)hip_stream);
}

loqt_status loqt_merge_requant_batched(int n_layers, const loqt_merge_desc* descs, void* ws, size_t ws_bytes,
                                       void* hip_stream) {
    if (n_layers < 0 || (n_layers > 0 && !descs)) return LOQT_INVALID_ARG;
    for (int i = 0; i < n_layers; ++i) {
        LOQT_TRY(check_merge(&descs[i].Wq, descs[i].codes_out, descs[i].absmax_out, &descs[i].Pq, descs[i].B,
                             descs[i].ld_B));
        LOQT_TRY(check_merge_ws(&descs[i].Wq, &descs[i].Pq, ws, ws_bytes));
    }
    // Layers that take the pre-pass form go out in groups: one launch expands the P_q of the group into the
    // workspace, one launch runs the merge tiles of all its layers.  A group holds as many consecutive layers as
    // the workspace has room for (at most MERGE_GROUP_MAX); with the minimum workspace that is one layer at a
    // time, the same kernels, the same bits.  Layers on the fused form (narrow weights) run one by one.
    hipStream_t st = (hipStream_t)hip_stream;
    int i = 0;
    while (i < n_layers) {
        if (!use_prepass_merge(descs[i].Wq.cols)) {
            LOQT_TRY(merge_checked(&descs[i].Wq, descs[i].codes_out, descs[i].absmax_out, &descs[i].Pq, descs[i].B,
                                   descs[i].ld_B, descs[i].s, ws, st));
            ++i;
            continue;
        }
        MergeGroupLayer layers[MERGE_GROUP_MAX];
        DequantGroupItem deq[MERGE_GROUP_MAX];
        int n = 0;
        size_t used = 0;
        while (i + n < n_layers && n < MERGE_GROUP_MAX && use_prepass_merge(descs[i + n].Wq.cols)) {
            const loqt_merge_desc& d = descs[i + n];
            const int64_t out = d.Wq.rows, in = d.Wq.cols, r = d.Pq.cols;
            const size_t need = merge_ws_bytes(out, in, r);
            if (n > 0 && used + need > ws_bytes) break;
            uint16_t* Pb = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(ws) + used);
            const int64_t ldr = (int64_t)round_up(r, 8);
            deq[n] = DequantGroupItem{d.Pq.codes, d.Pq.absmax, Pb, out, d.Pq.ld, ldr, (int)r};
            layers[n] = MergeGroupLayer{Pb, d.B, ldr, d.ld_B, d.Wq.codes, d.Wq.absmax, d.codes_out, d.absmax_out,
                                        d.Wq.ld, (int)out, (int)in, (int)r, d.s};
            used += need;
            ++n;
        }
        LOQT_HIP(launch_dequantize_grouped(deq, n, st, SLOT_PREPASS));
        LOQT_HIP(launch_merge_grouped(SLOT_MERGE, true, layers, n, st));
        i += n;
    }
    return LOQT_OK;
}

size_t loqt_merge_batched_workspace_bytes(int n_layers, const loqt_merge_desc* descs) {
    if (n_layers <= 0 || !descs) return 0;
    // the largest sum over MERGE_GROUP_MAX consecutive layers: with that much every group is full
    size_t best = 0;
    for (int i = 0; i < n_layers; ++i) {
        size_t sum = 0;
        for (int k = i; k < n_layers && k < i + MERGE_GROUP_MAX; ++k)
            sum += merge_ws_bytes(descs[k].Wq.rows, descs[k].Wq.cols, descs[k].Pq.cols);
        best = std::max(best, sum);
    }
    return best;
}

int loqt_resolved_path(int op, int64_t T, int64_t out, int64_t in) {
    if (op == LOQT_OP_MERGE) return use_prepass_merge(in) ? LOQT_PATH_PREPASS : LOQT_PATH_FUSED;
    if (!use_prepass(T)) return LOQT_PATH_FUSED;
    if (op == LOQT_OP_BWD) return use_folded_bwd(T, out, in) ? LOQT_PATH_FOLDED : LOQT_PATH_PREPASS;
    return use_folded(T, out, in) ? LOQT_PATH_FOLDED : LOQT_PATH_PREPASS;
}

loqt_status loqt_init_compensate(const float* W, int64_t ld_w, const float* P, int64_t ld_p, int64_t out,
                                 int64_t in, int64_t r, float s, int iters, int warm_start, uint8_t* codes_out,
                                 float* absmax_out, int64_t ld_q, loqt_bf16* B, int64_t ld_B, void* ws,
                                 size_t ws_bytes, void* hip_stream) {
    if (!W || !P || !codes_out || !absmax_out) return LOQT_INVALID_ARG;
    if (out < 0 || in < 0 || r < 0 || ld_w < 0 || ld_p < 0 || ld_q < 0) return LOQT_INVALID_ARG;
    if (iters < 1 || (warm_start != 0 && warm_start != 1)) return LOQT_INVALID_ARG;
    if (!(s > 0.f) || !(s <= 3.0e38f)) return LOQT_INVALID_ARG;  // also rejects NaN
    if (out == 0 || in == 0 || r == 0 || out > kMaxDim || in > kMaxDim || r > kMaxDim) return LOQT_BAD_SHAPE;
    if (ld_w % 4 != 0 || ld_w < in || ld_p % 4 != 0 || ld_p < r) return LOQT_BAD_SHAPE;
    if (ld_q % 64 != 0 || ld_q < in) return LOQT_BAD_SHAPE;
    LOQT_TRY(check_bf16(B, r, in, ld_B));
    if (!aligned(W, 16) || !aligned(P, 16) || !aligned(codes_out, 16) || !aligned(absmax_out, 4))
        return LOQT_MISALIGNED;
    if (!ws) return LOQT_INVALID_ARG;
    if (!aligned(ws, 256)) return LOQT_MISALIGNED;
    const InitWs L(out, in, r);
    if (ws_bytes < L.total) return LOQT_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    char* base = reinterpret_cast<char*>(ws);
    uint16_t* Pb = reinterpret_cast<uint16_t*>(base + L.Pb);
    uint16_t* E = reinterpret_cast<uint16_t*>(base + L.E);
    float* part = reinterpret_cast<float*>(base + L.partials);

    LOQT_HIP(launch_f32_to_bf16(P, out, r, ld_p, Pb, L.ldr, st));
    GemmParams p;
    for (int c = 0; c < iters; ++c) {
        // Q_c = q_NF4(W - s P B) and E = W - deq(Q_c); the first step of a cold start has B = 0
        const bool with_product = c > 0 || warm_start;
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(Pb, L.ldr, (int)out, with_product ? (int)r : 0);  // out x r, K contiguous
        p.B[0] = bf16_operand(B, ld_B, (int)in, with_product ? (int)r : 0);     // r x in: K x rows
        p.M = (int)out;
        p.N = (int)ld_q;  // reach the padding columns of the code matrix
        p.alpha = -s;
        p.out_codes = codes_out;
        p.out_absmax = absmax_out;
        p.w_ld = ld_q;
        p.w_cols = (int)in;
        p.w_f32 = W;
        p.w_f32_ld = ld_w;
        p.e_out = E;
        p.e_ld = L.lde;
        LOQT_HIP(launch_gemm_nt(SLOT_INIT_Q, EPI_COMP, false, true, p, st));
        // B = P^T E / s: P is out x r and E is out x in, both K x rows; contraction over `out` in slices
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(Pb, L.ldr, (int)r, (int)out);
        p.B[0] = bf16_operand(E, L.lde, (int)in, (int)out);
        p.M = (int)r;
        p.N = (int)in;
        p.alpha = 1.0f / s;
        p.C = part;
        p.ldc = L.ldp;
        p.splits = L.splits;
        LOQT_HIP(launch_gemm_nt(SLOT_INIT_B, EPI_F32_SPLITK, true, true, p, st));
        LOQT_HIP(launch_reduce_db(part, L.splits, r, in, L.ldp, B, LOQT_BF16, ld_B, 0, st));
    }
    return LOQT_OK;
}

// ---------------------------------------------------------------------------------------
// right-side projection variant: W_eff = deq(W_q) + s Bp deq(Q_q)^T
// ---------------------------------------------------------------------------------------
namespace {
// Qb = deq(Qq) (bf16, in x r) and We = deq(Wq) + s Bp Qb^T (bf16, out x in, pitch ldw)
loqt_status fold_weight_right(const loqt_nf4_mat* Wq, const loqt_nf4_mat* Qq, const loqt_bf16* Bp, int64_t ld_Bp,
                              float s, uint16_t* Qb, int64_t ldr, uint16_t* We, int64_t ldw, hipStream_t st) {
    const int64_t out = Wq->rows, in = Wq->cols, r = Qq->cols;
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(Bp, ld_Bp, (int)out, (int)r);  // out x r, K contiguous
    p.B[0] = bf16_operand(Qb, ldr, (int)in, (int)r);     // in x r: rows x K, K contiguous
    p.M = (int)out;
    p.N = (int)in;
    p.alpha = s;
    p.C = We;
    p.ldc = ldw;
    p.w_codes = Wq->codes;
    p.w_absmax = Wq->absmax;
    p.w_ld = Wq->ld;
    p.w_cols = (int)in;
    LOQT_HIP(launch_gemm_nt(SLOT_FOLD, EPI_FOLD, false, false, p, st));
    return LOQT_OK;
}
loqt_status check_ws(void* ws, size_t ws_bytes, size_t need) {
    if (!ws) return LOQT_INVALID_ARG;
    if (!aligned(ws, 256)) return LOQT_MISALIGNED;
    if (ws_bytes < need) return LOQT_WORKSPACE_TOO_SMALL;
    return LOQT_OK;
}
}  // namespace

loqt_status loqt_linear_fwd_right(const loqt_bf16* x, int64_t ld_x, int64_t T, const loqt_nf4_mat* Wq,
                                  const loqt_nf4_mat* Qq, const loqt_bf16* Bp, int64_t ld_Bp, float s,
                                  loqt_bf16* y, int64_t ld_y, void* ws, size_t ws_bytes, void* hip_stream) {
    LOQT_TRY(check_layer_right(Wq, Qq, Bp, ld_Bp));
    const int64_t out = Wq->rows, in = Wq->cols, r = Qq->cols;
    LOQT_TRY(check_bf16(x, T, in, ld_x));
    LOQT_TRY(check_bf16(y, T, out, ld_y));
    const RightWs L(LOQT_OP_FWD_RIGHT, T, out, in, r);
    LOQT_TRY(check_ws(ws, ws_bytes, L.total));
    hipStream_t st = (hipStream_t)hip_stream;
    char* base = reinterpret_cast<char*>(ws);
    uint16_t* Qb = reinterpret_cast<uint16_t*>(base + L.Qb);
    uint16_t* We = reinterpret_cast<uint16_t*>(base + L.We);
    LOQT_HIP(launch_dequantize(Qq->codes, Qq->absmax, in, r, Qq->ld, Qb, LOQT_BF16, L.ldr, st, SLOT_PREPASS));
    LOQT_TRY(fold_weight_right(Wq, Qq, Bp, ld_Bp, s, Qb, L.ldr, We, L.ldw, st));
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
    p.B[0] = bf16_operand(We, L.ldw, (int)out, (int)in);
    p.M = (int)T;
    p.N = (int)out;
    p.alpha = 1.0f;
    p.C = y;
    p.ldc = ld_y;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Y, EPI_BF16, false, false, p, st));
    return LOQT_OK;
}

loqt_status loqt_linear_bwd_right(const loqt_bf16* dy, int64_t ld_dy, const loqt_bf16* x, int64_t ld_x, int64_t T,
                                  const loqt_nf4_mat* Wq, const loqt_nf4_mat* Qq, const loqt_bf16* Bp,
                                  int64_t ld_Bp, float s, loqt_bf16* dx, int64_t ld_dx, void* dBp, int dBp_dtype,
                                  int64_t ld_dBp, int accumulate, void* ws, size_t ws_bytes, void* hip_stream) {
    LOQT_TRY(check_layer_right(Wq, Qq, Bp, ld_Bp));
    const int64_t out = Wq->rows, in = Wq->cols, r = Qq->cols;
    LOQT_TRY(check_bf16(dy, T, out, ld_dy));
    LOQT_TRY(check_bf16(x, T, in, ld_x));
    if (dx) LOQT_TRY(check_bf16(dx, T, in, ld_dx));
    if (!dBp) return LOQT_INVALID_ARG;
    if (dBp_dtype != LOQT_F32 && dBp_dtype != LOQT_BF16) return LOQT_INVALID_ARG;
    if (ld_dBp < r) return LOQT_BAD_SHAPE;
    if (!aligned(dBp, dBp_dtype == LOQT_BF16 ? 2 : 4)) return LOQT_MISALIGNED;
    const RightWs L(LOQT_OP_BWD_RIGHT, T, out, in, r);
    LOQT_TRY(check_ws(ws, ws_bytes, L.total));
    hipStream_t st = (hipStream_t)hip_stream;
    char* base = reinterpret_cast<char*>(ws);
    uint16_t* Qb = reinterpret_cast<uint16_t*>(base + L.Qb);
    uint16_t* We = reinterpret_cast<uint16_t*>(base + L.We);
    uint16_t* V = reinterpret_cast<uint16_t*>(base + L.V);
    float* part = reinterpret_cast<float*>(base + L.partials);
    LOQT_HIP(launch_dequantize(Qq->codes, Qq->absmax, in, r, Qq->ld, Qb, LOQT_BF16, L.ldr, st, SLOT_PREPASS));
    GemmParams p;
    // V = s x deq(Q): deq(Q) is in x r, i.e. K x rows
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
    p.B[0] = bf16_operand(Qb, L.ldr, (int)r, (int)in);
    p.M = (int)T;
    p.N = (int)r;
    p.alpha = s;
    p.C = V;
    p.ldc = L.ldr;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_U, EPI_BF16, false, true, p, st));
    if (dx) {
        // dx = dy W_eff, W_eff out x in: K x rows
        LOQT_TRY(fold_weight_right(Wq, Qq, Bp, ld_Bp, s, Qb, L.ldr, We, L.ldw, st));
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
        p.B[0] = bf16_operand(We, L.ldw, (int)in, (int)out);
        p.M = (int)T;
        p.N = (int)in;
        p.alpha = 1.0f;
        p.C = dx;
        p.ldc = ld_dx;
        LOQT_HIP(launch_gemm_nt(SLOT_GEMM_DX, EPI_BF16, false, true, p, st));
    }
    // dBp = dy^T V: dy is T x out and V is T x r, both K x rows; contraction over T in slices
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(dy, ld_dy, (int)out, (int)T);
    p.B[0] = bf16_operand(V, L.ldr, (int)r, (int)T);
    p.M = (int)out;
    p.N = (int)r;
    p.alpha = 1.0f;
    p.C = part;
    p.ldc = L.ldp;
    p.splits = L.splits;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_DB, EPI_F32_SPLITK, true, true, p, st));
    LOQT_HIP(launch_reduce_db(part, L.splits, out, r, L.ldp, dBp, dBp_dtype, ld_dBp, accumulate, st));
    return LOQT_OK;
}

loqt_status loqt_merge_requant_right(const loqt_nf4_mat* Wq, uint8_t* codes_out, float* absmax_out,
                                     const loqt_nf4_mat* Qq, const loqt_bf16* Bp, int64_t ld_Bp, float s, void* ws,
                                     size_t ws_bytes, void* hip_stream) {
    if (!codes_out || !absmax_out) return LOQT_INVALID_ARG;
    LOQT_TRY(check_layer_right(Wq, Qq, Bp, ld_Bp));
    if (!aligned(codes_out, 16) || !aligned(absmax_out, 4)) return LOQT_MISALIGNED;
    LOQT_TRY(check_out_alias(Wq, codes_out, absmax_out));
    const int64_t out = Wq->rows, in = Wq->cols, r = Qq->cols;
    const RightWs L(LOQT_OP_MERGE_RIGHT, 0, out, in, r);
    LOQT_TRY(check_ws(ws, ws_bytes, L.total));
    hipStream_t st = (hipStream_t)hip_stream;
    uint16_t* Qb = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(ws) + L.Qb);
    LOQT_HIP(launch_dequantize(Qq->codes, Qq->absmax, in, r, Qq->ld, Qb, LOQT_BF16, L.ldr, st, SLOT_PREPASS));
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(Bp, ld_Bp, (int)out, (int)r);  // rows of the tile are rows of W
    p.B[0] = bf16_operand(Qb, L.ldr, (int)in, (int)r);   // in x r: columns of the tile run along `in`
    p.M = (int)out;
    p.N = (int)Wq->ld;  // reach the padding columns (operand rows past `in` are never used)
    p.alpha = s;
    p.w_codes = Wq->codes;
    p.w_absmax = Wq->absmax;
    p.out_codes = codes_out;
    p.out_absmax = absmax_out;
    p.w_ld = Wq->ld;
    p.w_cols = (int)in;
    LOQT_HIP(launch_gemm_nt(SLOT_MERGE, EPI_MERGE, false, false, p, st));
    return LOQT_OK;
}

loqt_status loqt_merge_dense(const loqt_nf4_mat* Wq, const loqt_nf4_mat* Pq, const loqt_bf16* B, int64_t ld_B,
                             float s, float* W_out, int64_t ld_out, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!W_out) return LOQT_INVALID_ARG;
    LOQT_TRY(check_layer(Wq, Pq, B, ld_B));
    const int64_t out = Wq->rows, in = Wq->cols, r = Pq->cols;
    if (ld_out < 0) return LOQT_INVALID_ARG;
    if (ld_out % 4 != 0 || ld_out < in) return LOQT_BAD_SHAPE;
    if (!aligned(W_out, 16)) return LOQT_MISALIGNED;
    const MergeWs L(out, in, r);
    if (!ws) return LOQT_INVALID_ARG;
    if (!aligned(ws, 256)) return LOQT_MISALIGNED;
    if (ws_bytes < L.total) return LOQT_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)hip_stream;
    uint16_t* Pb = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(ws) + L.Pb);
    const int64_t ldr = (int64_t)round_up(r, 8);
    LOQT_HIP(launch_dequantize(Pq->codes, Pq->absmax, out, r, Pq->ld, Pb, LOQT_BF16, ldr, st, SLOT_PREPASS));
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(Pb, ldr, (int)out, (int)r);
    p.B[0] = bf16_operand(B, ld_B, (int)in, (int)r);  // r x in: K x rows
    p.M = (int)out;
    p.N = (int)in;
    p.alpha = s;
    p.C = W_out;
    p.ldc = ld_out;
    p.splits = 1;
    p.w_codes = Wq->codes;
    p.w_absmax = Wq->absmax;
    p.w_ld = Wq->ld;
    p.w_cols = (int)in;
    LOQT_HIP(launch_gemm_nt(SLOT_MERGE_DENSE, EPI_FOLD_F32, false, true, p, st));
    return LOQT_OK;
}

loqt_status loqt_adam_step(loqt_bf16* B, int64_t ld_B, int64_t rows, int64_t cols, const void* grad, int grad_dtype,
                           int64_t ld_grad, float* m, float* v, int64_t ld_mv, float lr, float beta1, float beta2,
                           float eps, int64_t step, void* hip_stream) {
    if (!grad || !m || !v) return LOQT_INVALID_ARG;
    if (grad_dtype != LOQT_F32 && grad_dtype != LOQT_BF16) return LOQT_INVALID_ARG;
    if (step < 1 || !(lr >= 0.f) || !(eps >= 0.f) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        return LOQT_INVALID_ARG;
    LOQT_TRY(check_bf16(B, rows, cols, ld_B));
    if (ld_grad < cols || ld_mv < cols) return LOQT_BAD_SHAPE;
    if (!aligned(grad, grad_dtype == LOQT_BF16 ? 2 : 4) || !aligned(m, 4) || !aligned(v, 4)) return LOQT_MISALIGNED;
    // bias corrections in double on the host
    const double bc1 = 1.0 / (1.0 - pow((double)beta1, (double)step));
    const double bc2 = 1.0 / (1.0 - pow((double)beta2, (double)step));
    LOQT_HIP(launch_adam(B, ld_B, grad, grad_dtype, ld_grad, m, v, ld_mv, rows, cols, lr, beta1, beta2, eps,
                         (float)bc1, (float)bc2, (hipStream_t)hip_stream));
    return LOQT_OK;
}

loqt_status loqt_merge_schedule(double tau, double psi, int64_t cap, int n, int64_t* steps_out) {
    if (!steps_out || n < 0) return LOQT_INVALID_ARG;
    if (!(tau >= 1.0) || !(psi >= 1.0) || cap < 1) return LOQT_INVALID_ARG;
    int64_t t = 0;
    for (int i = 0; i < n; ++i) {
        const double gap = floor(tau + pow(psi, (double)i));  // +inf once psi^i overflows: capped below
        t += gap >= (double)cap ? cap : (int64_t)gap;
        steps_out[i] = t;
    }
    return LOQT_OK;
}

// ---------------------------------------------------------------------------------------
// LoQT-nq: W and P in bf16, no quantisation anywhere
// ---------------------------------------------------------------------------------------
namespace {
loqt_status check_layer_nq(const loqt_bf16* W, int64_t ld_W, const loqt_bf16* P, int64_t ld_P, const loqt_bf16* B,
                           int64_t ld_B, int64_t out, int64_t in, int64_t r) {
    LOQT_TRY(check_bf16(W, out, in, ld_W));
    LOQT_TRY(check_bf16(P, out, r, ld_P));
    LOQT_TRY(check_bf16(B, r, in, ld_B));
    return LOQT_OK;
}
}  // namespace

// W_eff = bf16(W + s P B) for the unquantised layer (the product of loqt_merge_nq, written to `We`, pitch ld_we,
// instead of over W)
static hipError_t fold_nq(const loqt_bf16* W, int64_t ld_W, const loqt_bf16* P, int64_t ld_P, const loqt_bf16* B,
                          int64_t ld_B, int64_t out, int64_t in, int64_t r, float s, uint16_t* We, int64_t ld_we,
                          hipStream_t st) {
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A[0] = bf16_operand(P, ld_P, (int)out, (int)r);
    p.B[0] = bf16_operand(B, ld_B, (int)in, (int)r);  // r x in: K x rows
    p.M = (int)out;
    p.N = (int)in;
    p.alpha = s;
    p.C = We;
    p.ldc = ld_we;
    p.w_bf16 = W;
    p.w_bf16_ld = ld_W;
    return launch_gemm_nt(SLOT_FOLD, EPI_ACC_BF16, false, true, p, st);
}

loqt_status loqt_linear_fwd_nq(const loqt_bf16* x, int64_t ld_x, int64_t T, const loqt_bf16* W, int64_t ld_W,
                               const loqt_bf16* P, int64_t ld_P, const loqt_bf16* B, int64_t ld_B, int64_t out,
                               int64_t in, int64_t r, float s, loqt_bf16* y, int64_t ld_y, void* ws,
                               size_t ws_bytes, void* hip_stream) {
    LOQT_TRY(check_layer_nq(W, ld_W, P, ld_P, B, ld_B, out, in, r));
    LOQT_TRY(check_bf16(x, T, in, ld_x));
    LOQT_TRY(check_bf16(y, T, out, ld_y));
    const bool folded = use_folded(T, out, in);
    LOQT_TRY(check_ws(ws, ws_bytes, bf16_bytes(T, r) + (folded ? bf16_bytes(out, in) : 0)));
    hipStream_t st = (hipStream_t)hip_stream;
    uint16_t* U = reinterpret_cast<uint16_t*>(ws);
    const int64_t ld_u = (int64_t)round_up(r, 8);
    GemmParams p;
    if (folded) {  // y = x W_eff^T with the rank-r term folded into a transient copy of the weight
        uint16_t* We = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(ws) + bf16_bytes(T, r));
        const int64_t ld_we = (int64_t)round_up(in, 8);
        LOQT_HIP(fold_nq(W, ld_W, P, ld_P, B, ld_B, out, in, r, s, We, ld_we, st));
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
        p.B[0] = bf16_operand(We, ld_we, (int)out, (int)in);
        p.M = (int)T;
        p.N = (int)out;
        p.alpha = 1.0f;
        p.C = y;
        p.ldc = ld_y;
        LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Y, EPI_BF16, false, false, p, st));
        return LOQT_OK;
    }
    memset(&p, 0, sizeof(p));  // U = s x B^T
    p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
    p.B[0] = bf16_operand(B, ld_B, (int)r, (int)in);
    p.M = (int)T;
    p.N = (int)r;
    p.alpha = s;
    p.C = U;
    p.ldc = ld_u;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_U, EPI_BF16, false, false, p, st));
    memset(&p, 0, sizeof(p));  // y = [x | U] [W | P]^T
    p.A[0] = bf16_operand(x, ld_x, (int)T, (int)in);
    p.B[0] = bf16_operand(W, ld_W, (int)out, (int)in);
    p.A[1] = bf16_operand(U, ld_u, (int)T, (int)r);
    p.B[1] = bf16_operand(P, ld_P, (int)out, (int)r);
    p.M = (int)T;
    p.N = (int)out;
    p.alpha = 1.0f;
    p.C = y;
    p.ldc = ld_y;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Y, EPI_BF16, false, false, p, st));
    return LOQT_OK;
}

loqt_status loqt_linear_bwd_nq(const loqt_bf16* dy, int64_t ld_dy, const loqt_bf16* x, int64_t ld_x, int64_t T,
                               const loqt_bf16* W, int64_t ld_W, const loqt_bf16* P, int64_t ld_P,
                               const loqt_bf16* B, int64_t ld_B, int64_t out, int64_t in, int64_t r, float s,
                               loqt_bf16* dx, int64_t ld_dx, void* dB, int dB_dtype, int64_t ld_dB, int accumulate,
                               void* ws, size_t ws_bytes, void* hip_stream) {
    LOQT_TRY(check_layer_nq(W, ld_W, P, ld_P, B, ld_B, out, in, r));
    LOQT_TRY(check_bf16(dy, T, out, ld_dy));
    LOQT_TRY(check_bf16(x, T, in, ld_x));
    if (dx) LOQT_TRY(check_bf16(dx, T, in, ld_dx));
    if (!dB) return LOQT_INVALID_ARG;
    if (dB_dtype != LOQT_F32 && dB_dtype != LOQT_BF16) return LOQT_INVALID_ARG;
    if (ld_dB < in) return LOQT_BAD_SHAPE;
    if (!aligned(dB, dB_dtype == LOQT_BF16 ? 2 : 4)) return LOQT_MISALIGNED;
    const BwdWs L(T, out, in, r);  // only its split choice and slice pitch are used here
    const size_t z_bytes = bf16_bytes(T, r);
    const bool folded = dx && use_folded(T, out, in);
    LOQT_TRY(check_ws(ws, ws_bytes, z_bytes + (L.total - L.partials) + (folded ? bf16_bytes(out, in) : 0)));
    hipStream_t st = (hipStream_t)hip_stream;
    uint16_t* Z = reinterpret_cast<uint16_t*>(ws);
    float* part = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + z_bytes);
    uint16_t* We = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(ws) + z_bytes + (L.total - L.partials));
    const int64_t ld_we = (int64_t)round_up(in, 8);
    if (folded) LOQT_HIP(fold_nq(W, ld_W, P, ld_P, B, ld_B, out, in, r, s, We, ld_we, st));
    const int64_t ld_z = (int64_t)round_up(r, 8);
    GemmParams p;
    memset(&p, 0, sizeof(p));  // Z = s dy P: P is out x r, i.e. K x rows
    p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
    p.B[0] = bf16_operand(P, ld_P, (int)r, (int)out);
    p.M = (int)T;
    p.N = (int)r;
    p.alpha = s;
    p.C = Z;
    p.ldc = ld_z;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_Z, EPI_BF16, false, true, p, st));
    if (dx) {  // dx = [dy | Z] [W ; B]: W is out x in and B is r x in, both K x rows; folded: dx = dy W_eff
        memset(&p, 0, sizeof(p));
        p.A[0] = bf16_operand(dy, ld_dy, (int)T, (int)out);
        p.B[0] = folded ? bf16_operand(We, ld_we, (int)in, (int)out) : bf16_operand(W, ld_W, (int)in, (int)out);
        if (!folded) {
            p.A[1] = bf16_operand(Z, ld_z, (int)T, (int)r);
            p.B[1] = bf16_operand(B, ld_B, (int)in, (int)r);
        }
        p.M = (int)T;
        p.N = (int)in;
        p.alpha = 1.0f;
        p.C = dx;
        p.ldc = ld_dx;
        LOQT_HIP(launch_gemm_nt(SLOT_GEMM_DX, EPI_BF16, false, true, p, st));
    }
    memset(&p, 0, sizeof(p));  // dB = Z^T x over slices of T
    p.A[0] = bf16_operand(Z, ld_z, (int)r, (int)T);
    p.B[0] = bf16_operand(x, ld_x, (int)in, (int)T);
    p.M = (int)r;
    p.N = (int)in;
    p.alpha = 1.0f;
    p.C = part;
    p.ldc = L.ldp;
    p.splits = L.splits;
    LOQT_HIP(launch_gemm_nt(SLOT_GEMM_DB, EPI_F32_SPLITK, true, true, p, st));
    LOQT_HIP(launch_reduce_db(part, L.splits, r, in, L.ldp, dB, dB_dtype, ld_dB, accumulate, st));
    return LOQT_OK;
}

loqt_status loqt_merge_nq(loqt_bf16* W, int64_t ld_W, const loqt_bf16* P, int64_t ld_P, const loqt_bf16* B,
                          int64_t ld_B, int64_t out, int64_t in, int64_t r, float s, void* hip_stream) {
    LOQT_TRY(check_layer_nq(W, ld_W, P, ld_P, B, ld_B, out, in, r));
    GemmParams p;
    memset(&p, 0, sizeof(p));  // W <- bf16(W + s P B), in place
    p.A[0] = bf16_operand(P, ld_P, (int)out, (int)r);
    p.B[0] = bf16_operand(B, ld_B, (int)in, (int)r);  // r x in: K x rows
    p.M = (int)out;
    p.N = (int)in;
    p.alpha = s;
    p.C = W;
    p.ldc = ld_W;
    p.w_bf16 = W;
    p.w_bf16_ld = ld_W;
    LOQT_HIP(launch_gemm_nt(SLOT_MERGE, EPI_ACC_BF16, false, true, p, (hipStream_t)hip_stream));
    return LOQT_OK;
}

size_t loqt_absmax_dq_workspace_bytes(int64_t n) {
    return n <= 0 ? 0 : round_up((size_t)dq_partials(n) * sizeof(double), 256);
}

loqt_status loqt_absmax_dq_compress(const float* absmax, int64_t n, uint8_t* codes8, float* c1, float* mean, void* ws,
                                    size_t ws_bytes, void* hip_stream) {
    if (!absmax || !codes8 || !c1 || !mean) return LOQT_INVALID_ARG;
    if (n <= 0 || n > ((int64_t)1 << 40)) return LOQT_BAD_SHAPE;
    if (!aligned(absmax, 4) || !aligned(c1, 4) || !aligned(mean, 4)) return LOQT_MISALIGNED;
    LOQT_TRY(check_ws(ws, ws_bytes, loqt_absmax_dq_workspace_bytes(n)));
    if (!aligned(ws, 8)) return LOQT_MISALIGNED;
    LOQT_HIP(launch_dq_compress(absmax, n, codes8, c1, mean, reinterpret_cast<double*>(ws), (hipStream_t)hip_stream));
    return LOQT_OK;
}

int64_t loqt_absmax_dq_static_max_n(void) { return dq_static_max_n(); }

loqt_status loqt_absmax_dq_compress_static(const float* absmax, int64_t n, uint8_t* codes8, float* c1, float* mean,
                                           void* hip_stream) {
    if (!absmax || !codes8 || !c1 || !mean) return LOQT_INVALID_ARG;
    if (n <= 0) return LOQT_BAD_SHAPE;
    if (n > dq_static_max_n()) return LOQT_STATIC_SCRATCH_TOO_SMALL;
    if (!aligned(absmax, 4) || !aligned(c1, 4) || !aligned(mean, 4)) return LOQT_MISALIGNED;
    LOQT_HIP(launch_dq_compress_static(absmax, n, codes8, c1, mean, (hipStream_t)hip_stream));
    return LOQT_OK;
}

loqt_status loqt_absmax_dq_expand(const uint8_t* codes8, const float* c1, const float* mean, int64_t n, float* absmax_out,
                                  void* hip_stream) {
    if (!codes8 || !c1 || !mean || !absmax_out) return LOQT_INVALID_ARG;
    if (n <= 0 || n > ((int64_t)1 << 40)) return LOQT_BAD_SHAPE;
    if (!aligned(c1, 4) || !aligned(mean, 4) || !aligned(absmax_out, 4)) return LOQT_MISALIGNED;
    LOQT_HIP(launch_dq_expand(codes8, c1, mean, n, absmax_out, (hipStream_t)hip_stream));
    return LOQT_OK;
}

loqt_status loqt_prepare(void) {
    LOQT_HIP(prepare_nt_kernels());
    LOQT_HIP(prepare_fused_kernels());
    void* scratch_ptr = nullptr;
    LOQT_HIP(dq_static_scratch(&scratch_ptr));
    return LOQT_OK;
}

loqt_status loqt_set_path(int path) {
    if (path < LOQT_PATH_AUTO || path > LOQT_PATH_FOLDED) return LOQT_INVALID_ARG;
    g_path = path;
    return LOQT_OK;
}

loqt_status loqt_set_tile(int tile) {
    if (tile < LOQT_TILE_AUTO || tile > LOQT_TILE_128x128) return LOQT_INVALID_ARG;
    g_nt_tile_override = tile;
    return LOQT_OK;
}

loqt_status loqt_plan_product(int64_t M, int64_t N, int64_t Nx, int64_t* n_large, double* rounds) {
    if (M <= 0 || N <= 0 || Nx < 0 || M > ((int64_t)1 << 30) || N > ((int64_t)1 << 30) || Nx > ((int64_t)1 << 30))
        return LOQT_BAD_SHAPE;
    const BF16Plan plan = plan_bf16_product(M, N, Nx);
    if (n_large) *n_large = plan.n1;
    if (rounds) *rounds = plan.cost;
    return LOQT_OK;
}

void loqt_timing_enable(int on) {
    if (on) {
        if (!g_timing.begin) {
            g_timing.begin = new hipEvent_t[LOQT_TIMING_MAX_EVENTS];
            g_timing.end = new hipEvent_t[LOQT_TIMING_MAX_EVENTS];
            g_timing.slot = new int[LOQT_TIMING_MAX_EVENTS];
        }
        g_timing.n = 0;
        g_timing.on = true;
    } else {
        g_timing.on = false;
    }
}

int loqt_timing_slots(void) { return SLOT_COUNT; }

loqt_status loqt_timing_read(int slot, const char** name, int64_t* launches, double* total_ms) {
    if (slot < 0 || slot >= SLOT_COUNT || !name || !launches || !total_ms) return LOQT_INVALID_ARG;
    *name = kSlotNames[slot];
    *launches = 0;
    *total_ms = 0.0;
    for (int i = 0; i < g_timing.n; ++i) {
        if (g_timing.slot[i] != slot) continue;
        if (hipEventSynchronize(g_timing.end[i]) != hipSuccess) return LOQT_LAUNCH_FAILED;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_timing.begin[i], g_timing.end[i]) != hipSuccess) return LOQT_LAUNCH_FAILED;
        *launches += 1;
        *total_ms += ms;
    }
    return LOQT_OK;
}

}  // extern "C"
