/*
 * loqt.h -- C ABI of the MI355X (gfx950) LoQT hot-path library.
 *
 * LoQT ("Low-Rank Adapters for Quantized Pretraining", arxiv 2405.16528) trains a linear
 * layer whose frozen weight W (out x in) and projection P (out x r) are stored in NF4 and
 * whose only trainable tensor is the 16-bit factor B (r x in).  This library implements the
 * three things every training run spends its time in:
 *
 *   forward   y  = x deq(W_q)^T + s (x B^T) deq(P_q)^T              (paper sec. 2.2, 2.4)
 *   backward  dx = dy deq(W_q) + s (dy deq(P_q)) B
 *             dB = s deq(P_q)^T dy^T x     (G^B = P^T G^W, sec. 2.2; no full dW is formed)
 *   merge     W_q <- q_NF4( deq(W_q) + s deq(P_q) B )               (Alg. 1 line 5, sec. 2.4)
 *
 * plus the NF4 block codec itself (sec. 5.1).  Matrices use the PyTorch orientation
 * (y = x W^T): W is out x in, P is out x r, B is r x in, x is T x in, y and dy are T x out.
 *
 * Conventions common to every call
 *   - every data pointer is a DEVICE pointer (the descriptor structs themselves and the
 *     descriptor array of the batched merge live in HOST memory);
 *   - the caller owns every buffer; the library never allocates, frees or keeps a pointer;
 *   - all matrices are row-major with an explicit row pitch ("ld", in elements);
 *     a buffer of `rows` rows spans rows*ld elements;
 *   - bf16 matrices: ld % 8 == 0 and a 16-byte aligned base (so that rows stay 16-byte
 *     aligned); the logical column count is arbitrary;
 *   - work is enqueued on the given hipStream_t (passed as void*; NULL = the null stream)
 *     and the call returns without synchronising;
 *   - arguments are checked on the host; on error a status is returned and NOTHING is
 *     launched.  No exceptions, no state kept between calls, results are bit-deterministic;
 *   - inputs must be finite;
 *   - the calls can be recorded into a HIP graph (stream capture): they allocate nothing, record
 *     no memset nodes and synchronise with nothing.  The first launch of each kernel configuration
 *     in a process sets its LDS size with hipFuncSetAttribute: call loqt_prepare() once before the
 *     first capture (or run every call once eagerly with the shapes in question).
 *
 * NF4 storage (sec. 5.1: blocks of 64 weights, one scale M_beta = max |w| per block)
 *   codes  : rows x ld nibbles, two per byte.  Row i starts at byte i*ld/2; element j of
 *            the row is in byte j/2, EVEN j in the HIGH nibble.  ld % 64 == 0, ld >= cols.
 *            The nibble value is the index into the ascending 16-level NF4 table.
 *   absmax : fp32, ld/64 per row; entry [i*(ld/64) + j/64] scales elements 64*(j/64)..+63 of
 *            row i.  Blocks run along a row and never straddle rows; when cols % 64 != 0 the
 *            last block of a row is short.  (rows = 1, cols = numel gives the flat blocking.)
 *   Writers in this library fill nibbles cols..ld-1 with code 7 (the level 0.0) and give
 *   blocks that lie wholly in that padding absmax 0.  Readers never depend on it.
 *   An all-zero block is stored as absmax 0 / code 7.
 */
#ifndef LOQT_H
#define LOQT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int loqt_status;
enum {
    LOQT_OK = 0,
    LOQT_INVALID_ARG = 1,         /* NULL pointer, negative size, unknown enum value */
    LOQT_BAD_SHAPE = 2,           /* pitch rule violated, operand shapes inconsistent, size 0 */
    LOQT_MISALIGNED = 3,          /* base pointer alignment rule violated */
    LOQT_WORKSPACE_TOO_SMALL = 4, /* ws_bytes < loqt_workspace_bytes(...) */
    LOQT_LAUNCH_FAILED = 5,       /* HIP reported an error at launch */
    LOQT_STATIC_SCRATCH_TOO_SMALL = 6 /* an allocation-free entry point was given more than its fixed scratch holds */
};

typedef uint16_t loqt_bf16; /* raw bfloat16 bits */

/* A read-only NF4 matrix (device pointers, see "NF4 storage" above). */
typedef struct loqt_nf4_mat {
    const uint8_t *codes;
    const float *absmax;
    int64_t rows, cols; /* logical shape */
    int64_t ld;         /* row pitch in nibbles, multiple of 64 */
} loqt_nf4_mat;

enum { LOQT_F32 = 0, LOQT_BF16 = 1 };                 /* output dtypes */
enum { LOQT_OP_FWD = 0, LOQT_OP_BWD = 1, LOQT_OP_MERGE = 2, LOQT_OP_INIT = 3,
       LOQT_OP_FWD_RIGHT = 4, LOQT_OP_BWD_RIGHT = 5, LOQT_OP_MERGE_RIGHT = 6,
       LOQT_OP_FWD_NQ = 7, LOQT_OP_BWD_NQ = 8, LOQT_OP_FWD_SAVE = 9, LOQT_OP_BWD_SAVED = 10 };

/* Human-readable name of a status code (static string). */
const char *loqt_status_string(loqt_status st);

/*
 * nf4_quantize -- q_NF4 of sec. 5.1.
 *   w      : fp32, rows x cols, pitch ld_w (elements; ld_w % 4 == 0, 16-byte aligned base)
 *   codes  : out, rows * ld_q / 2 bytes;  absmax: out, rows * ld_q / 64 floats
 * For every block beta of 64 consecutive elements of a row: M = max |w| (exact), and for
 * each element the code is argmin_i |w/M - q_i| evaluated in exact arithmetic (ties to the
 * lower index).  An all-zero block gives M = 0 and code 7.  Padding as described above.
 */
loqt_status nf4_quantize(const float *w, int64_t rows, int64_t cols, int64_t ld_w,
                         uint8_t *codes, float *absmax, int64_t ld_q, void *hip_stream);

/*
 * nf4_dequantize -- q_NF4^{-1} of sec. 5.1: out[i][j] = M_beta * q[code].
 *   out_dtype LOQT_F32 : one IEEE fp32 multiply (round to nearest even), ld_out % 4 == 0
 *   out_dtype LOQT_BF16: that fp32 value rounded to nearest even bf16,    ld_out % 8 == 0
 * Only columns 0..cols-1 of each output row are written.
 */
loqt_status nf4_dequantize(const uint8_t *codes, const float *absmax, int64_t rows, int64_t cols,
                           int64_t ld_q, void *out, int out_dtype, int64_t ld_out,
                           void *hip_stream);

/*
 * Bytes of device workspace the given operation needs for these sizes (0 is possible).
 * The workspace must be 256-byte aligned; its contents are scratch.  Two calls that share a
 * workspace must be ordered on the same stream.  The figure covers both implementations (see
 * loqt_set_path in loqt_debug.h), so it does not depend on which one runs:
 *   FWD  : U = s x B^T (T x r bf16); pre-pass paths: + bf16 copies of deq(W_q) (or the folded
 *          weight) and deq(P_q)
 *   BWD  : Z = s dy deq(P_q) (T x r bf16), fp32 slices of dB; pre-pass paths: + the same two copies
 *   FWD_SAVE, BWD_SAVED: loqt_linear_fwd_save / loqt_linear_bwd_saved: as FWD / BWD without the copy of the
 *          weight (it lives in the caller's w_eff) and, forward, without U
 *   MERGE: pre-pass path: bf16 deq(P_q) (T is ignored)
 *   INIT : loqt_init_compensate: bf16 copy of P, the residual W - deq(Q_c) in bf16, fp32 slices of
 *          B (T is ignored)
 *   FWD_RIGHT, BWD_RIGHT, MERGE_RIGHT: the right-side variant below, with r = columns of Q_q:
 *          bf16 deq(Q_q); forward and backward + the folded weight (out x in bf16); backward +
 *          V = s x deq(Q_q) (T x r bf16) and fp32 slices of dBp
 *   FWD_NQ, BWD_NQ: the unquantised variant below: U resp. Z (T x r bf16), the fp32 slices of dB and
 *          the folded weight (out x in bf16)
 */
size_t loqt_workspace_bytes(int op, int64_t T, int64_t out, int64_t in, int64_t r);

/*
 * loqt_linear_fwd -- forward pass of the layer (sec. 2.2 "y = xW + xPB", with W and P
 * dequantised from NF4 on the fly, sec. 2.4; s is the scale of Alg. 1 line 5).
 *   y[T x out] = x[T x in] deq(Wq)^T + s * (x B^T) deq(Pq)^T
 *   Wq: out x in, Pq: out x r, B: r x in (pitch ld_B), x pitch ld_x, y pitch ld_y.
 * Products take bf16 operands (dequantised values rounded to nearest even) and accumulate in
 * fp32; y is rounded to bf16 once.  The intermediate s*x*B^T is kept in bf16 in `ws`.
 */
loqt_status loqt_linear_fwd(const loqt_bf16 *x, int64_t ld_x, int64_t T,
                            const loqt_nf4_mat *Wq, const loqt_nf4_mat *Pq,
                            const loqt_bf16 *B, int64_t ld_B, float s,
                            loqt_bf16 *y, int64_t ld_y,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * loqt_linear_bwd -- backward pass (sec. 2.2: the only weight gradient is G^B = P^T G^W).
 *   Z  = s * dy deq(Pq)                          (T x r, kept in bf16 in `ws`, used twice)
 *   dx = dy deq(Wq) + Z B                        (T x in, bf16; pass dx = NULL to skip it)
 *   dB = Z^T x                                   (r x in; dB_dtype LOQT_F32 or LOQT_BF16)
 *   accumulate != 0: dB_out = dB_in + dB (gradient accumulation), else dB_out = dB.
 * The full out x in gradient of W is never formed.  dB is summed in fp32 in a fixed order.
 */
loqt_status loqt_linear_bwd(const loqt_bf16 *dy, int64_t ld_dy, const loqt_bf16 *x, int64_t ld_x,
                            int64_t T, const loqt_nf4_mat *Wq, const loqt_nf4_mat *Pq,
                            const loqt_bf16 *B, int64_t ld_B, float s,
                            loqt_bf16 *dx, int64_t ld_dx,
                            void *dB, int dB_dtype, int64_t ld_dB, int accumulate,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * loqt_linear_fwd_save / loqt_linear_bwd_saved -- the same forward and backward pass (sec. 2.2, 2.4)
 * for callers that can afford to keep the transient 16-bit weight between the two: the forward call
 * also leaves
 *   W_eff[out x in] = bf16( fl32(deq(Wq)) + s * deq(Pq) B )          (w_eff, pitch ld_weff, caller-owned)
 * and the backward call takes it back instead of rebuilding it from the 4-bit codes:
 *   Z = s * dy deq(Pq),  dx = dy W_eff,  dB = Z^T x.
 * y, dx and dB are those of the two calls above when they run the folded form (same kernels, same
 * bits).  w_eff must hold out rows of ld_weff >= in elements (ld_weff % 8 == 0, 16-byte aligned) and
 * must not be touched between the two calls; `in` tells the backward call its width.  Any number of
 * forward / backward pairs may reuse one w_eff while Wq, Pq, B and s stay the same (the micro-batches
 * of a gradient-accumulation step, sec. 3.3).  Workspace sizes: LOQT_OP_FWD_SAVE / LOQT_OP_BWD_SAVED.
 */
loqt_status loqt_linear_fwd_save(const loqt_bf16 *x, int64_t ld_x, int64_t T,
                                 const loqt_nf4_mat *Wq, const loqt_nf4_mat *Pq,
                                 const loqt_bf16 *B, int64_t ld_B, float s,
                                 loqt_bf16 *y, int64_t ld_y, loqt_bf16 *w_eff, int64_t ld_weff,
                                 void *ws, size_t ws_bytes, void *hip_stream);
loqt_status loqt_linear_bwd_saved(const loqt_bf16 *dy, int64_t ld_dy, const loqt_bf16 *x, int64_t ld_x,
                                  int64_t T, const loqt_nf4_mat *Pq, int64_t in, float s,
                                  const loqt_bf16 *w_eff, int64_t ld_weff,
                                  loqt_bf16 *dx, int64_t ld_dx,
                                  void *dB, int dB_dtype, int64_t ld_dB, int accumulate,
                                  void *ws, size_t ws_bytes, void *hip_stream);

/*
 * loqt_merge_requant -- the periodic merge (Alg. 1 line 5; sec. 2.4: dequantise W_q and P_q,
 * add P B, quantise again, one layer at a time).
 *   W_new = deq(Wq) + s * deq(Pq) B   (fp32: fl32(M*q) + fp32-accumulated bf16 product)
 *   (codes_out, absmax_out) = nf4_quantize(W_new), same pitch Wq->ld.
 * codes_out / absmax_out may alias Wq->codes / Wq->absmax (in-place merge); they must not
 * partially overlap them.  B is not modified (re-initialising it is the caller's business).
 */
loqt_status loqt_merge_requant(const loqt_nf4_mat *Wq, uint8_t *codes_out, float *absmax_out,
                               const loqt_nf4_mat *Pq, const loqt_bf16 *B, int64_t ld_B, float s,
                               void *ws, size_t ws_bytes, void *hip_stream);

/* One layer of a batched merge (host struct; pointers inside are device pointers). */
typedef struct loqt_merge_desc {
    loqt_nf4_mat Wq;
    uint8_t *codes_out;
    float *absmax_out;
    loqt_nf4_mat Pq;
    const loqt_bf16 *B;
    int64_t ld_B;
    float s;
} loqt_merge_desc;

/*
 * loqt_merge_requant_batched -- loqt_merge_requant over n_layers layers (descs: HOST array; Alg. 1 line 5
 * for a whole block or model, sec. 2.4 "layer by layer").  Layers are independent; every descriptor is
 * checked before the first launch.  The layers go out in groups of consecutive layers: one launch expands
 * the P_q of a group into the workspace and one launch runs the merge tiles of all its layers, so that a
 * layer's ramp-up, last partly filled round and launch gap are filled with the next layer's tiles.  A group
 * holds as many layers as the workspace has room for (at most 24).  ws_bytes must be at least the largest
 * loqt_workspace_bytes(LOQT_OP_MERGE, ...) of any layer (then every group is one layer);
 * loqt_merge_batched_workspace_bytes returns the size with which every group is full.  Results do not
 * depend on the grouping: bit for bit those of n_layers calls of loqt_merge_requant.
 */
loqt_status loqt_merge_requant_batched(int n_layers, const loqt_merge_desc *descs,
                                       void *ws, size_t ws_bytes, void *hip_stream);
size_t loqt_merge_batched_workspace_bytes(int n_layers, const loqt_merge_desc *descs);

/*
 * Right-side projection variant (sec. 2.2: the one-sided projection is P^T G when the weight has
 * no more rows than columns and G Q otherwise, with the same argument for the right-side factor).  The
 * fixed NF4 projection sits on the input side and the trainable 16-bit factor on the output side:
 *     W_eff = deq(Wq) + s * Bp deq(Qq)^T        Wq: out x in,  Qq: in x r,  Bp: out x r (pitch ld_Bp)
 *   loqt_linear_fwd_right    y  = x W_eff^T  = x deq(Wq)^T + s (x deq(Qq)) Bp^T
 *   loqt_linear_bwd_right    dx = dy W_eff   = dy deq(Wq) + s (dy Bp) deq(Qq)^T      (dx may be NULL)
 *                            dBp (out x r, LOQT_F32 or LOQT_BF16, pitch ld_dBp >= r, optional +=)
 *                                = s dy^T (x deq(Qq))       (G^Bp = G^W Q; no full dW is formed)
 *   loqt_merge_requant_right W_q <- nf4_quantize( deq(Wq) + s Bp deq(Qq)^T ), aliasing rules of
 *                            loqt_merge_requant; Bp is not modified
 * Arguments, tolerances and error behaviour are those of the left-side calls above.  One
 * implementation for every size: deq(Qq) is expanded to bf16 and the rank-r term is folded into a
 * bf16 copy of the weight once per call (2 out in r flop), then y and dx are single products.
 */
loqt_status loqt_linear_fwd_right(const loqt_bf16 *x, int64_t ld_x, int64_t T,
                                  const loqt_nf4_mat *Wq, const loqt_nf4_mat *Qq,
                                  const loqt_bf16 *Bp, int64_t ld_Bp, float s,
                                  loqt_bf16 *y, int64_t ld_y,
                                  void *ws, size_t ws_bytes, void *hip_stream);
loqt_status loqt_linear_bwd_right(const loqt_bf16 *dy, int64_t ld_dy, const loqt_bf16 *x, int64_t ld_x,
                                  int64_t T, const loqt_nf4_mat *Wq, const loqt_nf4_mat *Qq,
                                  const loqt_bf16 *Bp, int64_t ld_Bp, float s,
                                  loqt_bf16 *dx, int64_t ld_dx,
                                  void *dBp, int dBp_dtype, int64_t ld_dBp, int accumulate,
                                  void *ws, size_t ws_bytes, void *hip_stream);
loqt_status loqt_merge_requant_right(const loqt_nf4_mat *Wq, uint8_t *codes_out, float *absmax_out,
                                     const loqt_nf4_mat *Qq, const loqt_bf16 *Bp, int64_t ld_Bp,
                                     float s, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * loqt_init_compensate -- error-compensated initialisation of B (Alg. 2 lines 5-11; sec. 2.5
 * "Compensating for Quantization Errors"): with the projection P fixed, find a quantised weight Q
 * and a factor B such that Q + s P B approximates the full-precision weight W, alternating
 *     Q_c = nf4_quantize( fl32( W - s P B ) )          (B = 0 at a cold start: Q_1 = q(W))
 *     B   = P^+ ( W - deq(Q_c) ) / s                   (least squares: argmin_B |Q_c + s P B - W|_F)
 * for `iters` steps (the paper uses at most five).  Of the three forms the paper prints for the
 * B update this is the one that minimises its stated objective.  It differs from the algorithm box as
 * printed (B <- P^+(W_hat - Q_c) with W_hat = W - P B, which for orthonormal P is this update minus the
 * previous B) from the second iteration on: taken literally that line makes |Q + P B - W| go back up on
 * every second iteration and end above this loop's (shown with the CPU oracle in
 * tests/test_oracle_init.py), so it is read as the least-squares step it names.  P^+ is taken as P^T: P must have
 * orthonormal columns (Alg. 2 line 3: left singular vectors), which is a precondition, not checked.
 *   W  : fp32 out x in,  pitch ld_w (ld_w % 4 == 0, 16-byte aligned base); read only
 *   P  : fp32 out x r,   pitch ld_p (ld_p % 4 == 0, 16-byte aligned base); read only.  The caller
 *        obtains P_q with nf4_quantize(P); the loop itself uses the unquantised P, as Alg. 2 does
 *   s  : scale of the low-rank term, > 0;  iters >= 1
 *   warm_start : 0 = start from B = 0 (Alg. 2 line 5; the contents of B are ignored);
 *                1 = start from the B passed in
 *   codes_out, absmax_out : out, the last Q_c in NF4 storage with pitch ld_q (ld_q % 64 == 0)
 *   B  : bf16 r x in, pitch ld_B; in (warm start) and out (the B that matches Q_c)
 * Products run on bf16 copies of P, B and the residual with fp32 accumulation; the quantiser is the
 * exact one of nf4_quantize.  With iters = 1 and a cold start the codes equal nf4_quantize(W) bit
 * for bit; later steps can differ from an exact evaluation by one level where W - s P B sits within
 * the product's rounding error of a decision point.
 */
loqt_status loqt_init_compensate(const float *W, int64_t ld_w, const float *P, int64_t ld_p,
                                 int64_t out, int64_t in, int64_t r, float s, int iters,
                                 int warm_start, uint8_t *codes_out, float *absmax_out, int64_t ld_q,
                                 loqt_bf16 *B, int64_t ld_B, void *ws, size_t ws_bytes,
                                 void *hip_stream);

/*
 * LoQT-nq -- the method without quantisation (the paper's "LoQT-nq": W and P stay in 16 bits).  Same
 * layer, same gradients, with bf16 matrices W (out x in, pitch ld_W) and P (out x r, pitch ld_P) in
 * place of the NF4 ones:
 *   loqt_linear_fwd_nq   y  = x W^T + s (x B^T) P^T
 *   loqt_linear_bwd_nq   dx = dy W + s (dy P) B  (dx may be NULL),  dB = s P^T dy^T x  (as loqt_linear_bwd)
 *   loqt_merge_nq        W <- bf16( fp32(W) + s * P B ), in place, round to nearest even (Alg. 1 line 5)
 * Nothing is dequantised.  With few tokens the rank-r term is carried as a second K segment of the
 * products ([x | U] [W | P]^T and [dy | Z] [W ; B]) and no pass over the weights precedes them; from
 * T (in + out) >= out * in on it is folded into a transient copy of the
 * weight in the workspace, W_eff = bf16(W + s P B), as in the quantised layer, and y = x W_eff^T,
 * dx = dy W_eff are single products.
 */
loqt_status loqt_linear_fwd_nq(const loqt_bf16 *x, int64_t ld_x, int64_t T,
                               const loqt_bf16 *W, int64_t ld_W, const loqt_bf16 *P, int64_t ld_P,
                               const loqt_bf16 *B, int64_t ld_B, int64_t out, int64_t in, int64_t r,
                               float s, loqt_bf16 *y, int64_t ld_y,
                               void *ws, size_t ws_bytes, void *hip_stream);
loqt_status loqt_linear_bwd_nq(const loqt_bf16 *dy, int64_t ld_dy, const loqt_bf16 *x, int64_t ld_x,
                               int64_t T, const loqt_bf16 *W, int64_t ld_W, const loqt_bf16 *P,
                               int64_t ld_P, const loqt_bf16 *B, int64_t ld_B, int64_t out, int64_t in,
                               int64_t r, float s, loqt_bf16 *dx, int64_t ld_dx,
                               void *dB, int dB_dtype, int64_t ld_dB, int accumulate,
                               void *ws, size_t ws_bytes, void *hip_stream);
loqt_status loqt_merge_nq(loqt_bf16 *W, int64_t ld_W, const loqt_bf16 *P, int64_t ld_P,
                          const loqt_bf16 *B, int64_t ld_B, int64_t out, int64_t in, int64_t r,
                          float s, void *hip_stream);

/*
 * loqt_merge_dense -- Alg. 1 line 5 as printed: W <- W_Q + s P_Q B in full precision, the input of
 * Alg. 2's Initialize (a new P from the gradient, then loqt_init_compensate on this W).
 *   W_out[out x in] (fp32, pitch ld_out, ld_out % 4 == 0, 16-byte aligned) =
 *       fl32(M * q[code]) + s * (fp32-accumulated bf16 product deq(Pq) B), one fused multiply-add;
 * nf4_quantize(W_out) reproduces loqt_merge_requant bit for bit.  Workspace: LOQT_OP_MERGE.
 */
loqt_status loqt_merge_dense(const loqt_nf4_mat *Wq, const loqt_nf4_mat *Pq, const loqt_bf16 *B,
                             int64_t ld_B, float s, float *W_out, int64_t ld_out,
                             void *ws, size_t ws_bytes, void *hip_stream);

/*
 * loqt_absmax_dq_compress / loqt_absmax_dq_expand -- double quantisation of the block scales (sec. 2.4:
 * the quantisation state is itself quantised again, as in the NF4 paper).
 * The paper gives no format; the one implemented is the cited method's description: the scales, being
 * positive, have their mean subtracted and are stored as 8-bit floats in blocks of 256 with one fp32
 * constant per block.  With M[0..n) the fp32 scales of an NF4 matrix taken as a flat array (absmax with
 * its padding, rows * ld / 64 values):
 *     mean = fl32( sum M / n )                         (fp64 sum in a fixed order)
 *     d_j  = fl32(M_j - mean);   c1_b = max |d_j| over block b = 256 consecutive scales
 *     code_j = E4M3( fl32( fl32(d_j / c1_b) * 448 ) )  (+-0 when c1_b = 0)
 *     M'_j = fl32( fl32( fl32(E4M3^-1(code_j) * c1_b) / 448 ) + mean )
 * E4M3: 1 sign, 4 exponent, 3 mantissa bits, bias 7, no infinities, largest value 448, subnormals
 * m * 2^-9; round to nearest, ties to the even code.  Storage: 8 bits per scale + 32 bits per 256
 * scales + 32 bits, i.e. 0.5 + 1/64 + 1/4096 bytes per weight instead of 0.5 + 1/16.  The layer calls
 * take fp32 scales: expand before use, compress what a merge wrote.  |M' - M| <= c1_b / 28 (half a step
 * at the top of the range) and about |M - mean| / 16 in general, so the weights change: this is a lossy
 * storage option, not part of the bit-exact codec contract.
 *   absmax, absmax_out : n fp32 scales (device);  codes8 : n bytes;  c1 : ceil(n / 256) floats;
 *   mean : one float (device), written by compress, read by expand
 *   ws   : loqt_absmax_dq_workspace_bytes(n) bytes of scratch, 8-byte aligned (compress only)
 */
size_t loqt_absmax_dq_workspace_bytes(int64_t n);
loqt_status loqt_absmax_dq_compress(const float *absmax, int64_t n, uint8_t *codes8, float *c1, float *mean,
                                    void *ws, size_t ws_bytes, void *hip_stream);
loqt_status loqt_absmax_dq_expand(const uint8_t *codes8, const float *c1, const float *mean, int64_t n,
                                  float *absmax_out, void *hip_stream);

/*
 * loqt_absmax_dq_compress_static -- loqt_absmax_dq_compress for callers that cannot allocate device
 * memory or bring a workspace: code recorded under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments without `ws`, same kernels, same bits in codes8, c1 and mean.  The
 * partial sums of the mean go to a fixed 64 KB array inside the library's device image (one copy per GPU,
 * held until the process ends), which bounds the call at loqt_absmax_dq_static_max_n() = 2^25 scales
 * (2^31 weights); a larger n returns LOQT_STATIC_SCRATCH_TOO_SMALL and launches nothing.  The call
 * allocates and frees nothing and records no memset.  The array's device address is looked up on the
 * first call on each GPU (with the calling thread's current device, which must be the stream's).  All calls on
 * one GPU share the array: they must be ordered (one stream, or events); calls that overlap on one GPU race.
 */
int64_t loqt_absmax_dq_static_max_n(void);
loqt_status loqt_absmax_dq_compress_static(const float *absmax, int64_t n, uint8_t *codes8, float *c1,
                                           float *mean, void *hip_stream);

/*
 * loqt_adam_step -- the update between merges (Alg. 1 line 9: B_{t+1} = B_t - rho(G^B_t), rho = Adam;
 * the paper names the optimiser only, so this is the published algorithm with bias correction and no
 * weight decay):
 *     m = beta1 m + (1 - beta1) g ;  v = beta2 v + (1 - beta2) g^2
 *     B = B - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *   B    : bf16 rows x cols (pitch ld_B), updated in place (fp32 arithmetic, one rounding to bf16)
 *   grad : LOQT_F32 or LOQT_BF16, pitch ld_grad >= cols (what loqt_linear_bwd wrote into dB)
 *   m, v : fp32 moments, pitch ld_mv >= cols, updated in place (zero them before step 1, and again
 *          whenever B is re-initialised after a merge)
 *   step : 1, 2, ...;  lr >= 0, 0 <= beta < 1, eps >= 0
 * Works for either factor (B of the left form, Bp of the right form).
 */
loqt_status loqt_adam_step(loqt_bf16 *B, int64_t ld_B, int64_t rows, int64_t cols,
                           const void *grad, int grad_dtype, int64_t ld_grad,
                           float *m, float *v, int64_t ld_mv,
                           float lr, float beta1, float beta2, float eps, int64_t step,
                           void *hip_stream);

/*
 * loqt_merge_schedule -- the steps at which W is updated (sec. 2.5 last paragraph: intervals that
 * start at tau and grow by a factor psi; hyper-parameter appendix: tau = 100, psi = 1.2; the
 * ablation of update intervals caps them at 2500).  HOST function, no GPU work:
 *     gap_i = min(cap, floor(tau + psi^i)),   steps_out[i] = gap_0 + ... + gap_i,   i = 0..n-1
 * (the text also prints T_i = tau + psi^i for the steps themselves; growing intervals are the
 * reading that matches the ablation, whose intervals start at 100 and reach 2500).  steps_out: HOST array of n entries.
 */
loqt_status loqt_merge_schedule(double tau, double psi, int64_t cap, int n, int64_t *steps_out);

/*
 * loqt_prepare -- optional set-up for callers that record their first call into a HIP graph (or want the first
 * call of a serving loop to cost what the others do).  Every GEMM kernel of the library needs its LDS size raised
 * above the default once per process; without this call that happens at the first launch of each kernel
 * configuration, which is not allowed while a stream is being captured.  loqt_prepare does it for all of them on
 * the calling thread's current device and looks up the device address of the fixed scratch of
 * loqt_absmax_dq_compress_static.  It launches nothing and allocates nothing; it may be called more than once.
 * (The calls above keep no other state: implementation and tile choices are functions of the sizes.  The
 * test / tuning overrides of those choices and the per-kernel timers are declared in loqt_debug.h.)
 */
loqt_status loqt_prepare(void);

#ifdef __cplusplus
}
#endif
#endif /* LOQT_H */
