"""CPU oracle for the LoQT quantized low-rank linear layer (arxiv 2405.16528).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check
and the cpu_baseline leg of the benchmark may import it.  It shares no code,
table generator or helper with the HIP library; it never calls it.

Everything is the plain definition, evaluated in numpy float64 in one pass:

  codec  (paper sec. 5.1 "Neural Network Quantization and NF4"):
      M_beta = max_{w in beta} |w_32|          blocks beta of 64 consecutive weights
      code   = argmin_i | w / M_beta - q_i |   q_0..q_15 the NF4 levels
      deq    = M_beta * q_code
  layer  (paper sec. 2.2 "Equivalence of Gradient Updates", forward y = xW + xPB,
          G^B = (xP)^T dL/dy = P^T G^W; sec. 2.4 "Quantized Training": W and P are
          kept in NF4 and dequantised before the products; Alg. 1 line 5 scale s):
      W_eff = deq(W_q) + s * deq(P_q) @ B      (out x in), PyTorch layout
      y  = x @ W_eff^T ;  dx = dy @ W_eff ;  dB = s * deq(P_q)^T @ dy^T @ x
  merge  (Alg. 1 line 5, sec. 2.4, sec. 2.5 first paragraph):
      W_new = deq(W_q) + s * deq(P_q) @ B ;  (codes', absmax') = q_NF4(W_new)

  right  (sec. 2.2 first paragraph: the gradient is projected from the left, P^T G, when the weight
          has no more rows than columns, and from the right, G Q, otherwise): the projection sits on the input side,
      W_eff = deq(W_q) + s * Bp @ deq(Q_q)^T   Q in x r fixed (NF4), Bp out x r trainable;
      y = x @ W_eff^T ; dx = dy @ W_eff ; dBp = s * dy^T @ (x @ deq(Q_q))
  nq     (the paper's LoQT-nq, "no quantization": the same layer with W and P kept in 16 bits):
      W_eff = W + s * P @ B with W, P bf16;  merge: W <- bf16(W + s P B)
  init   (Alg. 2 lines 5-11, sec. 2.5 "Compensating for Quantization Errors"): with P
          fixed, alternate  Q_c = q_NF4(W_hat) ;  B = P^+ (W - Q_c) / s ;
          W_hat = W - s P B,  so that Q_c + s P B approximates W.

  step   (Alg. 1 line 9: B_{t+1} = B_t - rho(G^B_t), rho = Adam; sec. 2.5 last paragraph and
          the hyper-parameter appendix: W is updated at steps T_i whose gaps are tau + psi^i).

  dq     (sec. 2.4 says that the quantisation state is itself quantised again, as in the NF4 paper): the fp32
          block scales of an NF4 matrix are themselves stored in 8 bits.  PARITY UNPINNED BY THE PAPER:
          it gives no format.  Reading taken (the cited method's own description: the scales, being
          positive, have their mean subtracted and are quantised to 8-bit floats in blocks of 256 with one
          fp32 constant per block): d = fl32(M - mean); c1 = max |d| over 256 consecutive scales;
          code = E4M3( fl32( fl32(d / c1) * 448 ) ), E4M3 the 8-bit float with 4 exponent and 3 mantissa
          bits, bias 7, no infinities, largest value 448, round to nearest even, saturating;
          M' = fl32( fl32( fl32(E4M3^-1(code) * c1) / 448 ) + mean ).

Layout convention used by every function here ("logical" form, no padding):
  codes  : uint8 array (rows, cols), one code 0..15 per element
  absmax : float32 array (rows, ceil(cols/64)); blocks run along a row and never
           straddle rows; a short last block covers the elements present.
pack_nf4 / unpack_nf4 convert to and from the byte layout of the C ABI.

Readings of points the paper leaves open (each one is also listed in the design
notes of the repository):
  * orientation: PyTorch layout, W out x in, P out x r, B r x in, x T x in;
  * s multiplies the low-rank term in forward, backward and merge alike;
  * argmin is taken in exact real arithmetic, ties go to the lower index;
  * an all-zero block stores absmax 0 and code 7 (the level 0.0);
  * the quantiser's input is fp32 (M_beta is defined on 32-bit values), so the
    merge rounds W_new to fp32 once (from the fp64 sum) before quantising;
  * the 16 level values are not printed in the paper (it defers to QLoRA); the
    table below is the published NF4 data type, typed in by hand, and pinned in
    the tests against its construction from normal quantiles.
  * compensation loop (Alg. 2): the algorithm box prints B <- P^+(W_hat - Q_c), the
    text B = P^+(Q - W); only B = P^+(W - Q_c) minimises the stated objective
    |Q + P B - W| (a least-squares problem in B), and it is the box's own first
    iteration (W_hat = W), so that is what every iteration computes here.  P is the
    unquantised projection of Alg. 2 line 3 (the box uses P, not P_q, in the loop);
    s divides B so that the layer's W_q + s P B is what approximates W.
  * Adam (the paper only names it): the published algorithm with bias correction,
    m = b1 m + (1-b1) g, v = b2 v + (1-b2) g^2, B -= lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps);
    no weight decay; pinned against torch.optim.Adam.
  * update schedule: the text gives T_i = tau + psi^i once as the steps themselves and once
    (appendix, and the ablation, whose intervals start at 100 and grow up to 2500) as growing intervals; intervals
    are the reading taken: gap_i = min(cap, floor(tau + psi^i)), T_i = gap_0 + ... + gap_i.
Parity status: every function below is pinned by tests/test_oracle_*.py against
closed forms, brute force in rational arithmetic, library routines and
invariants.  One group is PARITY UNPINNED by the paper: absmax_dq_compress /
absmax_dq_expand / e4m3_* (the paper gives no format for the re-quantised scales; the
arithmetic of the reading stated above is pinned, the reading itself cannot be).
"""
from __future__ import annotations

import numpy as np

BLOCK = 64

# The NF4 levels (QLoRA's "4-bit NormalFloat"), ascending; index = code.
NF4_LEVELS = np.array(
    [
        -1.0,
        -0.6961928009986877,
        -0.5250730514526367,
        -0.39491748809814453,
        -0.28444138169288635,
        -0.18477343022823334,
        -0.09105003625154495,
        0.0,
        0.07958029955625534,
        0.16093020141124725,
        0.24611230194568634,
        0.33791524171829224,
        0.44070982933044434,
        0.5626170039176941,
        0.7229568362236023,
        1.0,
    ],
    dtype=np.float64,
)


# ----------------------------------------------------------------------------
# bf16 <-> float helpers (bf16 travels as raw uint16 bit patterns)
# ----------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bfloat16 bit patterns, as float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round finite float32 to bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    return ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)


# ----------------------------------------------------------------------------
# codec (sec. 5.1)
# ----------------------------------------------------------------------------
def nf4_quantize(w: np.ndarray):
    """q_NF4 of a float32 matrix, blocks of 64 along each row (sec. 5.1).

    Returns (codes uint8 (rows, cols), absmax float32 (rows, ceil(cols/64))).
    code = #{ j in 0..14 : 2 w > (q_j + q_{j+1}) * M_beta }: this is the argmin of
    |w/M_beta - q_i| in real arithmetic (w/M > midpoint  <=>  2w > (q_j+q_{j+1}) M
    for M > 0) with ties resolved to the lower index.  q_j + q_{j+1} has at most 29
    significant bits and M_beta 24, so the product is exact in float64 and no
    rounding takes place anywhere in the decision.
    """
    w = np.asarray(w)
    assert w.dtype == np.float32 and w.ndim == 2
    rows, cols = w.shape
    nblk = -(-cols // BLOCK)
    wp = np.zeros((rows, nblk * BLOCK), dtype=np.float32)
    wp[:, :cols] = w
    wp = wp.reshape(rows, nblk, BLOCK)
    absmax = np.max(np.abs(wp), axis=2)  # exact, float32
    mid2 = NF4_LEVELS[:-1] + NF4_LEVELS[1:]  # 15 doubled midpoints, exact in fp64
    w2 = 2.0 * wp.astype(np.float64)
    m64 = absmax.astype(np.float64)
    codes = np.zeros(wp.shape, dtype=np.uint8)
    for j in range(15):
        codes += w2 > (mid2[j] * m64)[:, :, None]
    codes[absmax == 0.0] = 7  # all-zero block: level 0.0
    codes = codes.reshape(rows, nblk * BLOCK)[:, :cols]
    return np.ascontiguousarray(codes), absmax


def nf4_dequantize_f64(codes: np.ndarray, absmax: np.ndarray) -> np.ndarray:
    """M_beta * q_code as the exact real product (float64; 24 x 24 bits fit)."""
    rows, cols = codes.shape
    scale = np.repeat(absmax.astype(np.float64), BLOCK, axis=1)[:, :cols]
    return NF4_LEVELS[codes] * scale


def nf4_dequantize_f32(codes: np.ndarray, absmax: np.ndarray) -> np.ndarray:
    """fp32 output of the stand-alone decoder: the exact product rounded once."""
    return nf4_dequantize_f64(codes, absmax).astype(np.float32)


def nf4_dequantize_bf16(codes: np.ndarray, absmax: np.ndarray) -> np.ndarray:
    """bf16 output (bit patterns): the fp32 output rounded to nearest even."""
    return f32_to_bf16_rne(nf4_dequantize_f32(codes, absmax))


def pack_nf4(codes: np.ndarray, absmax: np.ndarray, ld: int):
    """Logical form -> C-ABI byte layout with row pitch `ld` nibbles (ld % 64 == 0).

    Row i starts at byte i*ld/2; element j sits in byte j//2, even j in the HIGH
    nibble; positions cols..ld-1 hold code 7; absmax has ld/64 entries per row,
    0.0 for blocks that lie entirely in the padding.
    """
    rows, cols = codes.shape
    assert ld % BLOCK == 0 and ld >= cols
    full = np.full((rows, ld), 7, dtype=np.uint8)
    full[:, :cols] = codes
    packed = (full[:, 0::2] << 4) | full[:, 1::2]
    am = np.zeros((rows, ld // BLOCK), dtype=np.float32)
    am[:, : absmax.shape[1]] = absmax
    return np.ascontiguousarray(packed.astype(np.uint8)), am


def unpack_nf4(packed: np.ndarray, absmax: np.ndarray, cols: int):
    """C-ABI byte layout -> logical form (drops the padding)."""
    rows = packed.shape[0]
    full = np.empty((rows, packed.shape[1] * 2), dtype=np.uint8)
    full[:, 0::2] = packed >> 4
    full[:, 1::2] = packed & 0xF
    nblk = -(-cols // BLOCK)
    return np.ascontiguousarray(full[:, :cols]), np.ascontiguousarray(absmax[:, :nblk])


# ----------------------------------------------------------------------------
# layer (sec. 2.2, 2.4; Alg. 1)
# ----------------------------------------------------------------------------
def loqt_linear_fwd(x, Wq, Pq, B, s):
    """y = x deq(W_q)^T + s (x B^T) deq(P_q)^T   in float64.

    x: (T, in) bf16 bits; Wq = (codes, absmax) of (out, in); Pq of (out, r);
    B: (r, in) bf16 bits.  Returns float64 (T, out).
    """
    xd = bf16_to_f64(x)
    Bd = bf16_to_f64(B)
    Wd = nf4_dequantize_f64(*Wq)
    Pd = nf4_dequantize_f64(*Pq)
    U = xd @ Bd.T
    return xd @ Wd.T + s * (U @ Pd.T)


def loqt_linear_bwd(dy, x, Wq, Pq, B, s):
    """dx = dy deq(W_q) + s (dy deq(P_q)) B ;  dB = s deq(P_q)^T dy^T x   (float64).

    The weight gradient goes to B alone (sec. 2.2: G^B = P^T G^W).
    """
    dyd = bf16_to_f64(dy)
    xd = bf16_to_f64(x)
    Bd = bf16_to_f64(B)
    Wd = nf4_dequantize_f64(*Wq)
    Pd = nf4_dequantize_f64(*Pq)
    Z = dyd @ Pd
    dx = dyd @ Wd + s * (Z @ Bd)
    dB = s * (Z.T @ xd)
    return dx, dB


def loqt_merge_f64(Wq, Pq, B, s):
    """The unquantised merged weight deq(W_q) + s deq(P_q) B in float64 (Alg. 1 l.5)."""
    return nf4_dequantize_f64(*Wq) + s * (nf4_dequantize_f64(*Pq) @ bf16_to_f64(B))


def loqt_merge_requant(Wq, Pq, B, s):
    """W_q <- q_NF4( fp32( deq(W_q) + s deq(P_q) B ) ).  Returns (codes, absmax)."""
    return nf4_quantize(loqt_merge_f64(Wq, Pq, B, s).astype(np.float32))


# ----------------------------------------------------------------------------
# right-side projection variant (sec. 2.2: one-sided projection G Q when m > n)
# ----------------------------------------------------------------------------
def loqt_right_weff_f64(Wq, Qq, Bp, s):
    """deq(W_q) + s Bp deq(Q_q)^T in float64.  Wq of (out, in), Qq of (in, r), Bp (out, r) bf16 bits."""
    return nf4_dequantize_f64(*Wq) + s * (bf16_to_f64(Bp) @ nf4_dequantize_f64(*Qq).T)


def loqt_linear_fwd_right(x, Wq, Qq, Bp, s):
    """y = x deq(W_q)^T + s (x deq(Q_q)) Bp^T   (float64); x (T, in) bf16 bits."""
    xd = bf16_to_f64(x)
    V = xd @ nf4_dequantize_f64(*Qq)
    return xd @ nf4_dequantize_f64(*Wq).T + s * (V @ bf16_to_f64(Bp).T)


def loqt_linear_bwd_right(dy, x, Wq, Qq, Bp, s):
    """dx = dy deq(W_q) + s (dy Bp) deq(Q_q)^T ;  dBp = s dy^T (x deq(Q_q))   (float64).

    The weight gradient goes to Bp alone: G^Bp = G^W Q, the right-sided projection of sec. 2.2.
    """
    dyd = bf16_to_f64(dy)
    xd = bf16_to_f64(x)
    Qd = nf4_dequantize_f64(*Qq)
    dx = dyd @ nf4_dequantize_f64(*Wq) + s * ((dyd @ bf16_to_f64(Bp)) @ Qd.T)
    dBp = s * (dyd.T @ (xd @ Qd))
    return dx, dBp


def loqt_merge_requant_right(Wq, Qq, Bp, s):
    """W_q <- q_NF4( fp32( deq(W_q) + s Bp deq(Q_q)^T ) )  (Alg. 1 line 5 for the right-side form)."""
    return nf4_quantize(loqt_right_weff_f64(Wq, Qq, Bp, s).astype(np.float32))


# ----------------------------------------------------------------------------
# LoQT-nq: the layer without quantisation (W and P in bf16)
# ----------------------------------------------------------------------------
def loqt_linear_fwd_nq(x, W, P, B, s):
    """y = x W^T + s (x B^T) P^T  (float64); W (out, in), P (out, r), B (r, in), x (T, in): bf16 bits."""
    xd = bf16_to_f64(x)
    return xd @ bf16_to_f64(W).T + s * ((xd @ bf16_to_f64(B).T) @ bf16_to_f64(P).T)


def loqt_linear_bwd_nq(dy, x, W, P, B, s):
    """dx = dy W + s (dy P) B ;  dB = s P^T dy^T x  (float64)."""
    dyd, xd = bf16_to_f64(dy), bf16_to_f64(x)
    Z = dyd @ bf16_to_f64(P)
    return dyd @ bf16_to_f64(W) + s * (Z @ bf16_to_f64(B)), s * (Z.T @ xd)


def loqt_merge_nq_f64(W, P, B, s):
    """W + s P B in float64 (Alg. 1 line 5 without quantisation)."""
    return bf16_to_f64(W) + s * (bf16_to_f64(P) @ bf16_to_f64(B))


def loqt_merge_nq(W, P, B, s):
    """W <- bf16(fp32(W + s P B)), round to nearest even; returns bf16 bits."""
    return f32_to_bf16_rne(loqt_merge_nq_f64(W, P, B, s).astype(np.float32))


# ----------------------------------------------------------------------------
# error-compensated initialisation of B (Alg. 2 lines 5-11, sec. 2.5)
# ----------------------------------------------------------------------------
def loqt_init_compensate(W, P, s, iters, B0=None):
    """The compensation loop of Alg. 2 with P fixed.

    W: (out, in) float32, the weight to be represented; P: (out, r) float32 (Alg. 2
    line 3: the first r left singular vectors of the gradient); s: the scale of the
    low-rank term; iters >= 1 compensation steps; B0: optional (r, in) float64 start
    (Alg. 2 line 5 starts from B = 0).  Each step:
        Q_c   = q_NF4(fp32(W_hat))               W_hat = W - s P B  (= W when B = 0)
        B     = P^+ (W - deq(Q_c)) / s           least squares: argmin_B |Q_c + s P B - W|_F
    Returns (codes, absmax) of the last Q_c, the matching B (float64) and the list of
    objectives |deq(Q_c) + s P B - W|_F after each step.  P^+ is numpy's Moore-Penrose
    pseudo-inverse in float64.
    """
    W = np.asarray(W)
    P = np.asarray(P)
    assert W.dtype == np.float32 and P.dtype == np.float32 and iters >= 1
    Wd = W.astype(np.float64)
    Pd = P.astype(np.float64)
    Pinv = np.linalg.pinv(Pd)
    B = np.zeros((P.shape[1], W.shape[1])) if B0 is None else np.asarray(B0, dtype=np.float64)
    history = []
    codes = absmax = None
    for _ in range(iters):
        W_hat = Wd - s * (Pd @ B)
        codes, absmax = nf4_quantize(W_hat.astype(np.float32))
        Q = nf4_dequantize_f64(codes, absmax)
        B = (Pinv @ (Wd - Q)) / s
        history.append(float(np.linalg.norm(Q + s * (Pd @ B) - Wd)))
    return codes, absmax, B, history


# ----------------------------------------------------------------------------
# the step between merges (Alg. 1 line 9) and the merge schedule (sec. 2.5)
# ----------------------------------------------------------------------------
def adam_step(B, g, m, v, lr, beta1, beta2, eps, t):
    """One Adam update of B (float64 arrays; t = 1, 2, ... is the step count).  Returns (B, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return B - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def merge_schedule(tau, psi, cap, n):
    """The first n steps T_i at which W is updated: gaps min(cap, floor(tau + psi**i)), accumulated."""
    steps, t = [], 0
    for i in range(n):
        t += min(int(cap), int(np.floor(tau + psi ** i)))
        steps.append(t)
    return steps


def loqt_merge_dense_f32(Wq, Pq, B, s):
    """Alg. 1 line 5 as printed: W <- W_Q + s P_Q B, kept in full precision (fp32 of the fp64 sum);
    the input of Alg. 2's Initialize."""
    return loqt_merge_f64(Wq, Pq, B, s).astype(np.float32)


# ---------------------------------------------------------------------------------------------
# double quantisation of the block scales (sec. 2.4; format: see the header, parity unpinned)
# ---------------------------------------------------------------------------------------------
E4M3_MAX = 448.0
DQ_BLOCK = 256


def e4m3_decode(code: np.ndarray) -> np.ndarray:
    """8-bit float, 1 sign / 4 exponent / 3 mantissa bits, bias 7, no infinities -> float32 (exact).
    Exponent field 0 holds the subnormals m * 2^-9; code 0x7f / 0xff is the NaN of the format."""
    code = np.asarray(code, dtype=np.uint8).astype(np.int64)
    sign = np.where(code & 0x80, -1.0, 1.0)
    e = (code >> 3) & 0xF
    m = code & 0x7
    mag = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    out = sign * mag
    out = np.where((e == 15) & (m == 7), np.nan, out)
    return out.astype(np.float32)


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest representable E4M3 value, ties to the even mantissa, saturating at +-448.
    Plain definition: among the 253 finite codes pick the one whose value is nearest; on a tie the code
    with the even mantissa bit pattern; the sign bit follows the sign of x (so -0.0 -> 0x80)."""
    x = np.asarray(x, dtype=np.float32)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    pos = codes[codes < 0x80]
    vals = e4m3_decode(pos).astype(np.float64)  # ascending with the code
    a = np.minimum(np.abs(x.astype(np.float64)), E4M3_MAX)
    hi = np.searchsorted(vals, a, side="left")          # first value >= a
    hi = np.minimum(hi, len(vals) - 1)
    lo = np.maximum(hi - 1, 0)
    dlo, dhi = a - vals[lo], vals[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((pos[hi] & 1) == 0))
    mag = np.where(pick_hi, pos[hi], pos[lo]).astype(np.uint8)
    mag = np.where(a == vals[hi], pos[hi], mag).astype(np.uint8)
    sign = (np.signbit(x)).astype(np.uint8) << 7
    return (mag | sign).astype(np.uint8)


def absmax_dq_compress(absmax: np.ndarray, mean=None):
    """Block scales (any shape, taken flat, fp32) -> (codes uint8 [n], c1 float32 [ceil(n/256)], mean float32).
    `mean` may be supplied (the format stores it, so any fp32 next to the true mean is a valid choice);
    by default it is the fp64 mean rounded to fp32."""
    a = np.asarray(absmax, dtype=np.float32).reshape(-1)
    n = a.size
    if mean is None:
        mean = np.float32(a.astype(np.float64).sum() / max(n, 1))
    mean = np.float32(mean)
    d = (a - mean).astype(np.float32)
    nb = (n + DQ_BLOCK - 1) // DQ_BLOCK
    c1 = np.zeros(nb, dtype=np.float32)
    codes = np.zeros(n, dtype=np.uint8)
    for b in range(nb):
        blk = d[b * DQ_BLOCK:(b + 1) * DQ_BLOCK]
        c = np.float32(np.max(np.abs(blk)))
        c1[b] = c
        if c > 0:
            t = (blk / c).astype(np.float32)
            u = (t * np.float32(E4M3_MAX)).astype(np.float32)
            codes[b * DQ_BLOCK:b * DQ_BLOCK + blk.size] = e4m3_encode(u)
        else:
            codes[b * DQ_BLOCK:b * DQ_BLOCK + blk.size] = e4m3_encode(blk)  # +-0
    return codes, c1, mean


def absmax_dq_expand(codes: np.ndarray, c1: np.ndarray, mean) -> np.ndarray:
    codes = np.asarray(codes, dtype=np.uint8).reshape(-1)
    v = e4m3_decode(codes)
    cc = np.repeat(np.asarray(c1, dtype=np.float32), DQ_BLOCK)[:codes.size]
    t = (v * cc).astype(np.float32)
    t = (t / np.float32(E4M3_MAX)).astype(np.float32)
    return (t + np.float32(mean)).astype(np.float32)
