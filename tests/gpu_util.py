"""Helpers for the GPU parity tests: move seeded numpy inputs to the device in the ABI's
layouts and bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import binding as L


def rup(v, a):
    return (v + a - 1) // a * a


def bf16_dev(bits: np.ndarray, ld=None) -> torch.Tensor:
    """uint16 bit patterns (rows, cols) -> bf16 view of a (rows, ld) device buffer, cols kept."""
    rows, cols = bits.shape
    ld = ld or rup(cols, 8)
    buf = np.zeros((rows, ld), dtype=np.uint16)
    buf[:, :cols] = bits
    t = torch.from_numpy(buf.view(np.int16)).cuda().view(torch.bfloat16)
    return t[:, :cols]


def bf16_empty(rows, cols, ld=None, fill=None) -> torch.Tensor:
    ld = ld or rup(cols, 8)
    t = torch.empty((rows, ld), dtype=torch.bfloat16, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t[:, :cols]


def bf16_host(t: torch.Tensor) -> np.ndarray:
    """bf16 device view -> uint16 bit patterns."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def nf4_dev(codes: np.ndarray, absmax: np.ndarray, ld=None) -> L.NF4Tensor:
    rows, cols = codes.shape
    ld = ld or rup(cols, 64)
    packed, am = O.pack_nf4(codes, absmax, ld)
    return L.NF4Tensor(torch.from_numpy(packed).cuda(), torch.from_numpy(am).cuda(), rows, cols, ld)


def nf4_host(q: L.NF4Tensor):
    """device NF4 -> logical (codes, absmax) plus the raw padded arrays."""
    packed = q.codes.cpu().numpy()
    am = q.absmax.cpu().numpy()
    c, a = O.unpack_nf4(packed, am, q.cols)
    return c, a, packed, am


def workspace(op, T, out, inp, r) -> torch.Tensor:
    n = L.loqt_workspace_bytes(op, T, out, inp, r)
    return torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")


def max_err_over_rms(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.abs(got - ref).max() / np.sqrt(np.mean(ref ** 2)))


def bf16_output_report(got_bits: np.ndarray, ref: np.ndarray, comp_budget: float = 1.2e-2):
    """Element-wise check of a bf16 output against the oracle's float64 values, for tensors so large that the
    output format itself, not the computation, sets the largest error: a result in [2^k, 2^(k+1)) is stored to
    within half a step, 2^(k-8), i.e. up to 2^-8 of its own size, which at five standard deviations is 2e-2 of the
    RMS all by itself.  Every element must satisfy
        |got - ref| <= 2^-8 |ref| + comp_budget * RMS(ref)
    (final rounding + the error of the bf16-operand products: the weight is rounded to bf16 once, a relative error of
    about 1.6e-3 rms per term, which over a contraction gives 1.6e-3 RMS per output and six times that as the
    largest of 10^8), which is tighter than 2e-2 * RMS for every element below 2 RMS, 95 % of them, and admits beyond
    that only what the format needs.  Returns (max |err| / RMS, the same figure for
    the oracle's own values rounded to bf16: the floor of the format, number of elements over 2e-2 * RMS)."""
    got = O.bf16_to_f64(got_bits)
    rms = float(np.sqrt(np.mean(ref ** 2)))
    err = np.abs(got - ref)
    bound = np.abs(ref) * 2.0 ** -8 + comp_budget * rms
    worst = int(np.argmax(err - bound))
    assert err.flat[worst] <= bound.flat[worst], (
        f"element {np.unravel_index(worst, err.shape)}: |err| {err.flat[worst]:.4e} > bound {bound.flat[worst]:.4e} "
        f"(ref {ref.flat[worst]:.6g}, got {got.flat[worst]:.6g}, rms {rms:.4e})")
    floor = np.abs(O.bf16_to_f64(O.f32_to_bf16_rne(ref.astype(np.float32))) - ref).max() / rms
    return float(err.max() / rms), float(floor), int(np.count_nonzero(err > 2e-2 * rms))


def weff_check(weff_bits: np.ndarray, Wq, Pq, B_bits: np.ndarray, s: float):
    """W_eff = bf16( fl32(deq(W_q)) + s * (bf16-operand, fp32-accumulated product deq(P_q) B) ) against the float64
    merge, element by element: half a bf16 step of the result (at most 2^-8 of it) plus the worst case of the
    product (every dequantised P entry rounded to bf16: 2^-8 relative; fp32 accumulation over r terms) and of the
    fp32 roundings of deq(W) and of the sum."""
    Wm = O.loqt_merge_f64(Wq, Pq, B_bits, s)
    got = O.bf16_to_f64(weff_bits)
    Pd = np.abs(O.nf4_dequantize_f64(*Pq))
    r = Pd.shape[1]
    E = abs(s) * (Pd @ np.abs(O.bf16_to_f64(B_bits))) * (2.0 ** -8 + (r + 2) * 2.0 ** -24) + np.abs(Wm) * 2.0 ** -22
    bound = (np.abs(Wm) + E) * 2.0 ** -8 + E
    err = np.abs(got - Wm)
    worst = int(np.argmax(err - bound))
    assert err.flat[worst] <= bound.flat[worst], (
        f"W_eff element {np.unravel_index(worst, err.shape)}: |err| {err.flat[worst]:.4e} > bound "
        f"{bound.flat[worst]:.4e} (ref {Wm.flat[worst]:.6g}, got {got.flat[worst]:.6g})")
    return float(err.max() / np.sqrt(np.mean(Wm ** 2)))
