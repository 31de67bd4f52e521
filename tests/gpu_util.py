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
