"""The whole method end to end on a synthetic regression task (Alg. 1 + Alg. 2): initialise from the gradient's
top singular vectors with error compensation, train B with Adam, merge at scheduled steps, re-initialise.

One driver, two back ends: the oracle (fp64, CPU) and the HIP library.  The task itself (inputs, teacher,
loss, the SVD that picks P) is harness code shared by both; every step of the method runs in the back end.
The CPU test checks that the oracle's loop learns; the GPU test checks that the library follows the same
loss curve."""
import numpy as np
import pytest

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

OUT, INP, R, T, S, LR = 256, 384, 32, 512, 0.5, 2e-3
STEPS = 45


def _task():
    rng = synth.rng_for(0, "loop")
    W0 = synth.normal_f32(rng, (OUT, INP), 0.02)
    D = (rng.standard_normal((OUT, 8)) @ rng.standard_normal((8, INP))) * 0.004
    return W0, W0.astype(np.float64) + D


def _batch(t):
    return synth.normal_bf16(synth.rng_for(0, "loop-x", str(t)), (T, INP), 1.0)


def _top_r(G):
    U, _, _ = np.linalg.svd(G, full_matrices=False)  # Alg. 2 lines 2-3 (the caller's job in this library)
    return np.ascontiguousarray(U[:, :R]).astype(np.float32)


class OracleBackend:
    def init(self, W, P):
        self.c, self.a, B, _ = O.loqt_init_compensate(W, P, S, 5)
        self.Pq = O.nf4_quantize(P)
        self.Bb = O.f32_to_bf16_rne(B.astype(np.float32))
        self.m, self.v, self.k = np.zeros_like(B), np.zeros_like(B), 0

    def fwd(self, x):
        return O.loqt_linear_fwd(x, (self.c, self.a), self.Pq, self.Bb, S)

    def bwd_and_step(self, dy, x):
        _, dB = O.loqt_linear_bwd(dy, x, (self.c, self.a), self.Pq, self.Bb, S)
        self.k += 1
        Bn, self.m, self.v = O.adam_step(O.bf16_to_f64(self.Bb), dB, self.m, self.v, LR, 0.9, 0.999, 1e-8, self.k)
        self.Bb = O.f32_to_bf16_rne(Bn.astype(np.float32))  # B lives in 16 bits

    def merge_dense(self):
        return O.loqt_merge_dense_f32((self.c, self.a), self.Pq, self.Bb, S)

    def schedule(self, n):
        return O.merge_schedule(14, 1.0, 2500, n)


class DeviceBackend:
    def __init__(self):
        import torch
        from tests import gpu_util as G
        from paper_2405_16528_amd import binding as L
        self.torch, self.G, self.L = torch, G, L
        self.ws = {op: G.workspace(op, T, OUT, INP, R) for op in (L.OP_FWD, L.OP_BWD, L.OP_MERGE, L.OP_INIT)}
        self.B = G.bf16_empty(R, INP)
        self.dB = torch.empty((R, INP), dtype=torch.float32, device="cuda")
        self.m = torch.zeros((R, INP), dtype=torch.float32, device="cuda")
        self.v = torch.zeros_like(self.m)
        self.y = G.bf16_empty(T, OUT)
        self.Wq = L.NF4Tensor.empty(OUT, INP)

    def init(self, W, P):
        torch, L = self.torch, self.L
        Wd, Pd = torch.from_numpy(W).cuda(), torch.from_numpy(P).cuda()
        L.loqt_init_compensate(Wd, Pd, S, 5, self.B, out=self.Wq, ws=self.ws[L.OP_INIT])
        self.Pq = L.nf4_quantize(Pd)
        self.m.zero_()
        self.v.zero_()
        self.k = 0

    def fwd(self, x):
        L, G = self.L, self.G
        L.loqt_linear_fwd(G.bf16_dev(x), self.Wq, self.Pq, self.B, S, self.y, self.ws[L.OP_FWD])
        return O.bf16_to_f64(G.bf16_host(self.y))

    def bwd_and_step(self, dy, x):
        L, G = self.L, self.G
        L.loqt_linear_bwd(G.bf16_dev(dy), G.bf16_dev(x), self.Wq, self.Pq, self.B, S, None, self.dB, False,
                          self.ws[L.OP_BWD])
        self.k += 1
        L.loqt_adam_step(self.B, self.dB, self.m, self.v, LR, self.k)

    def merge_dense(self):
        torch, L = self.torch, self.L
        Wd = torch.empty((OUT, INP), dtype=torch.float32, device="cuda")
        L.loqt_merge_dense(self.Wq, self.Pq, self.B, S, Wd, ws=self.ws[L.OP_MERGE])
        return Wd.cpu().numpy()

    def schedule(self, n):
        return self.L.loqt_merge_schedule(n, tau=14.0, psi=1.0, cap=2500)


def run_loop(be):
    W0, Wstar = _task()
    merges = set(be.schedule(3))
    assert merges == {15, 30, 45}

    def grad_w(y, xd):  # dL/dW of the harness loss 0.5 * mean over tokens of |y - y*|^2, bf16 dy as the layer sees it
        dy = O.f32_to_bf16_rne(((y - xd @ Wstar.T) / T).astype(np.float32))
        return dy, O.bf16_to_f64(dy).T @ xd

    x = _batch(0)
    xd = O.bf16_to_f64(x)
    _, G0 = grad_w(xd @ W0.astype(np.float64).T, xd)       # Alg. 1 line 1: the gradient at the starting weight
    be.init(W0, _top_r(G0))
    losses = []
    for t in range(1, STEPS + 1):
        x = _batch(t)
        xd = O.bf16_to_f64(x)
        y = be.fwd(x)
        losses.append(0.5 * float(np.mean((y - xd @ Wstar.T) ** 2)))
        dy, Gw = grad_w(y, xd)
        be.bwd_and_step(dy, x)                              # Alg. 1 line 9
        if t in merges and t < STEPS:
            W = be.merge_dense()                            # Alg. 1 line 5
            be.init(W, _top_r(Gw))                          # Alg. 1 lines 6-7, Alg. 2
    return losses


_oracle_losses = None


def oracle_losses():
    global _oracle_losses
    if _oracle_losses is None:
        _oracle_losses = run_loop(OracleBackend())
    return _oracle_losses


def test_oracle_loop_learns_and_survives_merges():
    L = oracle_losses()
    assert L[-1] < 0.5 * L[0]
    # the loss keeps falling from one merge interval to the next, and a merge (steps 15, 30) does not set it back
    assert np.mean(L[30:45]) < np.mean(L[15:30]) < np.mean(L[0:15])
    assert L[15] < L[13] * 1.02 and L[30] < L[28] * 1.02


@pytest.mark.gpu
def test_device_loop_follows_the_oracle_loss_curve():
    Ld = run_loop(DeviceBackend())
    Lo = oracle_losses()
    rel = max(abs(a - b) / b for a, b in zip(Ld, Lo))
    print("loss device", ["%.4e" % v for v in Ld[::5]], "oracle", ["%.4e" % v for v in Lo[::5]], f"max rel diff {rel:.2e}")
    assert rel <= 1e-2
    assert Ld[-1] < 0.5 * Ld[0]
