"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times
(path option AUTO): outputs the oracle can compute one by one are sampled -- token rows of y
and dx, (rank block x column block) patches of dB, rows of the merged weight."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth
from tests.test_gpu_layer import TOL, _merge_policy_check

pytestmark = pytest.mark.gpu

CASES = [
    ("60m_layer", "layer"),
    ("130m_block", "q"), ("130m_block", "gate"), ("130m_block", "down"),
    ("1b_block", "o"), ("1b_block", "up"), ("1b_block", "down"),   # 5461: odd sizes, K and N tails
    ("7b_block", "q"), ("7b_block", "gate"), ("7b_block", "down"),
    ("13b_block", "v"), ("13b_block", "down"),
]


def _blocks(rng, n, k):
    """k distinct 64-blocks of range(n), the last (possibly short) one always included."""
    nb = -(-n // 64)
    pick = set([nb - 1]) | set(rng.choice(nb, size=min(k, nb), replace=False).tolist())
    return sorted(pick)


def _cols(blocks, n):
    return np.concatenate([np.arange(64 * b, min(64 * b + 64, n)) for b in blocks])


@pytest.mark.parametrize("workload,layer", CASES)
def test_full_size_sampled(workload, layer):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    L.set_path(L.PATH_AUTO)
    wl = synth.WORKLOADS[workload]
    (_, out, inp), = [p for p in wl.projections if p[0] == layer]
    T, r, s = wl.T, wl.r, 0.5
    lay = synth.make_layer(workload, layer, out, inp, r, T, seed=0)
    Wq, Pq = O.nf4_quantize(lay.W), O.nf4_quantize(lay.P)
    rng = synth.rng_for(0, "fullsize-samples", workload, layer)

    x, dy, B = G.bf16_dev(lay.x), G.bf16_dev(lay.dy), G.bf16_dev(lay.B)
    Wd, Pd = G.nf4_dev(*Wq), G.nf4_dev(*Pq)
    y = G.bf16_empty(T, out, fill=float("nan"))
    dx = G.bf16_empty(T, inp, fill=float("nan"))
    dB = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
    ws = L.workspace(L.OP_BWD, T, out, inp, r)
    ws_f = L.workspace(L.OP_FWD, T, out, inp, r)
    L.loqt_linear_fwd(x, Wd, Pd, B, s, y, ws_f)
    L.loqt_linear_bwd(dy, x, Wd, Pd, B, s, dx, dB, False, ws)
    merged = L.loqt_merge_requant(Wd, Pd, B, s, out=L.NF4Tensor.empty(out, inp))
    torch.cuda.synchronize()
    assert not torch.isnan(y.float()).any() and not torch.isnan(dx.float()).any() and not torch.isnan(dB).any()

    # y and dx on sampled tokens (always the first and the last one)
    I = np.unique(np.concatenate([[0, T - 1], rng.choice(T, size=min(T, 128), replace=False)]))
    y_ref = O.loqt_linear_fwd(lay.x[I], Wq, Pq, lay.B, s)
    dx_ref, _ = O.loqt_linear_bwd(lay.dy[I], lay.x[I], Wq, Pq, lay.B, s)
    Id = torch.from_numpy(I).cuda()
    ey = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(y[Id])), y_ref)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dx[Id])), dx_ref)

    # dB on sampled (rank block, column block) patches: dB[R, J] = s deq(P)[:, R]^T dy^T x[:, J]
    Rb, Jb = _blocks(rng, r, 2), _blocks(rng, inp, 3)
    R, J = _cols(Rb, r), _cols(Jb, inp)
    _, dB_ref = O.loqt_linear_bwd(lay.dy, np.ascontiguousarray(lay.x[:, J]),
                                  (np.ascontiguousarray(Wq[0][:, J]), np.ascontiguousarray(Wq[1][:, Jb])),
                                  (np.ascontiguousarray(Pq[0][:, R]), np.ascontiguousarray(Pq[1][:, Rb])),
                                  np.ascontiguousarray(lay.B[R][:, J]), s)
    got = dB[torch.from_numpy(R).cuda()][:, torch.from_numpy(J).cuda()].cpu().numpy().astype(np.float64)
    eb = G.max_err_over_rms(got, dB_ref)
    print(f"{workload}/{layer} T={T} {out}x{inp} r={r}: err/rms y {ey:.2e} dx {ex:.2e} dB {eb:.2e}")
    assert ey <= TOL and ex <= TOL and eb <= TOL

    # the calls bench.py times by default (the bf16 weight kept between the passes, the merge of the block as
    # one batched call) run the same kernels on the same operands as the calls checked above: identical bits
    if workload == "7b_block":
        w_eff = G.bf16_empty(out, inp, fill=float("nan"))
        y2 = G.bf16_empty(T, out, fill=float("nan"))
        dx2 = G.bf16_empty(T, inp, fill=float("nan"))
        dB2 = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
        L.loqt_linear_fwd_save(x, Wd, Pd, B, s, y2, w_eff, ws_f)
        L.loqt_linear_bwd_saved(dy, x, Pd, s, w_eff, dx2, dB2, False, ws)
        merged2 = L.NF4Tensor.empty(out, inp)
        descs = L.make_merge_descs([(Wd, merged2, Pd, B, s)])
        L.loqt_merge_requant_batched(descs)
        torch.cuda.synchronize()
        assert torch.equal(y2, y) and torch.equal(dx2, dx) and torch.equal(dB2, dB)
        assert torch.equal(merged2.codes, merged.codes) and torch.equal(merged2.absmax, merged.absmax)
        del w_eff, y2, dx2, dB2, merged2

    # merge on sampled rows of W
    Orows = np.unique(np.concatenate([[0, out - 1], rng.choice(out, size=min(out, 48), replace=False)]))
    c, a, _, _ = G.nf4_host(merged)
    rate = _merge_policy_check(c[Orows], a[Orows], (Wq[0][Orows], Wq[1][Orows]), (Pq[0][Orows], Pq[1][Orows]),
                               lay.B, s)
    print(f"    merge code mismatch rate on {len(Orows)} rows: {rate:.2e}")
    assert rate <= 1e-3
