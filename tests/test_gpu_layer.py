"""GPU parity of loqt_linear_fwd / loqt_linear_bwd / loqt_merge_requant against the oracle on
shapes that span several tiles in every dimension and end in ragged tails."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-2  # max |err| <= TOL * RMS(reference): the bound stated for bf16 outputs and gradients


@pytest.fixture(params=["fused", "prepass", "folded"], autouse=True)
def path(request):
    """Every test runs once per implementation (NF4 expanded inside the GEMM / by a pre-pass)."""
    from paper_2405_16528_amd import binding as L
    L.set_path({"fused": L.PATH_FUSED, "prepass": L.PATH_PREPASS, "folded": L.PATH_FOLDED}[request.param])
    yield request.param
    L.set_path(L.PATH_AUTO)


def _setup(T, out, inp, r, seed, sigma_B=1e-3, name="layer"):
    from tests import gpu_util as G
    lay = synth.make_layer(name, "l", out, inp, r, T, seed)
    if sigma_B != 1e-3:
        lay.B = synth.normal_bf16(synth.rng_for(seed, name, "Bbig"), (r, inp), sigma_B)
    Wq = O.nf4_quantize(lay.W)
    Pq = O.nf4_quantize(lay.P)
    dev = dict(x=G.bf16_dev(lay.x), dy=G.bf16_dev(lay.dy), B=G.bf16_dev(lay.B),
               Wq=G.nf4_dev(*Wq), Pq=G.nf4_dev(*Pq))
    return lay, Wq, Pq, dev


SHAPES = [
    # T, out, in, r
    (256, 512, 512, 128),      # the 60M layer
    (300, 520, 456, 128),      # ragged M and N, K tail of 8
    (130, 300, 1000, 64),      # K tail not a multiple of 8... (1000 % 64 = 40)
    (515, 1100, 333, 192),     # odd in: pitch padded to 336, K tail 13
    (1000, 5461 // 4, 768, 256),
    (70, 130, 40, 32),         # every contraction shorter than one k-tile (one tail tile per K segment)
    (200, 192, 128, 40),       # whole k-tiles in the first K segment, a lone tail tile in the second
]


@pytest.mark.parametrize("T,out,inp,r", SHAPES)
@pytest.mark.parametrize("s", [1.0, 0.25])
def test_fwd_bwd_parity(T, out, inp, r, s):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    lay, Wq, Pq, d = _setup(T, out, inp, r, seed=T + out, sigma_B=2e-2)
    y = G.bf16_empty(T, out, fill=float("nan"))
    ws = G.workspace(L.OP_FWD, T, out, inp, r)
    L.loqt_linear_fwd(d["x"], d["Wq"], d["Pq"], d["B"], s, y, ws)
    dx = G.bf16_empty(T, inp, fill=float("nan"))
    dB = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
    ws2 = G.workspace(L.OP_BWD, T, out, inp, r)
    L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], s, dx, dB, False, ws2)
    torch.cuda.synchronize()
    y_ref = O.loqt_linear_fwd(lay.x, Wq, Pq, lay.B, s)
    dx_ref, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, s)
    ey = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(y)), y_ref)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dx)), dx_ref)
    eb = G.max_err_over_rms(dB.cpu().numpy().astype(np.float64), dB_ref)
    print(f"T={T} out={out} in={inp} r={r} s={s}: err/rms y {ey:.2e} dx {ex:.2e} dB {eb:.2e}")
    assert ey <= TOL and ex <= TOL and eb <= TOL


def test_bwd_options_accumulate_bf16_and_no_dx():
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    T, out, inp, r = 300, 260, 200, 64
    lay, Wq, Pq, d = _setup(T, out, inp, r, seed=9)
    ws = G.workspace(L.OP_BWD, T, out, inp, r)
    _, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, 0.5)
    # fp32 accumulate on top of an existing gradient, dx skipped
    base = synth.normal_f32(synth.rng_for(9, "dBbase"), (r, inp), float(np.sqrt(np.mean(dB_ref ** 2))))
    dB = torch.from_numpy(base.copy()).cuda()
    L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], 0.5, None, dB, True, ws)
    # bf16 output without accumulation
    dB16 = G.bf16_empty(r, inp, fill=float("nan"))
    L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], 0.5, None, dB16, False, ws)
    torch.cuda.synchronize()
    assert G.max_err_over_rms(dB.cpu().numpy().astype(np.float64), base + dB_ref) <= TOL
    assert G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dB16)), dB_ref) <= TOL


def test_results_are_deterministic():
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    T, out, inp, r = 700, 640, 520, 128
    lay, Wq, Pq, d = _setup(T, out, inp, r, seed=11)
    outs = []
    for _ in range(2):
        y = G.bf16_empty(T, out)
        dx = G.bf16_empty(T, inp)
        dB = torch.empty((r, inp), dtype=torch.float32, device="cuda")
        L.loqt_linear_fwd(d["x"], d["Wq"], d["Pq"], d["B"], 1.0, y, G.workspace(L.OP_FWD, T, out, inp, r))
        L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], 1.0, dx, dB, False,
                          G.workspace(L.OP_BWD, T, out, inp, r))
        m = L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], 1.0, out=L.NF4Tensor.empty(out, inp))
        torch.cuda.synchronize()
        outs.append((y.clone(), dx.clone(), dB.clone(), m.codes.clone(), m.absmax.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# --------------------------------------------------------------------------------- merge
def _merge_policy_check(c, a, Wq, Pq, B, s):
    """Codes may differ from the oracle's only where the bf16-operand product's worst-case
    error can move the normalised value across a decision threshold, and then by one level."""
    c_ref, a_ref = O.loqt_merge_requant(Wq, Pq, B, s)
    Wm = O.loqt_merge_f64(Wq, Pq, B, s)
    out, inp = c_ref.shape
    nblk = a_ref.shape[1]
    # worst-case error of the device's product: each dequantised P entry is rounded to bf16
    # (8 significant bits: relative error up to 2^-8), fp32 accumulation adds (r + 2) * 2^-24 of the absolute sum
    Pd = np.abs(O.nf4_dequantize_f64(*Pq))
    r = Pd.shape[1]
    E = abs(s) * (Pd @ np.abs(O.bf16_to_f64(B))) * (2.0 ** -8 + (r + 2) * 2.0 ** -24) + np.abs(Wm) * 2.0 ** -22
    pad = nblk * 64 - inp
    Ep = np.pad(E, ((0, 0), (0, pad))).reshape(out, nblk, 64)
    Emax = Ep.max(axis=2)
    a64 = a_ref.astype(np.float64)
    assert np.all(np.abs(a.astype(np.float64) - a64) <= Emax + 1e-30), "absmax outside the error bound"
    diff = c.astype(np.int32) - c_ref.astype(np.int32)
    bad = np.argwhere(diff != 0)
    rate = len(bad) / c.size
    mids = (O.NF4_LEVELS[:-1] + O.NF4_LEVELS[1:]) * 0.5
    for (o, i) in bad:
        assert abs(diff[o, i]) == 1, f"code off by {diff[o, i]} at {(o, i)}"
        am = a64[o, i // 64]
        t = Wm[o, i] / am
        mid = mids[min(c[o, i], c_ref[o, i])]
        # |t| <= 1: the scale's own error moves t by at most Emax/am
        tol = (E[o, i] + Emax[o, i // 64]) / am * 1.01
        assert abs(t - mid) <= tol, f"code differs at {(o, i)} though t is {abs(t - mid):.3e} from the threshold (tol {tol:.3e})"
    return rate


@pytest.mark.parametrize("out,inp,r,ld", [(512, 512, 128, None), (300, 456, 64, 512), (1100, 333, 192, None),
                                          (260, 2048, 256, None),
                                          (392, 264, 8, None),   # rank 8: eight terms per sum, little averaging
                                          (300, 200, 64, 512)])  # pitch exceeds `in` by more than two tiles
def test_merge_parity(out, inp, r, ld):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    lay, Wq, Pq, d = _setup(8, out, inp, r, seed=out + inp)
    d["Wq"] = G.nf4_dev(*Wq, ld)
    # B = 0: codes and absmax come back unchanged, bit for bit
    B0 = G.bf16_dev(np.zeros_like(lay.B))
    m0 = L.loqt_merge_requant(d["Wq"], d["Pq"], B0, 0.5, out=L.NF4Tensor.empty(out, inp, ld))
    torch.cuda.synchronize()
    assert torch.equal(m0.codes, d["Wq"].codes) and torch.equal(m0.absmax, d["Wq"].absmax)
    # general case, out of place, two scales
    for s in (1.0, 0.25):
        m = L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], s, out=L.NF4Tensor.empty(out, inp, ld))
        torch.cuda.synchronize()
        c, a, packed, am = G.nf4_host(m)
        rate = _merge_policy_check(c, a, Wq, Pq, lay.B, s)
        print(f"merge {out}x{inp} r={r} s={s}: code mismatch rate {rate:.2e}")
        assert rate <= 1e-3
        if m.ld > inp:  # padding written as level 0 / absmax 0
            p_ref, am_ref = O.pack_nf4(c, a, m.ld)
            assert np.array_equal(packed, p_ref) and np.array_equal(am, am_ref)
    # in place gives the same bits as out of place
    inplace = L.NF4Tensor(d["Wq"].codes.clone(), d["Wq"].absmax.clone(), out, inp, d["Wq"].ld)
    L.loqt_merge_requant(inplace, d["Pq"], d["B"], 0.25)
    torch.cuda.synchronize()
    assert torch.equal(inplace.codes, m.codes) and torch.equal(inplace.absmax, m.absmax)


def test_merge_large_update_parity():
    # an update as large as the weight itself (every block's scale changes)
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    out, inp, r = 384, 640, 128
    lay, Wq, Pq, d = _setup(8, out, inp, r, seed=21, sigma_B=5e-2)
    m = L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], 1.0, out=L.NF4Tensor.empty(out, inp))
    torch.cuda.synchronize()
    c, a, _, _ = G.nf4_host(m)
    rate = _merge_policy_check(c, a, Wq, Pq, lay.B, 1.0)
    assert not np.array_equal(a, Wq[1])
    # the rate scales with |update| / absmax: 2^-9 relative error of a product as large as the
    # weight moves t by ~5e-4, and about 15 thresholds per unit of t are in reach
    assert rate <= 1e-2


def test_merge_exact_case_bit_exact():
    # operands chosen so that every product and partial sum is exact in bf16 x bf16 -> fp32
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    rng = synth.rng_for(7, "exact")
    out, inp, r = 300, 448, 128
    wc = rng.choice(np.array([0, 7, 15], dtype=np.uint8), (out, inp))
    wc[:, 0::64] = 15
    wam = (np.float32(2.0) ** rng.integers(-12, -9, (out, inp // 64))).astype(np.float32)
    pc = rng.choice(np.array([0, 7, 15], dtype=np.uint8), (out, r))
    pc[:, 0::64] = 15
    pam = np.full((out, r // 64), 2.0 ** -5, dtype=np.float32)
    B = synth.to_bf16_bits((rng.integers(-4, 5, (r, inp)) * 2.0 ** -10).astype(np.float32))
    c_ref, a_ref = O.loqt_merge_requant((wc, wam), (pc, pam), B, 0.5)
    m = L.loqt_merge_requant(G.nf4_dev(wc, wam), G.nf4_dev(pc, pam), G.bf16_dev(B), 0.5,
                             out=L.NF4Tensor.empty(out, inp))
    torch.cuda.synchronize()
    c, a, _, _ = G.nf4_host(m)
    assert np.array_equal(a, a_ref) and np.array_equal(c, c_ref)
    assert len(np.unique(c)) >= 12


def test_merge_batched_matches_single():
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    layers, singles = [], []
    for i, (out, inp, r) in enumerate([(256, 320, 64), (130, 512, 128), (512, 192, 64)]):
        lay, Wq, Pq, d = _setup(8, out, inp, r, seed=30 + i)
        singles.append(L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], 0.5, out=L.NF4Tensor.empty(out, inp)))
        dst = L.NF4Tensor.empty(out, inp)
        layers.append((d["Wq"], dst, d["Pq"], d["B"], 0.5))
    descs = L.make_merge_descs(layers)
    L.loqt_merge_requant_batched(descs)
    torch.cuda.synchronize()
    for (_, dst, _, _, _), ref in zip(layers, singles):
        assert torch.equal(dst.codes, ref.codes) and torch.equal(dst.absmax, ref.absmax)


def test_merge_batched_grouped_launches_mixed_list():
    """The batched merge runs the wide weights (1024 columns and more) of a list as grouped launches of at most 24
    weights and the narrow ones one by one.  A list of 27 weights of mixed shapes -- ragged rows and columns, column
    counts that are not multiples of 64, narrow weights in between, in place and into separate outputs -- must give
    the bits of 27 single calls (Alg. 1 line 5 per layer; the grouping is only a launch layout)."""
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    shapes = [(300, 1088, 64), (130, 1500, 128), (512, 192, 64), (260, 1024, 32), (64, 2112, 96), (200, 1030, 40)]
    base = [_setup(8, out, inp, r, seed=70 + i) for i, (out, inp, r) in enumerate(shapes)]
    layers, singles = [], []
    for k in range(27):
        i = k % len(shapes)
        out, inp, r = shapes[i]
        lay, Wq, Pq, d = base[i]
        s = 0.25 + 0.125 * (k % 3)
        src = L.NF4Tensor(d["Wq"].codes.clone(), d["Wq"].absmax.clone(), out, inp, d["Wq"].ld)
        singles.append(L.loqt_merge_requant(src, d["Pq"], d["B"], s, out=L.NF4Tensor.empty(out, inp)))
        in_place = (k % 2) == 1
        dst = None if in_place else L.NF4Tensor.empty(out, inp)
        layers.append((src, dst, d["Pq"], d["B"], s))
    descs = L.make_merge_descs(layers)
    ws = torch.empty(L.merge_descs_workspace_bytes(descs), dtype=torch.uint8, device="cuda")
    L.loqt_merge_requant_batched(descs, ws)
    torch.cuda.synchronize()
    for k, ((src, dst, _, _, _), ref) in enumerate(zip(layers, singles)):
        got = dst if dst is not None else src
        assert torch.equal(got.codes, ref.codes) and torch.equal(got.absmax, ref.absmax), f"layer {k} {shapes[k % len(shapes)]}"


@pytest.mark.parametrize("T,out,inp,r", [(4096, 2048, 256, 512), (4100, 2056, 264, 500)])
def test_bwd_with_z_in_two_slices(T, out, inp, r):
    """Z = s dy deq(P) (sec. 2.2) with T x r outputs that would fill no more than half of the compute units is
    formed as two fp32 slices of the contraction over `out` and summed in a fixed order.  Shapes that take this
    form (64 to 128 tiles of 256x128, out >= 2048), one of them ragged in every dimension with a contraction
    that ends inside a k-tile; dx and dB against the oracle, and the same bits on a second call."""
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    s = 0.5
    lay, Wq, Pq, d = _setup(T, out, inp, r, seed=T + r, sigma_B=2e-2)
    res = []
    for _ in range(2):
        dx = G.bf16_empty(T, inp, fill=float("nan"))
        dB = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
        L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], s, dx, dB, False,
                          G.workspace(L.OP_BWD, T, out, inp, r))
        torch.cuda.synchronize()
        res.append((dx, dB))
    dx_ref, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, s)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(res[0][0])), dx_ref)
    eb = G.max_err_over_rms(res[0][1].cpu().numpy().astype(np.float64), dB_ref)
    print(f"two-slice Z T={T} out={out} in={inp} r={r}: err/rms dx {ex:.2e} dB {eb:.2e}")
    assert ex <= TOL and eb <= TOL
    assert torch.equal(res[0][0].view(torch.int16), res[1][0].view(torch.int16)) and torch.equal(res[0][1], res[1][1])
