"""GPU parity of the half-precision storage of the per-edge path weights (egnn_radial_weights_f16,
egnn_tp_segsum_f16, EGNN_OPT_W_FP16) against the oracle run with its weights rounded the same way (w_dtype=float16).

Rounding w to half precision is a quantisation decided by floating point: the GPU takes it on its fp32 value of w,
the oracle on its fp64 value, and a weight within the fp32 evaluation error of a rounding boundary lands on the
neighbouring code (a step of 2^-11 of that weight instead of an error of ~1e-6 of it).  The tests therefore split the
path where the decision is taken:
  * the codes themselves: equal to the oracle's, except where the oracle's value lies within the fp32 stage tolerance
    of the boundary between the two codes (and then only the neighbouring code is accepted);
  * the consumer (S4) fed with codes made by the oracle, so that both sides use identical weights: fp32 bar;
  * the composite calls: layer outputs (sums over ~10^2 edges x paths average the few flipped codes out) at the 1e-4
    bar; H_ij blocks (one edge each, nothing averages) within the size of the rounding itself in the max norm and
    far below it in the root-mean-square, where the rare flips do not dominate.
"""
import os
import numpy as np
import pytest

from paper_2507_03840_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_03840_amd import binding
    binding.load_library()
    return binding


def unpack_w16(words, n_cols):
    """int32 [n][32 * groups] -> float64 [n][n_cols] (layout of egnn_radial_weights_f16)."""
    u = np.ascontiguousarray(words).view(np.uint32)
    n, rw = u.shape
    lo = (u & 0xffff).astype(np.uint16).view(np.float16).reshape(n, rw // 32, 1, 32)
    hi = (u >> 16).astype(np.uint16).view(np.float16).reshape(n, rw // 32, 1, 32)
    return np.concatenate([lo, hi], axis=2).reshape(n, rw * 2)[:, :n_cols].astype(np.float64)


def pack_w16(w, fill=0.0):
    """float [n][n_cols] -> int32 words in the same layout (values rounded to half precision, nearest even)."""
    n, nc = w.shape
    groups = (nc + 63) // 64
    full = np.full((n, groups * 64), fill, np.float64)
    full[:, :nc] = w
    codes = full.astype(np.float16).view(np.uint16).astype(np.uint32).reshape(n, groups, 2, 32)
    return (codes[:, :, 0, :] | (codes[:, :, 1, :] << 16)).reshape(n, groups * 32).view(np.int32)


def test_pack_unpack_roundtrip_host():
    rng = np.random.default_rng(0)
    for nc in (8, 24, 64, 96, 1344):
        w = rng.standard_normal((5, nc))
        assert np.array_equal(unpack_w16(pack_w16(w), nc), w.astype(np.float16).astype(np.float64))


def _edge_setup(B, lmax, E, n, n_owned, n_rbf, r_cut, seed, which):
    from oracle import egnn_oracle as O
    w = synth.small_cluster(n, n_owned, lmax, E, n_rbf, r_cut, seed)
    g = U.oracle_graph(w)
    paths = O.tp_paths(lmax, lmax, lmax if which == 0 else O.L_READOUT)
    rng = np.random.default_rng([seed, 5])
    W = synth.layer_weights(rng, lmax, E, n_rbf, 64, len(paths))
    m = B.Egnn(lmax, E, n_rbf, r_cut, 4.0, orb_l=w.orb_l)
    pos = B.to_device(w.pos)
    gd = m.egnn_nlist(pos, n_owned, w.box, w.pbc)
    rhat_d = m.egnn_edge_geometry(gd, pos, w.box)[0]
    r = O.edge_vectors(w.pos, w.box, g[0], g[1], g[2])
    d = np.sqrt((r * r).sum(axis=1))
    w64 = O.radial_weights(d, W["W_r1"], W["W_r2"], paths, E, n_rbf, r_cut).reshape(len(d), -1)
    return w, g, m, gd, pos, rhat_d, W, w64, paths


@pytest.mark.parametrize("lmax,E,n,which", [(2, 8, 70, 0), (1, 8, 50, 0), (2, 16, 90, 1), (3, 32, 150, 0),
                                            (4, 32, 120, 1), (4, 64, 100, 0), (2, 128, 60, 0), (0, 8, 40, 0)])
def test_radial_weights_f16_codes(B, lmax, E, n, which):
    """Every stored code is the oracle's, or its neighbour where the oracle's value sits on a rounding boundary."""
    w, g, m, gd, pos, rhat_d, W, w64, paths = _edge_setup(B, lmax, E, n, n, 8, 4.0, 70 + lmax, which)
    words = m.egnn_radial_weights_f16(which, rhat_d, B.to_device(W["W_r1"]), B.to_device(W["W_r2"])).cpu().numpy()
    assert words.shape == (len(g[0]), 32 * ((w64.shape[1] + 63) // 64))
    got = unpack_w16(words, w64.shape[1])
    want = w64.astype(np.float16).astype(np.float64)
    same = got == want
    delta = 2e-5 * np.abs(w64).max()          # tolerance of the fp32 evaluation of w (the S3 stage test's bar)
    # a differing code must be the neighbour on the side of w64, and w64 within delta of the midpoint of the two
    mid = 0.5 * (got + want)
    ok = same | ((np.abs(w64 - mid) <= delta) & (np.abs(got - want) <= np.spacing(np.abs(want).astype(np.float16)).astype(np.float64) * 1.0001))
    frac = 1.0 - same.mean()
    print(f"lmax {lmax} E {E} which {which}: {same.size} codes, {frac:.2e} differ from the fp64 decision", flush=True)
    assert ok.all() and frac < 0.02


@pytest.mark.parametrize("lmax,E,n,n_owned", [(2, 8, 70, 50), (1, 16, 60, 60), (3, 32, 150, 100), (4, 32, 100, 100),
                                              (4, 64, 100, 80), (2, 128, 60, 60), (0, 16, 40, 40)])
def test_tp_segsum_f16_with_oracle_made_codes(B, lmax, E, n, n_owned):
    """S4 on half-precision weights packed on the host from the oracle's rounded values: identical weights on both
    sides, fp32 bar.  Unused halves of the last group hold NaN to show that they are not read."""
    from oracle import egnn_oracle as O
    w, g, m, gd, pos, rhat_d, W, w64, paths = _edge_setup(B, lmax, E, n, n_owned, 8, 4.0, 80 + lmax, 0)
    wr = w64.astype(np.float16).astype(np.float64)
    rng = np.random.default_rng(9)
    h = synth.node_features(rng, n, lmax, E)
    a = m.egnn_tp_segsum_f16(gd, rhat_d, B.to_device(h), B.to_device(pack_w16(wr, fill=np.nan)))
    ref = O.edge_messages_sum(g, w.pos, w.box, h.astype(np.float64),
                              lambda d, k0, k1, p: wr[k0:k1].reshape(k1 - k0, len(paths), E), lmax, lmax, 4.0)
    assert U.rel_err(a.cpu().numpy(), ref) < 2e-5


@pytest.mark.parametrize("lmax,E,n,n_owned", [(2, 8, 70, 50), (1, 16, 60, 60), (3, 32, 150, 100), (4, 32, 100, 100),
                                              (4, 64, 100, 80), (2, 128, 60, 60), (0, 16, 40, 40)])
def test_tp_segsum_f16h_features_and_weights_in_half_precision(B, lmax, E, n, n_owned):
    """S4 with the gathered features in half precision as well (egnn_tp_segsum_f16h).  The features are rounded on the
    device by egnn_pack_rows(half) with the identity index list -- bit-exact against numpy's rounding -- and the
    weights are packed from the oracle's rounded values, so both sides use identical inputs: fp32 bar against the
    oracle run on the rounded features and weights."""
    import torch
    from oracle import egnn_oracle as O
    w, g, m, gd, pos, rhat_d, W, w64, paths = _edge_setup(B, lmax, E, n, n_owned, 8, 4.0, 90 + lmax, 0)
    wr = w64.astype(np.float16).astype(np.float64)
    rng = np.random.default_rng(10)
    h = synth.node_features(rng, n, lmax, E)
    h[0, 0, 0] = 70000.0          # beyond the half-precision range: infinity on both sides of the rounding test
    h[1, 0, 0] = 3.0e-8           # below the smallest subnormal's half: zero
    h[2, 0, 0] = 6.1e-5           # subnormal range
    h16 = m.egnn_pack_rows(B.to_device(h), torch.arange(n, dtype=torch.int32, device="cuda"), half=True)
    assert h16.dtype == torch.float16
    with np.errstate(over="ignore"):
        expect = h.astype(np.float16)
    assert np.array_equal(h16.cpu().numpy().view(np.uint16), expect.view(np.uint16))
    h16[0, 0, 0] = 1.5            # (a finite value again for the sums)
    hr = h16.cpu().numpy().astype(np.float64)
    a = m.egnn_tp_segsum_f16h(gd, rhat_d, h16, B.to_device(pack_w16(wr, fill=np.nan)))
    ref = O.edge_messages_sum(g, w.pos, w.box, hr, lambda d, k0, k1, p: wr[k0:k1].reshape(k1 - k0, len(paths), E),
                              lmax, lmax, 4.0)
    e = U.rel_err(a.cpu().numpy(), ref)
    # what the rounding of the features itself costs, for the record (not a bar)
    h_full = h.astype(np.float64)
    h_full[0, 0, 0] = 1.5
    full = O.edge_messages_sum(g, w.pos, w.box, h_full, lambda d, k0, k1, p: wr[k0:k1].reshape(k1 - k0, len(paths), E),
                               lmax, lmax, 4.0)
    print(f"  lmax {lmax} E {E}: rel err {e:.2e} (rounding the features moves the result by "
          f"{np.abs(ref - full).max() / np.abs(full).max():.1e})", flush=True)
    assert e < 2e-5


def _rms(a):
    return float(np.sqrt(np.mean(np.square(a))))


def _check_composite_H(got, H_half, H_full, label):
    """Max norm: within the size of the rounding itself; rms: far below it."""
    scale = np.abs(H_full).max()
    e_half, e_full = np.abs(got - H_half).max() / scale, np.abs(got - H_full).max() / scale
    r_half, r_round = _rms(got - H_half), _rms(H_half - H_full)
    print(f"{label}: H max err vs rounded-weight oracle {e_half:.2e} (vs unrounded {e_full:.2e}); "
          f"rms {r_half / scale:.2e} vs rms of the rounding effect {r_round / scale:.2e}", flush=True)
    assert e_half < 2.0 ** -11 and e_half <= e_full
    assert r_half < 0.25 * r_round


@pytest.mark.parametrize("lmax,E,periodic,n,n_owned", [(0, 8, False, 40, 40), (1, 16, True, 120, 120),
                                                        (2, 64, False, 100, 60), (3, 16, True, 150, 90),
                                                        (4, 128, False, 60, 40), (4, 8, False, 70, 70),
                                                        (3, 32, True, 260, 200), (4, 32, False, 200, 150),
                                                        (4, 64, True, 180, 120), (1, 8, False, 33, 33),
                                                        (2, 32, False, 33, 33), (0, 32, False, 50, 50)])
def test_w_fp16_small_shapes(B, lmax, E, periodic, n, n_owned):
    w = synth.small_cluster(n, n_owned, lmax, E, 6, 4.0, 60 + lmax, periodic=periodic)
    w.n_layers = 2
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = max(1.0, U.mean_degree(g, w.n_owned))
    m, graph, xs, H = U.gpu_forward(w, wt, agg, w_fp16=True)
    xs_ref, H_ref = U.oracle_forward(w, wt, g, agg, w_dtype=np.float16)
    xs_full, H_full = U.oracle_forward(w, wt, g, agg)
    for t in range(2):
        assert U.rel_err(xs[t].cpu().numpy(), xs_ref[t]) < U.TOL
    _check_composite_H(H.cpu().numpy().astype(np.float64), H_ref, H_full, f"lmax {lmax} E {E}")


@pytest.mark.parametrize("index", [1, 2])
def test_w_fp16_configs_full(B, index):
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    m, graph, xs, H = U.gpu_forward(w, wt, agg, w_fp16=True)
    xs_ref, H_ref = U.oracle_forward(w, wt, g, agg, w_dtype=np.float16)
    xs_full, H_full = U.oracle_forward(w, wt, g, agg)
    for t in range(w.n_layers):
        e = U.rel_err(xs[t].cpu().numpy(), xs_ref[t])
        print(f"config {index} layer {t} (half-precision w): rel err {e:.2e}", flush=True)
        assert e < U.TOL
    _check_composite_H(H.cpu().numpy().astype(np.float64), H_ref, H_full, f"config {index}")


@pytest.mark.parametrize("index", [3, 4])
def test_w_fp16_fullsize_sampled_rows(B, index):
    """First layer and readout of the full-size configurations, both applied to the layer-0 features."""
    import torch
    path = os.path.join(GOLDEN, f"config{index}_w16_samples.npz")
    assert os.path.exists(path), f"run tests/golden/make_golden.py w16:{index}"
    gold = np.load(path)
    w = synth.workload(index)
    wt = U.model_weights(w)
    m = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, float(gold["agg"]), n_layers=w.n_layers, orb_l=w.orb_l)
    m.egnn_set_option(B.OPT_W_FP16, 1)
    pos = B.to_device(w.pos)
    graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
    assert graph.n_edges == int(gold["n_edges"])
    ws = m.workspace(graph)
    x = B.to_device(wt["x0"])
    m.egnn_species_embed(B.to_device(w.species), B.to_device(wt["table"]), x)
    y = m.egnn_layer_forward(graph, pos, w.box, x, B.to_device(wt["layers"][0]), ws)
    got = y[torch.from_numpy(gold["nodes"]).cuda()].cpu().numpy().astype(np.float64)
    scale = np.abs(gold["x1_rows"]).max()
    e_half = np.abs(got - gold["x1_rows"]).max() / scale
    e_full = np.abs(got - gold["x1_rows_full"]).max() / scale
    print(f"config {index} layer (half-precision w): vs rounded-weight oracle {e_half:.2e}, vs unrounded {e_full:.2e}",
          flush=True)
    assert e_half < U.TOL and e_half < e_full
    H = m.egnn_readout_hij(graph, pos, w.box, x, B.to_device(wt["readout"]), ws)
    got = H[torch.from_numpy(gold["edges"]).cuda()].cpu().numpy().astype(np.float64)
    _check_composite_H(got, gold["H_rows"], gold["H_rows_full"], f"config {index}")


def test_w_fp16_leaves_given_weights_and_stage_calls_alone(B):
    """Caller-supplied edge weights are fp32 whatever the option says."""
    from oracle import egnn_oracle as O
    w = synth.small_cluster(80, 80, 2, 16, 8, 4.0, 41)
    g = U.oracle_graph(w)
    rng = np.random.default_rng(3)
    P = len(O.tp_paths(2, 2, 2))
    W = synth.layer_weights(rng, 2, 16, 8, 64, P)
    x = synth.node_features(rng, 80, 2, 16)
    we = synth.normal(rng, (len(g[0]), P, 16))
    m = B.Egnn(2, 16, 8, w.r_cut, 5.0)
    m.egnn_set_option(B.OPT_W_FP16, 1)
    pos = B.to_device(w.pos)
    gd = m.egnn_nlist(pos, 80, w.box, w.pbc)
    ws = m.workspace(gd)
    y = m.egnn_layer_forward(gd, pos, w.box, B.to_device(x), B.to_device(W), ws, w_edge=B.to_device(we))
    ref = O.layer_forward(g, w.pos, w.box, x, W, 2, 2, 16, 8, w.r_cut, 5.0, w_edge=we)
    assert U.rel_err(y.cpu().numpy(), ref) < 1e-5
