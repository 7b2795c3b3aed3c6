"""GPU parity: every stage and the composite calls of the C ABI against the fp64 oracle, element by element.

Bar: integer outputs (edge list, CSR index, shifts) bit-exact; floating-point outputs
max|gpu - oracle| / max|oracle| <= 1e-4 per tensor (fp32 path vs fp64 oracle).
"""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from paper_2507_03840_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
TOL = U.TOL


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2507_03840_amd import binding
    binding.load_library()
    return binding


def _cluster(n, n_owned, lmax, E, n_rbf=8, r_cut=4.0, seed=0, periodic=False, density=0.05):
    return synth.small_cluster(n, n_owned, lmax, E, n_rbf, r_cut, seed, periodic, density)


def _graph_to_device(B, g, n_owned, n_total):
    src, dst, shift, row_ptr = g
    return B.Graph(B.to_device(src), B.to_device(dst), B.to_device(row_ptr), B.to_device(shift), n_owned, n_total)


# ------------------------------------------------------------------------------------------ S1
@pytest.mark.parametrize("cell_list", [True, False])
@pytest.mark.parametrize("case", ["open", "periodic", "halo", "config1", "config2", "empty", "single", "slab", "line"])
def test_nlist_bit_exact(B, case, cell_list):
    """Edge list, CSR index and periodic shifts against the brute-force oracle, for both search strategies."""
    print("case", case, flush=True)
    if case == "config1":
        w = synth.workload(1)
    elif case == "config2":
        w = synth.workload(2)
    elif case == "empty":
        w = _cluster(5, 0, 1, 8, seed=3)
    elif case == "single":
        w = _cluster(1, 1, 1, 8, seed=3)
    elif case == "slab":      # periodic in x, y only, many cells along x, halo atoms: the shape of config 4
        w = _cluster(900, 600, 1, 8, r_cut=3.0, seed=6, periodic=True, density=0.05)
        w.pbc = np.array([1, 1, 0], np.uint8)
    elif case == "line":      # all atoms on a line: two axes with zero extent
        w = _cluster(50, 50, 1, 8, r_cut=3.0, seed=7)
        w.pos[:, 1:] = 0.25
    else:
        w = _cluster(333, 200 if case == "halo" else 333, 1, 8, r_cut=5.0, seed=4, periodic=(case == "periodic"))
    m = B.Egnn(1, 8, 8, w.r_cut, 1.0)
    g = m.egnn_nlist(B.to_device(w.pos), w.n_owned, w.box, w.pbc, cell_list=cell_list)
    src, dst, shift, row_ptr = U.oracle_graph(w)
    assert g.n_edges == len(src)
    assert np.array_equal(g.row_ptr.cpu().numpy(), row_ptr)
    assert np.array_equal(g.src.cpu().numpy(), src)
    assert np.array_equal(g.dst.cpu().numpy(), dst)
    assert np.array_equal(g.shift.cpu().numpy().reshape(-1, 3), shift.reshape(-1, 3))


def test_nlist_rejects_small_periodic_box(B):
    w = _cluster(20, 20, 1, 8, r_cut=4.0, seed=1, periodic=True)
    m = B.Egnn(1, 8, 8, 40.0, 1.0)
    with pytest.raises(B.EgnnError) as e:
        m.egnn_nlist(B.to_device(w.pos), 20, w.box, w.pbc)
    assert e.value.code == -2


def test_nlist_fill_rejects_another_workspace(B):
    """The fill pass reuses the cells the count pass left in the workspace: a different workspace or position
    pointer is refused (EGNN_EINVAL) instead of walking cells that were never built."""
    import ctypes as C
    import torch
    w = _cluster(300, 300, 1, 8, r_cut=4.0, seed=2)
    m = B.Egnn(1, 8, 8, w.r_cut, 1.0)
    pos = B.to_device(w.pos)
    n = w.n_total
    nbytes = m.egnn_nlist_workspace_bytes(n)
    ws1 = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ws2 = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    row_ptr = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    n_edges = C.c_int64()
    box = (C.c_float * 3)(*[float(v) for v in w.box])
    pbc = (C.c_uint8 * 3)(*[int(v) for v in w.pbc])
    ptr = lambda t: C.c_void_p(t.data_ptr())
    assert m.lib.egnn_nlist_count(m.ctx, ptr(pos), n, n, box, pbc, ptr(row_ptr), C.byref(n_edges), ptr(ws1),
                                  C.c_size_t(nbytes), None) == 0
    src = torch.empty(n_edges.value, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    args = lambda ws, p: (m.ctx, ptr(p), n, n, box, pbc, ptr(row_ptr), C.c_int64(n_edges.value), ptr(src), ptr(dst),
                          None, ptr(ws), C.c_size_t(nbytes), None)
    assert m.lib.egnn_nlist_fill(*args(ws2, pos)) == -1
    assert m.lib.egnn_nlist_fill(*args(ws1, pos.clone())) == -1
    assert m.lib.egnn_nlist_fill(*args(ws1, pos)) == 0
    torch.cuda.synchronize()
    g = U.oracle_graph(w)
    assert np.array_equal(src.cpu().numpy(), g[0]) and np.array_equal(dst.cpu().numpy(), g[1])


# ------------------------------------------------------------------------------------------ S2
@pytest.mark.parametrize("lmax", [0, 1, 2, 3, 4])
def test_edge_geometry(B, lmax):
    w = _cluster(150, 150, lmax, 8, n_rbf=16, r_cut=5.0, seed=lmax, periodic=True)
    g = U.oracle_graph(w)
    m = B.Egnn(lmax, 8, 16, w.r_cut, 1.0)
    gd = _graph_to_device(B, g, w.n_owned, w.n_total)
    rhat_d, Y, rbf, fc = m.egnn_edge_geometry(gd, B.to_device(w.pos), w.box, True, True, True)
    r = O.edge_vectors(w.pos, w.box, g[0], g[1], g[2])
    d = np.linalg.norm(r, axis=1)
    assert len(d) > 1000
    assert np.abs(rhat_d.cpu().numpy()[:, :3] - r / d[:, None]).max() < 2e-7
    assert np.abs(rhat_d.cpu().numpy()[:, 3] / d - 1).max() < 2e-7
    assert U.rel_err(Y.cpu().numpy(), O.sph_harm_real(lmax, r / d[:, None])) < 1e-5
    assert np.abs(rbf.cpu().numpy() - O.radial_basis(d, 16, w.r_cut)).max() < 1e-5
    assert np.abs(fc.cpu().numpy() - O.envelope(d, w.r_cut)).max() < 1e-6


# ------------------------------------------------------------------------------------------ S3
@pytest.mark.parametrize("lmax,E,n_rbf,which", [(2, 16, 8, 0), (3, 32, 16, 0), (4, 32, 16, 0), (4, 64, 16, 0),
                                                 (3, 32, 16, 1), (1, 8, 5, 0), (2, 128, 32, 1)])
def test_radial_weights(B, lmax, E, n_rbf, which):
    w = _cluster(120, 120, lmax, E, n_rbf=n_rbf, r_cut=5.0, seed=10 + lmax, periodic=False)
    g = U.oracle_graph(w)
    n_e = len(g[0])
    assert n_e % 256 != 0 and n_e > 600     # several 256-edge tiles and a ragged tail
    paths = O.tp_paths(lmax, lmax, lmax if which == 0 else 4)
    rng = np.random.default_rng(5)
    W = synth.layer_weights(rng, lmax, E, n_rbf, 64, len(paths))
    m = B.Egnn(lmax, E, n_rbf, w.r_cut, 1.0)
    gd = _graph_to_device(B, g, w.n_owned, w.n_total)
    rhat_d, *_ = m.egnn_edge_geometry(gd, B.to_device(w.pos), w.box)
    wk = m.egnn_radial_weights(which, rhat_d, B.to_device(W["W_r1"]), B.to_device(W["W_r2"]))
    r = O.edge_vectors(w.pos, w.box, g[0], g[1], g[2])
    ref = O.radial_weights(np.linalg.norm(r, axis=1), W["W_r1"], W["W_r2"], paths, E, n_rbf, w.r_cut)
    assert wk.shape == ref.shape
    assert U.rel_err(wk.cpu().numpy(), ref) < 2e-5


# ------------------------------------------------------------------------------------------ S5
@pytest.mark.parametrize("lmax,E,two", [(0, 8, False), (2, 16, True), (3, 32, False), (4, 32, True), (4, 64, True),
                                         (1, 128, True)])
def test_node_mix(B, lmax, E, two):
    rng = np.random.default_rng(lmax * 10 + E)
    n = 77
    x1, x2 = synth.node_features(rng, n, lmax, E), synth.node_features(rng, n, lmax, E)
    W1 = synth.normal(rng, (lmax + 1, E, E), E ** -0.5)
    W2 = synth.normal(rng, (lmax + 1, E, E), E ** -0.5)
    m = B.Egnn(lmax, E, 8, 4.0, 1.0)
    y = m.egnn_node_mix(B.to_device(x1), B.to_device(W1), B.to_device(x2) if two else None,
                        B.to_device(W2) if two else None)
    ref = O.mix_channels(x1, W1, lmax) + (O.mix_channels(x2, W2, lmax) if two else 0.0)
    assert U.rel_err(y.cpu().numpy(), ref) < 1e-5


@pytest.mark.parametrize("lmax,E,two,n", [(4, 64, True, 7777), (4, 32, False, 15001), (2, 64, True, 33333)])
def test_node_mix_many_tiles(B, lmax, E, two, n):
    """Enough rows that a workgroup of the matrix-core kernel walks several row tiles (the next tile's rows in flight
    during the products of the current one), with a last tile that is partly or wholly past the end."""
    rng = np.random.default_rng(n)
    x1, x2 = synth.node_features(rng, n, lmax, E), synth.node_features(rng, n, lmax, E)
    W1 = synth.normal(rng, (lmax + 1, E, E), E ** -0.5)
    W2 = synth.normal(rng, (lmax + 1, E, E), E ** -0.5)
    m = B.Egnn(lmax, E, 8, 4.0, 1.0)
    y = m.egnn_node_mix(B.to_device(x1), B.to_device(W1), B.to_device(x2) if two else None,
                        B.to_device(W2) if two else None)
    ref = O.mix_channels(x1, W1, lmax) + (O.mix_channels(x2, W2, lmax) if two else 0.0)
    assert U.rel_err(y.cpu().numpy(), ref) < 1e-5
    y2 = m.egnn_node_mix(B.to_device(x1), B.to_device(W1), B.to_device(x2) if two else None,
                         B.to_device(W2) if two else None)
    assert np.array_equal(y.cpu().numpy(), y2.cpu().numpy())


# ------------------------------------------------------------------------------------------ S4
@pytest.mark.parametrize("lmax,E", [(0, 8), (1, 16), (2, 16), (3, 32), (4, 32), (4, 64), (2, 128)])
def test_tp_segsum_given_weights(B, lmax, E):
    """Messages with per-edge weights supplied by the caller; includes a node without incoming edges."""
    w = _cluster(90, 70, lmax, E, r_cut=4.5, seed=20 + lmax, periodic=False)
    w.pos[0] += 100.0          # owned atom 0 far away: empty row
    g = U.oracle_graph(w)
    assert g[3][1] == g[3][0] and len(g[0]) > 500
    rng = np.random.default_rng(6)
    paths = O.tp_paths(lmax, lmax, lmax)
    h = synth.node_features(rng, w.n_total, lmax, E)
    we = synth.normal(rng, (len(g[0]), len(paths), E))
    agg = 9.0
    m = B.Egnn(lmax, E, 8, w.r_cut, agg)
    gd = _graph_to_device(B, g, w.n_owned, w.n_total)
    rhat_d, *_ = m.egnn_edge_geometry(gd, B.to_device(w.pos), w.box)
    a = m.egnn_tp_segsum(gd, rhat_d, B.to_device(h), B.to_device(we))
    ref = O.edge_messages_sum(g, w.pos, w.box, h.astype(np.float64), lambda d, k0, k1, p: we[k0:k1].astype(np.float64),
                              lmax, lmax, agg)
    assert np.all(a[0].cpu().numpy() == 0)
    assert U.rel_err(a.cpu().numpy(), ref) < 2e-5
    # bit-identical on a second run (no atomics)
    a2 = m.egnn_tp_segsum(gd, rhat_d, B.to_device(h), B.to_device(we))
    assert np.array_equal(a.cpu().numpy(), a2.cpu().numpy())


def test_tp_segsum_edge_along_polar_axis(B):
    """Edges exactly along +z and -z: the azimuth is undefined there."""
    lmax, E = 4, 32
    pos = np.array([[0, 0, 0], [0, 0, 1.5], [0, 0, -1.7], [1.2, 0, 0], [0, -1.1, 0]], np.float32)
    box, pbc = np.ones(3, np.float32) * 50, np.zeros(3, np.uint8)
    g = O.neighbour_list(pos, 1, box, pbc, 2.0)
    assert len(g[0]) == 4
    rng = np.random.default_rng(8)
    paths = O.tp_paths(lmax, lmax, lmax)
    h = synth.node_features(rng, 5, lmax, E)
    we = synth.normal(rng, (4, len(paths), E))
    m = B.Egnn(lmax, E, 8, 2.0, 1.0)
    gd = _graph_to_device(B, g, 1, 5)
    rhat_d, *_ = m.egnn_edge_geometry(gd, B.to_device(pos), box)
    a = m.egnn_tp_segsum(gd, rhat_d, B.to_device(h), B.to_device(we))
    ref = O.edge_messages_sum(g, pos, box, h.astype(np.float64), lambda d, k0, k1, p: we[k0:k1].astype(np.float64),
                              lmax, lmax, 1.0)
    assert U.rel_err(a.cpu().numpy(), ref) < 2e-5


# ------------------------------------------------------------------------------------------ whole model
@pytest.mark.parametrize("fused", [False, True, 2])
@pytest.mark.parametrize("index", [1, 2])
def test_model_forward_configs_full(B, index, fused):
    """Configs 1 and 2 in full: species embedding, all layers, H_ij readout, every element; once through the materialised weight tensor
    (default) and once with the fused radial-weights + message kernel."""
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    m, graph, xs, H = U.gpu_forward(w, wt, agg, fused=fused)
    assert np.array_equal(graph.src.cpu().numpy(), g[0]) and np.array_equal(graph.dst.cpu().numpy(), g[1])
    xs_ref, H_ref = U.oracle_forward(w, wt, g, agg)
    for t in range(w.n_layers):
        e = U.rel_err(xs[t].cpu().numpy(), xs_ref[t])
        print(f"config {index} layer {t}: rel err {e:.2e}", flush=True)
        assert e < TOL
    e = U.rel_err(H.cpu().numpy(), H_ref)
    print(f"config {index} H_ij: rel err {e:.2e}  max|H| {np.abs(H_ref).max():.3f}", flush=True)
    assert e < TOL and H.shape == (len(g[0]), 13, 13)


@pytest.mark.parametrize("lmax,E,periodic,n,n_owned", [(0, 8, False, 40, 40), (1, 16, True, 120, 120),
                                                        (2, 64, False, 100, 60), (3, 16, True, 150, 90),
                                                        (4, 128, False, 60, 40), (4, 8, False, 70, 70),
                                                        (3, 32, True, 260, 200), (4, 32, False, 200, 150),
                                                        (4, 64, True, 180, 120), (0, 16, False, 40, 30),
                                                        (2, 32, False, 33, 33)])
def test_model_forward_small_shapes(B, lmax, E, periodic, n, n_owned):
    _model_forward_small(B, lmax, E, periodic, n, n_owned, False)


@pytest.mark.parametrize("lmax,E,n,n_owned,r_cut", [(1, 16, 120, 120, 4.0), (2, 64, 100, 60, 4.0), (3, 32, 150, 90, 4.0),
                                                     (4, 16, 70, 70, 4.0), (0, 32, 50, 50, 4.0), (4, 64, 90, 70, 4.0),
                                                     (1, 8, 60, 60, 4.0), (4, 128, 60, 40, 4.0), (3, 8, 150, 90, 4.0),
                                                     # up to ~300 incoming edges per node: several 128-edge tiles, ragged tails
                                                     (2, 8, 330, 25, 9.5), (4, 16, 330, 12, 9.5)])
def test_model_forward_small_shapes_fused(B, lmax, E, n, n_owned, r_cut):
    _model_forward_small(B, lmax, E, False, n, n_owned, True, r_cut)


@pytest.mark.parametrize("lmax,E,n,n_owned,r_cut", [(1, 16, 120, 120, 4.0), (2, 64, 100, 60, 4.0), (3, 32, 150, 90, 4.0),
                                                     (4, 16, 70, 70, 4.0), (0, 32, 50, 50, 4.0), (4, 64, 90, 70, 4.0),
                                                     (1, 8, 60, 60, 4.0), (4, 128, 60, 40, 4.0), (3, 8, 150, 90, 4.0),
                                                     # up to ~300 incoming edges per node: more than one round of 224
                                                     (2, 8, 330, 25, 9.5), (4, 16, 330, 12, 9.5)])
def test_model_forward_small_shapes_fused_lane(B, lmax, E, n, n_owned, r_cut):
    """The second fused design (weights produced on the matrix cores in the registers of the consuming lane)."""
    _model_forward_small(B, lmax, E, False, n, n_owned, 2, r_cut)


@pytest.mark.parametrize("fused", [1, 2])
@pytest.mark.parametrize("r_cut", [2.0, 2.6])
def test_fused_sparse_graph(B, r_cut, fused):
    """Few edges per node, and nodes without any."""
    _model_forward_small(B, 2, 16, False, 200, 150, fused, r_cut)


@pytest.mark.parametrize("s1,s2", [(1e-4, 1e-6), (30.0, 1e5), (1.0, 3e-9), (2e-3, 4e7)])
def test_radial_weight_scales(B, s1, s2):
    """The radial contraction (S3, and the second fused design) cuts its matrix-core operands into half-precision
    pieces; their scalings come from the weights, so tiny and huge radial weights keep fp32-level accuracy."""
    w = _cluster(120, 90, 3, 16, n_rbf=6, r_cut=4.0, seed=77)
    w.n_layers = 1
    wt = U.model_weights(w)
    wt["layers"][0]["W_r1"] = (wt["layers"][0]["W_r1"] * np.float32(s1)).astype(np.float32)
    wt["layers"][0]["W_r2"] = (wt["layers"][0]["W_r2"] * np.float32(s2)).astype(np.float32)
    wt["layers"][0]["W_self"] = np.zeros_like(wt["layers"][0]["W_self"])     # the output is the message term alone
    g = U.oracle_graph(w)
    agg = max(1.0, U.mean_degree(g, w.n_owned))
    wt["readout"]["W_r1"] = (wt["readout"]["W_r1"] * np.float32(s1)).astype(np.float32)
    wt["readout"]["W_r2"] = (wt["readout"]["W_r2"] * np.float32(s2)).astype(np.float32)
    xs_ref, H_ref = U.oracle_forward(w, wt, g, agg)
    assert np.abs(xs_ref[0]).max() > 0 and np.abs(H_ref).max() > 0
    errs = []
    for fused in (0, 2):
        m, graph, xs, H = U.gpu_forward(w, wt, agg, fused=fused)
        errs.append(U.rel_err(xs[0].cpu().numpy(), xs_ref[0]))
        if fused == 0:
            errs.append(U.rel_err(H.cpu().numpy(), H_ref))
    print("rel err two-kernel %.2e (H_ij %.2e), fused %.2e" % tuple(errs), flush=True)
    assert max(errs) < 1e-5


def _model_forward_small(B, lmax, E, periodic, n, n_owned, fused, r_cut=4.0):
    """Small ragged cases over every supported degree and channel width, with halo rows, two layers, readout."""
    w = _cluster(n, n_owned, lmax, E, n_rbf=6, r_cut=r_cut, seed=30 + lmax, periodic=periodic)
    w.n_layers = 2
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = max(1.0, U.mean_degree(g, w.n_owned))
    m, graph, xs, H = U.gpu_forward(w, wt, agg, fused=fused)
    xs_ref, H_ref = U.oracle_forward(w, wt, g, agg)
    for t in range(2):
        assert U.rel_err(xs[t].cpu().numpy(), xs_ref[t]) < TOL
    assert U.rel_err(H.cpu().numpy(), H_ref) < TOL


def test_layer_forward_with_given_edge_weights_and_errors(B):
    import torch
    w = _cluster(80, 80, 2, 16, r_cut=4.0, seed=41)
    g = U.oracle_graph(w)
    rng = np.random.default_rng(3)
    P = len(O.tp_paths(2, 2, 2))
    W = synth.layer_weights(rng, 2, 16, 8, 64, P)
    x = synth.node_features(rng, 80, 2, 16)
    we = synth.normal(rng, (len(g[0]), P, 16))
    m = B.Egnn(2, 16, 8, w.r_cut, 5.0)
    gd = _graph_to_device(B, g, 80, 80)
    ws = m.workspace(gd, with_weights=False)
    Wd = B.to_device(W)
    y = m.egnn_layer_forward(gd, B.to_device(w.pos), w.box, B.to_device(x), Wd, ws, w_edge=B.to_device(we))
    ref = O.layer_forward(g, w.pos, w.box, x, W, 2, 2, 16, 8, w.r_cut, 5.0, w_edge=we)
    assert U.rel_err(y.cpu().numpy(), ref) < TOL
    # workspace too small -> EGNN_EWS, nothing launched
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.EgnnError) as e:
        m.egnn_layer_forward(gd, B.to_device(w.pos), w.box, B.to_device(x), Wd, small)
    assert e.value.code == -3
    # aliasing input and output is refused
    xd = B.to_device(x)
    with pytest.raises(B.EgnnError) as e:
        m.egnn_layer_forward(gd, B.to_device(w.pos), w.box, xd, Wd, m.workspace(gd), out=xd)
    assert e.value.code == -1


@pytest.mark.parametrize("fused", [0, 1, 2])
def test_empty_graph_layer(B, fused):
    """No edges at all: the layer reduces to the self term."""
    w = _cluster(6, 6, 2, 16, r_cut=0.5, seed=2, density=0.001)
    g = U.oracle_graph(w)
    assert len(g[0]) == 0
    rng = np.random.default_rng(4)
    W = synth.layer_weights(rng, 2, 16, 8, 64, len(O.tp_paths(2, 2, 2)))
    x = synth.node_features(rng, 6, 2, 16)
    m = B.Egnn(2, 16, 8, w.r_cut, 1.0)
    m.egnn_set_option(B.OPT_FUSED, fused)
    graph = m.egnn_nlist(B.to_device(w.pos), 6, w.box, w.pbc)
    assert graph.n_edges == 0
    y = m.egnn_layer_forward(graph, B.to_device(w.pos), w.box, B.to_device(x), B.to_device(W), m.workspace(graph))
    assert U.rel_err(y.cpu().numpy(), O.mix_channels(x, W["W_self"], 2)) < 1e-5
