"""GPU parity of the SO(2) form of the message transform (egnn_so2_message_sum) against oracle/so2_oracle.py."""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from oracle import so2_oracle as S
from paper_2507_03840_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
TOL = U.TOL


@pytest.fixture(scope="module")
def B():
    from paper_2507_03840_amd import binding
    binding.load_library()
    return binding


def so2_weights(rng, lmax, E, n_rbf):
    """Every matrix ~ N(0, 1/fan_in) (fan_in doubled for m > 0, where two blocks feed each output)."""
    shapes = S.so2_shapes(lmax, E)
    W0 = synth.normal(rng, shapes[0], shapes[0][1] ** -0.5)
    Wr = [synth.normal(rng, s, (2 * s[1]) ** -0.5) for s in shapes[1:]]
    Wi = [synth.normal(rng, s, (2 * s[1]) ** -0.5) for s in shapes[1:]]
    W_e = synth.normal(rng, (E, n_rbf), n_rbf ** -0.5)
    return W_e, W0, Wr, Wi


def run_case(B, w, seed=0):
    g = U.oracle_graph(w)
    agg = max(1.0, U.mean_degree(g, w.n_owned))
    rng = np.random.default_rng([w.seed if hasattr(w, "seed") and w.seed else 0, 7, seed])
    x = synth.node_features(rng, w.n_total, w.lmax, w.channels)
    W_e, W0, Wr, Wi = so2_weights(rng, w.lmax, w.channels, w.n_rbf)
    ref = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, w.lmax, w.channels, w.n_rbf, w.r_cut, agg)
    m = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, agg)
    flat = S.so2_pack(W0, Wr, Wi)
    assert flat.size == m.egnn_so2_weight_count()
    graph = m.egnn_nlist(B.to_device(w.pos), w.n_owned, w.box, w.pbc)
    assert np.array_equal(graph.src.cpu().numpy(), g[0])
    import torch
    ws = torch.empty(m.egnn_so2_workspace_bytes(graph.n_edges), dtype=torch.uint8, device="cuda")
    a = m.egnn_so2_message_sum(graph, B.to_device(w.pos), w.box, B.to_device(x), B.to_device(W_e), B.to_device(flat), ws)
    return a.cpu().numpy(), ref, len(g[0])


@pytest.mark.parametrize("lmax,E,periodic,n,n_owned,r_cut", [
    (0, 8, False, 40, 40, 4.0), (1, 16, True, 120, 120, 4.0), (2, 32, False, 100, 60, 4.0), (3, 8, True, 150, 90, 4.0),
    (4, 16, False, 70, 70, 4.0), (4, 32, False, 90, 50, 4.0), (2, 64, False, 60, 40, 4.0),
    # many incoming edges per node, more than 448 edges in all (several row blocks of the GEMM, ragged tail)
    (3, 16, False, 330, 12, 9.5), (1, 128, False, 40, 25, 4.0)])
def test_so2_message_sum_small(B, lmax, E, periodic, n, n_owned, r_cut):
    print("case", lmax, E, periodic, n, n_owned, r_cut, flush=True)
    w = synth.small_cluster(n, n_owned, lmax, E, 6, r_cut, 50 + lmax, periodic)
    a, ref, n_e = run_case(B, w)
    assert n_e > 0 and np.abs(ref).max() > 0.05
    e = U.rel_err(a, ref)
    print(f"  {n_e} edges, rel err {e:.2e}", flush=True)
    assert e < TOL


def test_so2_message_sum_config1(B):
    w = synth.workload(1)
    a, ref, n_e = run_case(B, w)
    e = U.rel_err(a, ref)
    print(f"config 1: {n_e} edges, rel err {e:.2e}", flush=True)
    assert e < TOL


def test_so2_message_sum_empty_graph_and_errors(B):
    import torch
    w = synth.small_cluster(5, 5, 2, 8, 6, 0.5, 3)          # cutoff shorter than any distance: no edges
    g = U.oracle_graph(w)
    assert len(g[0]) == 0
    a, ref, _ = run_case(B, w)
    assert a.shape == ref.shape and np.all(a == 0.0)
    m = B.Egnn(2, 8, 6, 4.0, 1.0)
    w2 = synth.small_cluster(30, 30, 2, 8, 6, 4.0, 4)
    graph = m.egnn_nlist(B.to_device(w2.pos), 30, w2.box, w2.pbc)
    x = torch.zeros((30, 9, 8), device="cuda")
    We = torch.zeros((8, 6), device="cuda")
    Wf = torch.zeros(m.egnn_so2_weight_count(), device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.EgnnError) as err:
        m.egnn_so2_message_sum(graph, B.to_device(w2.pos), w2.box, x, We, Wf, small)
    assert err.value.code == -3        # workspace too small
