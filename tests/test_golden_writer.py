"""The stored full-size oracle values come from tests/golden/make_golden.py, which spreads the oracle's loops over
processes.  These CPU tests check, on config 1 with chunk sizes small enough that every loop has several chunks and
a ragged last one, that the chains composed there equal the oracle's own composite calls."""
import importlib.util
import os
import sys

import numpy as np

from oracle import egnn_oracle as O
from paper_2507_03840_amd import synth
from tests import gpu_util as U

_spec = importlib.util.spec_from_file_location(
    "make_golden", os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "make_golden.py"))
MG = importlib.util.module_from_spec(_spec)
sys.modules["make_golden"] = MG          # worker processes unpickle its functions by this name
_spec.loader.exec_module(MG)


def _config1():
    w = synth.workload(1)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    return w, wt, g, U.mean_degree(g, w.n_owned)


def test_parallel_layer_and_readout_equal_the_oracle_calls(monkeypatch):
    w, wt, g, agg = _config1()
    monkeypatch.setattr(MG, "CHUNK", 10)           # 64 nodes -> 7 chunks, the last of 4
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    y = MG.layer_parallel(2, w, g, x, wt["layers"][0], agg)
    ref = O.layer_forward(g, w.pos, w.box, x, wt["layers"][0], w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, agg)
    assert np.abs(y - ref).max() <= 1e-13 * np.abs(ref).max()
    xs_ref, H_ref = U.oracle_forward(w, wt, g, agg)
    assert np.array_equal(xs_ref[0], ref)
    MG._state.update(w=w, g=g, x=y, Wr=wt["readout"])
    for k in (0, 17, len(g[0]) - 1):
        k0, part = MG._readout_chunk((k, k + 1))
        assert k0 == k and np.abs(part[0] - H_ref[k]).max() <= 1e-13 * np.abs(H_ref).max()


def test_parallel_training_chain_equals_the_oracle_training_step(monkeypatch):
    w, wt, g, agg = _config1()
    monkeypatch.setattr(MG, "CHUNK", 10)
    monkeypatch.setattr(MG, "EDGE_CHUNK", 300)     # 1,384 edges -> 5 chunks, the last of 184
    T = synth.normal(np.random.default_rng([w.seed, 99]), (len(g[0]), w.n_orb, w.n_orb))
    got = MG.training_parallel(2, w, wt, g, agg, T)
    ref = U.oracle_training_step(w, wt, g, agg, T)
    assert abs(got["loss"] / ref["loss"] - 1) < 1e-13
    assert set(got["grads"]) == set(ref["grads"])
    for k, v in ref["grads"].items():
        assert np.abs(got["grads"][k] - v).max() <= 1e-13 * max(np.abs(v).max(), 1e-300), k


def test_aimed_samples_cover_the_rows_named():
    w = synth.small_cluster(90, 50, 2, 4, 6, 4.0, 3, False)
    g = O.neighbour_list(w.pos, w.n_owned, w.box, w.pbc, w.r_cut)
    rng = np.random.default_rng(0)
    nodes = MG.aimed_nodes(w, g, rng, w.n_owned)
    deg = np.diff(g[3])
    for j in (0, w.n_owned - 1, int(np.argmin(deg)), int(np.argmax(deg)), int(np.argmin(w.pos[:w.n_owned, 2])),
              int(np.argmax(w.pos[:w.n_owned, 0]))):
        assert j in nodes
    assert nodes.max() < w.n_owned and len(np.unique(nodes)) == len(nodes)
    rows = MG.aimed_nodes(w, g, rng, w.n_total)
    assert w.n_owned in rows and w.n_total - 1 in rows
    edges = MG.aimed_edges(g, rng)
    n_e = len(g[0])
    assert 0 in edges and all(k in edges for k in range(n_e - 64, n_e)) and edges.max() == n_e - 1
    x = np.zeros((3, 9, 2)); x[1, 5, 1] = -7.0; x[2, 0, 0] = 2.0
    assert MG.maxabs_per_degree(x, 2).tolist() == [2.0, 0.0, 7.0]
    H = np.zeros((2, 4, 4)); H[1, 0, 3] = 5.0; H[0, 2, 0] = -3.0
    assert MG.maxabs_per_shell_block(H, [0, 1]).tolist() == [[0.0, 5.0], [3.0, 0.0]]


def _sum_parts(parts):
    total = None
    for p in parts:
        if total is None:
            total = [np.array(v, dtype=np.float64, copy=True) for v in p]
        else:
            for acc, v in zip(total, p):
                acc += v
    return total


def test_so2_backward_chunks_sum_to_the_oracle_adjoints(monkeypatch):
    """The writers of config3_so2_backward.npz and config3_so2_blocks_backward.npz split the adjoints over edge ranges
    (message sum, edge block) and destination-node ranges (node block) and add the parts up: on config 1 the sums equal
    the oracle's own calls over the whole graph."""
    from oracle import so2_oracle as S
    w, wt, g, agg = _config1()
    L, E = w.lmax, w.channels
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    Wso2 = synth.so2_weights(np.random.default_rng([w.seed, 777]), L, E, w.n_rbf)
    da = U.so2_da(w)
    n_e = len(g[0])
    # message sum: edge ranges with a ragged last one
    MG._state.update(w=w, g=g, x=x, Wso2=Wso2, agg=agg, da=da)
    parts = [MG._so2_backward_chunk((k0, min(n_e, k0 + 500))) for k0 in range(0, n_e, 500)]
    flat = _sum_parts([[p[0], p[1], p[2]] + list(p[3]) + list(p[4]) for p in parts])
    ref = S.so2_message_sum_backward(g, w.pos, w.box, x, *Wso2, L, E, w.n_rbf, w.r_cut, agg, da)
    ref_flat = [ref[0], ref[1], ref[2]] + list(ref[3]) + list(ref[4])
    for a, b in zip(flat, ref_flat):
        assert np.abs(a - b).max() <= 1e-12 * np.abs(b).max()
    # the two blocks
    gg, xb, T, Wn, We, w_att = U.block_inputs(w)
    edges = MG.aimed_edges(g, np.random.default_rng(1))
    dT_out = U.blocks_dT_out(w, n_e)
    MG._state.update(w=w, g=g, x=xb, T=T, Wn=Wn, We=We, w_att=w_att, da=da, dT_out=dT_out, edges=edges)
    node_parts = [MG._blocks_backward_nodes((j0, min(w.n_owned, j0 + 10))) for j0 in range(0, w.n_owned, 10)]
    ref = S.so2_node_block_backward(g, w.pos, w.box, xb, T, Wn[1], Wn[2], Wn[3], w_att, L, E, w.r_cut, da)
    dx = _sum_parts([[p[0]] for p in node_parts])[0]
    assert np.abs(dx - ref[0]).max() <= 1e-12 * np.abs(ref[0]).max()
    wsum = _sum_parts([p[2][:-1] for p in node_parts])          # (the last member lists the edges at the kink)
    for a, b in zip(wsum, [ref[2]] + list(ref[3]) + list(ref[4]) + [ref[5]]):
        assert np.abs(a - b).max() <= 1e-12 * np.abs(b).max()
    for pick, rows in (p[1] for p in node_parts):
        assert np.array_equal(rows, ref[1][pick])
    assert sorted(np.concatenate([p[1][0] for p in node_parts]).tolist()) == edges.tolist()
    monkeypatch.setattr(MG, "EDGE_PIECE", 120)     # several oracle calls per job, a ragged last one
    edge_parts = [MG._blocks_backward_edges((k0, min(n_e, k0 + 500))) for k0 in range(0, n_e, 500)]
    ref = S.so2_edge_block_backward(g, w.pos, w.box, xb, T, We[1], We[2], We[3], L, E, w.r_cut, dT_out)
    dx = _sum_parts([[p[0]] for p in edge_parts])[0]
    assert np.abs(dx - ref[0]).max() <= 1e-12 * np.abs(ref[0]).max()
    for a, b in zip(_sum_parts([p[2] for p in edge_parts]), [ref[2]] + list(ref[3]) + list(ref[4])):
        assert np.abs(a - b).max() <= 1e-12 * np.abs(b).max()
    for pick, rows in (p[1] for p in edge_parts):
        assert np.abs(rows - ref[1][pick]).max() <= 1e-13 * np.abs(ref[1]).max()
