"""Pins of the node block, edge block, attention and gate of oracle/so2_oracle.py."""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from oracle import so2_oracle as S
from tests.test_oracle_so2 import _rot, _setup


def _edge_lengths(w, g):
    r = O.edge_vectors(w.pos, w.box, g[0], g[1], g[2])
    return r, np.sqrt((r * r).sum(axis=1))


def test_initial_edge_embedding_reproduces_the_message_sum():
    """With T_edge = its initial value (L = 0 plane W_e B(d), zeros elsewhere) the full-content messages are the ones
    of so2_message_sum (which is pinned to the Clebsch-Gordan product)."""
    lmax, E, n_rbf, r_cut = 3, 4, 6, 4.0
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E)
    r, d = _edge_lengths(w, g)
    T = S.edge_embedding_init(d, W_e, lmax, E, n_rbf, r_cut)
    assert np.all(T[:, 1:, :] == 0) and np.allclose(T[:, 0, :], O.radial_basis(d, n_rbf, r_cut) @ W_e.T)
    Y_old = S.so2_messages(g[0], g[1], r, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut)
    Y_new = S.so2_messages(g[0], g[1], r, x, None, W0, Wr, Wi, lmax, E, 0, r_cut, T_edge=T)
    assert np.allclose(Y_old, Y_new, atol=1e-13)
    # uniform attention (w_att = 0): the node block is the plain mean, i.e. the message sum rescaled per node
    a_sum = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, 1.0)
    a_att = S.so2_node_block(g, w.pos, w.box, x, T, W0, Wr, Wi, np.zeros(E), lmax, E, r_cut)
    deg = np.diff(g[3]).astype(float)
    assert deg.min() > 0 and np.allclose(a_att * deg[:, None, None], a_sum, atol=1e-12)


def test_attention_weights_closed_forms():
    rng = np.random.default_rng(3)
    E = 5
    w_att = rng.standard_normal(E)
    y0 = rng.standard_normal((7, E))
    row_ptr = np.array([0, 2, 2, 7])
    al = S.attention_weights(y0, w_att, row_ptr)
    lrelu = lambda t: np.where(t > 0, t, 0.2 * t)
    s = lrelu(y0) @ w_att
    # two edges: a logistic function of the score difference
    assert al[0] == pytest.approx(1.0 / (1.0 + np.exp(s[1] - s[0])), abs=1e-14) and al[0] + al[1] == pytest.approx(1.0)
    assert al[2:].sum() == pytest.approx(1.0) and np.all(al > 0)
    assert np.allclose(al[2:] / al[2], np.exp(s[2:] - s[2]), atol=1e-13)
    # adding a constant to all scores of a node changes nothing; very large scores do not overflow
    big = S.attention_weights(y0 * 1e4, w_att, row_ptr)
    assert np.all(np.isfinite(big)) and big[:2].sum() == pytest.approx(1.0)
    # negative inputs are scaled by 0.2
    one = S.attention_weights(np.array([[-1.0], [0.0]]), np.array([1.0]), np.array([0, 2]))
    assert one[0] == pytest.approx(1.0 / (1.0 + np.exp(0.2)))


@pytest.mark.parametrize("lmax", [1, 3])
def test_blocks_are_equivariant(lmax):
    """Rotating positions, node embeddings and edge embeddings rotates the outputs of both blocks; the attention
    weights are invariant."""
    E, r_cut = 4, 4.0
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, seed=2)
    rng = np.random.default_rng(7)
    T = rng.standard_normal((len(g[0]), (lmax + 1) ** 2, E))
    w_att = rng.standard_normal(E)
    R = _rot(rng)
    Dm = O.wigner_d_block(lmax, R)
    c = w.pos.astype(np.float64).mean(axis=0)
    pos2 = ((w.pos.astype(np.float64) - c) @ R.T + c).astype(np.float32)
    x2 = np.einsum("ab,nbc->nac", Dm, x)
    T2 = np.einsum("ab,nbc->nac", Dm, T)
    g2 = O.neighbour_list(pos2, w.n_owned, w.box, w.pbc, r_cut)
    if not (np.array_equal(g2[0], g[0]) and np.array_equal(g2[1], g[1])):
        pytest.skip("rounding of the rotated positions moved a pair across the cutoff")
    a1 = S.so2_node_block(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut)
    a2 = S.so2_node_block(g2, pos2, w.box, x2, T2, W0, Wr, Wi, w_att, lmax, E, r_cut)
    assert np.allclose(a2, np.einsum("ab,nbc->nac", Dm, a1), atol=2e-6 * np.abs(a1).max())
    t1 = S.so2_edge_block(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut)
    t2 = S.so2_edge_block(g2, pos2, w.box, x2, T2, W0, Wr, Wi, lmax, E, r_cut)
    assert np.allclose(t2, np.einsum("ab,nbc->nac", Dm, t1), atol=2e-6 * np.abs(t1).max())
    assert np.abs(a1).max() > 1e-2 and np.abs(t1 - T).max() > 1e-2


def test_edge_embedding_enters_every_degree():
    """A change of T_edge in degree l changes the message: the edge slot of the weights is read for every l."""
    lmax, E, r_cut = 2, 4, 4.0
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, seed=4)
    rng = np.random.default_rng(8)
    T = rng.standard_normal((len(g[0]), 9, E))
    base = S.so2_edge_block(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut)
    for l in range(lmax + 1):
        T2 = T.copy()
        T2[:, O.sl(l), :] += 1.0
        assert np.abs(S.so2_edge_block(g, w.pos, w.box, x, T2, W0, Wr, Wi, lmax, E, r_cut) - base - (T2 - T)).max() > 1e-3
    # zero weights: the block is the identity; k_range gives the same rows
    Z0, Zr, Zi = np.zeros_like(W0), [np.zeros_like(a) for a in Wr], [np.zeros_like(a) for a in Wi]
    assert np.array_equal(S.so2_edge_block(g, w.pos, w.box, x, T, Z0, Zr, Zi, lmax, E, r_cut), T)
    assert np.array_equal(S.so2_edge_block(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, k_range=(3, 9)), base[3:9])
    # nodes= gives the same rows of the node block
    w_att = rng.standard_normal(E)
    a = S.so2_node_block(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut)
    assert np.array_equal(S.so2_node_block(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut, nodes=[5, 1]), a[[5, 1]])


def test_gate_closed_forms_and_equivariance():
    rng = np.random.default_rng(9)
    lmax, E = 3, 5
    x = rng.standard_normal((6, 16, E))
    W_g = rng.standard_normal((lmax, E, E))
    y = S.gate(x, W_g, lmax)
    assert np.allclose(y[:, 0, :], x[:, 0, :] / (1 + np.exp(-x[:, 0, :])))
    # zero scalars: every higher degree is halved, the scalar plane stays zero
    x0 = x.copy(); x0[:, 0, :] = 0
    y0 = S.gate(x0, W_g, lmax)
    assert np.allclose(y0[:, 1:, :], 0.5 * x0[:, 1:, :]) and np.all(y0[:, 0, :] == 0)
    # the gate of (degree l, channel c) is sigmoid(sum_c' W_g[l-1][c][c'] x[0][c'])
    n, l, c = 2, 2, 3
    gate = 1 / (1 + np.exp(-(W_g[l - 1][c] @ x[n, 0, :])))
    assert np.allclose(y[n, O.sl(l), c], x[n, O.sl(l), c] * gate)
    Dm = O.wigner_d_block(lmax, _rot(rng))
    assert np.allclose(S.gate(np.einsum("ab,nbc->nac", Dm, x), W_g, lmax), np.einsum("ab,nbc->nac", Dm, y), atol=1e-12)


def _fd_check(loss, grads, values, rng, h=1e-4, rel=2e-7):
    """Central differences of a scalar loss along a random direction and along one entry of every argument.
    grads / values: dicts by argument name (a value may be a list of arrays: then one member at a time)."""
    for name, grad in grads.items():
        members = list(range(len(grad))) if isinstance(grad, list) else [None]
        for mem in members:
            g = grad[mem] if mem is not None else grad
            base = values[name][mem] if mem is not None else values[name]

            def moved(t):
                if mem is None:
                    return {name: base + t}
                return {name: [v + (t if i == mem else 0) for i, v in enumerate(values[name])]}

            v = rng.standard_normal(g.shape)
            idx = tuple(rng.integers(0, s) for s in g.shape)
            e = np.zeros(g.shape)
            e[idx] = 1.0
            for direction, expect in ((v, float((g * v).sum())), (e, float(g[idx]))):
                fd = (loss(**moved(h * direction)) - loss(**moved(-h * direction))) / (2 * h)
                assert fd == pytest.approx(expect, rel=rel, abs=1e-8), (name, mem)


def _block_setup(lmax, E, seed):
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, seed=seed)
    rng = np.random.default_rng(40 + seed)
    T = rng.standard_normal((len(g[0]), (lmax + 1) ** 2, E))
    return w, g, x, T, W0, Wr, Wi, rng


def test_edge_block_backward_is_the_derivative_of_the_forward():
    lmax, E, r_cut = 2, 4, 4.0
    w, g, x, T, W0, Wr, Wi, rng = _block_setup(lmax, E, 5)
    dT_out = rng.standard_normal(T.shape)
    vals = dict(x=x, T=T, W0=W0, Wr=Wr, Wi=Wi)

    def loss(**kw):
        a = dict(vals, **kw)
        return float((S.so2_edge_block(g, w.pos, w.box, a["x"], a["T"], a["W0"], a["Wr"], a["Wi"], lmax, E, r_cut) * dT_out).sum())

    dx, dT_in, dW0, dWr, dWi = S.so2_edge_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, dT_out)
    # the map is linear in (x, T) and in each weight group: the difference quotient is exact up to rounding
    _fd_check(loss, dict(x=dx, T=dT_in, W0=dW0, Wr=dWr, Wi=dWi), vals, rng, h=1e-3, rel=1e-8)
    # zero weights: the block is the identity on T, and so is its adjoint
    z = S.so2_edge_block_backward(g, w.pos, w.box, x, T, 0 * W0, [0 * a for a in Wr], [0 * a for a in Wi], lmax, E, r_cut, dT_out)
    assert np.array_equal(z[1], dT_out) and not z[0].any()


def test_node_block_backward_is_the_derivative_of_the_forward():
    lmax, E, r_cut = 2, 4, 4.0
    w, g, x, T, W0, Wr, Wi, rng = _block_setup(lmax, E, 6)
    w_att = rng.standard_normal(E)
    da = rng.standard_normal((w.n_owned, (lmax + 1) ** 2, E))
    vals = dict(x=x, T=T, W0=W0, Wr=Wr, Wi=Wi, w_att=w_att)

    def loss(**kw):
        a = dict(vals, **kw)
        return float((S.so2_node_block(g, w.pos, w.box, a["x"], a["T"], a["W0"], a["Wr"], a["Wi"], a["w_att"], lmax, E,
                                       r_cut) * da).sum())

    dx, dT, dW0, dWr, dWi, dw_att = S.so2_node_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut, da)
    # not linear (softmax, LeakyReLU): small steps; a kink of the LeakyReLU inside a step would show as a 1e-4 mismatch
    _fd_check(loss, dict(x=dx, T=dT, W0=dW0, Wr=dWr, Wi=dWi, w_att=dw_att), vals, rng, h=1e-5, rel=2e-6)
    # with w_att = 0 the weights are 1 / degree whatever the messages: no gradient flows through the scores
    dx0, dT0, *_rest, dw0 = S.so2_node_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, 0 * w_att, lmax, E, r_cut, da)
    deg = np.diff(g[3])
    gY_scale = np.repeat(1.0 / deg, deg)
    lin = S.so2_edge_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, da[g[1]] * gY_scale[:, None, None])
    assert np.allclose(dx0, lin[0], atol=1e-12) and np.allclose(dT0, lin[1] - da[g[1]] * gY_scale[:, None, None], atol=1e-12)
    assert np.abs(dw0).max() > 0          # (the scores still depend on w_att to first order)


def test_gate_backward_is_the_derivative_of_the_forward():
    lmax, E = 3, 5
    rng = np.random.default_rng(11)
    x = rng.standard_normal((6, (lmax + 1) ** 2, E))
    W_g = rng.standard_normal((lmax, E, E)) / np.sqrt(E)
    dy = rng.standard_normal(x.shape)
    vals = dict(x=x, W_g=W_g)

    def loss(**kw):
        a = dict(vals, **kw)
        return float((S.gate(a["x"], a["W_g"], lmax) * dy).sum())

    dx, dW = S.gate_backward(x, W_g, lmax, dy)
    _fd_check(loss, dict(x=dx, W_g=dW), vals, rng, h=1e-5, rel=1e-6)
    # lmax = 0: SiLU alone, derivative sigma(x) (1 + x (1 - sigma(x)))
    x0 = rng.standard_normal((4, 1, E))
    d0, _ = S.gate_backward(x0, np.zeros((0, E, E)), 0, np.ones_like(x0))
    s = 1 / (1 + np.exp(-x0))
    assert np.allclose(d0, s * (1 + x0 * (1 - s)), atol=1e-14)


def test_layer_step_chain_is_the_derivative_of_the_loss():
    """The chain of adjoints that the GPU training-step test compares against (tests/gpu_util.oracle_so2_layer_step):
    central differences of the composed loss with respect to x, T and one weight of every group."""
    from tests import gpu_util as U
    lmax, E = 2, 4
    w, g, x, T, W0, Wr, Wi, rng = _block_setup(lmax, E, 8)
    Wn = (None, W0, Wr, Wi)
    We = (None,) + tuple(S_ for S_ in (rng.standard_normal(W0.shape) / 6, [rng.standard_normal(a.shape) / 6 for a in Wr],
                                       [rng.standard_normal(a.shape) / 6 for a in Wi]))
    w_att = rng.standard_normal(E)
    W_g = rng.standard_normal((lmax, E, E)) / 2
    th = rng.standard_normal((w.n_owned, (lmax + 1) ** 2, E))
    tT = rng.standard_normal(T.shape)
    loss, gr = U.oracle_so2_layer_step(w, g, x, T, Wn, We, w_att, W_g, th, tT)
    h = 1e-5

    def fd(make):
        return (U.oracle_so2_layer_step(*make(+h), grads=False) - U.oracle_so2_layer_step(*make(-h), grads=False)) / (2 * h)

    v = rng.standard_normal(x.shape)
    assert fd(lambda t: (w, g, x + t * v, T, Wn, We, w_att, W_g, th, tT)) == pytest.approx((gr["x"] * v).sum(), rel=1e-6)
    v = rng.standard_normal(T.shape)
    assert fd(lambda t: (w, g, x, T + t * v, Wn, We, w_att, W_g, th, tT)) == pytest.approx((gr["T"] * v).sum(), rel=1e-6)
    v = rng.standard_normal(W0.shape)
    assert fd(lambda t: (w, g, x, T, (None, W0 + t * v, Wr, Wi), We, w_att, W_g, th, tT)) == pytest.approx(
        (gr["Wn"][0] * v).sum(), rel=1e-6)
    v = rng.standard_normal(We[2][0].shape)
    assert fd(lambda t: (w, g, x, T, Wn, (None, We[1], [We[2][0] + t * v] + list(We[2][1:]), We[3]), w_att, W_g, th,
                         tT)) == pytest.approx((gr["We"][1][0] * v).sum(), rel=1e-6)
    v = rng.standard_normal(E)
    assert fd(lambda t: (w, g, x, T, Wn, We, w_att + t * v, W_g, th, tT)) == pytest.approx((gr["w_att"] * v).sum(), rel=1e-6)
    v = rng.standard_normal(W_g.shape)
    assert fd(lambda t: (w, g, x, T, Wn, We, w_att, W_g + t * v, th, tT)) == pytest.approx((gr["W_g"] * v).sum(), rel=1e-6)


def test_chunks_node_subsets_and_edge_ranges_do_not_change_the_results():
    """The oracle walks the edges in chunks, and the full-size tests ask it for a few destination nodes or a range of
    edges only: every such call returns the rows of the one-piece result."""
    lmax, E, r_cut, n_rbf = 2, 3, 4.0, 6
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, n=16, n_owned=11, seed=9)
    rng = np.random.default_rng(2)
    n_e = len(g[0])
    assert n_e > 40
    T = rng.standard_normal((n_e, (lmax + 1) ** 2, E))
    w_att = rng.standard_normal(E)
    # message sum: chunks of 7 edges, and a subset of nodes (one of them asked for twice)
    a = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, 3.0)
    a7 = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, 3.0, chunk=7)
    nodes = [10, 0, 4, 4]
    an = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, 3.0, nodes=nodes)
    assert np.abs(a7 - a).max() < 1e-13 and an.shape == (4,) + a.shape[1:] and np.abs(an - a[nodes]).max() < 1e-13
    assert np.abs(a[nodes]).min(axis=(1, 2)).max() > 0
    # its adjoint in chunks of 7 edges
    da = rng.standard_normal(a.shape)
    full = S.so2_message_sum_backward(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, 3.0, da)
    part = S.so2_message_sum_backward(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, 3.0, da, chunk=7)
    flat = lambda t: np.concatenate([np.ravel(v) for v in (t if isinstance(t, (list, tuple)) else [t])])
    for u, v in zip(full, part):
        assert np.abs(flat(u) - flat(v)).max() < 1e-12 * max(1.0, np.abs(flat(u)).max())
    # node block on a subset of nodes; edge block in chunks and on a range of edges
    nb = S.so2_node_block(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut)
    nbn = S.so2_node_block(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut, nodes=nodes)
    assert np.abs(nbn - nb[nodes]).max() < 1e-13
    eb = S.so2_edge_block(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut)
    eb7 = S.so2_edge_block(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, chunk=7)
    ebr = S.so2_edge_block(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, k_range=(13, 37), chunk=5)
    assert np.abs(eb7 - eb).max() < 1e-13 and ebr.shape[0] == 24 and np.abs(ebr - eb[13:37]).max() < 1e-13
    dT_out = rng.standard_normal(T.shape)
    full = S.so2_edge_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, dT_out)
    part = S.so2_edge_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, lmax, E, r_cut, dT_out, chunk=7)
    for u, v in zip(full, part):
        assert np.abs(flat(u) - flat(v)).max() < 1e-12 * max(1.0, np.abs(flat(u)).max())


def test_near_kink_lists_the_edges_whose_score_inputs_are_within_the_margin():
    """so2_node_block_backward reports the edges with a scalar message channel closer to zero than kink_eps (where
    LeakyReLU' is a discrete decision): checked against the scalar channels of the messages themselves."""
    lmax, E, r_cut = 1, 4, 4.0
    w, g, x, T, W0, Wr, Wi, rng = _block_setup(lmax, E, 8)
    w_att = rng.standard_normal(E)
    da = rng.standard_normal((w.n_owned, (lmax + 1) ** 2, E))
    src, dst, shift, row_ptr = g
    r = O.edge_vectors(w.pos, w.box, src, dst, shift)
    y0 = S.so2_messages(src, dst, r, x, None, W0, Wr, Wi, lmax, E, 0, r_cut, T_edge=T, envelope=False)[:, 0, :]
    eps = float(np.sort(np.abs(y0).min(axis=1))[5]) * 1.0001      # six edges fall inside the margin
    want = np.nonzero((np.abs(y0) < eps).any(axis=1))[0].tolist()
    got = []
    S.so2_node_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut, da, near_kink=got, kink_eps=eps)
    assert sorted(got) == want and len(want) == 6 and max(want) > row_ptr[1]
    none = []
    S.so2_node_block_backward(g, w.pos, w.box, x, T, W0, Wr, Wi, w_att, lmax, E, r_cut, da, near_kink=none, kink_eps=0.0)
    assert none == []
