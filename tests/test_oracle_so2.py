"""Pins of the SO(2) message oracle (oracle/so2_oracle.py) against what the mathematics fixes."""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from oracle import so2_oracle as S
from paper_2507_03840_amd import synth


def _rot(rng):
    q, _ = np.linalg.qr(rng.standard_normal((3, 3)))
    return q * np.sign(np.linalg.det(q))


def _setup(lmax, E, n=14, n_owned=9, n_rbf=6, r_cut=4.0, seed=0):
    w = synth.small_cluster(n, n_owned, lmax, E, n_rbf, r_cut, seed)
    g = O.neighbour_list(w.pos, w.n_owned, w.box, w.pbc, w.r_cut)
    rng = np.random.default_rng(100 + seed)
    x = rng.standard_normal((n, (lmax + 1) ** 2, E))
    shapes = S.so2_shapes(lmax, E)
    W0 = rng.standard_normal(shapes[0]) / np.sqrt(shapes[0][1])
    Wr = [rng.standard_normal(s) / np.sqrt(2 * s[1]) for s in shapes[1:]]
    Wi = [rng.standard_normal(s) / np.sqrt(2 * s[1]) for s in shapes[1:]]
    W_e = rng.standard_normal((E, n_rbf)) / np.sqrt(n_rbf)
    return w, g, x, W_e, W0, Wr, Wi


def test_wigner_blocks_definition_and_component_convention():
    rng = np.random.default_rng(1)
    lmax = 4
    R = np.stack([_rot(rng) for _ in range(3)])
    D = S.wigner_blocks(lmax, R)
    for k in range(3):
        assert np.allclose(D[k], O.wigner_d_block(lmax, R[k]), atol=1e-11)          # same definition, other sample set
        assert np.allclose(D[k] @ D[k].T, np.eye((lmax + 1) ** 2), atol=1e-11)      # real orthogonal
    # homomorphism
    assert np.allclose(S.wigner_blocks(lmax, (R[0] @ R[1])[None])[0], D[0] @ D[1], atol=1e-10)
    # a rotation about z by a turns (x_{+m}, x_{-m}) by the angle m a and leaves m = 0 alone
    a = 0.37
    Rz = np.array([[np.cos(a), -np.sin(a), 0], [np.sin(a), np.cos(a), 0], [0, 0, 1.0]])
    Dz = S.wigner_blocks(lmax, Rz[None])[0]
    expect = np.zeros_like(Dz)
    for l in range(lmax + 1):
        c = l * l + l
        expect[c, c] = 1.0
        for m in range(1, l + 1):
            expect[c + m, c + m] = expect[c - m, c - m] = np.cos(m * a)
            expect[c + m, c - m] = np.sin(m * a) * (Dz[c + m, c - m] > 0) - np.sin(m * a) * (Dz[c + m, c - m] < 0)
            expect[c - m, c + m] = -expect[c + m, c - m]
    assert np.allclose(Dz, expect, atol=1e-11)
    # the sense of the turn is the same for every (l, m): one sign
    signs = {np.sign(Dz[l * l + l + m, l * l + l - m]) for l in range(1, lmax + 1) for m in range(1, l + 1)}
    assert len(signs) == 1


def test_bond_rotations_take_the_bond_to_z():
    rng = np.random.default_rng(2)
    v = rng.standard_normal((20, 3))
    v[0] = [0, 0, 1.0]
    v[1] = [0, 0, -1.0]
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    R = S.bond_rotations(v, gauge=rng.uniform(0, 6, 20))
    assert np.allclose(np.einsum("kab,kb->ka", R, v), np.tile([0, 0, 1.0], (20, 1)), atol=1e-12)
    assert np.allclose(np.einsum("kab,kcb->kac", R, R), np.tile(np.eye(3), (20, 1, 1)), atol=1e-12)
    assert np.allclose(np.linalg.det(R), 1.0)


@pytest.mark.parametrize("lmax", [1, 3])
def test_so2_gauge_independence(lmax):
    """Any rotation that takes the bond to z gives the same message: the layer commutes with turns about z."""
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, 3)
    a0 = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, 3, w.n_rbf, w.r_cut, 7.0)
    gauge = np.random.default_rng(5).uniform(0, 2 * np.pi, len(g[0]))
    a1 = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, 3, w.n_rbf, w.r_cut, 7.0, gauge=gauge)
    assert np.abs(a0).max() > 0.1
    assert np.allclose(a0, a1, atol=1e-11)


def test_so2_gauge_dependence_if_structure_is_broken():
    """Control for the test above: weights without the (Wr, Wi) structure do depend on the gauge."""
    lmax, E = 2, 2
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E)
    src, dst, shift, _ = g
    r = O.edge_vectors(w.pos, w.box, src, dst, shift)
    d = np.linalg.norm(r, axis=1)
    x = np.asarray(x)

    def broken(gauge):
        D = S.wigner_blocks(lmax, S.bond_rotations(r / d[:, None], gauge))
        M = np.concatenate([x[src], x[dst], np.zeros_like(x[src])], axis=2)
        Xp = np.einsum("kab,kbc->kac", D, M)
        Yp = S.so2_linear(Xp, W0, Wr, Wi, lmax, E)
        Yp[:, 3, :] += Xp[:, 1, :E]        # y_{1,+1} += x_{1,-1} with no partner term: not of the allowed form
        return np.einsum("kba,kbc->kac", D, Yp)

    g0 = broken(None)
    g1 = broken(np.full(len(src), 0.8))
    assert np.abs(g0 - g1).max() > 1e-3


@pytest.mark.parametrize("lmax,E", [(2, 3), (4, 2)])
def test_so2_equivariance(lmax, E):
    """Rotating the structure and the features rotates the result (proper rotations, open boundaries)."""
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, seed=3)
    a = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, w.n_rbf, w.r_cut, 5.0)
    Q = _rot(np.random.default_rng(9))
    DQ = O.wigner_d_block(lmax, Q)
    pos2 = (w.pos.astype(np.float64) @ Q.T)
    g2 = O.neighbour_list(pos2.astype(np.float32), w.n_owned, w.box, w.pbc, w.r_cut)
    assert np.array_equal(g2[0], g[0]) and np.array_equal(g2[1], g[1])
    a2 = S.so2_message_sum(g2, pos2.astype(np.float32), w.box, np.einsum("ab,nbc->nac", DQ, x), W_e, W0, Wr, Wi,
                           lmax, E, w.n_rbf, w.r_cut, 5.0)
    scale = np.abs(a).max()
    assert scale > 0.1
    assert np.abs(a2 - np.einsum("ab,nbc->nac", DQ, a)).max() < 2e-6 * scale      # positions went through fp32


def test_so2_lmax0_is_a_plain_linear_layer():
    lmax, E = 0, 5
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, seed=4)
    src, dst, shift, row_ptr = g
    a = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, [], [], lmax, E, w.n_rbf, w.r_cut, 3.0)
    r = O.edge_vectors(w.pos, w.box, src, dst, shift)
    d = np.linalg.norm(r, axis=1)
    ref = np.zeros((w.n_owned, 1, E))
    for k in range(len(src)):
        msg = np.concatenate([x[src[k], 0], x[dst[k], 0], W_e @ O.radial_basis(d[k:k + 1], w.n_rbf, w.r_cut)[0]])
        ref[dst[k], 0] += 0.5 * (1 + np.cos(np.pi * d[k] / w.r_cut)) * (W0 @ msg)
    assert np.allclose(a, ref / np.sqrt(3.0), atol=1e-12)


@pytest.mark.parametrize("lmax", [1, 2, 3])
def test_so2_layer_with_coupling_weights_is_the_tensor_product(lmax):
    """Sec. 2.1: aligned with the bond, the Clebsch-Gordan product with the harmonics of the bond direction becomes a
    linear layer per m.  With the weights of that layer read off the coupling coefficients (harmonics of z have only
    m = 0), the SO(2) oracle must reproduce the tensor-product oracle -- rotations, m indexing and signs included."""
    E = 3
    w, g, x, _, _, _, _ = _setup(lmax, E, seed=6)
    rng = np.random.default_rng(11)
    paths = O.tp_paths(lmax, lmax, lmax)
    wp = rng.standard_normal((len(paths), E))                     # one weight per (path, channel), same for all edges
    shapes = S.so2_shapes(lmax, E)
    W0 = np.zeros(shapes[0])
    Wr = [np.zeros(s) for s in shapes[1:]]
    Wi = [np.zeros(s) for s in shapes[1:]]
    for p, (l1, l2, l3) in enumerate(paths):
        T = O.cg_real(l1, l2, l3)[:, l2, :] * np.sqrt(2 * l2 + 1)    # [m1][m3]: coupling with Yhat_{l2}(z)
        for m1 in range(-l1, l1 + 1):
            for m3 in range(-l3, l3 + 1):
                if abs(m1) != abs(m3):
                    assert abs(T[l1 + m1, l3 + m3]) < 1e-14
        for c in range(E):
            W0[l3 * E + c, l1 * 3 * E + c] += wp[p, c] * T[l1, l3]
            for m in range(1, min(l1, l3) + 1):
                a, b = T[l1 + m, l3 + m], T[l1 + m, l3 - m]           # x_{+m} -> y_{+m},  x_{+m} -> y_{-m}
                assert abs(T[l1 - m, l3 - m] - a) < 1e-14 and abs(T[l1 - m, l3 + m] + b) < 1e-14
                Wr[m - 1][(l3 - m) * E + c, (l1 - m) * 3 * E + c] += wp[p, c] * a
                Wi[m - 1][(l3 - m) * E + c, (l1 - m) * 3 * E + c] += wp[p, c] * b
    W_e = np.zeros((E, w.n_rbf))
    a_so2 = S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, w.n_rbf, w.r_cut, 4.0)
    fn = lambda d, k0, k1, pl: O.envelope(d, w.r_cut)[:, None, None] * wp[None]
    a_tp = O.edge_messages_sum(g, w.pos, w.box, x, fn, lmax, lmax, 4.0)
    assert np.abs(a_tp).max() > 0.1
    assert np.allclose(a_so2, a_tp, atol=1e-11)


def test_so2_pack_order():
    lmax, E = 2, 2
    shapes = S.so2_shapes(lmax, E)
    assert shapes == [(6, 18), (4, 12), (2, 6)]
    W0 = np.arange(6 * 18).reshape(6, 18)
    Wr = [np.full(s, 10.0 + i) for i, s in enumerate(shapes[1:])]
    Wi = [np.full(s, 20.0 + i) for i, s in enumerate(shapes[1:])]
    flat = S.so2_pack(W0, Wr, Wi)
    assert flat.dtype == np.float32 and flat.size == 108 + 2 * 48 + 2 * 12
    assert flat[19] == 19 and flat[108] == 10 and flat[108 + 48] == 20 and flat[108 + 96] == 11 and flat[-1] == 21


def test_message_sum_backward_is_the_derivative_of_the_forward():
    """Central differences of L = <a, da> along random directions of every argument (the map is linear in x and in each
    weight group, so the difference quotient is exact up to rounding), and one entry of every group on its own."""
    lmax, E, n_rbf, r_cut, agg = 3, 4, 6, 4.0, 5.0
    w, g, x, W_e, W0, Wr, Wi = _setup(lmax, E, n_rbf=n_rbf, r_cut=r_cut, seed=3)
    rng = np.random.default_rng(9)
    da = rng.standard_normal((w.n_owned, (lmax + 1) ** 2, E))

    def loss(x=x, W_e=W_e, W0=W0, Wr=Wr, Wi=Wi):
        return float((S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, agg) * da).sum())

    dx, dW_e, dW0, dWr, dWi = S.so2_message_sum_backward(g, w.pos, w.box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, agg, da)
    assert dx.shape == x.shape and dW_e.shape == W_e.shape and dW0.shape == W0.shape
    h = 1e-3

    def check(grad, name, make):
        v = rng.standard_normal(grad.shape)
        fd = (loss(**{name: make(+h * v)}) - loss(**{name: make(-h * v)})) / (2 * h)
        assert fd == pytest.approx(float((grad * v).sum()), rel=1e-8, abs=1e-9), name
        # one entry alone: a misplaced index that a random direction could average out
        idx = tuple(rng.integers(0, s) for s in grad.shape)
        e = np.zeros(grad.shape)
        e[idx] = 1.0
        fd = (loss(**{name: make(+h * e)}) - loss(**{name: make(-h * e)})) / (2 * h)
        assert fd == pytest.approx(float(grad[idx]), rel=1e-8, abs=1e-9), (name, idx)

    check(dx, "x", lambda t: x + t)
    check(dW_e, "W_e", lambda t: W_e + t)
    check(dW0, "W0", lambda t: W0 + t)
    for m in range(lmax):
        check(dWr[m], "Wr", lambda t, m=m: [a + (t if i == m else 0) for i, a in enumerate(Wr)])
        check(dWi[m], "Wi", lambda t, m=m: [a + (t if i == m else 0) for i, a in enumerate(Wi)])
    # halo atoms receive a gradient through the source side only; an atom with no edge at all receives none
    src = g[0]
    untouched = np.setdiff1d(np.arange(len(x)), np.concatenate([src, g[1]]))
    assert np.all(dx[untouched] == 0)
