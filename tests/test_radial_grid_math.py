"""The reverse pass of the radial MLP has a route that reads the weight gradients once: it bins the rows of dw on a
grid of distances with six-point Lagrange weights and finishes with two small products over the grid points
(paper_2507_03840_amd/csrc/radial_grid.hip).  This CPU test writes that reformulation out in numpy, on the oracle's own
functions, and checks it against oracle.radial_weights_backward: the identity holds to the interpolation error, which
must stay far below the parity bar for weights up to the size at which the library switches to the exact route."""
import numpy as np
import pytest

from oracle import egnn_oracle as O

BINS, PTS = 2048, 6          # the library's grid


def lagrange6(t):
    """Weights of the grid points -2 .. 3 at position t in [0, 1) of the interval [0, 1]."""
    offs = np.arange(-2, 4)
    w = np.ones((len(t), PTS))
    for a, oa in enumerate(offs):
        for ob in offs:
            if ob != oa:
                w[:, a] *= (t - ob) / (oa - ob)
    return w


def grid_route(d, dw, W_r1, W_r2, paths, E, n_rbf, r_cut):
    h = r_cut / BINS
    nodes = (np.arange(BINS + PTS - 1) - 2) * h                       # node i <-> distance (i - 2) h
    m = np.clip(np.floor(d / h).astype(int), 0, BINS - 1)
    phi = lagrange6(d / h - m)
    alpha = np.repeat(O.path_norm(paths), E)
    X = dw.reshape(len(d), -1) * alpha[None, :]
    Z = np.zeros((len(nodes), X.shape[1]))
    for i in range(PTS):
        np.add.at(Z, m + i, phi[:, i:i + 1] * X)
    B = O.radial_basis(nodes, n_rbf, r_cut)
    fc = O.envelope(nodes, r_cut)
    pre = B @ W_r1.T
    sig = 1.0 / (1.0 + np.exp(-pre))
    G = fc[:, None] * pre * sig
    S = fc[:, None] * sig * (1.0 + pre * (1.0 - sig))
    dW_r2 = Z.T @ G
    U = Z @ W_r2
    dW_r1 = np.einsum("ij,ib->jb", S * U, B)
    return dW_r1, dW_r2


@pytest.mark.parametrize("w1_scale,bar", [(1.0, 1e-10), (8.0, 1e-9), (48.0, 1e-6)])
def test_grid_route_equals_the_adjoint(w1_scale, bar):
    rng = np.random.default_rng(5)
    lmax, E, n_rbf, r_cut, n_e = 2, 4, 16, 10.0, 6000
    paths = O.tp_paths(lmax, lmax, lmax)
    d = r_cut * rng.uniform(0.01, 1.0, n_e) ** (1.0 / 3.0)          # edge lengths of a uniform density
    dw = rng.standard_normal((n_e, len(paths), E))
    W_r1 = rng.standard_normal((64, n_rbf)) / 4.0 * w1_scale
    W_r2 = rng.standard_normal((len(paths) * E, 64)) / 8.0
    ref1, ref2 = O.radial_weights_backward(d, W_r1, W_r2, paths, E, n_rbf, r_cut, dw)
    got1, got2 = grid_route(d, dw, W_r1, W_r2, paths, E, n_rbf, r_cut)
    l1 = np.abs(W_r1).sum(axis=1).max()
    e1 = np.abs(got1 - ref1).max() / np.abs(ref1).max()
    e2 = np.abs(got2 - ref2).max() / np.abs(ref2).max()
    print(f"largest absolute row sum of W_r1 {l1:.0f}: dW_r1 {e1:.1e}, dW_r2 {e2:.1e}")
    assert l1 <= 256.0                      # all three lie inside the range the library gives to this route
    assert e1 < bar and e2 < bar


def test_lagrange_weights_reproduce_quintics_and_sum_to_one():
    t = np.linspace(0.0, 0.999, 50)
    w = lagrange6(t)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
    offs = np.arange(-2, 4)
    for deg in range(6):
        assert np.allclose(w @ offs.astype(float) ** deg, t ** deg, atol=1e-12)
