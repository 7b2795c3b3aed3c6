"""Pins for the oracle's reverse pass: central finite differences of the fp64 forward (CPU only)."""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from paper_2507_03840_amd import synth


def _model(lmax=2, E=2, n=9, n_owned=7, n_rbf=4, seed=0, n_layers=2):
    w = synth.small_cluster(n, n_owned, lmax, E, n_rbf, r_cut=3.6, seed=seed, density=0.06)
    rng = np.random.default_rng(seed + 7)
    P = len(O.tp_paths(lmax, lmax, lmax))
    P_ro = len(O.tp_paths(lmax, lmax, 4))
    _, n_out = O.readout_slots(w.orb_l)
    f64 = lambda d: {k: v.astype(np.float64) for k, v in d.items()}
    layers = [f64(synth.layer_weights(rng, lmax, E, n_rbf, 6, P)) for _ in range(n_layers)]
    ro = f64(synth.readout_weights(rng, lmax, E, n_rbf, 6, P_ro, sum(n_out)))
    x0 = synth.node_features(rng, n, lmax, E).astype(np.float64)
    halo = [synth.node_features(rng, n - n_owned, lmax, E).astype(np.float64) for _ in range(n_layers + 1)]
    g = O.neighbour_list(w.pos, n_owned, w.box, w.pbc, w.r_cut)
    T = rng.standard_normal((len(g[0]), 13, 13))
    return w, g, layers, ro, x0, halo, T


def _forward(w, g, layers, ro, x0, halo, T, agg=3.0):
    """Loss of the whole model and the tensors the reverse pass needs."""
    xs = [x0]
    x = x0
    for t, W in enumerate(layers):
        y = O.layer_forward(g, w.pos, w.box, x, W, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, agg)
        x = np.concatenate([y, halo[t + 1]], axis=0)
        xs.append(x)
    H = O.readout_hij(g, w.pos, w.box, x, ro, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l)
    return O.loss_mse(H, T), xs, H


def _backward(w, g, layers, ro, xs, H, T, agg=3.0):
    dH = O.loss_mse_backward(H, T)
    dx, g_ro = O.readout_backward(g, w.pos, w.box, xs[-1], ro, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut,
                                  w.orb_l, dH)
    g_layers = [None] * len(layers)
    for t in reversed(range(len(layers))):
        dx, g_layers[t] = O.layer_backward(g, w.pos, w.box, xs[t], layers[t], w.lmax, w.lmax, w.channels, w.n_rbf,
                                           w.r_cut, agg, dx[:w.n_owned])
    return dx, g_layers, g_ro


@pytest.mark.parametrize("lmax", [1, 2])
def test_gradients_match_central_differences(lmax):
    w, g, layers, ro, x0, halo, T = _model(lmax=lmax)
    assert len(g[0]) > 10 and w.n_total > w.n_owned
    L0, xs, H = _forward(w, g, layers, ro, x0, halo, T)
    dx0, g_layers, g_ro = _backward(w, g, layers, ro, xs, H, T)
    rng = np.random.default_rng(3)
    eps = 1e-4   # loss ~ 1, so roundoff ~1e-12 and truncation ~1e-8 relative

    def check(arr, grad, name):
        for _ in range(4):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            Lp = _forward(w, g, layers, ro, x0, halo, T)[0]
            arr[idx] = old - eps
            Lm = _forward(w, g, layers, ro, x0, halo, T)[0]
            arr[idx] = old
            fd = (Lp - Lm) / (2 * eps)
            scale = max(np.abs(grad).max(), 1e-12)
            assert abs(fd - grad[idx]) < 1e-6 * scale + 2e-12, (name, idx, fd, grad[idx])

    check(x0, dx0, "x0")
    for t, W in enumerate(layers):
        for k in W:
            check(W[k], g_layers[t][k], f"layer{t}.{k}")
    for k in ro:
        check(ro[k], g_ro[k], f"readout.{k}")
    # a gradient that vanishes identically would pass the relative test: make sure none does
    for t in range(len(layers)):
        assert all(np.abs(v).max() > 1e-8 for v in g_layers[t].values())
    assert all(np.abs(v).max() > 1e-8 for v in g_ro.values()) and np.abs(dx0).max() > 1e-8


def test_adjoint_identities():
    """<A x, y> = <x, A^T y> for the linear pieces, with random cotangents."""
    rng = np.random.default_rng(0)
    lmax, E, n = 3, 3, 11
    x = rng.standard_normal((n, 16, E)); dy = rng.standard_normal((n, 16, E)); W = rng.standard_normal((4, E, E))
    dx, dW = O.mix_channels_backward(x, W, dy, lmax)
    assert np.isclose(np.sum(O.mix_channels(x, W, lmax) * dy), np.sum(x * dx))
    assert np.isclose(np.sum(O.mix_channels(x, W, lmax) * dy), np.sum(W * dW))
    paths = O.tp_paths(lmax, lmax, lmax)
    v = rng.standard_normal((n, 3)); v /= np.linalg.norm(v, axis=1, keepdims=True)
    Y = O.sph_harm_real(lmax, v)
    w = rng.standard_normal((n, len(paths), E)); du = rng.standard_normal((n, 16, E))
    dh, dw = O.tensor_product_backward(x, Y, w, paths, du)
    u = O.tensor_product(x, Y, w, paths, lmax)
    assert np.isclose(np.sum(u * du), np.sum(x * dh)) and np.isclose(np.sum(u * du), np.sum(w * dw))
