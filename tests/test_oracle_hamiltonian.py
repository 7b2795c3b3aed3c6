"""Pins of oracle/hamiltonian_oracle.py (on-site blocks, padding, L1+L2 loss, assembly) against facts that do not
come from the oracle itself: closed forms of the Clebsch-Gordan coupling, rotation behaviour of orbital blocks, hand
values, central differences, and an entry-by-entry dense assembly."""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from oracle import hamiltonian_oracle as Hm
from paper_2507_03840_amd import synth

ORB_L = (0, 0, 1, 1, 2)


def _V(rng, orb_l, E):
    _, n_out = O.readout_slots(orb_l)
    return rng.standard_normal((sum(n_out), E))


def test_onsite_scalar_features_give_multiples_of_the_identity():
    """Only L = 0 features: a rotation-invariant block.  Shell pairs of different degree vanish and a pair of equal
    degree l is q * delta_{m m'} / sqrt(2l+1) (the coupling of two equal degrees to L = 0), q the collapsed scalar."""
    rng = np.random.default_rng(0)
    E, lmax = 6, 2
    x = np.zeros((3, (lmax + 1) ** 2, E))
    x[:, 0, :] = rng.standard_normal((3, E))
    V = _V(rng, ORB_L, E)
    H = Hm.onsite_hii(x, V, lmax, ORB_L)
    slots, n_out = O.readout_slots(ORB_L)
    off, n_orb = Hm.shell_orbitals(ORB_L)
    for a, la in enumerate(ORB_L):
        for b, lb in enumerate(ORB_L):
            blk = H[:, off[a]:off[a + 1], off[b]:off[b + 1]]
            if la != lb:
                assert np.abs(blk).max() == 0
            else:
                o = [s[3] for s in slots if s[0] == a and s[1] == b and s[2] == 0][0]
                q = x[:, 0, :] @ V[o]
                want = q[:, None, None] * np.eye(2 * la + 1)[None] / np.sqrt(2 * la + 1)
                assert np.allclose(np.abs(blk), np.abs(want), atol=1e-13)
                assert np.allclose(blk, want * np.sign(blk[0, 0, 0] * want[0, 0, 0]), atol=1e-13)   # one sign per (l)


def test_onsite_rotates_like_orbital_blocks():
    """x -> D x must give H -> (D_a H D_b^T) shell block by shell block (Sec. 2.2: entries of H are covariant)."""
    rng = np.random.default_rng(1)
    E, lmax = 5, 4
    x = rng.standard_normal((4, (lmax + 1) ** 2, E))
    V = _V(rng, ORB_L, E)
    q, _ = np.linalg.qr(rng.standard_normal((3, 3)))
    R = q * np.sign(np.linalg.det(q))
    D = O.wigner_d_block(lmax, R)
    H0 = Hm.onsite_hii(x, V, lmax, ORB_L)
    H1 = Hm.onsite_hii(np.einsum("ab,nbc->nac", D, x), V, lmax, ORB_L)
    off, n_orb = Hm.shell_orbitals(ORB_L)
    Dorb = np.zeros((n_orb, n_orb))
    for a, la in enumerate(ORB_L):
        Dorb[off[a]:off[a + 1], off[a]:off[a + 1]] = O.wigner_d_real(la, R)
    assert np.allclose(H1, np.einsum("ab,nbc,dc->nad", Dorb, H0, Dorb), atol=1e-12)
    assert np.abs(H0).max() > 0.1


def test_onsite_is_linear_in_each_collapsed_slot_and_ignores_degrees_above_lmax():
    """With l_max = 1 only L <= 1 slots act; zeroing their rows of V removes everything."""
    rng = np.random.default_rng(2)
    E, lmax = 4, 1
    x = rng.standard_normal((2, 4, E))
    V = _V(rng, ORB_L, E)
    slots, n_out = O.readout_slots(ORB_L)
    v_off = np.concatenate([[0], np.cumsum(n_out)])
    H = Hm.onsite_hii(x, V, lmax, ORB_L)
    V2 = V.copy()
    V2[v_off[2]:] = 7.0                       # rows of L = 2, 3, 4: no effect
    assert np.array_equal(Hm.onsite_hii(x, V2, lmax, ORB_L), H)
    V3 = V.copy()
    V3[:v_off[2]] = 0.0
    assert np.abs(Hm.onsite_hii(x, V3, lmax, ORB_L)).max() == 0
    # brute force over the definition for one node
    off, n_orb = Hm.shell_orbitals(ORB_L)
    want = np.zeros((n_orb, n_orb))
    for (a, b, L, o) in slots:
        if L > lmax:
            continue
        C = O.cg_real(ORB_L[a], ORB_L[b], L)
        for ma in range(2 * ORB_L[a] + 1):
            for mb in range(2 * ORB_L[b] + 1):
                for M in range(2 * L + 1):
                    qv = sum(V[v_off[L] + o][c] * x[1, L * L + M, c] for c in range(E))
                    want[off[a] + ma, off[b] + mb] += C[ma, mb, M] * qv
    assert np.allclose(H[1], want, atol=1e-13)


def test_species_bits_match_the_orbital_counts_of_the_paper():
    """Global list (s, s, p, p, d): 13 orbitals; (s, s, p, d) has 10 and (s, p) has 4 (Sec. 4.4, Sec. 6)."""
    bits = Hm.species_orbital_bits(ORB_L, [[0, 1, 2, 3, 4], [0, 1, 2, 4], [0, 2]])
    assert [bin(int(b)).count("1") for b in bits] == [13, 10, 4]
    assert int(bits[2]) == 0b0000000011101 and int(bits[0]) == (1 << 13) - 1
    assert Hm.bits_to_bool(bits, 13).sum(axis=1).tolist() == [13, 10, 4]


def test_loss_l1l2_hand_values_and_padding():
    H = np.zeros((1, 2, 2)); T = np.zeros((1, 2, 2))
    H[0] = [[1.0, -2.0], [0.5, 100.0]]
    row = np.array([0b11], np.uint32); col = np.array([0b01], np.uint32)     # second column is padding
    loss, g = Hm.loss_l1l2(H, T, row, col)
    assert loss == pytest.approx((1.0 + 0.5 + 1.0 + 0.25) / 2)
    assert np.allclose(g[0], [[(1 + 2) / 2, 0], [(1 + 1) / 2, 0]])
    loss_all, _ = Hm.loss_l1l2(H, T, row, np.array([0b11], np.uint32))
    assert loss_all == pytest.approx((1 + 2 + 0.5 + 100 + 1 + 4 + 0.25 + 1e4) / 4)
    # a target that is not zero: the loss measures H - T (zero at H = T, not at H = -T)
    T[0] = [[0.5, 1.0], [0.5, -3.0]]
    loss_t, g_t = Hm.loss_l1l2(H, T, row, col)
    assert loss_t == pytest.approx((0.5 + 0.0 + 0.25 + 0.0) / 2)
    assert np.allclose(g_t[0], [[(1 + 1) / 2, 0], [0, 0]])
    assert Hm.loss_l1l2(T, T, row, col)[0] == 0.0 and Hm.loss_l1l2(-T, T, row, col)[0] > 0.0


def test_loss_l1l2_gradient_by_central_differences():
    rng = np.random.default_rng(3)
    n_orb = 13
    H = rng.standard_normal((6, n_orb, n_orb)); T = rng.standard_normal((6, n_orb, n_orb))
    bits = Hm.species_orbital_bits(ORB_L, [[0, 1, 2, 3, 4], [0, 1, 2, 4], [0, 2]])
    row = bits[rng.integers(0, 3, 6)]; col = bits[rng.integers(0, 3, 6)]
    loss, g = Hm.loss_l1l2(H, T, row, col)
    eps = 1e-6
    for _ in range(40):
        k, a, b = rng.integers(0, 6), rng.integers(0, n_orb), rng.integers(0, n_orb)
        Hp, Hn = H.copy(), H.copy()
        Hp[k, a, b] += eps; Hn[k, a, b] -= eps
        fd = (Hm.loss_l1l2(Hp, T, row, col)[0] - Hm.loss_l1l2(Hn, T, row, col)[0]) / (2 * eps)
        assert fd == pytest.approx(g[k, a, b], abs=1e-8)
    m = Hm.block_mask(row, col, n_orb)
    assert np.all(g[~m] == 0) and np.all(g[m] != 0)


@pytest.mark.parametrize("n,n_owned,periodic", [(14, 14, False), (20, 12, False), (30, 30, True)])
def test_assembly_equals_entry_by_entry_dense_matrix(n, n_owned, periodic):
    rng = np.random.default_rng(4)
    w = synth.small_cluster(n, n_owned, 1, 4, 4, 3.0, 5, periodic=periodic)
    g = O.neighbour_list(w.pos, n_owned, w.box, w.pbc, w.r_cut)
    assert len(g[0]) > n
    species = rng.integers(0, 3, n)
    bits = Hm.species_orbital_bits(ORB_L, [[0, 1, 2, 3, 4], [0, 1, 2, 4], [0, 2]])
    H_edge = rng.standard_normal((len(g[0]), 13, 13)); H_node = rng.standard_normal((n_owned, 13, 13))
    orb_off, col_ptr, rows, vals = Hm.assemble_csc(g, species, bits, H_edge, H_node, n_owned, n)
    M = Hm.assemble_dense(g, species, bits, H_edge, H_node, n_owned, n)
    counts = np.array([13, 10, 4])[species]
    assert np.array_equal(np.diff(orb_off), counts) and M.shape == (counts.sum(), counts[:n_owned].sum())
    D = np.zeros_like(M)
    for c in range(len(col_ptr) - 1):
        r = rows[col_ptr[c]:col_ptr[c + 1]]
        assert np.all(np.diff(r) > 0)                       # ascending, no duplicates
        D[r, c] = vals[col_ptr[c]:col_ptr[c + 1]]
    assert np.array_equal(D, M)
    # every block of the graph is stored: per owned atom (1 + degree) blocks
    deg = np.diff(g[3])
    nnz = sum(counts[j] * (counts[j] + counts[g[0][g[3][j]:g[3][j + 1]]].sum()) for j in range(n_owned))
    assert len(vals) == nnz and col_ptr[-1] == nnz and deg.sum() == len(g[0])


def test_padding_zeroes_exactly_the_absent_orbitals():
    rng = np.random.default_rng(5)
    bits = Hm.species_orbital_bits(ORB_L, [[0, 1, 2, 3, 4], [0, 2]])
    H = rng.standard_normal((2, 13, 13))
    P = Hm.apply_padding(H, bits[[0, 1]], bits[[1, 1]])
    keep = [0, 2, 3, 4]
    assert np.count_nonzero(P[0]) == 13 * 4 and np.count_nonzero(P[1]) == 16
    assert np.array_equal(P[1][np.ix_(keep, keep)], H[1][np.ix_(keep, keep)])


def test_onsite_backward_by_central_differences():
    """f = sum(G * onsite_hii(x, V)) is bilinear in (x, V): central differences are exact up to rounding."""
    rng = np.random.default_rng(6)
    E, lmax, n = 4, 3, 3
    x = rng.standard_normal((n, (lmax + 1) ** 2, E))
    V = _V(rng, ORB_L, E)
    G = rng.standard_normal((n, 13, 13))
    dx, dV = Hm.onsite_backward(x, V, lmax, ORB_L, G)
    f = lambda xx, vv: float(np.sum(G * Hm.onsite_hii(xx, vv, lmax, ORB_L)))
    eps = 1e-4
    for _ in range(30):
        i, q, c = rng.integers(0, n), rng.integers(0, (lmax + 1) ** 2), rng.integers(0, E)
        xp, xn = x.copy(), x.copy()
        xp[i, q, c] += eps; xn[i, q, c] -= eps
        assert (f(xp, V) - f(xn, V)) / (2 * eps) == pytest.approx(dx[i, q, c], abs=1e-9)
        r = rng.integers(0, V.shape[0])
        Vp, Vn = V.copy(), V.copy()
        Vp[r, c] += eps; Vn[r, c] -= eps
        assert (f(x, Vp) - f(x, Vn)) / (2 * eps) == pytest.approx(dV[r, c], abs=1e-9)
    # rows of V for degrees above l_max get no gradient
    _, n_out = O.readout_slots(ORB_L)
    assert np.all(dV[sum(n_out[:lmax + 1]):] == 0) and np.abs(dV[:sum(n_out[:lmax + 1])]).min() > 0
