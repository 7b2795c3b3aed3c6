"""Pins of oracle/partition_oracle.py: hand-worked cut sequences from the neighbour-count rule of Algorithm 1,
closed-form partitions of uniform structures, balance and bookkeeping invariants."""
from math import ceil
import numpy as np
import pytest

from oracle import egnn_oracle as O
from oracle import partition_oracle as P
from paper_2507_03840_amd import synth


def _lattice(nx, ny, nz, a):
    g = np.stack(np.meshgrid(np.arange(nx), np.arange(ny), np.arange(nz), indexing="ij"), axis=-1).reshape(-1, 3)
    return (g + 0.25) * a, np.array([nx, ny, nz], float) * a


def test_get_cut_balances_the_summed_degree():
    coord = np.array([5.0, 1.0, 3.0, 2.0, 4.0])
    order, n_left, p = P.get_cut(coord, [1, 1, 1, 1, 4])        # sorted degrees: 1 1 1 4 1 -> left 3 | right 5 or 4 | 4... 
    assert order.tolist() == [1, 3, 2, 4, 0]
    # sums of the sorted sequence 1,1,1,4,1: left 1..4 atoms -> |1-7|, |2-6|, |3-5|, |7-1|  -> 3 atoms on the left
    assert n_left == 3 and p == 4.0
    # a tie takes the smaller left side; equal coordinates keep index order
    order, n_left, p = P.get_cut(np.array([0.0, 0.0, 1.0, 1.0]), [1, 1, 1, 1])
    assert order.tolist() == [0, 1, 2, 3] and n_left == 2 and p == 1.0
    order, n_left, _ = P.get_cut(np.array([0.0, 1.0, 2.0]), [1, 2, 1])      # |1-3| = |3-1|: tie -> 1
    assert n_left == 1


def test_cut_dimensions_follow_the_neighbour_count_rule():
    """Uniform periodic lattice, box 48^3, r_cut 10.  Worked by hand from NN[i] = 1 if the dimension has one cut, else
    ceil(2 r_cut / L[i]), lowest NN wins, highest index among equals:
      level 1: NN = (1,1,1) -> z;  then L_z ~ 24: NN_z = ceil(20/22) = 1 -> z again (tie with x, y, highest index);
      then L_z ~ 12 - a: NN_z = ceil(20/10) = 2 > 1 -> y (tie x, y);  then NN = (1, ceil(20/22) = 1, 2) -> y;
      then NN = (1, 2, 2) -> x;  then x (NN_x = 1 <= 2, unique minimum)."""
    pos, box = _lattice(24, 24, 24, 2.0)
    part, log = P.low_nn_partition(pos, np.ones(len(pos)), box, [1, 1, 1], 10.0, 6)
    by_level = {}
    for l, dim, n, n_left in log:
        by_level.setdefault(l, set()).add(dim)
        assert n_left * 2 == n                                   # uniform lattice: exact halves
    assert [by_level[l] for l in (6, 5, 4, 3, 2, 1)] == [{2}, {2}, {1}, {1}, {0}, {0}]
    counts = np.bincount(part, minlength=64)
    assert np.all(counts == len(pos) // 64)
    # every part is a brick of 6 x 6 x 6 lattice sites
    for q in range(64):
        ext = np.ptp(np.mod(pos[part == q] - pos[part == q][0] + 24.0, 48.0), axis=0)
        assert np.allclose(np.sort(ext), [10.0, 10.0, 10.0])


def test_few_parts_give_slabs_and_a_ring_of_neighbours():
    """The behaviour Sec. 4.4 describes for few ranks: a 1-D-like split, every part with two neighbours."""
    pos, box = _lattice(16, 16, 16, 2.5)                          # box 40, r_cut 8: two cuts keep NN_z = 1
    part, log = P.low_nn_partition(pos, np.ones(len(pos)), box, [1, 1, 1], 8.0, 2)
    assert {d for _, d, _, _ in log} == {2}
    g = O.neighbour_list(pos.astype(np.float32), len(pos), box.astype(np.float32), np.ones(3, np.uint8), 8.0)
    nb = P.neighbour_parts(part, g[0], g[1], 4)
    assert all(len(s) == 2 for s in nb)
    # the four slabs form a ring: q's neighbours are its two cyclic neighbours in z order
    zc = [np.mean(np.mod(pos[part == q][:, 2] - pos[part == 0][:, 2].min(), 40.0)) for q in range(4)]
    ring = np.argsort(zc)
    for t, q in enumerate(ring):
        assert nb[q] == {int(ring[(t - 1) % 4]), int(ring[(t + 1) % 4])}


def test_open_dimension_has_no_ring_to_open():
    """A slab that is not periodic in z: the first real cut may go through z at once (cuts starts at 1 there)."""
    pos, box = _lattice(8, 8, 32, 2.0)
    part, log = P.low_nn_partition(pos, np.ones(len(pos)), box, [1, 1, 0], 5.0, 1)
    assert log == [(1, 2, len(pos), len(pos) // 2)]
    assert pos[part == 0][:, 2].max() < pos[part == 1][:, 2].min()


def test_degree_balance_on_an_inhomogeneous_structure():
    """Every bisection balances the summed degree to within one atom's degree; all atoms are assigned once."""
    w = synth.small_cluster(400, 400, 1, 8, 4, 4.0, 11, periodic=True)
    g = O.neighbour_list(w.pos, 400, w.box, w.pbc, w.r_cut)
    deg = np.diff(g[3]).astype(float)
    part, log = P.low_nn_partition(w.pos, deg, w.box, w.pbc, w.r_cut, 3)
    assert part.min() == 0 and part.max() == 7 and np.all(np.bincount(part) > 0)
    sums = np.array([deg[part == q].sum() for q in range(8)])
    # three nested bisections, each off by at most the largest degree
    assert np.abs(sums - deg.sum() / 8).max() <= 3 * deg.max()
    for l, dim, n, n_left in log:
        assert 0 < n_left < n
    assert len(log) == 7


def test_more_parts_than_atoms_leaves_empty_parts_and_keeps_numbering():
    pos = np.array([[1.0, 1.0, 1.0], [5.0, 5.0, 5.0], [9.0, 9.0, 9.0]])
    part, _ = P.low_nn_partition(pos, [1, 1, 1], [12.0, 12.0, 12.0], [1, 1, 1], 3.0, 3)
    assert sorted(part.tolist()) == sorted(set(part.tolist())) and part.max() < 8


def test_pack_and_unpack_rows():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((10, 4, 8)).astype(np.float32)
    idx = np.array([7, 2, 2, 9])
    buf = P.pack_rows(x, idx, np.float16)
    assert buf.dtype == np.float16 and np.array_equal(buf, x[idx].astype(np.float16))
    full = np.zeros((12, 4, 8), np.float32)
    out = P.unpack_rows(full, 8, buf)
    assert np.array_equal(out[8:12], buf.astype(np.float32)) and np.all(out[:8] == 0)
