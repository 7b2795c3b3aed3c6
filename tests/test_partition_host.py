"""The library's Low-NN partitioner (host code, no GPU) against oracle/partition_oracle.py: identical parts and
identical cut logs, on lattices, amorphous structures, open and periodic boxes, inhomogeneous degrees."""
import numpy as np
import pytest

from oracle import egnn_oracle as O
from oracle import partition_oracle as P
from paper_2507_03840_amd import binding as B
from paper_2507_03840_amd import synth


def _compare(pos, deg, box, pbc, r_cut, levels):
    part, log = B.egnn_partition_low_nn(pos, deg, box, pbc, r_cut, levels)
    ref_part, ref_log = P.low_nn_partition(np.asarray(pos, np.float32), deg, np.asarray(box, np.float32), pbc, r_cut, levels)
    assert np.array_equal(part, ref_part)
    assert log.tolist() == [list(e) for e in ref_log]
    return part, log


@pytest.mark.parametrize("levels", [0, 1, 3, 6])
def test_uniform_lattice(levels):
    g = np.stack(np.meshgrid(np.arange(12), np.arange(12), np.arange(12), indexing="ij"), axis=-1).reshape(-1, 3)
    pos = ((g + 0.25) * 4.0).astype(np.float32)
    part, log = _compare(pos, np.ones(len(pos), np.int32), [48.0, 48.0, 48.0], [1, 1, 1], 10.0, levels)
    assert np.all(np.bincount(part, minlength=1 << levels) == len(pos) >> levels)


@pytest.mark.parametrize("periodic,levels,seed", [(True, 3, 1), (True, 5, 2), (False, 4, 3), (False, 1, 4)])
def test_amorphous_with_real_degrees(periodic, levels, seed):
    w = synth.small_cluster(600, 600, 1, 8, 4, 4.0, seed, periodic=periodic)
    g = O.neighbour_list(w.pos, 600, w.box, w.pbc, w.r_cut)
    deg = np.diff(g[3]).astype(np.int32)
    part, log = _compare(w.pos, deg, w.box, w.pbc, w.r_cut, levels)
    assert part.min() == 0 and part.max() == (1 << levels) - 1


def test_slab_open_in_one_dimension_and_duplicate_coordinates():
    rng = np.random.default_rng(5)
    pos = rng.uniform(0, 30, (500, 3)).astype(np.float32)
    pos[:, 0] = np.round(pos[:, 0])                # many equal x coordinates: ties resolved by arrival order
    deg = rng.integers(1, 50, 500).astype(np.int32)
    _compare(pos, deg, [30.0, 30.0, 30.0], [1, 1, 0], 6.0, 5)
    _compare(pos, deg, [30.0, 30.0, 30.0], [0, 0, 0], 6.0, 4)


def test_more_parts_than_atoms_and_bad_arguments():
    pos = np.array([[1, 1, 1], [5, 5, 5], [9, 9, 9]], np.float32)
    part, log = _compare(pos, np.ones(3, np.int32), [12.0, 12.0, 12.0], [1, 1, 1], 3.0, 3)
    assert len(set(part.tolist())) == 3
    with pytest.raises(B.EgnnError):
        B.egnn_partition_low_nn(pos, np.ones(3, np.int32), [12.0, 12.0, 12.0], [1, 1, 1], -1.0, 2)
    with pytest.raises(B.EgnnError):
        B.egnn_partition_low_nn(pos, np.ones(3, np.int32), [0.0, 12.0, 12.0], [1, 1, 1], 3.0, 2)


def test_config4_structure_into_64_parts():
    """The full structure behind config 4 (20,000 atoms): identical to the oracle, balanced, few neighbours."""
    w = synth.workload(4, check_cutoff=False)
    rng = np.random.default_rng(0)
    deg = rng.integers(150, 250, w.n_total).astype(np.int32)      # stand-in degrees (the real ones need the full graph)
    part, log = _compare(w.pos, deg, w.box, w.pbc, w.r_cut, 6)
    sums = np.array([deg[part == q].sum() for q in range(64)])
    assert sums.max() / sums.mean() < 1.02


def _morton_reference(pos, n_owned, cell):
    """The definition written out with numpy: cube of every atom, bits of the three cube indices interleaved (x lowest),
    stable sort of the owned atoms and of the halo atoms by that key."""
    p = np.asarray(pos, np.float32).astype(np.float64)
    q = np.clip(np.floor((p - p.min(axis=0)) / float(np.float32(cell))), 0, 1023).astype(np.int64)
    key = np.zeros(len(p), np.int64)
    for b in range(10):
        for a in range(3):
            key |= ((q[:, a] >> b) & 1) << (3 * b + a)
    own = np.argsort(key[:n_owned], kind="stable")
    halo = np.argsort(key[n_owned:], kind="stable") + n_owned
    return np.concatenate([own, halo]).astype(np.int32)


@pytest.mark.parametrize("n,n_owned,cell", [(500, 500, 2.0), (700, 450, 1.5), (64, 0, 3.0), (1, 1, 1.0), (300, 300, 0.01)])
def test_spatial_order_is_the_morton_walk_of_the_cubes(n, n_owned, cell):
    rng = np.random.default_rng(n)
    pos = (rng.random((n, 3)) * np.array([20.0, 12.0, 7.0]) - 3.0).astype(np.float32)
    pos[n // 2:n // 2 + 3] = pos[0]                               # atoms of one cube keep their order of arrival
    perm = B.egnn_spatial_order(pos, n_owned, cell)
    assert np.array_equal(np.sort(perm), np.arange(n))
    assert np.all(perm[:n_owned] < n_owned) and np.all(perm[n_owned:] >= n_owned)
    assert np.array_equal(perm, _morton_reference(pos, n_owned, cell))


def test_spatial_order_brings_neighbours_close_in_index():
    w = synth.small_cluster(4000, 4000, 1, 8, 4, 4.0, 3, periodic=False)
    rng = np.random.default_rng(0)
    pos = w.pos[rng.permutation(4000)]
    src, dst, _, _ = O.neighbour_list(pos[:1500], 1500, w.box, w.pbc, 3.0)     # (pairs among the first atoms: a sample)
    full = B.egnn_spatial_order(pos, 4000, 2.0)
    new_index = np.empty(4000, np.int64); new_index[full] = np.arange(4000)
    before = np.median(np.abs(src.astype(np.int64) - dst))
    after = np.median(np.abs(new_index[src] - new_index[dst]))        # (the curve has jumps: the median, not the mean)
    assert len(src) > 1000 and after < 0.1 * before


def test_spatial_order_rejects_bad_arguments():
    pos = np.zeros((4, 3), np.float32)
    for n_owned, cell in [(5, 1.0), (-1, 1.0), (2, 0.0), (2, -1.0), (2, float("nan"))]:
        with pytest.raises(B.EgnnError):
            B.egnn_spatial_order(pos, n_owned, cell)
    assert len(B.egnn_spatial_order(np.zeros((0, 3), np.float32), 0, 1.0)) == 0
