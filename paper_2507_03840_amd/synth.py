"""Seeded synthetic inputs: atomic structures, random features and random weights.

This module serves both the HIP path and the CPU oracle used by the tests.  It
holds none of the method's arithmetic: it draws atom positions, species, random
feature tensors and random weight tensors with numpy's PCG64 generator
(``numpy.random.default_rng(seed)``), and nothing else.  Sizes that depend on the
method (number of tensor-product paths, readout widths) are passed in by the
caller, who gets them from its own side.

The structures imitate the workloads of the paper (Sec. 3 "Implementation":
thousands of atoms, cutoffs of 10+ Angstrom, hundreds of neighbours per atom;
Sec. 6: 13 orbitals per atom = 2s + 2p + 1d), whose HfO2 / GeSbTe geometries are
not available:

  config 1  64 atoms, jittered diamond lattice, open boundaries, r_cut 6
  config 2  1,000 atoms, jittered diamond, periodic cube, r_cut 8
  config 3  3,000 atoms, amorphous-like (uniform + 2.0 A rejection), r_cut 10
  config 4  one rank's share of a slab: 12,000 owned + 8,000 halo atoms, r_cut 10
  config 5  config 3 plus random target blocks (training step)
"""
from dataclasses import dataclass, field
import numpy as np

SEED_BASE = 20250703
DIAMOND_A = 5.43
CUTOFF_SAFETY = 1e-9  # no pair may lie this close (relative, in d^2) to r_cut^2

# 8-atom conventional cell of the diamond structure (fractional coordinates)
_DIAMOND_BASIS = np.array(
    [[0, 0, 0], [0, .5, .5], [.5, 0, .5], [.5, .5, 0],
     [.25, .25, .25], [.25, .75, .75], [.75, .25, .75], [.75, .75, .25]], dtype=np.float64)


@dataclass
class Workload:
    """One synthetic configuration: structure + model hyper-parameters."""
    name: str
    index: int
    lmax: int
    channels: int
    n_rbf: int
    n_layers: int
    r_cut: float
    n_species: int
    readout: bool
    n_hidden: int = 64
    orb_l: tuple = (0, 0, 1, 1, 2)
    # filled by build():
    pos: np.ndarray = field(default=None, repr=False)       # f32 [n_total,3]
    species: np.ndarray = field(default=None, repr=False)   # i32 [n_total]
    box: np.ndarray = field(default=None, repr=False)       # f32 [3]
    pbc: np.ndarray = field(default=None, repr=False)       # u8  [3]
    n_owned: int = 0
    n_total: int = 0

    @property
    def seed(self):
        return SEED_BASE + self.index

    @property
    def n_orb(self):
        return int(sum(2 * l + 1 for l in self.orb_l))


def _diamond(cells, sigma, rng):
    nx, ny, nz = cells
    ii, jj, kk = np.meshgrid(np.arange(nx), np.arange(ny), np.arange(nz), indexing="ij")
    origin = np.stack([ii, jj, kk], -1).reshape(-1, 1, 3).astype(np.float64)
    frac = (origin + _DIAMOND_BASIS[None]).reshape(-1, 3)
    cell_idx = np.repeat(np.stack([ii, jj, kk], -1).reshape(-1, 3), 8, axis=0)
    pos = frac * DIAMOND_A + rng.normal(0.0, sigma, size=frac.shape)
    return pos, cell_idx


def _min_image(delta, box, pbc):
    for a in range(3):
        if pbc[a]:
            delta[..., a] -= box[a] * np.rint(delta[..., a] / box[a])
    return delta


def _amorphous(n, length, dmin, rng):
    """Sequential random insertion in a periodic cube with a minimum distance."""
    box = np.array([length] * 3)
    pts = np.empty((n, 3))
    k = 0
    while k < n:
        p = rng.uniform(0.0, length, size=3)
        if k:
            d = _min_image(pts[:k] - p, box, (1, 1, 1))
            if np.min(np.einsum("ij,ij->i", d, d)) < dmin * dmin:
                continue
        pts[k] = p
        k += 1
    return pts


def closest_to_cutoff(pos32, n_owned, box, pbc, r_cut):
    """min over pairs (i != j, j owned) of |d^2/r_cut^2 - 1|, from the fp32 data in fp64."""
    p = pos32.astype(np.float64)
    b = np.asarray(box, np.float64)
    rc2 = float(np.float32(r_cut)) ** 2
    worst = np.inf
    step = 512
    for j0 in range(0, n_owned, step):
        d = p[None, :, :] - p[j0:j0 + step, None, :]
        d = _min_image(d, b, pbc)
        rel = np.abs(np.einsum("jia,jia->ji", d, d) / rc2 - 1.0)
        worst = min(worst, float(rel.min()))
    return worst


def workload(index: int, check_cutoff: bool = True) -> Workload:
    """Build configuration `index` (1..5).  Deterministic in `index`."""
    presets = {
        1: Workload("tiny-diamond-64", 1, lmax=2, channels=16, n_rbf=8, n_layers=1, r_cut=6.0,
                    n_species=2, readout=True),
        2: Workload("diamond-1000", 2, lmax=3, channels=32, n_rbf=16, n_layers=2, r_cut=8.0,
                    n_species=3, readout=True),
        3: Workload("amorphous-3000", 3, lmax=4, channels=32, n_rbf=16, n_layers=3, r_cut=10.0,
                    n_species=2, readout=True),
        4: Workload("slab-12000+8000halo", 4, lmax=4, channels=64, n_rbf=16, n_layers=3, r_cut=10.0,
                    n_species=2, readout=False),
        5: Workload("amorphous-3000-train", 5, lmax=4, channels=32, n_rbf=16, n_layers=3, r_cut=10.0,
                    n_species=2, readout=True),
    }
    w = presets[index]
    struct_seed = SEED_BASE + (3 if index == 5 else index)  # config 5 reuses config 3's graph
    attempt = 0
    while True:
        rng = np.random.default_rng([struct_seed, attempt])
        if index == 1:
            pos, _ = _diamond((2, 2, 2), 0.05, rng)
            box = np.array([2 * DIAMOND_A] * 3)
            pbc = np.zeros(3, np.uint8)
            n_owned = len(pos)
        elif index == 2:
            pos, _ = _diamond((5, 5, 5), 0.1, rng)
            box = np.array([5 * DIAMOND_A] * 3)
            pbc = np.ones(3, np.uint8)
            n_owned = len(pos)
        elif index in (3, 5):
            length = (3000 / 0.05) ** (1.0 / 3.0)
            pos = _amorphous(3000, length, 2.0, rng)
            box = np.array([length] * 3)
            pbc = np.ones(3, np.uint8)
            n_owned = len(pos)
        else:
            pos, cell = _diamond((25, 10, 10), 0.1, rng)
            owned = (cell[:, 2] >= 2) & (cell[:, 2] <= 7)
            order = np.concatenate([np.nonzero(owned)[0], np.nonzero(~owned)[0]])
            pos = pos[order]
            box = np.array([25 * DIAMOND_A, 10 * DIAMOND_A, 10 * DIAMOND_A])
            pbc = np.array([1, 1, 0], np.uint8)
            n_owned = int(owned.sum())
        species = rng.integers(0, w.n_species, size=len(pos)).astype(np.int32)
        pos32 = pos.astype(np.float32)
        box32 = box.astype(np.float32)
        if not check_cutoff or closest_to_cutoff(pos32, n_owned, box32, pbc, w.r_cut) > CUTOFF_SAFETY:
            break
        attempt += 1
    w.pos, w.species, w.box, w.pbc = pos32, species, box32, pbc
    w.n_owned, w.n_total = n_owned, len(pos32)
    return w


def small_cluster(n_atoms, n_owned, lmax, channels, n_rbf, r_cut, seed, periodic=False, density=0.05):
    """A small random structure for unit tests (same recipe as config 3, any size)."""
    rng = np.random.default_rng([SEED_BASE, 77, seed])
    length = (n_atoms / density) ** (1.0 / 3.0)
    if periodic:
        length = max(length, 2.0 * r_cut * 1.001)
    pos = _amorphous(n_atoms, length, 1.5, rng)
    w = Workload(f"cluster-{n_atoms}", 0, lmax=lmax, channels=channels, n_rbf=n_rbf, n_layers=1,
                 r_cut=r_cut, n_species=2, readout=True)
    w.pos = pos.astype(np.float32)
    w.species = rng.integers(0, 2, size=n_atoms).astype(np.int32)
    w.box = np.array([length] * 3, np.float32)
    w.pbc = np.array([1, 1, 1] if periodic else [0, 0, 0], np.uint8)
    w.n_owned, w.n_total = n_owned, n_atoms
    return w


def normal(rng, shape, std=1.0):
    return (rng.standard_normal(size=shape) * std).astype(np.float32)


def layer_weights(rng, lmax, channels, n_rbf, n_hidden, n_paths):
    """Random weights of one message-passing layer, every W ~ N(0, 1/fan_in)."""
    E = channels
    return dict(
        W_pre=normal(rng, (lmax + 1, E, E), E ** -0.5),
        W_post=normal(rng, (lmax + 1, E, E), E ** -0.5),
        W_self=normal(rng, (lmax + 1, E, E), E ** -0.5),
        W_r1=normal(rng, (n_hidden, n_rbf), n_rbf ** -0.5),
        W_r2=normal(rng, (n_paths * E, n_hidden), n_hidden ** -0.5),
    )


def readout_weights(rng, lmax, channels, n_rbf, n_hidden, n_paths_ro, n_out_total):
    """Random weights of the H_ij readout; `n_out_total` = rows of the packed collapse matrix V."""
    E = channels
    return dict(
        W_s=normal(rng, (lmax + 1, E, E), E ** -0.5),
        W_t=normal(rng, (lmax + 1, E, E), E ** -0.5),
        W_r1=normal(rng, (n_hidden, n_rbf), n_rbf ** -0.5),
        W_r2=normal(rng, (n_paths_ro * E, n_hidden), n_hidden ** -0.5),
        V=normal(rng, (n_out_total, E), E ** -0.5),
    )


def node_features(rng, n_rows, lmax, channels):
    """x ~ N(0,1) on every (l, m, channel) so that every path is exercised."""
    return normal(rng, (n_rows, (lmax + 1) ** 2, channels))


def so2_weights(rng, lmax, channels, n_rbf):
    """Random weights of the SO(2) message transform: W_e [E][n_rbf], W_0, and (Wr_m, Wi_m) for m = 1..lmax with
    (lmax+1-m) E rows and (lmax+1-m) 3E columns; every matrix ~ N(0, 1/fan_in), two blocks feeding each output for m > 0."""
    E = channels
    shapes = [((lmax + 1 - m) * E, (lmax + 1 - m) * 3 * E) for m in range(lmax + 1)]
    W0 = normal(rng, shapes[0], shapes[0][1] ** -0.5)
    Wr = [normal(rng, s, (2 * s[1]) ** -0.5) for s in shapes[1:]]
    Wi = [normal(rng, s, (2 * s[1]) ** -0.5) for s in shapes[1:]]
    W_e = normal(rng, (E, n_rbf), n_rbf ** -0.5)
    return W_e, W0, Wr, Wi


def species_table(rng, n_species, channels):
    return normal(rng, (n_species, channels))
