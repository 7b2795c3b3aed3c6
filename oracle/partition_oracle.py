"""CPU oracle (plain Python / numpy) for the Low-NN partitioner and the halo pack / unpack.  TEST INFRASTRUCTURE ONLY.

Imported by tests/ only; shares no code with the library.

What it follows (arXiv 2507.03840, Sec. 4.4 and Appendix A, Algorithm 1): a recursive coordinate bisection of the atoms
into 2^l parts that (1) balances the summed node degree N_D of the two sides of every cut, as a stand-in for the
number of edges, (2) knows that the structure is periodic, and (3) cuts, at every level, the dimension in which a cut
is expected to add the fewest neighbouring parts.  Steps, in the algorithm's order and notation:

  Cut-Domain(l, pos, N_D, cuts):
    l = 0: the atoms are one finished part.
    L = extent of the (sub)domain in each dimension.
    If some dimension has no cut yet: take the lowest such dimension, let Get-Cut find its balanced cut position and
      make that position the origin O of the dimension; count the cut; go on with the same atoms and the same l.
      (One cut through a periodic ring does not divide it: it only fixes where the ring is opened.)
    Otherwise NN[i] = 1 where cuts[i] = 1 (the dimension still spans its whole period: halving it gives each half the
      other one as its only neighbour) and ceil(2 r_cut / L[i]) elsewhere; dim = argmin NN, the highest index among
      equal minima; Get-Cut splits the atoms at the balanced position; count the cut; recurse into the left and the
      right half with l - 1.
  Get-Cut(pos, N_D, dim, O): with the atoms ordered along dim (measured from the origin O, wrapped into the period),
      the position p where the summed N_D on the two sides is closest to equal; left = atoms before p, right = the rest.

Readings where the listing is silent or loose:
  * coordinates along a periodic dimension are (x - O) mod box; the origin found in the first phase replaces O = 0;
  * "closest to equal": over the ordered atoms, the number of atoms on the left, 1 .. N-1, that minimises
    |sum_left - sum_right|, the smallest such number on ties; atoms at equal coordinate keep the order in which they
    arrive (their index order at the top, the order of the parent's sort below); the
    cut position p (the new origin in the first phase) is the coordinate of the first atom of the right side;
  * `cuts` is handed down by value: each half keeps its own counts;
  * a dimension that is not periodic has no ring to open: it starts with cuts = 1 and origin = its smallest coordinate;
  * L[i] is max - min of the wrapped coordinates of the atoms of the (sub)domain (0 for a single atom; NN is then
    taken as a large number so that such a dimension is cut last);
  * parts are numbered in the order in which they are finished (left before right); a (sub)domain with fewer atoms
    than parts gives empty parts.
"""
from math import ceil
import numpy as np


def _wrapped(x, origin, box_d, periodic):
    return np.mod(x - origin, box_d) if periodic else x - origin


def get_cut(coord, n_d):
    """Number of atoms on the left (in the order of `coord`, stable) and the cut position."""
    order = np.argsort(coord, kind="stable")
    c = np.cumsum(np.asarray(n_d, np.float64)[order])
    total = c[-1]
    if len(order) < 2:
        return order, len(order), (coord[order[0]] if len(order) else 0.0)
    diff = np.abs(2.0 * c[:-1] - total)          # |left - right| for 1 .. N-1 atoms on the left
    n_left = int(np.argmin(diff)) + 1
    return order, n_left, float(coord[order[n_left]])


def low_nn_partition(pos, n_d, box, pbc, r_cut, levels):
    """part [N] in 0 .. 2^levels - 1, and the list of cut dimensions in the order the cuts were made (depth first)."""
    pos = np.asarray(pos, np.float64)
    n_d = np.asarray(n_d, np.float64)
    box = np.asarray(box, np.float64)
    part = np.full(len(pos), -1, np.int64)
    log = []
    counter = [0]

    def cut_domain(l, idx, cuts, origin):
        if l == 0:
            part[idx] = counter[0]
            counter[0] += 1
            return
        if len(idx) == 0:
            for _ in range(2 ** l):
                counter[0] += 1
            return
        cuts, origin = list(cuts), list(origin)
        while any(c == 0 for c in cuts):
            dim = min(d for d in range(3) if cuts[d] == 0)
            coord = _wrapped(pos[idx, dim], origin[dim], box[dim], True)
            _, _, p = get_cut(coord, n_d[idx])
            origin[dim] = origin[dim] + p
            cuts[dim] += 1
        coords = np.stack([_wrapped(pos[idx, d], origin[d], box[d], bool(pbc[d])) for d in range(3)], axis=1)
        L = coords.max(axis=0) - coords.min(axis=0)
        nn = []
        for d in range(3):
            if cuts[d] == 1:
                nn.append(1)
            else:
                nn.append(ceil(2.0 * r_cut / L[d]) if L[d] > 0 else 1 << 30)
        lowest = min(nn)
        dim = max(d for d in range(3) if nn[d] == lowest)
        order, n_left, _ = get_cut(coords[:, dim], n_d[idx])
        log.append((l, dim, len(idx), n_left))
        cuts[dim] += 1
        cut_domain(l - 1, idx[order[:n_left]], cuts, origin)
        cut_domain(l - 1, idx[order[n_left:]], cuts, origin)

    cuts0 = [0 if pbc[d] else 1 for d in range(3)]
    origin0 = [0.0 if pbc[d] else (float(pos[:, d].min()) if len(pos) else 0.0) for d in range(3)]
    cut_domain(levels, np.arange(len(pos)), cuts0, origin0)
    return part, log


def neighbour_parts(part, src, dst, n_parts):
    """For every part the set of other parts it receives node embeddings from (sources of its incoming edges)."""
    nb = [set() for _ in range(n_parts)]
    for i, j in zip(part[np.asarray(src)], part[np.asarray(dst)]):
        if i != j:
            nb[j].add(int(i))
    return nb


def pack_rows(x, idx, dtype=np.float32):
    """Send buffer: the rows idx of x, in that order, in the payload precision."""
    return np.asarray(x)[np.asarray(idx)].astype(dtype)


def unpack_rows(x_full, first_row, buf):
    """Received rows written behind the owned rows (halo rows follow the owned ones)."""
    out = np.array(x_full, np.float32, copy=True)
    out[first_row:first_row + len(buf)] = np.asarray(buf).astype(np.float32)
    return out
