"""CPU oracle (fp64, numpy) for the assembly of the predicted Hamiltonian.  TEST INFRASTRUCTURE ONLY.

Imported by tests/ and by bench.py's cpu_baseline leg only; shares no code with the HIP path.

What it follows (arXiv 2507.03840):
  * the nodes of the graph map to the diagonal blocks H_ii and the edges to the off-diagonal blocks H_ij; the final
    embeddings are collapsed along the embedding dimension (E -> 1) into coupled-basis blocks and taken back to the
    uncoupled (alpha, beta) orbital blocks by the inverse of the coupling of Eq. 1 (Sec. 3, last paragraph of "Message
    passing"; Fig. 2(e); Sec. 2.2);
  * the predicted blocks are padded: the network emits every block in one common shell list, while the number of
    orbitals per atom depends on the species (Sec. 2.2: N_orb = sum over species of atoms x orbitals per atom;
    Fig. 2(e); Sec. 4.4 has 10 and 4 orbitals for the two species of one material, Sec. 6 has 13 for all three of another);
  * training minimises a combined L1 + L2 loss over the elements of H (Sec. 6);
  * the uncoupled blocks are put together into the Hamiltonian matrix (Sec. 3, end of "Message passing").

Readings (the paper gives no formulas for these steps):
  * on-site block: q_i[o][M] = sum_c V_L[o][c] x_i[(L, M)][c] for the coupled degrees L <= l_max of the features
    (degrees above l_max have no feature to read and contribute nothing), uncoupled exactly like an edge block, with
    its own collapse weights packed like those of the edge readout;
  * species: one global shell list; a species owns a subset of its shells, given as a bit mask over the orbitals of the
    global list; a padded entry (row orbital absent on the source atom or column orbital absent on the destination atom)
    is zero in the output, carries no loss and no gradient;
  * loss = mean |H - T| + mean (H - T)^2 over the entries that are not padding (equal weights);
  * assembled matrix: columns = orbitals of the owned atoms (an atom owns the blocks of its incoming edges), rows =
    orbitals of all atoms (owned first, then halo), padding removed; stored column-compressed with the rows of a column
    ascending; every entry of a present block is stored, zero or not.  Block (i, j) = H_k of the edge i -> j (rows:
    source orbitals), block (j, j) = the on-site block.
"""
import numpy as np

from oracle import egnn_oracle as O

F64 = np.float64


def shell_orbitals(orb_l):
    """First orbital index of every shell of the global list, and the total."""
    off = np.concatenate([[0], np.cumsum([2 * l + 1 for l in orb_l])]).astype(int)
    return off, int(off[-1])


def species_orbital_bits(orb_l, shells_of_species):
    """Bit mask over the global orbital indices for each species (list of lists of shell indices)."""
    off, _ = shell_orbitals(orb_l)
    bits = []
    for shells in shells_of_species:
        b = 0
        for s in shells:
            for o in range(off[s], off[s + 1]):
                b |= 1 << o
        bits.append(b)
    return np.array(bits, np.uint32)


def bits_to_bool(bits, n_orb):
    """[n] uint32 -> [n][n_orb] bool."""
    return ((np.asarray(bits, np.uint32)[:, None] >> np.arange(n_orb, dtype=np.uint32)[None, :]) & 1).astype(bool)


def onsite_hii(x, V_node, lmax, orb_l):
    """H_i[(alpha, m_a), (beta, m_b)] for every row of x (Sec. 3; Fig. 2(e); inverse of Eq. 1)."""
    x = np.asarray(x, F64)
    slots, n_out = O.readout_slots(orb_l)
    v_off = np.concatenate([[0], np.cumsum(n_out)])
    V = np.asarray(V_node, F64)
    off, n_orb = shell_orbitals(orb_l)
    H = np.zeros((x.shape[0], n_orb, n_orb), F64)
    for (a, b, L, o) in slots:
        if L > lmax:
            continue
        q = np.einsum("c,nmc->nm", V[v_off[L] + o], x[:, O.sl(L), :])
        C = O.cg_real(orb_l[a], orb_l[b], L)
        H[:, off[a]:off[a + 1], off[b]:off[b + 1]] += np.einsum("abm,nm->nab", C, q)
    return H


def onsite_backward(x, V_node, lmax, orb_l, dH):
    """Adjoint of onsite_hii: returns (dx, dV_node) for a gradient dH w.r.t. the blocks (training needs the
    gradients of the forward pass, Sec. 4.1)."""
    x = np.asarray(x, F64)
    V = np.asarray(V_node, F64)
    dH = np.asarray(dH, F64)
    slots, n_out = O.readout_slots(orb_l)
    v_off = np.concatenate([[0], np.cumsum(n_out)])
    off, n_orb = shell_orbitals(orb_l)
    dx, dV = np.zeros_like(x), np.zeros_like(V)
    for (a, b, L, o) in slots:
        if L > lmax:
            continue
        C = O.cg_real(orb_l[a], orb_l[b], L)
        dq = np.einsum("abm,nab->nm", C, dH[:, off[a]:off[a + 1], off[b]:off[b + 1]])
        dV[v_off[L] + o] += np.einsum("nm,nmc->c", dq, x[:, O.sl(L), :])
        dx[:, O.sl(L), :] += dq[:, :, None] * V[v_off[L] + o][None, None, :]
    return dx, dV


def block_mask(row_bits, col_bits, n_orb):
    """[n][n_orb][n_orb] bool: entry present (not padding)."""
    return bits_to_bool(row_bits, n_orb)[:, :, None] & bits_to_bool(col_bits, n_orb)[:, None, :]


def apply_padding(H, row_bits, col_bits):
    H = np.asarray(H, F64)
    return np.where(block_mask(row_bits, col_bits, H.shape[1]), H, 0.0)


def loss_l1l2(H, T, row_bits, col_bits):
    """(loss, dloss/dH): mean |H - T| + mean (H - T)^2 over the entries that are not padding (Sec. 6)."""
    H, T = np.asarray(H, F64), np.asarray(T, F64)
    m = block_mask(row_bits, col_bits, H.shape[1])
    n = int(m.sum())
    d = np.where(m, H - T, 0.0)
    loss = (np.abs(d).sum() + (d * d).sum()) / n
    return float(loss), (np.sign(d) + 2.0 * d) / n


def assemble_csc(graph, species, orb_bits, H_edge, H_node, n_owned, n_total):
    """Column-compressed Hamiltonian.  Returns (orb_off [n_total + 1], col_ptr [n_cols + 1], row_idx, values)."""
    src, dst, shift, row_ptr = graph
    species = np.asarray(species)
    n_orb = H_node.shape[1]
    present = bits_to_bool(np.asarray(orb_bits, np.uint32)[species], n_orb)     # [n_total][n_orb]
    count = present.sum(axis=1)
    orb_off = np.concatenate([[0], np.cumsum(count)]).astype(np.int64)
    col_ptr, rows, vals = [0], [], []
    for j in range(n_owned):
        k0, k1 = int(row_ptr[j]), int(row_ptr[j + 1])
        blocks = {int(src[k]): np.asarray(H_edge[k], F64) for k in range(k0, k1)}
        assert j not in blocks and len(blocks) == k1 - k0
        blocks[j] = np.asarray(H_node[j], F64)
        atoms = sorted(blocks)
        for b in np.nonzero(present[j])[0]:
            for i in atoms:
                a = np.nonzero(present[i])[0]
                rows.append(orb_off[i] + np.arange(len(a)))
                vals.append(blocks[i][a, b])
            col_ptr.append(col_ptr[-1] + sum(int(count[i]) for i in atoms))
    cat = lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.zeros(0, dt)
    return orb_off, np.array(col_ptr, np.int64), cat(rows, np.int64), cat(vals, F64)


def assemble_dense(graph, species, orb_bits, H_edge, H_node, n_owned, n_total):
    """The same matrix written out densely, entry by entry ([all orbitals] x [orbitals of the owned atoms])."""
    src, dst, shift, row_ptr = graph
    n_orb = H_node.shape[1]
    present = bits_to_bool(np.asarray(orb_bits, np.uint32)[np.asarray(species)], n_orb)
    first = np.concatenate([[0], np.cumsum(present.sum(axis=1))])
    local = np.cumsum(present, axis=1) - 1           # position of a global orbital among the atom's own
    M = np.zeros((int(first[n_total]), int(first[n_owned])), F64)
    def put(i, j, blk):
        for a in range(n_orb):
            for b in range(n_orb):
                if present[i, a] and present[j, b]:
                    M[first[i] + local[i, a], first[j] + local[j, b]] += blk[a, b]
    for k in range(len(src)):
        put(int(src[k]), int(dst[k]), H_edge[k])
    for j in range(n_owned):
        put(j, j, H_node[j])
    return M
