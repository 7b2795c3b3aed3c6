"""CPU oracle (fp64, numpy) for the bond-aligned SO(2) form of the message transform.  TEST INFRASTRUCTURE ONLY.

Imported by tests/ only (and by nothing under paper_2507_03840_amd/); shares no code with the HIP path.

What it follows (arXiv 2507.03840): Fig. 2(a) bottom (a message is the concatenation of the two node embeddings
and the edge embedding), Fig. 2(d) and Sec. 3 "Message passing" (every message is rotated with the Wigner matrix of
its bond so that the bond lies on a fixed axis, split into its m components, each |m| goes through its own linear
layer that mixes the degrees l and takes 3E channels to E, and the result is rotated back), Sec. 2.1 end (this is
what turns the tensor product into linear layers), Sec. 3 "Initialization" (the L = 0 plane of an edge embedding
is the Gaussian expansion of the edge length) and the sum over incoming edges of Sec. 3.

Choices where the paper is silent (its references define the layer):
  * frame: any rotation R_k with R_k rhat_k = z; the result does not depend on which one (a linear layer of this
    form commutes with rotations about z), which test_so2_gauge checks;
  * components: with the real harmonics of egnn_oracle (m > 0 <-> cos, m < 0 <-> sin) a rotation about z by a turns
    (x_{+m}, x_{-m}) by the angle m a, so the layer of order m > 0 is
        y_{+m} = Wr_m x_{+m} - Wi_m x_{-m},   y_{-m} = Wi_m x_{+m} + Wr_m x_{-m}
    and y_0 = W_0 x_0, where x_{+-m} stacks the degrees l >= m and the 3E channels, y the degrees l >= m and E channels;
  * weights do not depend on the edge; the edge enters through its embedding e_k, whose L = 0 plane is W_e B(d_k)
    (W_e [E][n_rbf], a learnable linear map of the Gaussian basis) and whose other planes are zero (edge embeddings
    are not carried from layer to layer in this build);
  * each message is multiplied by the cosine envelope f_c(d_k) and the sum over incoming edges by agg_norm^-1/2 (the
    paper's attention weights are not part of this path).
"""
from math import sqrt
import numpy as np
from . import egnn_oracle as O

F64 = np.float64


def so2_shapes(lmax, E):
    """[(rows, cols)] of W_0, then of Wr_m = Wi_m for m = 1..lmax: rows (l_out - m) E + c_out, cols (l_in - m) 3E + g E + c_in."""
    return [((lmax + 1 - m) * E, (lmax + 1 - m) * 3 * E) for m in range(lmax + 1)]


def so2_pack(W0, Wr, Wi):
    """Flat fp32 layout of the C ABI: W_0, then Wr_1, Wi_1, Wr_2, Wi_2, ..., each row-major."""
    parts = [np.asarray(W0, np.float32).ravel()]
    for a, b in zip(Wr, Wi):
        parts += [np.asarray(a, np.float32).ravel(), np.asarray(b, np.float32).ravel()]
    return np.concatenate(parts)


def bond_rotations(rhat, gauge=None):
    """R [n][3][3] with R rhat = z (Rodrigues about rhat x z), optionally followed by a rotation about z by gauge[n]."""
    rhat = np.asarray(rhat, F64)
    n = len(rhat)
    z = np.array([0.0, 0.0, 1.0])
    R = np.zeros((n, 3, 3), F64)
    for k in range(n):
        v = np.cross(rhat[k], z)
        s, c = np.linalg.norm(v), float(rhat[k] @ z)
        if s < 1e-14:
            Rk = np.eye(3) if c > 0 else np.diag([1.0, -1.0, -1.0])     # rhat = -z: half turn about x
        else:
            K = np.array([[0, -v[2], v[1]], [v[2], 0, -v[0]], [-v[1], v[0], 0]]) / s
            Rk = np.eye(3) + s * K + (1 - c) * (K @ K)
        if gauge is not None:
            ca, sa = np.cos(gauge[k]), np.sin(gauge[k])
            Rk = np.array([[ca, -sa, 0], [sa, ca, 0], [0, 0, 1.0]]) @ Rk
        R[k] = Rk
    return R


def wigner_blocks(lmax, R):
    """D [n][(lmax+1)^2][(lmax+1)^2], block diagonal, with Y(R_k r) = D_k Y(r): solved from the harmonics themselves at a
    fixed set of sample directions (the same definition as egnn_oracle.wigner_d_real, batched over rotations)."""
    rng = np.random.default_rng(4321)
    n = len(R)
    dim = (lmax + 1) ** 2
    D = np.zeros((n, dim, dim), F64)
    v = rng.standard_normal((8 * (2 * lmax + 1), 3))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    Yv = O.sph_harm_real(lmax, v)                                      # [s][dim]
    rot = np.einsum("kab,sb->ksa", R, v)                               # R_k v_s
    Yr = O.sph_harm_real(lmax, rot.reshape(-1, 3)).reshape(n, len(v), dim)
    for l in range(lmax + 1):
        pinv = np.linalg.pinv(Yv[:, O.sl(l)])                          # [2l+1][s]
        D[:, O.sl(l), O.sl(l)] = np.einsum("as,ksb->kba", pinv, Yr[:, :, O.sl(l)])
    return D


def so2_linear(Xp, W0, Wr, Wi, lmax, E):
    """The per-|m| linear layers on bond-frame messages Xp [n][(lmax+1)^2][3E] -> [n][(lmax+1)^2][E]."""
    n = Xp.shape[0]
    Yp = np.zeros((n, (lmax + 1) ** 2, E), F64)
    ls0 = np.arange(lmax + 1)
    x0 = Xp[:, ls0 * ls0 + ls0, :].reshape(n, -1)                      # (l, channel) stacked
    Yp[:, ls0 * ls0 + ls0, :] = (x0 @ np.asarray(W0, F64).T).reshape(n, lmax + 1, E)
    for m in range(1, lmax + 1):
        ls = np.arange(m, lmax + 1)
        xp = Xp[:, ls * ls + ls + m, :].reshape(n, -1)
        xm = Xp[:, ls * ls + ls - m, :].reshape(n, -1)
        A, B = np.asarray(Wr[m - 1], F64), np.asarray(Wi[m - 1], F64)
        Yp[:, ls * ls + ls + m, :] = (xp @ A.T - xm @ B.T).reshape(n, len(ls), E)
        Yp[:, ls * ls + ls - m, :] = (xp @ B.T + xm @ A.T).reshape(n, len(ls), E)
    return Yp


def so2_messages(src, dst, r, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, gauge=None, T_edge=None, envelope=True):
    """One transformed message per edge, lab frame: f_c(d) D^T SO2Linear(D [x_src | x_dst | e]).
    T_edge [n][(lmax+1)^2][E]: full edge embeddings of these edges (W_e is then not used); envelope=False leaves
    the factor f_c(d) out."""
    x = np.asarray(x, F64)
    d = np.sqrt(np.einsum("ka,ka->k", r, r))
    D = wigner_blocks(lmax, bond_rotations(r / d[:, None], gauge))
    n, dim = len(src), (lmax + 1) ** 2
    M = np.zeros((n, dim, 3 * E), F64)
    M[:, :, :E] = x[src]
    M[:, :, E:2 * E] = x[dst]
    if T_edge is None:
        M[:, 0, 2 * E:] = O.radial_basis(d, n_rbf, r_cut) @ np.asarray(W_e, F64).T
    else:
        M[:, :, 2 * E:] = np.asarray(T_edge, F64)
    Xp = np.einsum("kab,kbc->kac", D, M)
    Yp = so2_linear(Xp, W0, Wr, Wi, lmax, E)
    Y = np.einsum("kba,kbc->kac", D, Yp)                               # D^T = D^-1
    return Y * O.envelope(d, r_cut)[:, None, None] if envelope else Y


def so2_message_sum(graph, pos, box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, agg_norm, gauge=None, chunk=4096,
                    nodes=None):
    """a_j = agg_norm^-1/2 sum over the incoming edges of owned node j of the transformed messages.
    nodes: if given, only these destination nodes are evaluated and only their rows returned (same arithmetic)."""
    src, dst, shift, row_ptr = graph
    n_owned = len(row_ptr) - 1
    if nodes is not None:
        out = np.zeros((len(nodes), (lmax + 1) ** 2, E), F64)
        for i, j in enumerate(nodes):
            k0, k1 = int(row_ptr[j]), int(row_ptr[j + 1])
            if k1 > k0:
                r = O.edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
                out[i] = so2_messages(src[k0:k1], dst[k0:k1], r, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut,
                                      None if gauge is None else gauge[k0:k1]).sum(axis=0)
        return out / sqrt(agg_norm)
    a = np.zeros((n_owned, (lmax + 1) ** 2, E), F64)
    for k0 in range(0, len(src), chunk):
        k1 = min(len(src), k0 + chunk)
        r = O.edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
        Y = so2_messages(src[k0:k1], dst[k0:k1], r, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut,
                         None if gauge is None else gauge[k0:k1])
        np.add.at(a, dst[k0:k1], Y)
    return a / sqrt(agg_norm)


def so2_linear_backward(Xp, gYp, W0, Wr, Wi, lmax, E):
    """Adjoint of so2_linear: (gXp, dW0, [dWr_m], [dWi_m]) from the bond-frame inputs Xp and the gradient gYp of the
    outputs.  With y_{+m} = Wr x_{+m} - Wi x_{-m}, y_{-m} = Wi x_{+m} + Wr x_{-m}:
        gx_{+m} = Wr^T gy_{+m} + Wi^T gy_{-m},   gx_{-m} = -Wi^T gy_{+m} + Wr^T gy_{-m},
        dWr = gy_{+m} x_{+m}^T + gy_{-m} x_{-m}^T,   dWi = -gy_{+m} x_{-m}^T + gy_{-m} x_{+m}^T   (summed over the edges)."""
    n = Xp.shape[0]
    gXp = np.zeros_like(Xp)
    ls0 = np.arange(lmax + 1)
    i0 = ls0 * ls0 + ls0
    x0 = Xp[:, i0, :].reshape(n, -1)
    g0 = gYp[:, i0, :].reshape(n, -1)
    gXp[:, i0, :] = (g0 @ np.asarray(W0, F64)).reshape(n, lmax + 1, -1)
    dW0 = g0.T @ x0
    dWr, dWi = [], []
    for m in range(1, lmax + 1):
        ls = np.arange(m, lmax + 1)
        ip, im = ls * ls + ls + m, ls * ls + ls - m
        xp, xm = Xp[:, ip, :].reshape(n, -1), Xp[:, im, :].reshape(n, -1)
        gp, gm = gYp[:, ip, :].reshape(n, -1), gYp[:, im, :].reshape(n, -1)
        A, B = np.asarray(Wr[m - 1], F64), np.asarray(Wi[m - 1], F64)
        gXp[:, ip, :] = (gp @ A + gm @ B).reshape(n, len(ls), -1)
        gXp[:, im, :] = (gm @ A - gp @ B).reshape(n, len(ls), -1)
        dWr.append(gp.T @ xp + gm.T @ xm)
        dWi.append(gm.T @ xp - gp.T @ xm)
    return gXp, dW0, dWr, dWi


def so2_message_sum_backward(graph, pos, box, x, W_e, W0, Wr, Wi, lmax, E, n_rbf, r_cut, agg_norm, da, chunk=4096):
    """Adjoint of so2_message_sum with respect to the node embeddings and the weights (positions are data):
    from da [n_owned][(lmax+1)^2][E] returns (dx [n_total][(lmax+1)^2][E], dW_e, dW0, [dWr_m], [dWi_m]).
    Every step of so2_messages is linear in (x, e) for fixed weights and linear in the weights for fixed inputs; the
    steps are undone in reverse order: the scale and the envelope, the rotation back (adjoint: D), the per-|m| linear
    layers (so2_linear_backward), the rotation into the bond frame (adjoint: D^T), the concatenation (its three
    column groups go to x[src], x[dst] and, through the L = 0 plane only, to W_e)."""
    src, dst, shift, row_ptr = graph
    x = np.asarray(x, F64)
    da = np.asarray(da, F64)
    dx = np.zeros_like(x)
    dW_e = np.zeros((E, n_rbf), F64)
    shapes = so2_shapes(lmax, E)
    dW0 = np.zeros(shapes[0], F64)
    dWr = [np.zeros(s, F64) for s in shapes[1:]]
    dWi = [np.zeros(s, F64) for s in shapes[1:]]
    dim = (lmax + 1) ** 2
    for k0 in range(0, len(src), chunk):
        k1 = min(len(src), k0 + chunk)
        s_, d_ = src[k0:k1], dst[k0:k1]
        r = O.edge_vectors(pos, box, s_, d_, shift[k0:k1])
        d = np.sqrt(np.einsum("ka,ka->k", r, r))
        D = wigner_blocks(lmax, bond_rotations(r / d[:, None]))
        B = O.radial_basis(d, n_rbf, r_cut)
        M = np.zeros((k1 - k0, dim, 3 * E), F64)
        M[:, :, :E] = x[s_]
        M[:, :, E:2 * E] = x[d_]
        M[:, 0, 2 * E:] = B @ np.asarray(W_e, F64).T
        Xp = np.einsum("kab,kbc->kac", D, M)
        gY = da[d_] * (O.envelope(d, r_cut) / sqrt(agg_norm))[:, None, None]
        gYp = np.einsum("kab,kbc->kac", D, gY)
        gXp, g0, gr, gi = so2_linear_backward(Xp, gYp, W0, Wr, Wi, lmax, E)
        gM = np.einsum("kba,kbc->kac", D, gXp)
        np.add.at(dx, s_, gM[:, :, :E])
        np.add.at(dx, d_, gM[:, :, E:2 * E])
        dW_e += gM[:, 0, 2 * E:].T @ B
        dW0 += g0
        for m in range(lmax):
            dWr[m] += gr[m]
            dWi[m] += gi[m]
    return dx, dW_e, dW0, dWr, dWi


# --------------------------------------------------------------------------------------
# The two blocks of a layer with the full message content (Sec. 3 "Message passing", Fig. 2(b), 2(c)): persistent edge
# embeddings, a node block that ends in an attention-weighted sum over incoming edges, an edge block without the sum.
#
# Choices where the paper is silent (it names the steps and leaves the formulas to its references):
#   * edge embeddings start with the L = 0 plane W_e B(d_k) and zeros elsewhere (Sec. 3 "Initialization") and are then
#     full tensors [(lmax+1)^2][E] that rotate like node embeddings;
#   * attention: one head; the score of an edge is s_k = w_att . LeakyReLU_0.2(y_k[L = 0]) from the rotation-invariant
#     plane of its transformed message (before the envelope), the weights are the softmax of the scores over the
#     incoming edges of the destination node, and a_j = sum_k alpha_k f_c(d_k) y_k;
#   * edge block: T'_k = T_k + f_c(d_k) y_k with its own SO(2) weights, no sum;
#   * gate: the L = 0 plane goes through SiLU; the plane of degree l >= 1 is multiplied, channel by channel, by
#     sigmoid(W_g[l-1] x[L = 0]) (scalars computed from the input's L = 0 plane gate the higher degrees).
# --------------------------------------------------------------------------------------
def edge_embedding_init(d, W_e, lmax, E, n_rbf, r_cut):
    T = np.zeros((len(d), (lmax + 1) ** 2, E), F64)
    T[:, 0, :] = O.radial_basis(np.asarray(d, F64), n_rbf, r_cut) @ np.asarray(W_e, F64).T
    return T


def attention_weights(y0, w_att, row_ptr, slope=0.2):
    """alpha [n_edges]: softmax over each destination segment of w_att . LeakyReLU(y0[k]);  y0 [n_edges][E]."""
    y0 = np.asarray(y0, F64)
    s = np.where(y0 > 0, y0, slope * y0) @ np.asarray(w_att, F64)
    alpha = np.zeros(len(s), F64)
    for j in range(len(row_ptr) - 1):
        k0, k1 = int(row_ptr[j]), int(row_ptr[j + 1])
        if k1 > k0:
            e = np.exp(s[k0:k1] - s[k0:k1].max())
            alpha[k0:k1] = e / e.sum()
    return alpha


def so2_node_block(graph, pos, box, x, T_edge, W0, Wr, Wi, w_att, lmax, E, r_cut, nodes=None):
    """a_j = sum over incoming edges of alpha_k f_c(d_k) y_k (owned nodes; `nodes`: only these rows)."""
    src, dst, shift, row_ptr = graph
    n_owned = len(row_ptr) - 1
    todo = range(n_owned) if nodes is None else nodes
    out = np.zeros((len(todo), (lmax + 1) ** 2, E), F64)
    for i, j in enumerate(todo):
        k0, k1 = int(row_ptr[j]), int(row_ptr[j + 1])
        if k1 == k0:
            continue
        r = O.edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
        Y = so2_messages(src[k0:k1], dst[k0:k1], r, x, None, W0, Wr, Wi, lmax, E, 0, r_cut, T_edge=T_edge[k0:k1],
                         envelope=False)
        alpha = attention_weights(Y[:, 0, :], w_att, np.array([0, k1 - k0]))
        fc = O.envelope(np.sqrt(np.einsum("ka,ka->k", r, r)), r_cut)
        out[i] = np.einsum("k,kac->ac", alpha * fc, Y)
    return out


def so2_edge_block(graph, pos, box, x, T_edge, W0, Wr, Wi, lmax, E, r_cut, k_range=None, chunk=4096):
    """T'_k = T_k + f_c(d_k) y_k for every edge (or those of k_range)."""
    src, dst, shift, row_ptr = graph
    a, b = (0, len(src)) if k_range is None else k_range
    out = np.zeros((b - a, (lmax + 1) ** 2, E), F64)
    for k0 in range(a, b, chunk):
        k1 = min(b, k0 + chunk)
        r = O.edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
        out[k0 - a:k1 - a] = np.asarray(T_edge[k0:k1], F64) + so2_messages(
            src[k0:k1], dst[k0:k1], r, x, None, W0, Wr, Wi, lmax, E, 0, r_cut, T_edge=T_edge[k0:k1])
    return out


def gate(x, W_g, lmax):
    """x [n][(lmax+1)^2][E], W_g [lmax][E][E]."""
    x = np.asarray(x, F64)
    out = np.zeros_like(x)
    x0 = x[:, 0, :]
    out[:, 0, :] = O.silu(x0)
    for l in range(1, lmax + 1):
        g = 1.0 / (1.0 + np.exp(-(x0 @ np.asarray(W_g[l - 1], F64).T)))
        out[:, O.sl(l), :] = x[:, O.sl(l), :] * g[:, None, :]
    return out


# --------------------------------------------------------------------------------------
# Adjoints of the two blocks and of the gate (Sec. 4.1: training needs the gradients of the forward pass).  Positions
# are data.  Each function undoes the steps of its forward function in reverse order; tests/test_oracle_so2_blocks.py
# pins them to central differences of the forward functions.
# --------------------------------------------------------------------------------------
def so2_messages_backward(src, dst, r, x, T_edge, W0, Wr, Wi, lmax, E, gY):
    """Adjoint of so2_messages(..., T_edge=T_edge, envelope=False) for the edges given: from gY [n][(lmax+1)^2][E]
    (gradient of the transformed messages, lab frame) returns (gM [n][(lmax+1)^2][3E], dW0, [dWr_m], [dWi_m]); the
    three column groups of gM belong to x[src], x[dst] and T_edge."""
    x = np.asarray(x, F64)
    d = np.sqrt(np.einsum("ka,ka->k", r, r))
    D = wigner_blocks(lmax, bond_rotations(r / d[:, None]))
    n, dim = len(src), (lmax + 1) ** 2
    M = np.zeros((n, dim, 3 * E), F64)
    M[:, :, :E] = x[src]
    M[:, :, E:2 * E] = x[dst]
    M[:, :, 2 * E:] = np.asarray(T_edge, F64)
    Xp = np.einsum("kab,kbc->kac", D, M)
    gYp = np.einsum("kab,kbc->kac", D, np.asarray(gY, F64))      # Y = D^T Y'
    gXp, dW0, dWr, dWi = so2_linear_backward(Xp, gYp, W0, Wr, Wi, lmax, E)
    return np.einsum("kba,kbc->kac", D, gXp), dW0, dWr, dWi      # X' = D M


def so2_edge_block_backward(graph, pos, box, x, T_edge, W0, Wr, Wi, lmax, E, r_cut, dT_out, chunk=4096):
    """Adjoint of so2_edge_block: from dT_out [n_edges][(lmax+1)^2][E] returns (dx [n_total][...], dT_in, dW0, [dWr_m],
    [dWi_m]).  T' = T + f_c y: the identity term passes dT_out on, the message term goes through so2_messages_backward
    with gY = f_c dT_out."""
    src, dst, shift, row_ptr = graph
    x = np.asarray(x, F64)
    dT_out = np.asarray(dT_out, F64)
    dx = np.zeros_like(x)
    dT_in = dT_out.copy()
    shapes = so2_shapes(lmax, E)
    dW0 = np.zeros(shapes[0], F64)
    dWr = [np.zeros(s, F64) for s in shapes[1:]]
    dWi = [np.zeros(s, F64) for s in shapes[1:]]
    for k0 in range(0, len(src), chunk):
        k1 = min(len(src), k0 + chunk)
        s_, d_ = src[k0:k1], dst[k0:k1]
        r = O.edge_vectors(pos, box, s_, d_, shift[k0:k1])
        fc = O.envelope(np.sqrt(np.einsum("ka,ka->k", r, r)), r_cut)
        gM, g0, gr, gi = so2_messages_backward(s_, d_, r, x, T_edge[k0:k1], W0, Wr, Wi, lmax, E,
                                               dT_out[k0:k1] * fc[:, None, None])
        np.add.at(dx, s_, gM[:, :, :E])
        np.add.at(dx, d_, gM[:, :, E:2 * E])
        dT_in[k0:k1] += gM[:, :, 2 * E:]
        dW0 += g0
        for m in range(lmax):
            dWr[m] += gr[m]
            dWi[m] += gi[m]
    return dx, dT_in, dW0, dWr, dWi


def so2_node_block_backward(graph, pos, box, x, T_edge, W0, Wr, Wi, w_att, lmax, E, r_cut, da, slope=0.2,
                            near_kink=None, kink_eps=0.0):
    """Adjoint of so2_node_block: from da [n_owned][(lmax+1)^2][E] returns (dx, dT_edge, dW0, [dWr_m], [dWi_m], dw_att).
    Per destination node j with incoming edges k: a_j = sum_k alpha_k f_c,k y_k, alpha = softmax(s), s_k = w_att .
    LeakyReLU(y_k[L = 0]).  Backwards: t_k = f_c,k <da_j, y_k> is the gradient of alpha_k; the softmax gives
    ds_k = alpha_k (t_k - sum_k' alpha_k' t_k'); the score gives dw_att += ds_k LeakyReLU(y0_k) and
    gY_k[L = 0] += ds_k w_att LeakyReLU'(y0_k); the weighted sum gives gY_k += alpha_k f_c,k da_j.
    near_kink: if a list is given, the ids of the edges that have a score input |y0_k[c]| < kink_eps are appended to it
    (LeakyReLU' jumps at zero: there a comparison in lower precision may legitimately take the other branch)."""
    src, dst, shift, row_ptr = graph
    x = np.asarray(x, F64)
    da = np.asarray(da, F64)
    w_att = np.asarray(w_att, F64)
    n_owned = len(row_ptr) - 1
    dx = np.zeros_like(x)
    dT = np.zeros((len(src), (lmax + 1) ** 2, E), F64)
    shapes = so2_shapes(lmax, E)
    dW0 = np.zeros(shapes[0], F64)
    dWr = [np.zeros(s, F64) for s in shapes[1:]]
    dWi = [np.zeros(s, F64) for s in shapes[1:]]
    dw_att = np.zeros(E, F64)
    for j in range(n_owned):
        k0, k1 = int(row_ptr[j]), int(row_ptr[j + 1])
        if k1 == k0:
            continue
        s_, d_ = src[k0:k1], dst[k0:k1]
        r = O.edge_vectors(pos, box, s_, d_, shift[k0:k1])
        Y = so2_messages(s_, d_, r, x, None, W0, Wr, Wi, lmax, E, 0, r_cut, T_edge=T_edge[k0:k1], envelope=False)
        y0 = Y[:, 0, :]
        alpha = attention_weights(y0, w_att, np.array([0, k1 - k0]), slope)
        fc = O.envelope(np.sqrt(np.einsum("ka,ka->k", r, r)), r_cut)
        t = fc * np.einsum("ac,kac->k", da[j], Y)
        ds = alpha * (t - np.dot(alpha, t))
        if near_kink is not None:
            near_kink.extend((k0 + np.nonzero((np.abs(y0) < kink_eps).any(axis=1))[0]).tolist())
        act = np.where(y0 > 0, y0, slope * y0)
        dw_att += ds @ act
        gY = (alpha * fc)[:, None, None] * da[j][None, :, :]
        gY[:, 0, :] += ds[:, None] * w_att[None, :] * np.where(y0 > 0, 1.0, slope)
        gM, g0, gr, gi = so2_messages_backward(s_, d_, r, x, T_edge[k0:k1], W0, Wr, Wi, lmax, E, gY)
        np.add.at(dx, s_, gM[:, :, :E])
        np.add.at(dx, d_, gM[:, :, E:2 * E])
        dT[k0:k1] = gM[:, :, 2 * E:]
        dW0 += g0
        for m in range(lmax):
            dWr[m] += gr[m]
            dWi[m] += gi[m]
    return dx, dT, dW0, dWr, dWi, dw_att


def gate_backward(x, W_g, lmax, dy):
    """Adjoint of gate: (dx, dW_g).  y[L=0] = SiLU(x0); y_l = x_l * g_l with g_l = sigmoid(W_g[l-1] x0), so
    dx_l = dy_l g_l, dg_l[c] = sum_m dy_l[m][c] x_l[m][c], dz_l = dg_l g_l (1 - g_l), dW_g[l-1] = sum_nodes dz_l x0^T,
    dx0 = dy0 SiLU'(x0) + sum_l W_g[l-1]^T dz_l."""
    x = np.asarray(x, F64)
    dy = np.asarray(dy, F64)
    x0 = x[:, 0, :]
    sg = 1.0 / (1.0 + np.exp(-x0))
    dx = np.zeros_like(x)
    dx[:, 0, :] = dy[:, 0, :] * (sg * (1.0 + x0 * (1.0 - sg)))
    dW = np.zeros((max(lmax, 0), x.shape[2], x.shape[2]), F64)
    for l in range(1, lmax + 1):
        Wl = np.asarray(W_g[l - 1], F64)
        g = 1.0 / (1.0 + np.exp(-(x0 @ Wl.T)))
        dx[:, O.sl(l), :] = dy[:, O.sl(l), :] * g[:, None, :]
        dz = np.einsum("nmc,nmc->nc", dy[:, O.sl(l), :], x[:, O.sl(l), :]) * g * (1.0 - g)
        dW[l - 1] = dz.T @ x0
        dx[:, 0, :] += dz @ Wl
    return dx, dW
