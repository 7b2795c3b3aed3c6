"""CPU oracle (fp64, numpy) for the equivariant message-passing hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition the HIP kernels are checked against.  It
is imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline
leg, and by nothing else; it shares no code with the HIP path.  All arithmetic is
fp64 on the fp32 inputs.

What it follows (arXiv 2507.03840):
  * graph of atoms with directed edges i -> j inside r_cut, periodic images
    included (Sec. 3 "Initialization of node and edge embeddings"; Sec. 4.4);
  * node tensors of shape (l_max+1)^2 x E per atom, (l, m) flattened, edge
    distances expanded in a Gaussian basis (same passage);
  * a message per directed edge built from the source embedding and the edge,
    transformed equivariantly and summed over the incoming edges of each node
    (Sec. 3 "Message passing"); the equivariant transform is written here in its
    general tensor-product form (Sec. 2.1, Sec. 2.2 and Eq. 1: Clebsch-Gordan
    coupling of |l1 m1>|l2 m2> into |L M>) rather than the bond-aligned SO(2)
    shortcut, which computes the same function;
  * "incoming edge" ownership: sums run only into owned nodes, halo nodes are
    read-only sources (Sec. 3 "Distribution", Fig. 2(f));
  * readout: channel collapse E -> 1, coupled blocks, inverse Clebsch-Gordan
    transform back to the (alpha, beta) orbital blocks H_ij (Fig. 2(e), Sec. 2.2,
    Sec. 3, 13 orbitals = 2s+2p+1d from Sec. 6).

The paper leaves the layer's details to its references; the choices made here
(radial MLP, path list, normalisation, conventions) are listed next to each
function.  Pins: tests/test_oracle_*.py check every function against closed
forms, quadrature, brute force and symmetry.  Nothing here is pinned to numbers
printed in the paper (it prints none for this layer): in that sense parity with
the paper's own network is unpinned.
"""
from functools import lru_cache
from math import factorial, sqrt, pi
import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# index helpers
# --------------------------------------------------------------------------------------
def sl(l):
    """Slice of degree l inside the flattened (l, m) axis, m = -l..l."""
    return slice(l * l, (l + 1) * (l + 1))


def tp_paths(l_in, l_sh, l_out):
    """Allowed couplings (l1, l2, l3): triangle rule and l1+l2+l3 even, lexicographic order.

    Sec. 2.2: l_a (x) l_b decomposes into L = |l_a-l_b| .. l_a+l_b.  The even-sum rule is the
    parity selection for features of parity (-1)^l coupled with spherical harmonics.
    """
    return [(l1, l2, l3)
            for l1 in range(l_in + 1) for l2 in range(l_sh + 1)
            for l3 in range(abs(l1 - l2), min(l1 + l2, l_out) + 1)
            if (l1 + l2 + l3) % 2 == 0]


def path_norm(paths):
    """alpha_p = 1/sqrt(number of paths that end in the same l3)."""
    count = {}
    for (_, _, l3) in paths:
        count[l3] = count.get(l3, 0) + 1
    return np.array([1.0 / sqrt(count[l3]) for (_, _, l3) in paths], F64)


# --------------------------------------------------------------------------------------
# O1  edge set (Sec. 3 "Initialization": edges i -> j within r_cut; Sec. 4.4: periodic)
# --------------------------------------------------------------------------------------
def neighbour_list(pos, n_owned, box, pbc, r_cut):
    """All ordered pairs (src i, dst j), i != j, j owned, |r_i + shift*box - r_j| < r_cut.

    Brute force over all pairs.  Minimum image on periodic axes (the box must be at least
    2*r_cut there, so the image is unique for every pair inside the cutoff).  Strict '<',
    fp64 on the fp32 inputs.  Output sorted by (dst, src); row_ptr is the CSR index over dst.
    """
    p = np.asarray(pos, np.float32).astype(F64)
    b = np.asarray(box, np.float32).astype(F64)
    rc2 = float(np.float32(r_cut)) ** 2
    n_total = p.shape[0]
    src, dst, shift = [], [], []
    row_ptr = np.zeros(n_owned + 1, np.int64)
    for j in range(n_owned):
        delta = p - p[j]
        image = np.zeros((n_total, 3), F64)
        for a in range(3):
            if pbc[a]:
                image[:, a] = -np.rint(delta[:, a] / b[a])
                delta[:, a] += image[:, a] * b[a]
        inside = np.einsum("ia,ia->i", delta, delta) < rc2
        inside[j] = False
        i = np.nonzero(inside)[0]
        src.append(i)
        dst.append(np.full(len(i), j))
        shift.append(image[i])
        row_ptr[j + 1] = row_ptr[j] + len(i)
    cat = lambda parts, dt, shape: (np.concatenate(parts).astype(dt) if parts else np.zeros(shape, dt))
    return (cat(src, np.int32, (0,)), cat(dst, np.int32, (0,)),
            cat(shift, np.int8, (0, 3)), row_ptr.astype(np.int32))


def edge_vectors(pos, box, src, dst, shift):
    """r_k = (source position, imaged) - (destination position), fp64."""
    p = np.asarray(pos, np.float32).astype(F64)
    b = np.asarray(box, np.float32).astype(F64)
    return p[src] + shift.astype(F64) * b - p[dst]


# --------------------------------------------------------------------------------------
# O2  real spherical harmonics (Sec. 2.2: orbitals transform like Y^l_m)
# --------------------------------------------------------------------------------------
def sph_harm_real(lmax, rhat):
    """Component-normalised real spherical harmonics Yhat = sqrt(4 pi) Y, shape [n, (lmax+1)^2].

    z is the polar axis, m runs -l..l; m > 0 carries cos(m phi), m < 0 carries sin(|m| phi),
    no Condon-Shortley sign in the real form.  With Q_l^m(z) = d^m P_l / dz^m:
      Y_l0 = N_l0 P_l(z),  Y_l,+m = sqrt2 N_lm Q_l^m(z) Re (x+iy)^m,  Y_l,-m = sqrt2 N_lm Q_l^m(z) Im (x+iy)^m,
      N_lm = sqrt((2l+1)/(4 pi) (l-m)!/(l+m)!).
    """
    r = np.asarray(rhat, F64)
    x, y, z = r[:, 0], r[:, 1], r[:, 2]
    n = r.shape[0]
    out = np.zeros((n, (lmax + 1) ** 2), F64)
    # Q[l][m] by the upward recurrence in l for fixed m
    Q = [[None] * (lmax + 1) for _ in range(lmax + 1)]
    for m in range(lmax + 1):
        dfact = 1.0
        for k in range(1, m + 1):
            dfact *= 2 * k - 1
        Q[m][m] = np.full(n, dfact)
        if m + 1 <= lmax:
            Q[m + 1][m] = (2 * m + 1) * z * Q[m][m]
        for l in range(m + 2, lmax + 1):
            Q[l][m] = ((2 * l - 1) * z * Q[l - 1][m] - (l + m - 1) * Q[l - 2][m]) / (l - m)
    xy = (x + 1j * y)
    for l in range(lmax + 1):
        for m in range(l + 1):
            N = sqrt((2 * l + 1) / (4 * pi) * factorial(l - m) / factorial(l + m))
            if m == 0:
                out[:, l * l + l] = N * Q[l][0]
            else:
                pw = xy ** m
                out[:, l * l + l + m] = sqrt(2.0) * N * Q[l][m] * pw.real
                out[:, l * l + l - m] = sqrt(2.0) * N * Q[l][m] * pw.imag
    return out * sqrt(4 * pi)


# --------------------------------------------------------------------------------------
# O3  Clebsch-Gordan coefficients (Eq. 1), real basis
# --------------------------------------------------------------------------------------
def cg_complex(j1, m1, j2, m2, J, M):
    """<j1 m1 j2 m2 | J M>, Condon-Shortley phases, Racah's closed formula."""
    if m1 + m2 != M or J < abs(j1 - j2) or J > j1 + j2 or abs(m1) > j1 or abs(m2) > j2 or abs(M) > J:
        return 0.0
    f = factorial
    pref = sqrt((2 * J + 1) * f(J + j1 - j2) * f(J - j1 + j2) * f(j1 + j2 - J) / f(j1 + j2 + J + 1))
    pref *= sqrt(f(J + M) * f(J - M) * f(j1 - m1) * f(j1 + m1) * f(j2 - m2) * f(j2 + m2))
    total = 0.0
    for k in range(0, j1 + j2 - J + 1):
        args = (k, j1 + j2 - J - k, j1 - m1 - k, j2 + m2 - k, J - j2 + m1 + k, J - j1 - m2 + k)
        if min(args) < 0:
            continue
        den = 1
        for a in args:
            den *= f(a)
        total += (-1) ** k / den
    return pref * total


def real_basis_change(l):
    """U[m, mu]: real Y_lm = sum_mu U[m, mu] Y_l^mu (complex, Condon-Shortley). Index = value + l."""
    U = np.zeros((2 * l + 1, 2 * l + 1), complex)
    U[l, l] = 1.0
    for m in range(1, l + 1):
        U[l + m, l + m] = (-1) ** m / sqrt(2)
        U[l + m, l - m] = 1 / sqrt(2)
        U[l - m, l + m] = -1j * (-1) ** m / sqrt(2)
        U[l - m, l - m] = 1j / sqrt(2)
    return U


@lru_cache(maxsize=None)
def cg_real(l1, l2, l3):
    """Real coupling tensor C[m1, m2, m3] (indices shifted by l), orthonormal in (m1 m2) per m3.

    C = sum U1 U2 conj(U3) <l1 mu1 l2 mu2 | l3 mu3>; this is real when l1+l2+l3 is even and
    purely imaginary when it is odd, in which case the imaginary part is taken.
    """
    cc = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1), F64)
    for a in range(-l1, l1 + 1):
        for b in range(-l2, l2 + 1):
            if abs(a + b) <= l3:
                cc[a + l1, b + l2, a + b + l3] = cg_complex(l1, a, l2, b, l3, a + b)
    t = np.einsum("ai,bj,ck,ijk->abc", real_basis_change(l1), real_basis_change(l2),
                  np.conj(real_basis_change(l3)), cc.astype(complex))
    return np.ascontiguousarray(t.real if (l1 + l2 + l3) % 2 == 0 else t.imag)


# --------------------------------------------------------------------------------------
# O4  radial part (Sec. 3: edge distances expanded in a Gaussian basis)
# --------------------------------------------------------------------------------------
def radial_basis(d, n_rbf, r_cut):
    """B_b(d) = exp(-(d-mu_b)^2 / (2 sigma^2)), mu_b = b r_cut/(n_b-1), sigma = r_cut/(n_b-1)."""
    rc = float(np.float32(r_cut))
    mu = np.arange(n_rbf, dtype=F64) * rc / (n_rbf - 1)
    sigma = rc / (n_rbf - 1)
    return np.exp(-((d[:, None] - mu[None, :]) ** 2) / (2 * sigma * sigma))


def envelope(d, r_cut):
    """Cosine cutoff f_c(d) = (1 + cos(pi d / r_cut)) / 2."""
    return 0.5 * (1.0 + np.cos(pi * d / float(np.float32(r_cut))))


def silu(t):
    return t / (1.0 + np.exp(-t))


def radial_weights(d, W_r1, W_r2, paths, channels, n_rbf, r_cut, w_dtype=None):
    """w[k, p, c] = f_c(d_k) alpha_p (W_r2 SiLU(W_r1 B(d_k)))[p*E + c]; no biases.

    w_dtype=np.float16 models the mixed-precision mode (Sec. 4.1: half-precision values, fp32 sums): the weights are
    rounded to half precision (round to nearest even) where they are stored; everything else stays as it is."""
    B = radial_basis(d, n_rbf, r_cut)
    g = silu(B @ np.asarray(W_r1, F64).T)
    w = (g @ np.asarray(W_r2, F64).T).reshape(len(d), len(paths), channels)
    w = w * envelope(d, r_cut)[:, None, None] * path_norm(paths)[None, :, None]
    return w if w_dtype is None else w.astype(w_dtype).astype(F64)


# --------------------------------------------------------------------------------------
# O5  message-passing layer
# --------------------------------------------------------------------------------------
def mix_channels(x, W, lmax):
    """y[n, (l,m), c] = sum_c' W[l, c, c'] x[n, (l,m), c']  (the per-degree linear of Fig. 2(d))."""
    x = np.asarray(x, F64)
    y = np.empty((x.shape[0], x.shape[1], W.shape[1]), F64)
    for l in range(lmax + 1):
        y[:, sl(l), :] = np.einsum("dc,nmc->nmd", np.asarray(W[l], F64), x[:, sl(l), :])
    return y


def tensor_product(h, Y, w, paths, l_out):
    """u[k, (l3,m3), c] = sum_p w[k,p,c] sum_{m1,m2} C_p[m1,m2,m3] h[k,(l1,m1),c] Y[k,(l2,m2)]   (Eq. 1)."""
    n, _, E = h.shape
    u = np.zeros((n, (l_out + 1) ** 2, E), F64)
    for p, (l1, l2, l3) in enumerate(paths):
        C = cg_real(l1, l2, l3)
        CY = np.einsum("abm,kb->kam", C, Y[:, sl(l2)])
        u[:, sl(l3), :] += w[:, p, None, :] * np.einsum("kam,kac->kmc", CY, h[:, sl(l1), :])
    return u


def species_embed(x, species, table):
    """Adds table[species_i] into the l = 0 plane (Sec. 3: the L=0 plane is initialised from Z_i)."""
    y = np.array(x, F64)
    y[:, 0, :] += np.asarray(table, F64)[species]
    return y


def edge_messages_sum(graph, pos, box, h, weights_fn, lmax, l_sh, agg_norm, chunk_nodes=64):
    """a_j = agg_norm^-1/2 sum_{k: dst(k)=j} TP(h_src(k), Yhat(rhat_k); w_k), owned j only."""
    src, dst, shift, row_ptr = graph
    n_owned = len(row_ptr) - 1
    paths = tp_paths(lmax, l_sh, lmax)
    a = np.zeros((n_owned, (lmax + 1) ** 2, h.shape[2]), F64)
    for j0 in range(0, n_owned, chunk_nodes):
        j1 = min(n_owned, j0 + chunk_nodes)
        k0, k1 = int(row_ptr[j0]), int(row_ptr[j1])
        if k1 == k0:
            continue
        r = edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
        d = np.sqrt(np.einsum("ka,ka->k", r, r))
        Y = sph_harm_real(l_sh, r / d[:, None])
        w = weights_fn(d, k0, k1, paths)
        u = tensor_product(h[src[k0:k1]], Y, w, paths, lmax)
        for j in range(j0, j1):
            a[j] = u[row_ptr[j] - k0:row_ptr[j + 1] - k0].sum(axis=0)
    return a / sqrt(agg_norm)


def layer_forward(graph, pos, box, x_in, W, lmax, l_sh, channels, n_rbf, r_cut, agg_norm, w_edge=None, w_dtype=None):
    """One message-passing layer.  x_in has n_total rows (owned first), returns the n_owned new rows.

    h = W_pre x (all nodes);  a_j as in edge_messages_sum;  x'_j = W_post a_j + W_self x_j.
    The destination's own embedding enters through W_self, the edge through the radial
    weights: a linear map of the concatenated message (Sec. 3) split into its three terms.
    """
    x = np.asarray(x_in, F64)
    h = mix_channels(x, W["W_pre"], lmax)
    if w_edge is None:
        fn = lambda d, k0, k1, paths: radial_weights(d, W["W_r1"], W["W_r2"], paths, channels, n_rbf, r_cut, w_dtype)
    else:
        fn = lambda d, k0, k1, paths: np.asarray(w_edge[k0:k1], F64)
    a = edge_messages_sum(graph, pos, box, h, fn, lmax, l_sh, agg_norm)
    n_owned = a.shape[0]
    return mix_channels(a, W["W_post"], lmax) + mix_channels(x[:n_owned], W["W_self"], lmax)


# --------------------------------------------------------------------------------------
# O6  H_ij readout
# --------------------------------------------------------------------------------------
L_READOUT = 4


def readout_slots(orb_l):
    """Enumerates o(alpha, beta, L): ordered shell pairs in row-major shell order, L ascending.

    Returns (slots, n_out) with slots = list of (alpha, beta, L, index within V_L) and n_out[L].
    """
    n_out = [0] * (L_READOUT + 1)
    slots = []
    for a, la in enumerate(orb_l):
        for b, lb in enumerate(orb_l):
            for L in range(abs(la - lb), la + lb + 1):
                slots.append((a, b, L, n_out[L]))
                n_out[L] += 1
    return slots, n_out


def readout_hij(graph, pos, box, x, W, lmax, l_sh, channels, n_rbf, r_cut, orb_l, k_range=None, w_dtype=None):
    """H_k[(alpha, m_a), (beta, m_b)] for edges k (rows: source-atom orbitals, cols: destination's).

    z_k = (W_s x)_src + (W_t x)_dst;  u_k = TP(z_k, Yhat_k; w_k) for L <= 4;
    q_k[o, M] = sum_c V_L[o, c] u_k[L, M, c]   (collapse E -> 1, Fig. 2(e));
    H_k = sum_{L,M} C^{(L,M)}_{(l_a m_a)(l_b m_b)} q_k[o(a,b,L), M]   (inverse of Eq. 1).
    """
    src, dst, shift, row_ptr = graph
    k0, k1 = (0, len(src)) if k_range is None else k_range
    xs = mix_channels(np.asarray(x, F64), W["W_s"], lmax)
    xt = mix_channels(np.asarray(x, F64), W["W_t"], lmax)
    paths = tp_paths(lmax, l_sh, L_READOUT)
    slots, n_out = readout_slots(orb_l)
    v_off = np.concatenate([[0], np.cumsum(n_out)])
    V = np.asarray(W["V"], F64)
    orb_off = np.concatenate([[0], np.cumsum([2 * l + 1 for l in orb_l])])
    n_orb = int(orb_off[-1])
    H = np.zeros((k1 - k0, n_orb, n_orb), F64)
    step = 8192
    for c0 in range(k0, k1, step):
        c1 = min(k1, c0 + step)
        r = edge_vectors(pos, box, src[c0:c1], dst[c0:c1], shift[c0:c1])
        d = np.sqrt(np.einsum("ka,ka->k", r, r))
        Y = sph_harm_real(l_sh, r / d[:, None])
        w = radial_weights(d, W["W_r1"], W["W_r2"], paths, channels, n_rbf, r_cut, w_dtype)
        z = xs[src[c0:c1]] + xt[dst[c0:c1]]
        u = tensor_product(z, Y, w, paths, L_READOUT)
        for (a, b, L, o) in slots:
            q = np.einsum("c,kmc->km", V[v_off[L] + o], u[:, sl(L), :])
            C = cg_real(orb_l[a], orb_l[b], L)
            H[c0 - k0:c1 - k0, orb_off[a]:orb_off[a + 1], orb_off[b]:orb_off[b + 1]] += \
                np.einsum("abm,km->kab", C, q)
    return H


def loss_mse(H, T):
    """Mean over all n_e * n_orb^2 entries of (H - T)^2."""
    diff = np.asarray(H, F64) - np.asarray(T, F64)
    return float(np.mean(diff * diff))


# --------------------------------------------------------------------------------------
# O7  reverse pass (training step; the paper leaves the gradients to its framework's automatic differentiation,
#     Sec. 4.1; here they are written out by hand, the adjoint of each function above in reverse order)
# --------------------------------------------------------------------------------------
def loss_mse_backward(H, T):
    """dL/dH for L = mean (H - T)^2."""
    diff = np.asarray(H, F64) - np.asarray(T, F64)
    return 2.0 * diff / diff.size


def mix_channels_backward(x, W, dy, lmax):
    """Adjoint of mix_channels: returns (dx, dW)."""
    x = np.asarray(x, F64)
    dx = np.zeros_like(x)
    dW = np.zeros(np.shape(W), F64)
    for l in range(lmax + 1):
        dW[l] = np.einsum("nmd,nmc->dc", dy[:, sl(l), :], x[:, sl(l), :])
        dx[:, sl(l), :] = np.einsum("dc,nmd->nmc", np.asarray(W[l], F64), dy[:, sl(l), :])
    return dx, dW


def tensor_product_backward(h, Y, w, paths, du):
    """Adjoint of tensor_product w.r.t. the features and the weights: returns (dh, dw)."""
    dh = np.zeros_like(h)
    dw = np.zeros_like(w)
    for p, (l1, l2, l3) in enumerate(paths):
        C = cg_real(l1, l2, l3)
        CY = np.einsum("abm,kb->kam", C, Y[:, sl(l2)])
        t = np.einsum("kam,kmc->kac", CY, du[:, sl(l3), :])
        dh[:, sl(l1), :] += w[:, p, None, :] * t
        dw[:, p, :] = np.einsum("kac,kac->kc", h[:, sl(l1), :], t)
    return dh, dw


def radial_weights_backward(d, W_r1, W_r2, paths, channels, n_rbf, r_cut, dw):
    """Adjoint of radial_weights w.r.t. its two matrices: returns (dW_r1, dW_r2)."""
    W_r1, W_r2 = np.asarray(W_r1, F64), np.asarray(W_r2, F64)
    B = radial_basis(d, n_rbf, r_cut)
    pre = B @ W_r1.T
    sig = 1.0 / (1.0 + np.exp(-pre))
    g = pre * sig
    dwl = (dw * envelope(d, r_cut)[:, None, None] * path_norm(paths)[None, :, None]).reshape(len(d), -1)
    dW_r2 = dwl.T @ g
    dpre = (dwl @ W_r2) * (sig * (1.0 + pre * (1.0 - sig)))
    return dpre.T @ B, dW_r2


def layer_backward(graph, pos, box, x_in, W, lmax, l_sh, channels, n_rbf, r_cut, agg_norm, dx_out):
    """Adjoint of layer_forward.  Returns (dx_in [n_total rows], dict of weight gradients)."""
    src, dst, shift, row_ptr = graph
    x = np.asarray(x_in, F64)
    n_owned = len(row_ptr) - 1
    paths = tp_paths(lmax, l_sh, lmax)
    h = mix_channels(x, W["W_pre"], lmax)
    # forward quantities needed again: a (for dW_post)
    fn = lambda d, k0, k1, pth: radial_weights(d, W["W_r1"], W["W_r2"], pth, channels, n_rbf, r_cut)
    a = edge_messages_sum(graph, pos, box, h, fn, lmax, l_sh, agg_norm)
    da, dW_post = mix_channels_backward(a, W["W_post"], dx_out, lmax)
    dx_self, dW_self = mix_channels_backward(x[:n_owned], W["W_self"], dx_out, lmax)
    dh = np.zeros_like(h)
    dW_r1 = np.zeros(np.shape(W["W_r1"]), F64)
    dW_r2 = np.zeros(np.shape(W["W_r2"]), F64)
    step = 4096
    for k0 in range(0, len(src), step):
        k1 = min(len(src), k0 + step)
        r = edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
        d = np.sqrt(np.einsum("ka,ka->k", r, r))
        Y = sph_harm_real(l_sh, r / d[:, None])
        w = radial_weights(d, W["W_r1"], W["W_r2"], paths, channels, n_rbf, r_cut)
        du = da[dst[k0:k1]] / sqrt(agg_norm)
        dh_k, dw_k = tensor_product_backward(h[src[k0:k1]], Y, w, paths, du)
        np.add.at(dh, src[k0:k1], dh_k)
        g1, g2 = radial_weights_backward(d, W["W_r1"], W["W_r2"], paths, channels, n_rbf, r_cut, dw_k)
        dW_r1 += g1
        dW_r2 += g2
    dx, dW_pre = mix_channels_backward(x, W["W_pre"], dh, lmax)
    dx[:n_owned] += dx_self
    return dx, dict(W_pre=dW_pre, W_post=dW_post, W_self=dW_self, W_r1=dW_r1, W_r2=dW_r2)


def readout_backward(graph, pos, box, x, W, lmax, l_sh, channels, n_rbf, r_cut, orb_l, dH):
    """Adjoint of readout_hij.  Returns (dx [n_total rows], dict of weight gradients)."""
    src, dst, shift, row_ptr = graph
    x = np.asarray(x, F64)
    xs = mix_channels(x, W["W_s"], lmax)
    xt = mix_channels(x, W["W_t"], lmax)
    paths = tp_paths(lmax, l_sh, L_READOUT)
    slots, n_out = readout_slots(orb_l)
    v_off = np.concatenate([[0], np.cumsum(n_out)])
    V = np.asarray(W["V"], F64)
    orb_off = np.concatenate([[0], np.cumsum([2 * l + 1 for l in orb_l])])
    dxs, dxt = np.zeros_like(xs), np.zeros_like(xt)
    dV = np.zeros_like(V)
    dW_r1 = np.zeros(np.shape(W["W_r1"]), F64)
    dW_r2 = np.zeros(np.shape(W["W_r2"]), F64)
    step = 4096
    for k0 in range(0, len(src), step):
        k1 = min(len(src), k0 + step)
        r = edge_vectors(pos, box, src[k0:k1], dst[k0:k1], shift[k0:k1])
        d = np.sqrt(np.einsum("ka,ka->k", r, r))
        Y = sph_harm_real(l_sh, r / d[:, None])
        w = radial_weights(d, W["W_r1"], W["W_r2"], paths, channels, n_rbf, r_cut)
        z = xs[src[k0:k1]] + xt[dst[k0:k1]]
        u = tensor_product(z, Y, w, paths, L_READOUT)
        du = np.zeros_like(u)
        for (a, b, L, o) in slots:
            C = cg_real(orb_l[a], orb_l[b], L)
            dq = np.einsum("abm,kab->km", C, dH[k0:k1, orb_off[a]:orb_off[a + 1], orb_off[b]:orb_off[b + 1]])
            dV[v_off[L] + o] += np.einsum("km,kmc->c", dq, u[:, sl(L), :])
            du[:, sl(L), :] += dq[:, :, None] * V[v_off[L] + o][None, None, :]
        dz, dw_k = tensor_product_backward(z, Y, w, paths, du)
        np.add.at(dxs, src[k0:k1], dz)
        np.add.at(dxt, dst[k0:k1], dz)
        g1, g2 = radial_weights_backward(d, W["W_r1"], W["W_r2"], paths, channels, n_rbf, r_cut, dw_k)
        dW_r1 += g1
        dW_r2 += g2
    dx1, dW_s = mix_channels_backward(x, W["W_s"], dxs, lmax)
    dx2, dW_t = mix_channels_backward(x, W["W_t"], dxt, lmax)
    return dx1 + dx2, dict(W_s=dW_s, W_t=dW_t, W_r1=dW_r1, W_r2=dW_r2, V=dV)


# --------------------------------------------------------------------------------------
# test tool: Wigner-D matrices from their defining property (Sec. 2.2)
# --------------------------------------------------------------------------------------
def wigner_d_real(l, R, rng=None):
    """D^l(R) with Y_l(R r) = D^l(R) Y_l(r) for all r, by least squares over random directions."""
    rng = np.random.default_rng(12345) if rng is None else rng
    v = rng.standard_normal((8 * (2 * l + 1), 3))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    A = sph_harm_real(l, v)[:, sl(l)]
    B = sph_harm_real(l, v @ np.asarray(R, F64).T)[:, sl(l)]
    X, *_ = np.linalg.lstsq(A, B, rcond=None)
    return X.T


def wigner_d_block(lmax, R):
    """Block-diagonal D over l = 0..lmax acting on the flattened (l, m) axis."""
    D = np.zeros(((lmax + 1) ** 2,) * 2, F64)
    for l in range(lmax + 1):
        D[sl(l), sl(l)] = wigner_d_real(l, R)
    return D
