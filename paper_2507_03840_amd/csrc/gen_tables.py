#!/usr/bin/env python3
"""Build step: writes csrc/egnn_gen.inc, the unrolled constants of the HIP tensor-product kernels.

The kernels evaluate the Clebsch-Gordan tensor product of a feature vector with the
spherical harmonics of the edge direction (Sec. 2.1, Sec. 2.2 and Eq. 1 of arXiv 2507.03840)
in the bond-aligned frame (Sec. 2.1 last paragraph, Fig. 2(d)): rotate the feature so that the
edge lies on the polar axis, where Yhat_{l2,m2} = sqrt(2 l2+1) delta_{m2,0} and every coupling
path collapses to a few constants, then rotate back.  The rotation is factored as

    D(R) = J^T Z(-theta) J Z(-phi),      R r_hat = z_hat,

with Z(a) the rotation about the polar axis (2x2 blocks of cos/sin m a) and J = D(R_x(pi/2)) a
constant sparse matrix per degree, so the only per-edge quantities are cos/sin of m*phi, m*theta.

Everything here is computed from scratch (complex spherical harmonics from scipy, Wigner
matrices from their defining property, coupling coefficients from ladder operators) and
checked against a dense evaluation before anything is written.  Conventions (shared with the
callers of the library, stated in include/egnn.h): z polar axis, m = -l..l, m>0 ~ cos(m phi),
m<0 ~ sin(|m| phi), component normalisation, real coupling tensor = real part (l1+l2+l3 even)
or imaginary part (odd) of the complex Condon-Shortley coefficients in the real basis.
"""
import os
import sys
from fractions import Fraction
from math import sqrt, pi
import numpy as np
from scipy.special import sph_harm_y

LMAX = 4
L_READOUT = 4
ORB_LMAX = 2


# ------------------------------------------------------------------ real harmonics and rotations
def real_sh(l, v):
    """Real orthonormal harmonics of degree l at unit vectors v (component order m = -l..l)."""
    x, y, z = v.T
    theta = np.arccos(np.clip(z, -1.0, 1.0))
    phi = np.arctan2(y, x)
    out = np.zeros((len(v), 2 * l + 1))
    for m in range(l + 1):
        Y = sph_harm_y(l, m, theta, phi)
        if m == 0:
            out[:, l] = Y.real
        else:
            out[:, l + m] = sqrt(2) * (-1) ** m * Y.real
            out[:, l - m] = sqrt(2) * (-1) ** m * Y.imag
    return out


def rotation_matrix_of_degree(l, R):
    """D with Y_l(R r) = D Y_l(r): least squares over many directions (exact up to rounding)."""
    rng = np.random.default_rng(2024 + l)
    v = rng.standard_normal((12 * (2 * l + 1), 3))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    X, *_ = np.linalg.lstsq(real_sh(l, v), real_sh(l, v @ R.T), rcond=None)
    return X.T


def rot_x(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[1, 0, 0], [0, c, -s], [0, s, c]])


def rot_y(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, 0, s], [0, 1, 0], [-s, 0, c]])


def rot_z(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, -s, 0], [s, c, 0], [0, 0, 1]])


def z_block(l, a):
    """Z(a) = D^l(R_z(a)) written out: the form the kernels apply."""
    Z = np.zeros((2 * l + 1, 2 * l + 1))
    Z[l, l] = 1.0
    for m in range(1, l + 1):
        c, s = np.cos(m * a), np.sin(m * a)
        Z[l + m, l + m], Z[l + m, l - m] = c, -s
        Z[l - m, l + m], Z[l - m, l - m] = s, c
    return Z


def j_matrix(l):
    J = rotation_matrix_of_degree(l, rot_x(pi / 2))
    J[np.abs(J) < 1e-12] = 0.0
    # the factorisation the kernels rely on
    for a in (0.3, -1.1, 2.5):
        assert np.allclose(rotation_matrix_of_degree(l, rot_z(a)), z_block(l, a), atol=1e-12)
        assert np.allclose(rotation_matrix_of_degree(l, rot_y(a)), J.T @ z_block(l, a) @ J, atol=1e-12)
    return J


# ------------------------------------------------------------------ coupling coefficients by ladder operators
def _ladder_down(j, m):
    """<j m-1| J_- |j m>^2 as an exact fraction."""
    return Fraction((j + m) * (j - m + 1))


def coupling_complex(j1, j2, J):
    """Table c[(m1, m2)] = <j1 m1 j2 m2 | J m1+m2> from the highest-weight state and J_-.

    |J J> = sum_m1 a(m1) |j1 m1>|j2 J-m1> with J_+|J J> = 0, a(j1) > 0 (Condon-Shortley)."""
    # highest weight: recursion a(m1-1) = -a(m1) * sqrt(up1(m1-1)) / sqrt(up2(m2)) from J_+ = J1_+ + J2_+
    hi = {}
    m1 = j1
    while m1 >= -j1 and abs(J - m1) > j2:
        m1 -= 1
    start = m1
    hi[start] = 1.0
    m1 = start
    while m1 - 1 >= -j1 and abs(J - (m1 - 1)) <= j2:
        m2 = J - m1
        up1 = float(_ladder_down(j1, m1)) ** 0.5            # <m1| J1+ |m1-1>
        up2 = float(_ladder_down(j2, m2 + 1)) ** 0.5        # <m2+1| J2+ |m2>
        hi[m1 - 1] = -hi[m1] * up2 / up1
        m1 -= 1
    norm = sqrt(sum(v * v for v in hi.values()))
    state = {(a, J - a): v / norm for a, v in hi.items()}
    assert state[(start, J - start)] > 0
    table = dict(state)
    M = J
    while M > -J:
        new = {}
        for (a, b), v in state.items():
            if a - 1 >= -j1:
                new[(a - 1, b)] = new.get((a - 1, b), 0.0) + v * float(_ladder_down(j1, a)) ** 0.5
            if b - 1 >= -j2:
                new[(a, b - 1)] = new.get((a, b - 1), 0.0) + v * float(_ladder_down(j2, b)) ** 0.5
        scale = float(_ladder_down(J, M)) ** 0.5
        state = {k: v / scale for k, v in new.items()}
        table.update(state)
        M -= 1
    return table


def to_real_basis(l):
    U = np.zeros((2 * l + 1, 2 * l + 1), complex)
    U[l, l] = 1
    r = 1 / sqrt(2)
    for m in range(1, l + 1):
        sgn = -1.0 if m % 2 else 1.0
        U[l + m, l + m], U[l + m, l - m] = sgn * r, r
        U[l - m, l + m], U[l - m, l - m] = -1j * sgn * r, 1j * r
    return U


def coupling_real(l1, l2, l3):
    T = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1), complex)
    for (a, b), v in coupling_complex(l1, l2, l3).items():
        T[a + l1, b + l2, a + b + l3] = v
    T = np.einsum("ai,bj,ck,ijk->abc", to_real_basis(l1), to_real_basis(l2), to_real_basis(l3).conj(), T)
    C = T.real if (l1 + l2 + l3) % 2 == 0 else T.imag
    other = T.imag if (l1 + l2 + l3) % 2 == 0 else T.real
    assert np.abs(other).max() < 1e-13
    C = np.where(np.abs(C) < 1e-13, 0.0, C)
    assert np.allclose(np.einsum("abm,abn->mn", C, C), np.eye(2 * l3 + 1), atol=1e-12)
    return C


def check_even_coupling_against_triple_integrals(l1, l2, l3, C):
    """Independent check of sign and scale for even paths: C is proportional to the integral of three
    real harmonics with a factor whose sign is (-1)^((l1+l2+l3)/2 - l3)."""
    t, wt = np.polynomial.legendre.leggauss(20)
    nphi = 41
    ph = 2 * pi * np.arange(nphi) / nphi
    T, P = np.meshgrid(t, ph, indexing="ij")
    s = np.sqrt(1 - T * T)
    pts = np.stack([s * np.cos(P), s * np.sin(P), T], -1).reshape(-1, 3)
    w = (wt[:, None] * np.full(nphi, 2 * pi / nphi)[None]).reshape(-1)
    G = np.einsum("n,na,nb,nc->abc", w, real_sh(l1, pts), real_sh(l2, pts), real_sh(l3, pts))
    G = G / np.sqrt(np.einsum("abm,abm->m", G, G))[None, None, :]
    sign = -1.0 if ((l1 + l2 + l3) // 2 - l3) % 2 else 1.0
    assert np.allclose(C, sign * G, atol=1e-11), (l1, l2, l3)


def tp_paths(l_in, l_sh, l_out):
    out = []
    for l1 in range(l_in + 1):
        for l2 in range(l_sh + 1):
            for l3 in range(abs(l1 - l2), min(l1 + l2, l_out) + 1):
                if (l1 + l2 + l3) % 2 == 0:
                    out.append((l1, l2, l3))
    return out


# ------------------------------------------------------------------ bond-frame form of one tensor product
def bond_frame_constants(l_in, l_sh, l_out):
    """For every (l1, l3): list over m = 0..min(l1,l3) of [(path index, K)] with
    K = sqrt(2 l2+1) C_p[m, 0, m]; in the bond frame out'[l3, +-m] += (sum_p w_p K) v'[l1, +-m]."""
    paths = tp_paths(l_in, l_sh, l_out)
    groups = {}
    for p, (l1, l2, l3) in enumerate(paths):
        C = coupling_real(l1, l2, l3)
        check_even_coupling_against_triple_integrals(l1, l2, l3, C)
        K = sqrt(2 * l2 + 1) * C[:, l2, :]
        off = K.copy()
        for m in range(-min(l1, l3), min(l1, l3) + 1):
            off[l1 + m, l3 + m] = 0.0
            assert abs(K[l1 + m, l3 + m] - K[l1 - m, l3 - m]) < 1e-12
        assert np.abs(off).max() < 1e-12
        for m in range(min(l1, l3) + 1):
            if abs(K[l1 + m, l3 + m]) > 1e-12:
                groups.setdefault((l1, l3), {}).setdefault(m, []).append((p, float(K[l1 + m, l3 + m])))
    return paths, groups


def emulate_bond_frame_tp(l_in, l_sh, l_out, groups, Jm, v, w, rhat):
    """numpy model of exactly what the kernel does for one edge and one channel."""
    x, y, z = rhat
    rho = sqrt(x * x + y * y)
    cphi, sphi = (x / rho, y / rho) if rho > 1e-20 else (1.0, 0.0)
    phi, theta = np.arctan2(sphi, cphi), np.arctan2(rho, z)
    vin = v.copy()
    for l in range(l_in + 1):
        s = slice(l * l, (l + 1) ** 2)
        vin[s] = Jm[l].T @ (z_block(l, -theta) @ (Jm[l] @ (z_block(l, -phi) @ v[s])))
    o = np.zeros((l_out + 1) ** 2)
    for (l1, l3), by_m in groups.items():
        for m, terms in by_m.items():
            g = sum(w[p] * k for p, k in terms)
            o[l3 * l3 + l3 + m] += g * vin[l1 * l1 + l1 + m]
            if m:
                o[l3 * l3 + l3 - m] += g * vin[l1 * l1 + l1 - m]
    for l in range(l_out + 1):
        s = slice(l * l, (l + 1) ** 2)
        o[s] = z_block(l, phi) @ (Jm[l].T @ (z_block(l, theta) @ (Jm[l] @ o[s])))
    return o


def dense_tp(l_in, l_sh, l_out, paths, v, w, rhat):
    o = np.zeros((l_out + 1) ** 2)
    for p, (l1, l2, l3) in enumerate(paths):
        Y = sqrt(4 * pi) * real_sh(l2, rhat[None])[0]
        o[l3 * l3:(l3 + 1) ** 2] += w[p] * np.einsum("abm,a,b->m", coupling_real(l1, l2, l3),
                                                      v[l1 * l1:(l1 + 1) ** 2], Y)
    return o


# ------------------------------------------------------------------ code emission
def f32(x):
    return repr(float(np.float32(x))) + "f"


def emit_matvec(name, M, doc):
    """In-place v <- M v on a (2l+1)-vector of registers, constants as literals."""
    n = M.shape[0]
    lines = [f"// {doc}", f"__device__ __forceinline__ void {name}(float* v) {{"]
    for i in range(n):
        terms = []
        for j in range(n):
            c = M[i, j]
            if c == 0.0:
                continue
            if abs(c - 1.0) < 1e-12:
                terms.append(f"v[{j}]")
            elif abs(c + 1.0) < 1e-12:
                terms.append(f"-v[{j}]")
            else:
                terms.append(f"{f32(c)} * v[{j}]")
        lines.append(f"  const float t{i} = {' + '.join(terms) if terms else '0.0f'};")
    for i in range(n):
        lines.append(f"  v[{i}] = t{i};")
    lines.append("}")
    return "\n".join(lines)


def emit_mid(l_in, l_sh, l_out, paths, groups):
    tag = f"{l_in}_{l_sh}_{l_out}"
    lines = [f"// bond-frame tensor product, paths P({l_in},{l_sh},{l_out}); o is overwritten",
             f"struct TpMid_{tag} {{",
             f"  static constexpr int L_IN = {l_in}, L_SH = {l_sh}, L_OUT = {l_out}, P = {len(paths)};",
             "  __device__ __forceinline__ static void run(const float* v, const float* w, float* o) {"]
    touched = set()
    for (l1, l3) in sorted(groups):
        for m in sorted(groups[(l1, l3)]):
            terms = groups[(l1, l3)][m]
            g = " + ".join(f"{f32(k)} * w[{p}]" for p, k in terms)
            lines.append(f"    {{ const float g = {g};")
            for mm in ([m, -m] if m else [0]):
                oi, vi = l3 * l3 + l3 + mm, l1 * l1 + l1 + mm
                op = "+=" if oi in touched else "="
                touched.add(oi)
                lines.append(f"      o[{oi}] {op} g * v[{vi}];")
            lines.append("    }")
    for oi in range((l_out + 1) ** 2):
        if oi not in touched:
            lines.append(f"    o[{oi}] = 0.0f;")
    lines.append("  }")
    # adjoint: given d(o) returns d(v) and d(w) (both overwritten)
    lines.append("  __device__ __forceinline__ static void run_bwd(const float* v, const float* w, const float* go,")
    lines.append("                                                 float* gv, float* gw) {")
    tv, tw = set(), set()
    for (l1, l3) in sorted(groups):
        for m in sorted(groups[(l1, l3)]):
            terms = groups[(l1, l3)][m]
            g = " + ".join(f"{f32(k)} * w[{p}]" for p, k in terms)
            pairs = [(l3 * l3 + l3 + mm, l1 * l1 + l1 + mm) for mm in ([m, -m] if m else [0])]
            dg = " + ".join(f"go[{oi}] * v[{vi}]" for oi, vi in pairs)
            lines.append(f"    {{ const float g = {g};")
            lines.append(f"      const float dg = {dg};")
            for oi, vi in pairs:
                lines.append(f"      gv[{vi}] {'+=' if vi in tv else '='} g * go[{oi}];")
                tv.add(vi)
            for p, k in terms:
                lines.append(f"      gw[{p}] {'+=' if p in tw else '='} {f32(k)} * dg;")
                tw.add(p)
            lines.append("    }")
    for vi in range((l_in + 1) ** 2):
        if vi not in tv:
            lines.append(f"    gv[{vi}] = 0.0f;")
    for p in range(len(paths)):
        if p not in tw:
            lines.append(f"    gw[{p}] = 0.0f;")
    lines.append("  }")
    # the same product split by input degree l1 (paths are ordered l1-major, so each piece uses one contiguous run of
    # weights): o is accumulated into, v is the degree-l1 block only, w the weights of that run
    first = [min(p for p, t in enumerate(paths) if t[0] == l1) for l1 in range(l_in + 1)]
    count = [sum(1 for t in paths if t[0] == l1) for l1 in range(l_in + 1)]
    lines.append(f"  static constexpr int CHUNK_FIRST[{l_in + 1}] = {{{', '.join(map(str, first))}}};")
    lines.append(f"  static constexpr int CHUNK_COUNT[{l_in + 1}] = {{{', '.join(map(str, count))}}};")
    lines.append(f"  static constexpr int CHUNK_MAX = {max(count)};")
    lines.append("  template <int L1> __device__ __forceinline__ static void run_l1(const float* v, const float* w, float* o);")
    lines.append("  template <int L1> __device__ __forceinline__ static void run_bwd_l1(const float* v, const float* w, const float* go,")
    lines.append("                                                                       float* gv, float* gw);")
    lines.append("};")
    for l1 in range(l_in + 1):
        lines.append(f"template <> __device__ __forceinline__ void TpMid_{tag}::run_l1<{l1}>(const float* v, const float* w, float* o) {{")
        for (a, l3) in sorted(groups):
            if a != l1:
                continue
            for m in sorted(groups[(a, l3)]):
                terms = groups[(a, l3)][m]
                g = " + ".join(f"{f32(k)} * w[{p - first[l1]}]" for p, k in terms)
                lines.append(f"  {{ const float g = {g};")
                for mm in ([m, -m] if m else [0]):
                    lines.append(f"    o[{l3 * l3 + l3 + mm}] += g * v[{l1 + mm}];")
                lines.append("  }")
        lines.append("}")
    # the adjoint split the same way: v and gv are the degree-l1 block only (gv overwritten), w and gw the run of
    # weights of that degree (gw overwritten), go the whole output gradient
    for l1 in range(l_in + 1):
        lines.append(f"template <> __device__ __forceinline__ void TpMid_{tag}::run_bwd_l1<{l1}>(const float* v, const float* w, const float* go,")
        lines.append("                                                                          float* gv, float* gw) {")
        tv, tw = set(), set()
        for (a, l3) in sorted(groups):
            if a != l1:
                continue
            for m in sorted(groups[(a, l3)]):
                terms = groups[(a, l3)][m]
                g = " + ".join(f"{f32(k)} * w[{p - first[l1]}]" for p, k in terms)
                pairs = [(l3 * l3 + l3 + mm, l1 + mm) for mm in ([m, -m] if m else [0])]
                dg = " + ".join(f"go[{oi}] * v[{vi}]" for oi, vi in pairs)
                lines.append(f"  {{ const float g = {g};")
                lines.append(f"    const float dg = {dg};")
                for oi, vi in pairs:
                    lines.append(f"    gv[{vi}] {'+=' if vi in tv else '='} g * go[{oi}];")
                    tv.add(vi)
                for p, k in terms:
                    q = p - first[l1]
                    lines.append(f"    gw[{q}] {'+=' if q in tw else '='} {f32(k)} * dg;")
                    tw.add(q)
                lines.append("  }")
        for vi in range(2 * l1 + 1):
            if vi not in tv:
                lines.append(f"  gv[{vi}] = 0.0f;")
        for q in range(count[l1]):
            if q not in tw:
                lines.append(f"  gw[{q}] = 0.0f;")
        lines.append("}")
    return "\n".join(lines)


def generate():
    Jm = {0: np.ones((1, 1))}
    out = ["// GENERATED by gen_tables.py -- do not edit.", "#pragma once", ""]
    for l in range(1, LMAX + 1):
        Jm[l] = j_matrix(l)
        out.append(emit_matvec(f"egnn_apply_J{l}", Jm[l], f"v <- J v, J = D^{l}(R_x(pi/2))"))
        out.append(emit_matvec(f"egnn_apply_Jt{l}", Jm[l].T, f"v <- J^T v, degree {l}"))
        out.append("")
    rng = np.random.default_rng(7)
    combos = [(l, l, l) for l in range(0, LMAX + 1)] + [(l, l, L_READOUT) for l in range(0, LMAX)]
    path_rows = []
    for (l_in, l_sh, l_out) in combos:
        paths, groups = bond_frame_constants(l_in, l_sh, l_out)
        # self-check of the whole bond-frame evaluation against the dense definition
        for trial in range(3):
            v = rng.standard_normal((l_in + 1) ** 2)
            w = rng.standard_normal(len(paths))
            r = rng.standard_normal(3)
            r /= np.linalg.norm(r)
            if trial == 2:
                r = np.array([0.0, 0.0, -1.0])
            a = emulate_bond_frame_tp(l_in, l_sh, l_out, groups, Jm, v, w, r)
            b = dense_tp(l_in, l_sh, l_out, paths, v, w, r)
            assert np.allclose(a, b, atol=1e-11), (l_in, l_sh, l_out, trial, np.abs(a - b).max())
        out.append(emit_mid(l_in, l_sh, l_out, paths, groups))
        out.append("")
        path_rows.append((l_in, l_sh, l_out, paths))
    # host tables: path lists and the real coupling tensors for the orbital uncoupling (l_a, l_b <= 2)
    out.append("#ifdef EGNN_GEN_HOST_TABLES")
    out.append("struct EgnnPathList { int l_in, l_sh, l_out, n; int l[64][3]; };")
    out.append(f"static const EgnnPathList egnn_path_lists[{len(path_rows)}] = {{")
    for (l_in, l_sh, l_out, paths) in path_rows:
        body = ", ".join("{%d,%d,%d}" % p for p in paths)
        out.append(f"  {{{l_in}, {l_sh}, {l_out}, {len(paths)}, {{{body}}}}},")
    out.append("};")
    out.append(f"static const int egnn_n_path_lists = {len(path_rows)};")
    n = ORB_LMAX + 1
    flat, offs = [], {}
    for la in range(n):
        for lb in range(n):
            for L in range(abs(la - lb), la + lb + 1):
                offs[(la, lb, L)] = len(flat)
                flat.extend(coupling_real(la, lb, L).reshape(-1).tolist())
    out.append(f"// real coupling tensors C[m_a][m_b][M] for l_a, l_b <= {ORB_LMAX}, flattened; offset -1 = not allowed")
    out.append(f"static const int egnn_cg_offset[{n}][{n}][{2 * ORB_LMAX + 1}] = {{")
    for la in range(n):
        rows = []
        for lb in range(n):
            rows.append("{" + ", ".join(str(offs.get((la, lb, L), -1)) for L in range(2 * ORB_LMAX + 1)) + "}")
        out.append("  {" + ", ".join(rows) + "},")
    out.append("};")
    out.append(f"static const double egnn_cg_values[{len(flat)}] = {{")
    for i in range(0, len(flat), 6):
        out.append("  " + ", ".join(repr(float(x)) for x in flat[i:i + 6]) + ",")
    out.append("};")
    out.append("#endif")
    return "\n".join(out) + "\n"


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    target = sys.argv[1] if len(sys.argv) > 1 else os.path.join(here, "egnn_gen.inc")
    text = generate()
    if not os.path.exists(target) or open(target).read() != text:
        with open(target, "w") as f:
            f.write(text)
    print(f"wrote {target} ({len(text.splitlines())} lines)")


if __name__ == "__main__":
    main()
