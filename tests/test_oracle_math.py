"""Pins for the SO(3) pieces of the fp64 oracle: each check compares the oracle with something fixed by
mathematics or by a library routine, not with the oracle itself."""
import itertools
import os

import numpy as np
import pytest

import oracle as O

RNG = np.random.default_rng(1234)


def Rz(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, -s, 0], [s, c, 0], [0, 0, 1.0]])


def Ry(a):
    c, s = np.cos(a), np.sin(a)
    return np.array([[c, 0, s], [0, 1.0, 0], [-s, 0, c]])


def sh_all(l, X):
    return np.stack([O.solid_harmonics(l, x) for x in X], axis=1)  # [2l+1][P]


# ---------------------------------------------------------------- solid harmonics

def test_solid_harmonics_closed_forms():
    """Racah-normalised real solid harmonics as Cartesian polynomials (textbook forms), order m=-l..l."""
    for _ in range(5):
        x, y, z = r = RNG.normal(size=3)
        r2 = r @ r
        s3 = np.sqrt(3.0)
        np.testing.assert_allclose(O.solid_harmonics(0, r), [1.0], atol=1e-14)
        np.testing.assert_allclose(O.solid_harmonics(1, r), [y, z, x], atol=1e-14)
        np.testing.assert_allclose(O.solid_harmonics(2, r),
                                   [s3 * x * y, s3 * y * z, 0.5 * (3 * z * z - r2), s3 * x * z,
                                    0.5 * s3 * (x * x - y * y)], atol=1e-13)
        l3 = O.solid_harmonics(3, r)
        np.testing.assert_allclose(l3[3], 0.5 * (5 * z ** 3 - 3 * z * r2), atol=1e-13)
        np.testing.assert_allclose(l3[6], np.sqrt(5.0 / 8.0) * (x ** 3 - 3 * x * y * y), atol=1e-13)
        np.testing.assert_allclose(l3[0], np.sqrt(5.0 / 8.0) * (3 * x * x * y - y ** 3), atol=1e-13)


def test_solid_harmonics_against_scipy():
    """Against scipy's complex harmonics (orthonormal, Condon-Shortley): Racah factor sqrt(4 pi/(2l+1))."""
    from scipy.special import sph_harm_y
    for l in range(7):
        for _ in range(3):
            r = RNG.normal(size=3)
            d = np.linalg.norm(r)
            theta, phi = np.arccos(r[2] / d), np.arctan2(r[1], r[0])
            mine = O.solid_harmonics(l, r) / d ** l
            fac = np.sqrt(4 * np.pi / (2 * l + 1))
            np.testing.assert_allclose(mine[l], fac * sph_harm_y(l, 0, theta, phi).real, atol=1e-13)
            for m in range(1, l + 1):
                Y = fac * sph_harm_y(l, m, theta, phi)
                np.testing.assert_allclose(mine[l + m], (-1) ** m * np.sqrt(2) * Y.real, atol=1e-13)
                np.testing.assert_allclose(mine[l - m], (-1) ** m * np.sqrt(2) * Y.imag, atol=1e-13)


def test_solid_harmonics_invariants():
    for l in range(7):
        r = RNG.normal(size=3)
        u = r / np.linalg.norm(r)
        assert abs(np.sum(O.solid_harmonics(l, u) ** 2) - 1.0) < 1e-13       # addition theorem at zero angle
        np.testing.assert_allclose(O.solid_harmonics(l, 1.7 * r), 1.7 ** l * O.solid_harmonics(l, r), rtol=1e-12)
        # pole sparsity (Lemma, Sec. 3.3): only m = 0 survives on the z-axis, with value d^l
        e0 = np.zeros(2 * l + 1)
        e0[l] = 2.5 ** l
        np.testing.assert_allclose(O.solid_harmonics(l, [0, 0, 2.5]), e0, atol=1e-12)


def test_solid_harmonics_are_harmonic():
    """Laplacian of r^l Y_lm vanishes (second differences of a polynomial of degree <= 6)."""
    hstep = 1e-3
    for l in range(5):
        r = RNG.normal(size=3)
        lap = -6 * O.solid_harmonics(l, r)
        for k in range(3):
            e = np.zeros(3)
            e[k] = hstep
            lap = lap + O.solid_harmonics(l, r + e) + O.solid_harmonics(l, r - e)
        assert np.abs(lap / hstep ** 2).max() < 1e-5 * max(1.0, np.abs(r).max() ** l * 50)


# ---------------------------------------------------------------- Clebsch-Gordan

def test_complex_cg_against_sympy():
    from sympy import S
    from sympy.physics.quantum.cg import CG
    for j1, j2 in itertools.product(range(4), range(3)):
        for j in range(abs(j1 - j2), j1 + j2 + 1):
            for m1 in range(-j1, j1 + 1):
                for m2 in range(-j2, j2 + 1):
                    m = m1 + m2
                    if abs(m) > j:
                        continue
                    ref = float(CG(S(j1), S(m1), S(j2), S(m2), S(j), S(m)).doit())
                    assert abs(O.cg_complex(j1, m1, j2, m2, j, m) - ref) < 1e-13


def test_complex_cg_unitarity():
    for j1, j2 in [(4, 1), (3, 2), (4, 4)]:
        for m1 in range(-j1, j1 + 1):
            for m2 in range(-j2, j2 + 1):
                tot = sum(O.cg_complex(j1, m1, j2, m2, j, m1 + m2) ** 2 for j in range(abs(j1 - j2), j1 + j2 + 1))
                assert abs(tot - 1.0) < 1e-12


def test_real_cg_textbook_vector_cases():
    """Two vectors a, b in (y,z,x) component order: scalar, cross and symmetric-traceless products."""
    a, b = RNG.normal(size=3), RNG.normal(size=3)
    av, bv = a[[1, 2, 0]], b[[1, 2, 0]]          # (y,z,x) ordering of the l=1 components

    def couple(lo):
        return np.einsum("oif,i,f->o", O.cg_real(1, 1, lo), av, bv)

    np.testing.assert_allclose(couple(0), [-(a @ b) / np.sqrt(3)], atol=1e-14)
    cr = np.cross(a, b)[[1, 2, 0]]
    c1 = couple(1)
    # the odd path is fixed up to one global sign (choice of -i vs +i); magnitude and direction are not
    assert min(np.abs(c1 - cr / np.sqrt(2)).max(), np.abs(c1 + cr / np.sqrt(2)).max()) < 1e-14
    c2 = couple(2)
    ax, ay, az = a
    bx, by, bz = b
    expect = np.array([(ax * by + ay * bx) / np.sqrt(2), (ay * bz + az * by) / np.sqrt(2),
                       (2 * az * bz - ax * bx - ay * by) / np.sqrt(6), (ax * bz + az * bx) / np.sqrt(2),
                       (ax * bx - ay * by) / np.sqrt(2)])
    np.testing.assert_allclose(c2, expect, atol=1e-14)
    # scalar times vector: (0 x 1 -> 1) is the plain product
    np.testing.assert_allclose(np.einsum("oif,i,f->o", O.cg_real(0, 1, 1), [2.0], bv), 2.0 * bv, atol=1e-14)


def test_real_cg_is_equivariant():
    a, b, g = RNG.uniform(-3, 3, size=3)
    for li, lf in [(1, 1), (2, 1), (3, 1), (4, 1), (2, 2), (3, 2), (4, 3)]:
        for lo in range(abs(li - lf), min(li + lf, 5) + 1):
            T = O.cg_real(li, lf, lo)
            u, v = RNG.normal(size=2 * li + 1), RNG.normal(size=2 * lf + 1)
            Di, Df, Do = (O.wigner_D_real(l, a, b, g) for l in (li, lf, lo))
            lhs = np.einsum("oif,i,f->o", T, Di @ u, Df @ v)
            rhs = Do @ np.einsum("oif,i,f->o", T, u, v)
            np.testing.assert_allclose(lhs, rhs, atol=1e-12)
            # unitary normalisation: sum over (mi,mf) of C^2 is 1 for every mo
            np.testing.assert_allclose(np.sum(T ** 2, axis=(1, 2)), 1.0, atol=1e-12)


# ---------------------------------------------------------------- Wigner-D

def test_wigner_D_definition_and_fit():
    """Y(R x) = D(R) Y(x); D also equals the least-squares fit Y(R X) Y(X)^+ on generic points."""
    X = RNG.normal(size=(40, 3))
    for l in range(6):
        a, b, g = RNG.uniform(-3, 3, size=3)
        R = Rz(a) @ Ry(b) @ Rz(g)
        D = O.wigner_D_real(l, a, b, g)
        YX, YRX = sh_all(l, X), sh_all(l, X @ R.T)
        np.testing.assert_allclose(D @ YX, YRX, atol=1e-11)
        Dfit = YRX @ np.linalg.pinv(YX)
        np.testing.assert_allclose(D, Dfit, atol=1e-10)
        np.testing.assert_allclose(D @ D.T, np.eye(2 * l + 1), atol=1e-12)


def test_wigner_D_degree_one_is_the_rotation_matrix():
    a, b, g = RNG.uniform(-3, 3, size=3)
    R = Rz(a) @ Ry(b) @ Rz(g)
    perm = [1, 2, 0]                               # (y,z,x)
    np.testing.assert_allclose(O.wigner_D_real(1, a, b, g), R[np.ix_(perm, perm)], atol=1e-14)


def test_wigner_D_homomorphism():
    X = RNG.normal(size=(40, 3))
    a1, b1, g1, a2, b2, g2 = RNG.uniform(-3, 3, size=6)
    R12 = Rz(a1) @ Ry(b1) @ Rz(g1) @ Rz(a2) @ Ry(b2) @ Rz(g2)
    for l in range(5):
        D12 = O.wigner_D_real(l, a1, b1, g1) @ O.wigner_D_real(l, a2, b2, g2)
        np.testing.assert_allclose(D12 @ sh_all(l, X), sh_all(l, X @ R12.T), atol=1e-11)


def test_alignment_rotation_gives_pole_sparsity():
    """D(R_ij) R^(l)(r) = d^l e_0 for the aligning rotation (Lemma, Sec. 3.3), any gauge angle."""
    for r in [RNG.normal(size=3), np.array([0, 0, 1.3]), np.array([0, 0, -0.7]), np.array([1.1, 0, 0]),
              np.array([1e-9, -1e-9, -2.0])]:
        th, ph = O.align_angles(r)
        d = np.linalg.norm(r)
        np.testing.assert_allclose(Ry(-th) @ Rz(-ph) @ r, [0, 0, d], atol=1e-12)
        for l in range(5):
            e0 = np.zeros(2 * l + 1)
            e0[l] = d ** l
            for chi in (0.0, 1.234):
                np.testing.assert_allclose(O.wigner_D_real(l, chi, -th, -ph) @ O.solid_harmonics(l, r), e0, atol=1e-11)


# ---------------------------------------------------------------- the re-indexing operator P

def test_P_sparsity_and_parity_rule():
    """At most one input order per output order; even L_Sigma keeps m, odd flips it and kills m_o = 0; the
    surviving coefficient is the complex CG <li |m|; lf 0 | lo |m|> (with sign(m_o) on odd paths)."""
    counts = {}
    for lf in (0, 1, 2, 3):
        for L in (1, 2, 4):
            nnz = 0
            for li in range(L + 1):
                for lo in range(abs(li - lf), min(li + lf, L) + 1):
                    src, coef, worst = O.P_path(li, lf, lo)
                    assert worst <= 1
                    odd = (li + lf + lo) % 2
                    for k, mo in enumerate(range(-lo, lo + 1)):
                        mi_expected = -mo if odd else mo
                        c = O.cg_complex(li, abs(mo), lf, 0, lo, abs(mo)) if abs(mo) <= li else 0.0
                        if odd:
                            c *= np.sign(mo)
                        if abs(c) < 1e-13:
                            assert src[k] == -1
                        else:
                            assert src[k] - li == mi_expected
                            assert abs(coef[k] - c) < 1e-13
                            nnz += 1
            counts[(lf, L)] = nnz
    assert counts[(1, 1)] == 4 and counts[(1, 2)] == 14 and counts[(1, 4)] == 52 and counts[(2, 4)] == 64


def test_P_worked_examples_from_the_paper():
    path = os.path.join(os.path.dirname(__file__), "golden", "eaas_worked_examples.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 4
    for li, lf, lo, mo, _, mi in rows:
        li, lf, lo, mo = int(li), int(lf), int(lo), int(mo)
        src, coef, _ = O.P_path(li, lf, lo)
        if mi == "none":
            assert src[mo + lo] == -1 and coef[mo + lo] == 0.0
        else:
            assert src[mo + lo] - li == int(mi) and abs(coef[mo + lo]) > 0.1
    # values under this repo's conventions: -1/sqrt3 for (1,1,0); +-1/sqrt2, opposite signs, for (1,1,1)
    assert abs(O.P_path(1, 1, 0)[1][0] + 1 / np.sqrt(3)) < 1e-14
    c = O.P_path(1, 1, 1)[1]
    assert abs(abs(c[0]) - 1 / np.sqrt(2)) < 1e-14 and abs(c[0] + c[2]) < 1e-14


# ---------------------------------------------------------------- EAAS identity

@pytest.mark.parametrize("lf", [0, 1, 2, 3])
def test_eaas_equals_dense_contraction_per_path(lf):
    """Proposition (Sec. 3.3): align, re-index, inverse-align equals the dense CG product, path by path."""
    L = 4
    n = (L + 1) ** 2
    for li in range(L + 1):
        for lo in range(abs(li - lf), min(li + lf, L) + 1):
            w = np.zeros((L + 1, L + 1))
            w[li, lo] = 1.0
            for r in [RNG.normal(size=3) * 2.0, np.array([0.0, 0.0, -1.5]), np.array([0.3, 0.0, 0.0])]:
                v = RNG.normal(size=(n, 2))
                dense = O.message(L, lf, w, v, r, "dense")
                # the dense route, retyped here from Eq. cg_product with the oracle's pinned CG and harmonics
                expect = np.zeros_like(v)
                expect[lo * lo:(lo + 1) ** 2] = np.einsum("oif,ic,f->oc", O.cg_real(li, lf, lo),
                                                          v[li * li:(li + 1) ** 2], O.solid_harmonics(lf, r))
                np.testing.assert_allclose(dense, expect, atol=1e-12)
                for chi in (0.0, 2.1):
                    np.testing.assert_allclose(O.message(L, lf, w, v, r, "eaas", chi), dense, atol=1e-12)


def test_eaas_all_paths_with_weights():
    L = 4
    n = (L + 1) ** 2
    for lf in (1, 2):
        w = RNG.uniform(0.5, 1.5, size=(L + 1, L + 1))
        v, r = RNG.normal(size=(n, 3)), RNG.normal(size=3) * 3
        np.testing.assert_allclose(O.message(L, lf, w, v, r, "eaas", 0.4), O.message(L, lf, w, v, r, "dense"),
                                   atol=1e-12)


def test_degree_one_message_is_linear_in_r():
    """l_f = 1 case of the node-centric factorization (Eq. e2former_final): msg(r_j - r_i) splits into a
    source term and a target term about any origin."""
    L = 3
    n = (L + 1) ** 2
    w = RNG.uniform(0.5, 1.5, size=(L + 1, L + 1))
    v = RNG.normal(size=(n, 2))
    ri, rj, o = RNG.normal(size=(3, 3))
    for mode in ("dense", "eaas"):
        lhs = O.message(L, 1, w, v, rj - ri, mode)
        rhs = O.message(L, 1, w, v, rj - o, mode) - O.message(L, 1, w, v, ri - o, mode)
        np.testing.assert_allclose(lhs, rhs, atol=1e-12)
