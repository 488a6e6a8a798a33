/*
 * fp64 CPU oracle for the node-centric equivariant attention forward pass of E2Former-V2.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a slow, plain restatement of the paper's definitions and is
 * only ever called by the tests, by the smoke check and by the benchmark's cpu_baseline leg.  It
 * shares no code, tables or constants with the HIP library and the HIP library never calls it.
 *
 * What is written out here, with the passage each part follows:
 *   - real solid harmonics R^(l)_m(r) = |r|^l Y_lm(r/|r|)            (Preliminaries, "Geometric encoding")
 *   - complex Clebsch-Gordan coefficients (Racah's closed formula) and the real-basis tensor
 *     obtained through the {m,-m} change of basis                     (Eq. cg_product; App. C, Eq. app-real-basis)
 *   - Wigner-D matrices of the real basis                             (Preliminaries; Sec. 3.3)
 *   - the edge message m_ij = v_j (x) R^(lf)(r_ij), once by the dense contraction and once through
 *     align -> re-index P -> inverse-align (EAAS)                     (Preliminaries; Def. of P, Prop. EAAS)
 *   - l-wise projections and invariant q,k                            (Sec. 3.2, Eq. qk)
 *   - alpha_ij = softmax_j(q.k/sqrt(d_k) + b(r)) * phi(r)             (Eq. attn), two-pass, and the
 *     streaming recurrences for mu, z, A                              (Sec. 3.4, Algorithm 1)
 *   - neighbour sets by all pairs and by a cell list.
 *
 * Conventions (readings where the paper is silent):
 *   - component index of (l,m) is l*l + l + m; features are h[atom][component][channel].
 *   - real basis: m<0 as printed in Eq. app-real-basis, m>0 x_m = (z_{-m} + (-1)^m z_m)/sqrt 2, so the
 *     l=1 components (m=-1,0,1) are proportional to (y,z,x).
 *   - Racah normalisation: Y_l0(z-axis) = 1 and sum_m Y_lm^2 = 1 on the unit sphere.
 *   - column convention: Y(R x) = D(R) Y(x); aligned features D(R) v; back rotation D(R)^T.
 *   - real CG tensor = U_o Cbar (U_i^dagger (x) U_f^dagger); it is real for even l_i+l_f+l_o and purely
 *     imaginary for odd, where its imaginary part is taken.
 *   - neighbour predicate evaluated in binary32 with a fixed operation order (no fused multiply-add):
 *     d2 = (dx*dx + dy*dy) + dz*dz < rc*rc, j != i, same segment, d2 > 0.
 *   - radial basis g_b(d) = exp(-gamma (d - mu_b)^2), mu_b = b rc/(B-1), gamma = (B-1)^2/(2 rc^2);
 *     bias b_h(d) = sum_b Wb[h][b] g_b(d); gate phi(d) = (1 + cos(pi d/rc))/2, outside the softmax.
 *   - head h owns channels [h C/H, (h+1) C/H) of every degree; d_k = (L+1) C/H.
 *   - an atom without neighbours gets a zero output.
 */
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define E2FO_MAX_L 8

static double fact(int n) {
    double f = 1.0;
    for (int i = 2; i <= n; ++i) f *= (double)i;
    return f;
}

/* ------------------------------------------------------------------ solid harmonics */

/* Associated Legendre function P_l^m(x), m >= 0, including the Condon-Shortley phase (-1)^m;
 * s = sqrt(1 - x^2) is passed in so that it keeps its accuracy next to the poles. */
static double assoc_legendre(int l, int m, double x, double s) {
    double pmm = 1.0;
    for (int i = 1; i <= m; ++i) pmm *= -(2.0 * i - 1.0) * s;
    if (l == m) return pmm;
    double pm1 = x * (2.0 * m + 1.0) * pmm;
    if (l == m + 1) return pm1;
    double pl = 0.0;
    for (int ll = m + 2; ll <= l; ++ll) {
        pl = (x * (2.0 * ll - 1.0) * pm1 - (ll + m - 1.0) * pmm) / (double)(ll - m);
        pmm = pm1;
        pm1 = pl;
    }
    return pl;
}

/* R^(l)_m(r) for m = -l..l (out has 2l+1 entries), Racah normalised real harmonics times |r|^l. */
void e2fo_solid_harmonics(int l, const double *r, double *out) {
    double d = sqrt(r[0] * r[0] + r[1] * r[1] + r[2] * r[2]);
    if (d == 0.0) {
        for (int m = -l; m <= l; ++m) out[m + l] = (l == 0) ? 1.0 : 0.0;
        return;
    }
    double ct = r[2] / d;
    double st = sqrt(r[0] * r[0] + r[1] * r[1]) / d;
    double phi = atan2(r[1], r[0]);
    double dl = pow(d, (double)l);
    out[l] = dl * assoc_legendre(l, 0, ct, st);
    for (int m = 1; m <= l; ++m) {
        /* complex Y_l^m = N P_l^m e^{i m phi}; x_{+m} = (-1)^m sqrt2 Re, x_{-m} = (-1)^m sqrt2 Im */
        double nlm = sqrt(fact(l - m) / fact(l + m));
        double p = assoc_legendre(l, m, ct, st);
        double sgn = (m & 1) ? -1.0 : 1.0;
        out[l + m] = dl * sgn * sqrt(2.0) * nlm * p * cos(m * phi);
        out[l - m] = dl * sgn * sqrt(2.0) * nlm * p * sin(m * phi);
    }
}

/* ------------------------------------------------------------------ Clebsch-Gordan */

/* <j1 m1; j2 m2 | j m> in the Condon-Shortley convention, Racah's closed formula. */
double e2fo_cg_complex(int j1, int m1, int j2, int m2, int j, int m) {
    if (m1 + m2 != m) return 0.0;
    if (j < abs(j1 - j2) || j > j1 + j2) return 0.0;
    if (abs(m1) > j1 || abs(m2) > j2 || abs(m) > j) return 0.0;
    double pre = (2.0 * j + 1.0) * fact(j + j1 - j2) * fact(j - j1 + j2) * fact(j1 + j2 - j) / fact(j1 + j2 + j + 1);
    pre *= fact(j + m) * fact(j - m) * fact(j1 - m1) * fact(j1 + m1) * fact(j2 - m2) * fact(j2 + m2);
    double sum = 0.0;
    for (int k = 0; k <= j1 + j2 - j; ++k) {
        int a = j1 + j2 - j - k, b = j1 - m1 - k, c = j2 + m2 - k, e = j - j2 + m1 + k, f = j - j1 - m2 + k;
        if (a < 0 || b < 0 || c < 0 || e < 0 || f < 0) continue;
        double term = 1.0 / (fact(k) * fact(a) * fact(b) * fact(c) * fact(e) * fact(f));
        sum += (k & 1) ? -term : term;
    }
    return sqrt(pre) * sum;
}

/* Unitary U with x = U z (complex basis z_mu, real basis x_m); U[(m+l)*(2l+1) + (mu+l)]. */
static void real_basis_U(int l, double complex *U) {
    int n = 2 * l + 1;
    for (int i = 0; i < n * n; ++i) U[i] = 0.0;
    const double s = 1.0 / sqrt(2.0);
    U[l * n + l] = 1.0;
    for (int m = 1; m <= l; ++m) {
        double sg = (m & 1) ? -1.0 : 1.0;
        /* m > 0 : x_m = (z_{-m} + (-1)^m z_m)/sqrt2 */
        U[(l + m) * n + (l - m)] = s;
        U[(l + m) * n + (l + m)] = sg * s;
        /* m < 0 (index -m): x_{-m} = i/sqrt2 (z_{-m} - (-1)^m z_{m}) */
        U[(l - m) * n + (l - m)] = I * s;
        U[(l - m) * n + (l + m)] = -I * sg * s;
    }
}

/* Real-basis CG tensor out[mo][mi][mf] (sizes 2lo+1, 2li+1, 2lf+1) for (li (x) lf -> lo). */
void e2fo_cg_real(int li, int lf, int lo, double *out) {
    int ni = 2 * li + 1, nf = 2 * lf + 1, no = 2 * lo + 1;
    double complex Ui[(2 * E2FO_MAX_L + 1) * (2 * E2FO_MAX_L + 1)];
    double complex Uf[(2 * E2FO_MAX_L + 1) * (2 * E2FO_MAX_L + 1)];
    double complex Uo[(2 * E2FO_MAX_L + 1) * (2 * E2FO_MAX_L + 1)];
    real_basis_U(li, Ui);
    real_basis_U(lf, Uf);
    real_basis_U(lo, Uo);
    int odd = (li + lf + lo) & 1;
    for (int mo = 0; mo < no; ++mo)
        for (int mi = 0; mi < ni; ++mi)
            for (int mf = 0; mf < nf; ++mf) {
                double complex acc = 0.0;
                for (int ui = -li; ui <= li; ++ui)
                    for (int uf = -lf; uf <= lf; ++uf) {
                        int uo = ui + uf;
                        if (abs(uo) > lo) continue;
                        double c = e2fo_cg_complex(li, ui, lf, uf, lo, uo);
                        if (c == 0.0) continue;
                        acc += Uo[mo * no + (uo + lo)] * c * conj(Ui[mi * ni + (ui + li)]) *
                               conj(Uf[mf * nf + (uf + lf)]);
                    }
                out[(mo * ni + mi) * nf + mf] = odd ? cimag(acc) : creal(acc);
            }
}

/* ------------------------------------------------------------------ Wigner-D (real basis) */

/* Wigner small-d d^j_{mp m}(beta), Wigner's sum formula. */
static double wigner_small_d(int j, int mp, int m, double beta) {
    double c = cos(0.5 * beta), s = sin(0.5 * beta);
    double pre = sqrt(fact(j + m) * fact(j - m) * fact(j + mp) * fact(j - mp));
    double sum = 0.0;
    for (int k = 0; k <= 2 * j; ++k) {
        int a = j + m - k, b = j - k - mp, e = k - m + mp;
        if (a < 0 || b < 0 || e < 0) continue;
        double term = pow(c, 2 * j - 2 * k + m - mp) * pow(s, 2 * k - m + mp) / (fact(a) * fact(k) * fact(b) * fact(e));
        sum += ((k - m + mp) & 1) ? -term : term;
    }
    return pre * sum;
}

/*
 * Real-basis D^(l)(R) for R = Rz(alpha) Ry(beta) Rz(gamma) (active rotations), defined by
 * Y(R x) = D(R) Y(x).  In the complex basis the matrix with that property is the conjugate of the
 * standard D^l_{m m'}(R) = e^{-i m alpha} d^l_{m m'}(beta) e^{-i m' gamma}.  out[(m+l)*(2l+1) + (m'+l)].
 */
void e2fo_wigner_D_real(int l, double alpha, double beta, double gamma, double *out) {
    int n = 2 * l + 1;
    double complex Dc[(2 * E2FO_MAX_L + 1) * (2 * E2FO_MAX_L + 1)];
    double complex U[(2 * E2FO_MAX_L + 1) * (2 * E2FO_MAX_L + 1)];
    double complex T[(2 * E2FO_MAX_L + 1) * (2 * E2FO_MAX_L + 1)];
    real_basis_U(l, U);
    for (int m = -l; m <= l; ++m)
        for (int mp = -l; mp <= l; ++mp)
            Dc[(m + l) * n + (mp + l)] = cexp(I * (m * alpha)) * wigner_small_d(l, m, mp, beta) * cexp(I * (mp * gamma));
    /* D_real = U Dc U^dagger */
    for (int a = 0; a < n; ++a)
        for (int b = 0; b < n; ++b) {
            double complex acc = 0.0;
            for (int k = 0; k < n; ++k) acc += U[a * n + k] * Dc[k * n + b];
            T[a * n + b] = acc;
        }
    for (int a = 0; a < n; ++a)
        for (int b = 0; b < n; ++b) {
            double complex acc = 0.0;
            for (int k = 0; k < n; ++k) acc += T[a * n + k] * conj(U[b * n + k]);
            out[a * n + b] = creal(acc);
        }
}

/* Polar angles of r: theta from +z, phi in the xy-plane.  R = Ry(-theta) Rz(-phi) takes r/|r| to +z. */
void e2fo_align_angles(const double *r, double *theta, double *phi) {
    double rho = sqrt(r[0] * r[0] + r[1] * r[1]);
    *theta = atan2(rho, r[2]);
    *phi = atan2(r[1], r[0]);
}

/* ------------------------------------------------------------------ edge message, two ways */

/* Everything about the coupling that does not depend on the pair: CG tensors and P, per path. */
typedef struct {
    int L, lf;
    double *cg[E2FO_MAX_L + 1][E2FO_MAX_L + 1];               /* [li][lo] -> [mo][mi][mf], NULL if no path */
    int src[E2FO_MAX_L + 1][E2FO_MAX_L + 1][2 * E2FO_MAX_L + 1]; /* P: contributing input order per mo */
    double coef[E2FO_MAX_L + 1][E2FO_MAX_L + 1][2 * E2FO_MAX_L + 1];
} coupling_tables;

/*
 * Re-indexing operator P for one path: the m_f = 0 slice of the real CG tensor.  For every output
 * order mo it returns the single contributing input order src[mo+lo] (as an offset 0..2li, or -1 when
 * the row is empty) and its coefficient coef[mo+lo].  Returns the largest number of non-negligible
 * entries found in any row (the paper states this is at most one).
 */
int e2fo_P_path(int li, int lf, int lo, int *src, double *coef) {
    int ni = 2 * li + 1, nf = 2 * lf + 1, no = 2 * lo + 1;
    double *cg = (double *)malloc(sizeof(double) * no * ni * nf);
    e2fo_cg_real(li, lf, lo, cg);
    int worst = 0;
    for (int mo = 0; mo < no; ++mo) {
        int cnt = 0;
        src[mo] = -1;
        coef[mo] = 0.0;
        for (int mi = 0; mi < ni; ++mi) {
            double c = cg[(mo * ni + mi) * nf + lf];
            if (fabs(c) > 1e-13) {
                ++cnt;
                src[mo] = mi;
                coef[mo] = c;
            }
        }
        if (cnt > worst) worst = cnt;
    }
    free(cg);
    return worst;
}

static void tables_init(coupling_tables *t, int L, int lf) {
    t->L = L;
    t->lf = lf;
    for (int li = 0; li <= L; ++li)
        for (int lo = 0; lo <= L; ++lo) {
            t->cg[li][lo] = NULL;
            if (lo < abs(li - lf) || lo > li + lf) continue;
            t->cg[li][lo] = (double *)malloc(sizeof(double) * (2 * lo + 1) * (2 * li + 1) * (2 * lf + 1));
            e2fo_cg_real(li, lf, lo, t->cg[li][lo]);
            e2fo_P_path(li, lf, lo, t->src[li][lo], t->coef[li][lo]);
        }
}

static void tables_free(coupling_tables *t) {
    for (int li = 0; li <= t->L; ++li)
        for (int lo = 0; lo <= t->L; ++lo) free(t->cg[li][lo]);
}

/*
 * Dense definition for all C channels of one pair:
 * msg[lo,mo][c] = sum_li w_path[li][lo] sum_{mi,mf} C^{(lo,mo)}_{(li,mi),(lf,mf)} v[li,mi][c] R^(lf)_mf(r).
 * v and msg are [(L+1)^2][C].
 */
static void message_dense(const coupling_tables *t, const double *w_path, const double *v, int C, const double *r,
                          double *msg) {
    int L = t->L, lf = t->lf, n = (L + 1) * (L + 1);
    double Rf[2 * E2FO_MAX_L + 1];
    e2fo_solid_harmonics(lf, r, Rf);
    for (int i = 0; i < n * C; ++i) msg[i] = 0.0;
    for (int li = 0; li <= L; ++li)
        for (int lo = 0; lo <= L; ++lo) {
            const double *cg = t->cg[li][lo];
            if (!cg) continue;
            int ni = 2 * li + 1, nf = 2 * lf + 1, no = 2 * lo + 1;
            double w = w_path[li * (L + 1) + lo];
            for (int mo = 0; mo < no; ++mo)
                for (int mi = 0; mi < ni; ++mi)
                    for (int mf = 0; mf < nf; ++mf) {
                        double f = w * cg[(mo * ni + mi) * nf + mf] * Rf[mf];
                        for (int c = 0; c < C; ++c) msg[(lo * lo + mo) * C + c] += f * v[(li * li + mi) * C + c];
                    }
        }
}

/*
 * EAAS route for all C channels of one pair: rotate v into the frame whose z-axis is r (D(R) with
 * R = Rz(chi) Ry(-theta) Rz(-phi); chi is the free gauge angle about the aligned axis), apply P with
 * the aligned encoding R^(lf)(R r) = d^lf e_0, rotate the result back with D(R)^T.
 */
static void message_eaas(const coupling_tables *t, const double *w_path, const double *v, int C, const double *r,
                         double chi, double *msg) {
    int L = t->L, lf = t->lf, n = (L + 1) * (L + 1);
    double theta, phi;
    e2fo_align_angles(r, &theta, &phi);
    double d = sqrt(r[0] * r[0] + r[1] * r[1] + r[2] * r[2]);
    double dlf = pow(d, (double)lf);
    int ld = (2 * L + 1) * (2 * L + 1);
    double *D = (double *)malloc(sizeof(double) * (L + 1) * ld);
    double *vt = (double *)calloc((size_t)n * C, sizeof(double));
    double *y = (double *)calloc((size_t)n * C, sizeof(double));
    for (int l = 0; l <= L; ++l) {
        double *Dl = D + l * ld;
        e2fo_wigner_D_real(l, chi, -theta, -phi, Dl);
        int nl = 2 * l + 1;
        for (int a = 0; a < nl; ++a)
            for (int b = 0; b < nl; ++b)
                for (int c = 0; c < C; ++c) vt[(l * l + a) * C + c] += Dl[a * nl + b] * v[(l * l + b) * C + c];
    }
    for (int li = 0; li <= L; ++li)
        for (int lo = 0; lo <= L; ++lo) {
            if (!t->cg[li][lo]) continue;
            double w = w_path[li * (L + 1) + lo];
            for (int mo = 0; mo < 2 * lo + 1; ++mo) {
                int mi = t->src[li][lo][mo];
                if (mi < 0) continue;
                double f = w * t->coef[li][lo][mo] * dlf;
                for (int c = 0; c < C; ++c) y[(lo * lo + mo) * C + c] += f * vt[(li * li + mi) * C + c];
            }
        }
    for (int i = 0; i < n * C; ++i) msg[i] = 0.0;
    for (int l = 0; l <= L; ++l) {
        const double *Dl = D + l * ld;
        int nl = 2 * l + 1;
        for (int b = 0; b < nl; ++b)
            for (int a = 0; a < nl; ++a)
                for (int c = 0; c < C; ++c) msg[(l * l + b) * C + c] += Dl[a * nl + b] * y[(l * l + a) * C + c];
    }
    free(D);
    free(vt);
    free(y);
}

/* Single-pair entry points for the tests: v, msg are [(L+1)^2][C]; mode 0 dense, 1 EAAS. */
void e2fo_message(int L, int lf, const double *w_path, const double *v, int C, const double *r, int mode, double chi,
                  double *msg) {
    coupling_tables t;
    tables_init(&t, L, lf);
    if (mode == 0)
        message_dense(&t, w_path, v, C, r, msg);
    else
        message_eaas(&t, w_path, v, C, r, chi, msg);
    tables_free(&t);
}

/* ------------------------------------------------------------------ neighbour sets */

/* The cutoff predicate, in binary32 with this exact operation order (built with -ffp-contract=off). */
static int within_cutoff(const double *pi_d, const double *pj_d, float rc2) {
    float pi[3] = {(float)pi_d[0], (float)pi_d[1], (float)pi_d[2]};
    float pj[3] = {(float)pj_d[0], (float)pj_d[1], (float)pj_d[2]};
    float dx = pj[0] - pi[0];
    float dy = pj[1] - pi[1];
    float dz = pj[2] - pi[2];
    float xx = dx * dx;
    float yy = dy * dy;
    float zz = dz * dz;
    float s = xx + yy;
    float d2 = s + zz;
    return (d2 < rc2) && (d2 > 0.0f);
}

static int cmp_int(const void *a, const void *b) {
    int x = *(const int *)a, y = *(const int *)b;
    return (x > y) - (x < y);
}

/*
 * Neighbour lists in CSR form, neighbours of each atom sorted by index.  offsets has N+1 entries;
 * *idx_out is malloc'ed here (release with e2fo_free).  use_cells = 0: all pairs inside each segment;
 * use_cells = 1: uniform cell list of edge rc(1+1e-6) per segment, 27-cell stencil.
 */
int e2fo_neighbor_list(const double *pos, const int32_t *seg_offsets, int N, int S, float cutoff, int use_cells,
                       int64_t *offsets, int32_t **idx_out) {
    (void)N;
    float rc2 = cutoff * cutoff;
    int64_t cap = 1024, cnt = 0;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * cap);
    offsets[0] = 0;
    for (int s = 0; s < S; ++s) {
        int a0 = seg_offsets[s], a1 = seg_offsets[s + 1];
        int ns = a1 - a0;
        int *cell_of = NULL, *cell_start = NULL, *order = NULL;
        int dims[3] = {1, 1, 1};
        double lo[3] = {0, 0, 0};
        /* a hair above the cutoff: the binary32 predicate can accept a pair whose exact |dx| exceeds rc by rounding */
        double edge = (double)cutoff * (1.0 + 1e-6);
        if (use_cells && ns > 0) {
            double hi[3];
            for (int k = 0; k < 3; ++k) lo[k] = hi[k] = pos[3 * a0 + k];
            for (int a = a0; a < a1; ++a)
                for (int k = 0; k < 3; ++k) {
                    if (pos[3 * a + k] < lo[k]) lo[k] = pos[3 * a + k];
                    if (pos[3 * a + k] > hi[k]) hi[k] = pos[3 * a + k];
                }
            for (int k = 0; k < 3; ++k) dims[k] = (int)floor((hi[k] - lo[k]) / edge) + 1;
            int nc = dims[0] * dims[1] * dims[2];
            cell_of = (int *)malloc(sizeof(int) * ns);
            cell_start = (int *)calloc((size_t)nc + 1, sizeof(int));
            order = (int *)malloc(sizeof(int) * ns);
            for (int a = a0; a < a1; ++a) {
                int c[3];
                for (int k = 0; k < 3; ++k) {
                    c[k] = (int)floor((pos[3 * a + k] - lo[k]) / edge);
                    if (c[k] >= dims[k]) c[k] = dims[k] - 1;
                }
                cell_of[a - a0] = (c[2] * dims[1] + c[1]) * dims[0] + c[0];
                cell_start[cell_of[a - a0] + 1]++;
            }
            for (int c = 0; c < nc; ++c) cell_start[c + 1] += cell_start[c];
            int *fill = (int *)calloc((size_t)nc, sizeof(int));
            for (int a = a0; a < a1; ++a) {
                int c = cell_of[a - a0];
                order[cell_start[c] + fill[c]++] = a;
            }
            free(fill);
        }
        for (int i = a0; i < a1; ++i) {
            int64_t begin = cnt;
            if (!use_cells) {
                for (int j = a0; j < a1; ++j) {
                    if (j == i || !within_cutoff(pos + 3 * i, pos + 3 * j, rc2)) continue;
                    if (cnt == cap) idx = (int32_t *)realloc(idx, sizeof(int32_t) * (cap *= 2));
                    idx[cnt++] = j;
                }
            } else {
                int c = cell_of[i - a0];
                int cx = c % dims[0], cy = (c / dims[0]) % dims[1], cz = c / (dims[0] * dims[1]);
                for (int dz = -1; dz <= 1; ++dz)
                    for (int dy = -1; dy <= 1; ++dy)
                        for (int dx = -1; dx <= 1; ++dx) {
                            int x = cx + dx, y = cy + dy, z = cz + dz;
                            if (x < 0 || y < 0 || z < 0 || x >= dims[0] || y >= dims[1] || z >= dims[2]) continue;
                            int cc = (z * dims[1] + y) * dims[0] + x;
                            for (int t = cell_start[cc]; t < cell_start[cc + 1]; ++t) {
                                int j = order[t];
                                if (j == i || !within_cutoff(pos + 3 * i, pos + 3 * j, rc2)) continue;
                                if (cnt == cap) idx = (int32_t *)realloc(idx, sizeof(int32_t) * (cap *= 2));
                                idx[cnt++] = j;
                            }
                        }
                qsort(idx + begin, (size_t)(cnt - begin), sizeof(int32_t), cmp_int);
            }
            offsets[i + 1] = cnt;
        }
        free(cell_of);
        free(cell_start);
        free(order);
    }
    *idx_out = idx;
    return 0;
}

void e2fo_free(void *p) { free(p); }

/* ------------------------------------------------------------------ the operator */

typedef struct {
    int L, C, H, B, lf;
    double cutoff;
} e2fo_config;

static double radial_gate(double d, double rc) { return 0.5 * (1.0 + cos(M_PI * d / rc)); }

static void radial_basis(double d, double rc, int B, double *g) {
    double bm1 = (B > 1) ? (double)(B - 1) : 1.0;
    double gamma = 0.5 * bm1 * bm1 / (rc * rc);
    for (int b = 0; b < B; ++b) {
        double mu = (double)b * rc / bm1;
        g[b] = exp(-gamma * (d - mu) * (d - mu));
    }
}

/* One l-wise projection of one atom: out[comp][co] = sum_ci W[l][co][ci] h[comp][ci]. */
static void project(const e2fo_config *cfg, const double *W, const double *h_atom, double *out) {
    int L = cfg->L, C = cfg->C;
    for (int l = 0; l <= L; ++l)
        for (int m = 0; m < 2 * l + 1; ++m) {
            const double *x = h_atom + (size_t)(l * l + m) * C;
            double *o = out + (size_t)(l * l + m) * C;
            for (int co = 0; co < C; ++co) {
                const double *w = W + ((size_t)l * C + co) * C;
                double acc = 0.0;
                for (int ci = 0; ci < C; ++ci) acc += w[ci] * x[ci];
                o[co] = acc;
            }
        }
}

/*
 * Forward pass for the listed target atoms (targets == NULL: all atoms, n_targets ignored).
 *   pos  double[N][3] (the cutoff predicate rounds them to binary32 first); h double[N][n][C]; seg_offsets int32[S+1];
 *   WQ1,WQ2,WK1,WK2,WV double[L+1][C][C] (out channel, in channel); Wb double[H][B];
 *   w_path double[L+1][L+1] indexed [li][lo];
 *   nbr_offsets/nbr_idx: CSR neighbour lists from e2fo_neighbor_list;
 *   edge_shift: NULL, or double[E][3] beside nbr_idx: the lattice translation of the neighbour's periodic image,
 *     r_ij = (pos[j] + edge_shift[e]) - pos[i]  (periodic boundaries; not in the paper, which states the operator
 *     for pair vectors r_ij as given);
 *   message_mode 0 = dense CG contraction, 1 = EAAS (gauge angle chi);
 *   softmax_mode 0 = two-pass softmax, 1 = streaming recurrences of Algorithm 1;
 *   score_mode 0 = the logit of Eq. kernel_score, s = tau q.k + b;
 *     1 = the logit with the non-linear pair feature of App. "Role of Non-linearity" (Eqs. app-nonlin-fea,
 *     app-nonlin-alpha), in this reading of it:  with Y^(l) the real harmonics of the unit pair vector, Q = W_Q1 h_i and
 *     V = W_V h_j, the product "within each angular order" is the invariant  a[l][c] = sum_m Q[l,m,c] Y^(l)_m  and
 *     b[l][c] = sum_m V[l,m,c] Y^(l)_m  (any pointwise sigma of an invariant keeps the operator equivariant),
 *     Fea = sigma(a || b) with sigma(x) = x / (1 + e^-x), and the triple product contracts q_i, k_j and both halves of
 *     Fea over (l, channel of the head):  s = tau sum_{l,c} q[l][c] k[l][c] (sigma(a[l][c]) + sigma(b[l][c])) + b_h(d);
 *   out double[n_targets][n][C].
 */
int e2fo_attn_forward(const e2fo_config *cfg, const double *pos, const double *h, int N, const double *WQ1,
                      const double *WQ2, const double *WK1, const double *WK2, const double *WV, const double *Wb,
                      const double *w_path, const int64_t *nbr_offsets, const int32_t *nbr_idx,
                      const double *edge_shift, const int32_t *targets, int n_targets, int message_mode,
                      int softmax_mode, double chi, int score_mode, double *out) {
    int L = cfg->L, C = cfg->C, H = cfg->H, B = cfg->B, lf = cfg->lf;
    if (L < 0 || L > E2FO_MAX_L || lf < 0 || lf > E2FO_MAX_L || C <= 0 || H <= 0 || C % H != 0 || B <= 0) return 1;
    int n = (L + 1) * (L + 1);
    int Ch = C / H;
    double tau = 1.0 / sqrt((double)((L + 1) * Ch));
    int nt = targets ? n_targets : N;
    coupling_tables tab;
    tables_init(&tab, L, lf);

    /* which atoms need projections: targets need q, their neighbours need k and v */
    char *need_q = (char *)calloc(N, 1), *need_kv = (char *)calloc(N, 1);
    for (int t = 0; t < nt; ++t) {
        int i = targets ? targets[t] : t;
        need_q[i] = 1;
        for (int64_t e = nbr_offsets[i]; e < nbr_offsets[i + 1]; ++e) need_kv[nbr_idx[e]] = 1;
    }
    double *q = (double *)calloc((size_t)N * (L + 1) * C, sizeof(double));
    double *k = (double *)calloc((size_t)N * (L + 1) * C, sizeof(double));
    double *v = (double *)calloc((size_t)N * n * C, sizeof(double));
    double *q1 = score_mode == 1 ? (double *)calloc((size_t)N * n * C, sizeof(double)) : NULL;   /* W_Q1 h of the targets */
#pragma omp parallel
    {
        double *p1 = (double *)malloc(sizeof(double) * n * C);
        double *p2 = (double *)malloc(sizeof(double) * n * C);
#pragma omp for schedule(dynamic, 16)
        for (int a = 0; a < N; ++a) {
            const double *ha = h + (size_t)a * n * C;
            if (need_q[a]) {
                project(cfg, WQ1, ha, p1);
                project(cfg, WQ2, ha, p2);
                if (q1) memcpy(q1 + (size_t)a * n * C, p1, sizeof(double) * n * C);
                for (int l = 0; l <= L; ++l)
                    for (int c = 0; c < C; ++c) {
                        double acc = 0.0;
                        for (int m = 0; m < 2 * l + 1; ++m) acc += p1[(l * l + m) * C + c] * p2[(l * l + m) * C + c];
                        q[((size_t)a * (L + 1) + l) * C + c] = acc;
                    }
            }
            if (need_kv[a]) {
                project(cfg, WK1, ha, p1);
                project(cfg, WK2, ha, p2);
                for (int l = 0; l <= L; ++l)
                    for (int c = 0; c < C; ++c) {
                        double acc = 0.0;
                        for (int m = 0; m < 2 * l + 1; ++m) acc += p1[(l * l + m) * C + c] * p2[(l * l + m) * C + c];
                        k[((size_t)a * (L + 1) + l) * C + c] = acc;
                    }
                project(cfg, WV, ha, v + (size_t)a * n * C);
            }
        }
        free(p1);
        free(p2);
    }

#pragma omp parallel
    {
        double *g = (double *)malloc(sizeof(double) * B);
        double *msg = (double *)malloc(sizeof(double) * n * C);
        double *Y = (double *)malloc(sizeof(double) * n);
#pragma omp for schedule(dynamic, 4)
        for (int t = 0; t < nt; ++t) {
            int i = targets ? targets[t] : t;
            int64_t e0 = nbr_offsets[i], e1 = nbr_offsets[i + 1];
            int K = (int)(e1 - e0);
            double *o = out + (size_t)t * n * C;
            for (int x = 0; x < n * C; ++x) o[x] = 0.0;
            if (K == 0) continue;
            double *s = (double *)malloc(sizeof(double) * K * H);
            double *gate = (double *)malloc(sizeof(double) * K);
            double *rij = (double *)malloc(sizeof(double) * K * 3);
            for (int e = 0; e < K; ++e) {
                int j = nbr_idx[e0 + e];
                double r[3];
                for (int x = 0; x < 3; ++x)
                    r[x] = (pos[3 * j + x] + (edge_shift ? edge_shift[3 * (e0 + e) + x] : 0.0)) - pos[3 * i + x];
                double d = sqrt(r[0] * r[0] + r[1] * r[1] + r[2] * r[2]);
                for (int x = 0; x < 3; ++x) rij[3 * e + x] = r[x];
                gate[e] = radial_gate(d, cfg->cutoff);
                radial_basis(d, cfg->cutoff, B, g);
                if (score_mode == 1) {
                    double rhat[3] = {r[0] / d, r[1] / d, r[2] / d};
                    for (int l = 0; l <= L; ++l) e2fo_solid_harmonics(l, rhat, Y + l * l);
                }
                for (int hh = 0; hh < H; ++hh) {
                    double dot = 0.0;
                    for (int l = 0; l <= L; ++l)
                        for (int c = hh * Ch; c < (hh + 1) * Ch; ++c) {
                            double fea = 1.0;
                            if (score_mode == 1) {
                                double a = 0.0, b = 0.0;
                                for (int m = 0; m < 2 * l + 1; ++m) {
                                    a += q1[((size_t)i * n + l * l + m) * C + c] * Y[l * l + m];
                                    b += v[((size_t)j * n + l * l + m) * C + c] * Y[l * l + m];
                                }
                                fea = a / (1.0 + exp(-a)) + b / (1.0 + exp(-b));
                            }
                            dot += q[((size_t)i * (L + 1) + l) * C + c] * k[((size_t)j * (L + 1) + l) * C + c] * fea;
                        }
                    double bias = 0.0;
                    for (int b = 0; b < B; ++b) bias += Wb[hh * B + b] * g[b];
                    s[e * H + hh] = tau * dot + bias;
                }
            }
            if (softmax_mode == 0) {
                /* alpha = softmax over the neighbours, then times the gate */
                double *alpha = (double *)malloc(sizeof(double) * K * H);
                for (int hh = 0; hh < H; ++hh) {
                    double mx = -INFINITY, z = 0.0;
                    for (int e = 0; e < K; ++e) mx = fmax(mx, s[e * H + hh]);
                    for (int e = 0; e < K; ++e) z += exp(s[e * H + hh] - mx);
                    for (int e = 0; e < K; ++e) alpha[e * H + hh] = exp(s[e * H + hh] - mx) / z * gate[e];
                }
                for (int e = 0; e < K; ++e) {
                    int j = nbr_idx[e0 + e];
                    const double *vj = v + (size_t)j * n * C;
                    if (message_mode == 0)
                        message_dense(&tab, w_path, vj, C, rij + 3 * e, msg);
                    else
                        message_eaas(&tab, w_path, vj, C, rij + 3 * e, chi, msg);
                    for (int x = 0; x < n; ++x)
                        for (int c = 0; c < C; ++c) o[x * C + c] += alpha[e * H + c / Ch] * msg[x * C + c];
                }
                free(alpha);
            } else {
                /* Algorithm 1: running max mu, normaliser z, accumulator A, per head */
                double *mu = (double *)malloc(sizeof(double) * H);
                double *z = (double *)malloc(sizeof(double) * H);
                for (int hh = 0; hh < H; ++hh) {
                    mu[hh] = -INFINITY;
                    z[hh] = 0.0;
                }
                for (int e = 0; e < K; ++e) {
                    int j = nbr_idx[e0 + e];
                    const double *vj = v + (size_t)j * n * C;
                    if (message_mode == 0)
                        message_dense(&tab, w_path, vj, C, rij + 3 * e, msg);
                    else
                        message_eaas(&tab, w_path, vj, C, rij + 3 * e, chi, msg);
                    for (int hh = 0; hh < H; ++hh) {
                        double sv = s[e * H + hh];
                        double mun = fmax(mu[hh], sv);
                        double scale = exp(mu[hh] - mun), pe = exp(sv - mun);
                        z[hh] = z[hh] * scale + pe;
                        for (int x = 0; x < n; ++x)
                            for (int c = hh * Ch; c < (hh + 1) * Ch; ++c)
                                o[x * C + c] = o[x * C + c] * scale + pe * gate[e] * msg[x * C + c];
                        mu[hh] = mun;
                    }
                }
                for (int c = 0; c < C; ++c)
                    for (int x = 0; x < n; ++x) o[x * C + c] /= z[c / Ch];
                free(mu);
                free(z);
            }
            free(s);
            free(gate);
            free(rij);
        }
        free(g);
        free(msg);
        free(Y);
    }
    free(q1);
    tables_free(&tab);
    free(need_q);
    free(need_kv);
    free(q);
    free(k);
    free(v);
    return 0;
}

/* Number of OpenMP threads the parallel loops above use (reported next to timings). */
#ifdef _OPENMP
#include <omp.h>
int e2fo_num_threads(void) { return omp_get_max_threads(); }
/* Thread count of the loops over target atoms (timing aid: the benchmark reports the oracle on all cores and on one). */
void e2fo_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int e2fo_num_threads(void) { return 1; }
void e2fo_set_num_threads(int n) { (void)n; }
#endif
