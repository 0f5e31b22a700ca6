/*
 * kge_oracle.c -- plain, slow CPU oracle for one mini-batch step of knowledge-graph-embedding training.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It exists so that the GPU library can be checked against
 * something obviously correct.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * build, load or call it.  It shares no code, header, table or helper with the GPU library.
 *
 * What it computes (paper sections in brackets):
 *   - the score of a triple (h, r, t) for TransE (L1 or L2), TransR, DistMult, ComplEx, RotatE and RESCAL  [Table 1]
 *   - negatives obtained by replacing the head or the tail of a positive triple              [Sec. 2]
 *   - joint negative sampling: positives are grouped into consecutive sets of size g and all members of a
 *     set share the same k corrupting entities                                               [Sec. 3.3]
 *   - the logistic loss  log(1 + exp(-y f))  with y = +1 on positives and -1 on negatives    [Sec. 2]
 *   - or the pairwise ranking loss  max(0, gamma - f(positive) + f(negative))                [Sec. 2]
 *   - the gradients of that loss with respect to every embedding row that took part          [Sec. 3.1 step 3]
 *   - the update of exactly those rows by Adagrad                                            [Sec. 3.1 step 4]
 *
 * How: every (positive, negative) pair is scored on its own, directly from the table rows, with the Table 1
 * formula written out.  There is no grouping into matrix products, no splitting of the score into two
 * parts, no blocking or fusion.  All arithmetic is fp64; embedding tables and optimizer state are stored as
 * fp32 (one rounding when a value is written back).
 *
 * Readings taken where the paper is silent (each is listed with its reason in the design notes):
 *   - distance models use  f = gamma - distance ; DistMult and ComplEx do not use gamma
 *   - TransE-L2 uses the un-squared norm (Table 1 and Sec. 3.3 agree on that)
 *   - RotatE uses gamma - sum_j |h_j r_j - t_j| (modulus per complex coordinate); the literally printed
 *     squared norm is available through rotate_squared
 *   - a row of ComplEx / RotatE entities is [real parts | imaginary parts]; a RotatE relation row holds
 *     phases in radians; a RESCAL relation row holds the D x D matrix M_r row by row (rel_dim = D * D); a TransR
 *     relation row holds the translation r (D numbers) followed by the D x D projection M_r row by row
 *     (rel_dim = D + D * D: relations live in a space of the entities' dimension)
 *   - TransR is used as printed in Table 1, with the squared norm: f = gamma - |M_r h + r - M_r t|_2^2
 *   - loss = (1/b) sum_i [ softplus(-f+_i) + sum_j w_ij softplus(f-_ij) ],  w_ij = 1/k, or the softmax over
 *     j of (adv_temperature * f-_ij) treated as a constant when adv_temperature > 0
 *   - ranking loss = (1/b) sum_i sum_j w_ij max(0, gamma - f+_i + f-_ij): every positive is paired with its own k
 *     negatives, with the same weights and the same 1/b as the logistic loss; its margin is the gamma that the
 *     distance models also carry inside f (where it cancels: gamma + dist+ - dist-); the sub-gradient at the kink
 *     (margin term exactly 0) is 0
 *   - the optimizer is element-wise Adagrad:  S += g^2 ; theta -= lr * g / (sqrt(S) + eps), where g is the
 *     sum of all contributions to that row within the step
 *   - where a norm or modulus is exactly zero its sub-gradient is taken to be zero
 *
 * In bf16_inputs mode the score of a (positive, negative) pair is, as in Sec. 3.3, a function of
 * o = h + r (or its analogue for the other models and the other side) and the corrupting row n; both are
 * rounded to bfloat16 (round to nearest even) before the pair function is evaluated, and so is the
 * per-pair backward coefficient.  Positives, loss and the update stay unrounded.
 *
 * parity pins (tests/test_oracle_*.py): hand-worked scores, central finite differences of the loss,
 * equality of the per-pair scores with the split form of Sec. 3.3 evaluated by numpy matrix products,
 * special values of the loss, the Adagrad closed form, brute-force duplicate counting; the bfloat16 rounding
 * against exact values (ties, the largest finite number, inf / nan) and two independent conversions; the
 * bf16_inputs branch against the Sec. 3.3 products written out in numpy on operands rounded by one of those; the
 * condition measure of grad_triple_mag against a hand-worked case, against |gradient| and against float32
 * re-evaluations of the same gradient under several orders of summation.  Copies of this file with a planted
 * mistake (truncating rounding, halved measure, unrounded coefficient) are compiled by the tests and must fail.
 *
 * Compiled with -fopenmp this file is also the all-cores timing baseline of the benchmark (ko_loss_grad deals
 * the positives to the threads); the parity oracle is always the build without OpenMP.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { KO_TRANSE_L2 = 0, KO_TRANSE_L1 = 1, KO_DISTMULT = 2, KO_COMPLEX = 3, KO_ROTATE = 4, KO_RESCAL = 5, KO_TRANSR = 6 };
enum { KO_NEG_TAIL = 0, KO_NEG_HEAD = 1 };
enum { KO_LOSS_LOGISTIC = 0, KO_LOSS_RANKING = 1 };

typedef struct {
    int32_t model;
    int32_t ent_dim;         /* numbers per entity row   */
    int32_t rel_dim;         /* numbers per relation row */
    int32_t neg_side;        /* KO_NEG_TAIL: (h, r, n);  KO_NEG_HEAD: (n, r, t) */
    int32_t tables_f64;      /* tables hold double instead of float (finite-difference tests) */
    int32_t bf16_inputs;     /* see header comment */
    int32_t rotate_squared;  /* RotatE as printed in Table 1: gamma - sum_j |h_j r_j - t_j|^2 */
    int32_t split_form;      /* evaluate negatives through the Sec. 3.3 split without any rounding (tests) */
    int32_t loss;            /* KO_LOSS_LOGISTIC or KO_LOSS_RANKING (the two losses of Sec. 2) */
    double gamma;
    double adv_temperature;
} ko_params;

/* ------------------------------------------------------------------------------------------------ */
/* helpers                                                                                            */

static void fetch_row(const void *table, int is_f64, int64_t row, int dim, double *out) {
    if (is_f64) {
        const double *src = (const double *)table + row * (int64_t)dim;
        for (int d = 0; d < dim; ++d) out[d] = src[d];
    } else {
        const float *src = (const float *)table + row * (int64_t)dim;
        for (int d = 0; d < dim; ++d) out[d] = (double)src[d];
    }
}

/* index of id in the ascending list ids[0..n); ids == NULL means the identity (dense tables) */
static int64_t slot_of(const int64_t *ids, int64_t n, int64_t id) {
    if (!ids) return id;
    int64_t lo = 0, hi = n - 1;
    while (lo <= hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (ids[mid] == id) return mid;
        if (ids[mid] < id) lo = mid + 1; else hi = mid - 1;
    }
    return -1;
}

static double softplus(double x) { return (x > 0 ? x : 0) + log1p(exp(-fabs(x))); }
static double sigmoid(double x) {
    if (x >= 0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

/* bfloat16 rounding (nearest, ties to even) of a value that is first held as fp32 */
static double round_bf16(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* the same, callable from the tests that pin it */
double ko_round_bf16(double x) { return round_bf16(x); }

/* ------------------------------------------------------------------------------------------------ */
/* Table 1: score of one triple from its three rows                                                   */

static double score_triple(const ko_params *p, const double *h, const double *r, const double *t) {
    const int D = p->ent_dim;
    double acc = 0.0;
    switch (p->model) {
    case KO_TRANSE_L2:
        for (int d = 0; d < D; ++d) { double u = h[d] + r[d] - t[d]; acc += u * u; }
        return p->gamma - sqrt(acc);
    case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) acc += fabs(h[d] + r[d] - t[d]);
        return p->gamma - acc;
    case KO_DISTMULT:
        for (int d = 0; d < D; ++d) acc += h[d] * r[d] * t[d];
        return acc;
    case KO_COMPLEX: {
        const int C = D / 2;
        for (int j = 0; j < C; ++j) {
            double hr_re = h[j] * r[j] - h[C + j] * r[C + j];
            double hr_im = h[j] * r[C + j] + h[C + j] * r[j];
            acc += hr_re * t[j] + hr_im * t[C + j]; /* Re( (h r) conj(t) ) */
        }
        return acc;
    }
    case KO_ROTATE: {
        const int C = D / 2;
        for (int j = 0; j < C; ++j) {
            double c = cos(r[j]), s = sin(r[j]);
            double q_re = h[j] * c - h[C + j] * s - t[j];
            double q_im = h[j] * s + h[C + j] * c - t[C + j];
            double m2 = q_re * q_re + q_im * q_im;
            acc += p->rotate_squared ? m2 : sqrt(m2);
        }
        return p->gamma - acc;
    }
    case KO_RESCAL: /* h^T M t, M[a][c] = r[a * D + c] */
        for (int a = 0; a < D; ++a)
            for (int c = 0; c < D; ++c) acc += h[a] * r[(int64_t)a * D + c] * t[c];
        return acc;
    case KO_TRANSR: { /* u = M h + r - M t, M[a][c] = r[D + a * D + c]; gamma - |u|^2 */
        const double *M = r + D;
        for (int a = 0; a < D; ++a) {
            double u = r[a];
            for (int c = 0; c < D; ++c) u += M[(int64_t)a * D + c] * (h[c] - t[c]);
            acc += u * u;
        }
        return p->gamma - acc;
    }
    default: return NAN;
    }
}

/* gh += coef * df/dh, gr += coef * df/dr, gt += coef * df/dt  for one triple */
static void grad_triple(const ko_params *p, const double *h, const double *r, const double *t, double coef,
                        double *gh, double *gr, double *gt) {
    const int D = p->ent_dim;
    switch (p->model) {
    case KO_TRANSE_L2: {
        double s = 0.0;
        for (int d = 0; d < D; ++d) { double u = h[d] + r[d] - t[d]; s += u * u; }
        double dist = sqrt(s);
        if (dist == 0.0) return;
        for (int d = 0; d < D; ++d) {
            double e = (h[d] + r[d] - t[d]) / dist;  /* d(dist)/du */
            gh[d] -= coef * e; gr[d] -= coef * e; gt[d] += coef * e;
        }
        return;
    }
    case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) {
            double u = h[d] + r[d] - t[d];
            double e = (u > 0) - (u < 0);
            gh[d] -= coef * e; gr[d] -= coef * e; gt[d] += coef * e;
        }
        return;
    case KO_DISTMULT:
        for (int d = 0; d < D; ++d) {
            gh[d] += coef * r[d] * t[d];
            gr[d] += coef * h[d] * t[d];
            gt[d] += coef * h[d] * r[d];
        }
        return;
    case KO_COMPLEX: {
        const int C = D / 2;
        for (int j = 0; j < C; ++j) {
            double hre = h[j], him = h[C + j], rre = r[j], rim = r[C + j], tre = t[j], tim = t[C + j];
            gh[j]     += coef * ( rre * tre + rim * tim);
            gh[C + j] += coef * (-rim * tre + rre * tim);
            gr[j]     += coef * ( hre * tre + him * tim);
            gr[C + j] += coef * (-him * tre + hre * tim);
            gt[j]     += coef * ( hre * rre - him * rim);
            gt[C + j] += coef * ( hre * rim + him * rre);
        }
        return;
    }
    case KO_ROTATE: {
        const int C = D / 2;
        for (int j = 0; j < C; ++j) {
            double c = cos(r[j]), s = sin(r[j]);
            double p_re = h[j] * c - h[C + j] * s, p_im = h[j] * s + h[C + j] * c; /* h rotated by theta */
            double q_re = p_re - t[j], q_im = p_im - t[C + j];
            double e_re, e_im; /* d(term_j)/dq, term_j = |q| or |q|^2 */
            if (p->rotate_squared) { e_re = 2 * q_re; e_im = 2 * q_im; }
            else {
                double m = sqrt(q_re * q_re + q_im * q_im);
                if (m == 0.0) continue;
                e_re = q_re / m; e_im = q_im / m;
            }
            /* f = gamma - sum term_j */
            gt[j]     += coef * e_re;
            gt[C + j] += coef * e_im;
            gh[j]     -= coef * ( e_re * c + e_im * s);
            gh[C + j] -= coef * (-e_re * s + e_im * c);
            gr[j]     -= coef * (-e_re * p_im + e_im * p_re);
        }
        return;
    }
    case KO_RESCAL:
        for (int a = 0; a < D; ++a)
            for (int c = 0; c < D; ++c) {
                const double m = r[(int64_t)a * D + c];
                gh[a] += coef * m * t[c];
                gt[c] += coef * h[a] * m;
                gr[(int64_t)a * D + c] += coef * h[a] * t[c];
            }
        return;
    case KO_TRANSR: { /* f = gamma - sum_a u_a^2, u = M (h - t) + r:  df/du_a = -2 u_a */
        const double *M = r + D;
        for (int a = 0; a < D; ++a) {
            double u = r[a];
            for (int c = 0; c < D; ++c) u += M[(int64_t)a * D + c] * (h[c] - t[c]);
            const double e = -2.0 * u * coef;
            gr[a] += e;
            for (int c = 0; c < D; ++c) {
                gh[c] += e * M[(int64_t)a * D + c];
                gt[c] -= e * M[(int64_t)a * D + c];
                gr[D + (int64_t)a * D + c] += e * (h[c] - t[c]);
            }
        }
        return;
    }
    default: return;
    }
}

/*
 * Condition measure for the parity tests (not part of the method): an upper estimate, per element, of the
 * magnitudes of the terms that the gradient contribution of one triple is built from.  Where grad_triple forms
 * coef * (x - y) this adds |coef| * (|x| + |y|), so that (unit roundoff) * (sum of these over all triples) bounds
 * the error of evaluating the same gradient in a shorter floating-point format, including cancellation inside
 * a single contribution.  For TransE-L1 a coordinate whose difference is within roundoff of zero may get the
 * other sign in a shorter format; its whole contribution is then charged (scaled so that 2^-20 of it covers it).
 */
static void grad_triple_mag(const ko_params *p, const double *h, const double *r, const double *t, double coef,
                            double *mh, double *mr, double *mt) {
    const int D = p->ent_dim;
    const double ac = fabs(coef);
    switch (p->model) {
    case KO_TRANSE_L2: {
        double s = 0.0;
        for (int d = 0; d < D; ++d) { double u = h[d] + r[d] - t[d]; s += u * u; }
        double dist = sqrt(s);
        if (dist == 0.0) return;
        for (int d = 0; d < D; ++d) {
            double m = ac * (fabs(h[d]) + fabs(r[d]) + fabs(t[d])) / dist;
            mh[d] += m; mr[d] += m; mt[d] += m;
        }
        return;
    }
    case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) {
            double u = h[d] + r[d] - t[d], scale = fabs(h[d]) + fabs(r[d]) + fabs(t[d]);
            double m = fabs(u) <= 9.5367431640625e-07 * scale ? 2.0 * ac * 1048576.0 : ac;
            mh[d] += m; mr[d] += m; mt[d] += m;
        }
        return;
    case KO_DISTMULT:
        for (int d = 0; d < D; ++d) {
            mh[d] += ac * fabs(r[d] * t[d]);
            mr[d] += ac * fabs(h[d] * t[d]);
            mt[d] += ac * fabs(h[d] * r[d]);
        }
        return;
    case KO_COMPLEX: {
        const int C = D / 2;
        for (int j = 0; j < C; ++j) {
            double hre = fabs(h[j]), him = fabs(h[C + j]), rre = fabs(r[j]), rim = fabs(r[C + j]);
            double tre = fabs(t[j]), tim = fabs(t[C + j]);
            mh[j] += ac * (rre * tre + rim * tim); mh[C + j] += ac * (rim * tre + rre * tim);
            mr[j] += ac * (hre * tre + him * tim); mr[C + j] += ac * (him * tre + hre * tim);
            mt[j] += ac * (hre * rre + him * rim); mt[C + j] += ac * (hre * rim + him * rre);
        }
        return;
    }
    case KO_ROTATE: {
        const int C = D / 2;
        for (int j = 0; j < C; ++j) {
            double c = cos(r[j]), s = sin(r[j]);
            double p_re = h[j] * c - h[C + j] * s, p_im = h[j] * s + h[C + j] * c;
            double q_re = p_re - t[j], q_im = p_im - t[C + j];
            double m = p->rotate_squared ? 0.5 : sqrt(q_re * q_re + q_im * q_im);
            if (m == 0.0) continue;
            /* magnitudes of the terms of q_re, q_im, divided by |q| (the direction e = q / |q|) */
            double T_re = (fabs(h[j] * c) + fabs(h[C + j] * s) + fabs(t[j])) / m;
            double T_im = (fabs(h[j] * s) + fabs(h[C + j] * c) + fabs(t[C + j])) / m;
            mt[j] += ac * T_re; mt[C + j] += ac * T_im;
            mh[j] += ac * (T_re * fabs(c) + T_im * fabs(s));
            mh[C + j] += ac * (T_re * fabs(s) + T_im * fabs(c));
            mr[j] += ac * (T_re * fabs(p_im) + T_im * fabs(p_re));
        }
        return;
    }
    case KO_RESCAL:
        for (int a = 0; a < D; ++a)
            for (int c = 0; c < D; ++c) {
                const double m = fabs(r[(int64_t)a * D + c]);
                mh[a] += ac * m * fabs(t[c]);
                mt[c] += ac * fabs(h[a]) * m;
                mr[(int64_t)a * D + c] += ac * fabs(h[a] * t[c]);
            }
        return;
    case KO_TRANSR: { /* magnitudes of the terms of u_a, times the factors they are multiplied with */
        const double *M = r + D;
        for (int a = 0; a < D; ++a) {
            double T = fabs(r[a]);
            for (int c = 0; c < D; ++c) T += fabs(M[(int64_t)a * D + c]) * (fabs(h[c]) + fabs(t[c]));
            const double e = 2.0 * T * ac;
            mr[a] += e;
            for (int c = 0; c < D; ++c) {
                mh[c] += e * fabs(M[(int64_t)a * D + c]);
                mt[c] += e * fabs(M[(int64_t)a * D + c]);
                mr[D + (int64_t)a * D + c] += e * (fabs(h[c]) + fabs(t[c]));
            }
        }
        return;
    }
    default: return;
    }
}

/* ------------------------------------------------------------------------------------------------ */
/* bf16_inputs mode: the Sec. 3.3 split.  o depends on the uncorrupted entity a and the relation only. */

/* o for a positive: tail side a = h, head side a = t */
static void split_o(const ko_params *p, const double *a, const double *r, double *o) {
    const int D = p->ent_dim, C = D / 2;
    const int head = p->neg_side == KO_NEG_HEAD;
    switch (p->model) {
    case KO_TRANSE_L2: case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) o[d] = head ? a[d] - r[d] : a[d] + r[d];
        break;
    case KO_DISTMULT:
        for (int d = 0; d < D; ++d) o[d] = a[d] * r[d];
        break;
    case KO_COMPLEX: case KO_ROTATE:
        for (int j = 0; j < C; ++j) {
            double rre, rim;
            if (p->model == KO_ROTATE) { rre = cos(r[j]); rim = sin(r[j]); } else { rre = r[j]; rim = r[C + j]; }
            if (head) rim = -rim; /* a * conj(r) */
            o[j]     = a[j] * rre - a[C + j] * rim;
            o[C + j] = a[j] * rim + a[C + j] * rre;
        }
        break;
    case KO_RESCAL: /* tail side: h^T M n = (M^T h) . n ; head side: n^T M t = n . (M t) */
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int x = 0; x < D; ++x)
            for (int c = 0; c < D; ++c) {
                if (head) o[x] += r[(int64_t)x * D + c] * a[c];
                else o[c] += a[x] * r[(int64_t)x * D + c];
            }
        break;
    }
}

/* score of a pair from o and the corrupting row x */
static double pair_score(const ko_params *p, const double *o, const double *x) {
    const int D = p->ent_dim, C = D / 2;
    double acc = 0.0;
    switch (p->model) {
    case KO_TRANSE_L2:
        for (int d = 0; d < D; ++d) { double u = o[d] - x[d]; acc += u * u; }
        return p->gamma - sqrt(acc);
    case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) acc += fabs(o[d] - x[d]);
        return p->gamma - acc;
    case KO_DISTMULT: case KO_COMPLEX: case KO_RESCAL:
        for (int d = 0; d < D; ++d) acc += o[d] * x[d];
        return acc;
    case KO_ROTATE:
        for (int j = 0; j < C; ++j) {
            double q_re = o[j] - x[j], q_im = o[C + j] - x[C + j];
            double m2 = q_re * q_re + q_im * q_im;
            acc += p->rotate_squared ? m2 : sqrt(m2);
        }
        return p->gamma - acc;
    }
    return NAN;
}

/* go += coef * dpsi/do, gx += coef * dpsi/dx */
static void pair_grad(const ko_params *p, const double *o, const double *x, double coef, double *go, double *gx) {
    const int D = p->ent_dim, C = D / 2;
    switch (p->model) {
    case KO_TRANSE_L2: {
        double s = 0.0;
        for (int d = 0; d < D; ++d) { double u = o[d] - x[d]; s += u * u; }
        double dist = sqrt(s);
        if (dist == 0.0) return;
        for (int d = 0; d < D; ++d) { double e = (o[d] - x[d]) / dist; go[d] -= coef * e; gx[d] += coef * e; }
        return;
    }
    case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) { double u = o[d] - x[d]; double e = (u > 0) - (u < 0); go[d] -= coef * e; gx[d] += coef * e; }
        return;
    case KO_DISTMULT: case KO_COMPLEX: case KO_RESCAL:
        for (int d = 0; d < D; ++d) { go[d] += coef * x[d]; gx[d] += coef * o[d]; }
        return;
    case KO_ROTATE:
        for (int j = 0; j < C; ++j) {
            double q_re = o[j] - x[j], q_im = o[C + j] - x[C + j], e_re, e_im;
            if (p->rotate_squared) { e_re = 2 * q_re; e_im = 2 * q_im; }
            else {
                double m = sqrt(q_re * q_re + q_im * q_im);
                if (m == 0.0) continue;
                e_re = q_re / m; e_im = q_im / m;
            }
            go[j] -= coef * e_re; go[C + j] -= coef * e_im;
            gx[j] += coef * e_re; gx[C + j] += coef * e_im;
        }
        return;
    }
}

/* ga += J_a^T go, gr += J_r^T go for o = split_o(a, r) */
static void split_o_backward(const ko_params *p, const double *a, const double *r, const double *go, double *ga, double *gr) {
    const int D = p->ent_dim, C = D / 2;
    const int head = p->neg_side == KO_NEG_HEAD;
    switch (p->model) {
    case KO_TRANSE_L2: case KO_TRANSE_L1:
        for (int d = 0; d < D; ++d) { ga[d] += go[d]; gr[d] += head ? -go[d] : go[d]; }
        break;
    case KO_DISTMULT:
        for (int d = 0; d < D; ++d) { ga[d] += go[d] * r[d]; gr[d] += go[d] * a[d]; }
        break;
    case KO_COMPLEX:
        for (int j = 0; j < C; ++j) {
            double rre = r[j], rim = head ? -r[C + j] : r[C + j];
            /* o_re = a_re rre - a_im rim ; o_im = a_re rim + a_im rre */
            ga[j]     += go[j] * rre + go[C + j] * rim;
            ga[C + j] += -go[j] * rim + go[C + j] * rre;
            double d_rre = go[j] * a[j] + go[C + j] * a[C + j];
            double d_rim = -go[j] * a[C + j] + go[C + j] * a[j];
            gr[j] += d_rre;
            gr[C + j] += head ? -d_rim : d_rim;
        }
        break;
    case KO_ROTATE:
        for (int j = 0; j < C; ++j) {
            double rre = cos(r[j]), rim = sin(r[j]);
            if (head) rim = -rim;
            double o_re = a[j] * rre - a[C + j] * rim, o_im = a[j] * rim + a[C + j] * rre;
            ga[j]     += go[j] * rre + go[C + j] * rim;
            ga[C + j] += -go[j] * rim + go[C + j] * rre;
            /* tail side do/dtheta = i o ; head side do/dtheta = -i o */
            double d_th = -go[j] * o_im + go[C + j] * o_re;
            gr[j] += head ? -d_th : d_th;
        }
        break;
    case KO_RESCAL:
        for (int x = 0; x < D; ++x)
            for (int c = 0; c < D; ++c) {
                const double m = r[(int64_t)x * D + c];
                if (head) { ga[c] += go[x] * m; gr[(int64_t)x * D + c] += go[x] * a[c]; }  /* o = M a */
                else { ga[x] += m * go[c]; gr[(int64_t)x * D + c] += a[x] * go[c]; }        /* o = M^T a */
            }
        break;
    }
}

/* ------------------------------------------------------------------------------------------------ */
/* loss and gradients of one mini-batch                                                               */

/* acc[slot] += v */
static void add_rows(double *acc, int64_t slot, int dim, const double *v) {
    double *dst = acc + slot * (int64_t)dim;
    for (int d = 0; d < dim; ++d) dst[d] += v[d];
}

/* scratch rows of one worker */
typedef struct {
    double *hv, *tv, *nv, *rv, *ov, *go, *th, *tt, *tr, *fneg, *w;
} ko_scratch;

static int scratch_alloc(ko_scratch *s, int De, int Dr, int64_t k) {
    const size_t nr = (size_t)(Dr > De ? Dr : De), nk = (size_t)(k > 0 ? k : 1);
    memset(s, 0, sizeof(*s));
    s->hv = malloc(sizeof(double) * De); s->tv = malloc(sizeof(double) * De); s->nv = malloc(sizeof(double) * De);
    s->rv = malloc(sizeof(double) * nr);
    s->ov = malloc(sizeof(double) * De); s->go = malloc(sizeof(double) * De);
    s->th = malloc(sizeof(double) * De); s->tt = malloc(sizeof(double) * De);
    s->tr = malloc(sizeof(double) * nr);
    s->fneg = malloc(sizeof(double) * nk); s->w = malloc(sizeof(double) * nk);
    return s->hv && s->tv && s->nv && s->rv && s->ov && s->go && s->th && s->tt && s->tr && s->fneg && s->w;
}

static void scratch_free(ko_scratch *s) {
    free(s->hv); free(s->tv); free(s->nv); free(s->rv); free(s->ov); free(s->go); free(s->fneg); free(s->w);
    free(s->th); free(s->tt); free(s->tr);
}

/* what ko_loss_grad was asked for, and where a worker adds its results */
typedef struct {
    const ko_params *p;
    const void *E, *R;
    const int64_t *h, *r, *t, *neg;
    int64_t b, k, chunk;
    const double *w_fixed;
    double *pos_score, *neg_score, *w_out;
    const int64_t *ent_ids, *rel_ids;
    int64_t n_ent_slots, n_rel_slots;
} ko_batch;

typedef struct {
    double total;                    /* this worker's share of the loss */
    double *dE, *dR, *aE, *aR, *mE, *mR; /* accumulators (see ko_loss_grad); dE == NULL: no gradients wanted */
} ko_acc;

/* Positive i with its k negatives: scores, weights, loss term, and (if wanted) every gradient contribution.
 * Returns 0, or -2 if an id has no slot. */
static int one_positive(const ko_batch *q, int64_t i, ko_scratch *s, ko_acc *acc) {
    const ko_params *p = q->p;
    const int De = p->ent_dim, Dr = p->rel_dim, f64 = p->tables_f64;
    const int head_side = p->neg_side == KO_NEG_HEAD;
    const int use_split = p->bf16_inputs || p->split_form;
    const int64_t b = q->b, k = q->k;
    const int64_t *h = q->h, *r = q->r, *t = q->t, *neg = q->neg;
    double *hv = s->hv, *tv = s->tv, *nv = s->nv, *rv = s->rv, *ov = s->ov, *go = s->go;
    double *th = s->th, *tt = s->tt, *tr = s->tr, *fneg = s->fneg, *w = s->w;
    double *dE = acc->dE, *dR = acc->dR, *aE = acc->aE, *aR = acc->aR, *mE = acc->mE, *mR = acc->mR;

    const int64_t c = i / q->chunk;
    fetch_row(q->E, f64, h[i], De, hv);
    fetch_row(q->R, f64, r[i], Dr, rv);
    fetch_row(q->E, f64, t[i], De, tv);
    const double fpos = score_triple(p, hv, rv, tv);
    if (q->pos_score) q->pos_score[i] = fpos;

    if (use_split) {
        split_o(p, head_side ? tv : hv, rv, ov);
        if (p->bf16_inputs) for (int d = 0; d < De; ++d) ov[d] = round_bf16(ov[d]);
    }
    /* scores of this positive's k negatives */
    for (int64_t j = 0; j < k; ++j) {
        fetch_row(q->E, f64, neg[c * k + j], De, nv);
        if (use_split) {
            if (p->bf16_inputs) for (int d = 0; d < De; ++d) nv[d] = round_bf16(nv[d]);
            fneg[j] = pair_score(p, ov, nv);
        } else {
            fneg[j] = head_side ? score_triple(p, nv, rv, tv) : score_triple(p, hv, rv, nv);
        }
        if (q->neg_score) q->neg_score[i * k + j] = fneg[j];
    }
    /* weights of the negatives: uniform, or softmax of temperature * score (held constant) */
    if (q->w_fixed) {
        for (int64_t j = 0; j < k; ++j) w[j] = q->w_fixed[i * k + j];
    } else if (p->adv_temperature > 0 && k > 0) {
        double mx = -INFINITY, z = 0.0;
        for (int64_t j = 0; j < k; ++j) if (p->adv_temperature * fneg[j] > mx) mx = p->adv_temperature * fneg[j];
        for (int64_t j = 0; j < k; ++j) { w[j] = exp(p->adv_temperature * fneg[j] - mx); z += w[j]; }
        for (int64_t j = 0; j < k; ++j) w[j] /= z;
    } else {
        for (int64_t j = 0; j < k; ++j) w[j] = 1.0 / (double)k;
    }
    if (q->w_out) for (int64_t j = 0; j < k; ++j) q->w_out[i * k + j] = w[j];

    double li, cpos;
    if (p->loss == KO_LOSS_RANKING) {
        /* pairwise ranking loss: the positive against each of its negatives, margin gamma */
        double active = 0.0;
        li = 0.0;
        for (int64_t j = 0; j < k; ++j) {
            const double m = p->gamma - fpos + fneg[j];
            if (m > 0) { li += w[j] * m; active += w[j]; }
        }
        cpos = -active / (double)b;
    } else {
        /* logistic loss: y = +1 for the positive, y = -1 for each negative */
        li = softplus(-fpos);
        for (int64_t j = 0; j < k; ++j) li += w[j] * softplus(fneg[j]);
        cpos = -sigmoid(-fpos) / (double)b; /* d/df softplus(-f) / b */
    }
    acc->total += li / (double)b;

    if (!dE) return 0;
    const int64_t sh = slot_of(q->ent_ids, q->n_ent_slots, h[i]);
    const int64_t st = slot_of(q->ent_ids, q->n_ent_slots, t[i]);
    const int64_t sr = slot_of(q->rel_ids, q->n_rel_slots, r[i]);
    if (sh < 0 || st < 0 || sr < 0) return -2;
    /* every triple's contribution is formed in scratch rows (th, tr, tt) and then added to the rows'
     * accumulators; the optional aE / aR receive the magnitudes of the terms involved (a condition
     * measure used by the parity tests, not part of the method) */
    memset(th, 0, sizeof(double) * De); memset(tr, 0, sizeof(double) * Dr); memset(tt, 0, sizeof(double) * De);
    grad_triple(p, hv, rv, tv, cpos, th, tr, tt);
    add_rows(dE, sh, De, th); add_rows(dR, sr, Dr, tr); add_rows(dE, st, De, tt);
    if (aE) grad_triple_mag(p, hv, rv, tv, cpos, aE + sh * De, aR + sr * Dr, aE + st * De);
    if (use_split) memset(go, 0, sizeof(double) * De);
    for (int64_t j = 0; j < k; ++j) {
        const int64_t n = neg[c * k + j];
        const int64_t sn = slot_of(q->ent_ids, q->n_ent_slots, n);
        if (sn < 0) return -2;
        double cneg = w[j] * sigmoid(fneg[j]) / (double)b; /* d/df softplus(f) * w / b */
        fetch_row(q->E, f64, n, De, nv);
        if (p->loss == KO_LOSS_RANKING) {
            const double m = p->gamma - fpos + fneg[j];
            cneg = m > 0 ? w[j] / (double)b : 0.0;
            double big = fabs(fpos) > fabs(fneg[j]) ? fabs(fpos) : fabs(fneg[j]);
            if (aE && fabs(m) <= 2e-5 * (big > 1 ? big : 1)) { /* undecided in fp32: see aE above */
                const double flip = 1048576.0 * w[j] / (double)b;
                grad_triple_mag(p, hv, rv, tv, flip, aE + sh * De, aR + sr * Dr, aE + st * De);
                if (head_side) grad_triple_mag(p, nv, rv, tv, flip, aE + sn * De, aR + sr * Dr, aE + st * De);
                else grad_triple_mag(p, hv, rv, nv, flip, aE + sh * De, aR + sr * Dr, aE + sn * De);
            }
        }
        memset(th, 0, sizeof(double) * De); memset(tr, 0, sizeof(double) * Dr); memset(tt, 0, sizeof(double) * De);
        if (aE) {
            if (head_side) grad_triple_mag(p, nv, rv, tv, cneg, aE + sn * De, aR + sr * Dr, aE + st * De);
            else grad_triple_mag(p, hv, rv, nv, cneg, aE + sh * De, aR + sr * Dr, aE + sn * De);
        }
        if (mE && mR) { /* this pair's measure alone, then the element-wise maximum */
            memset(th, 0, sizeof(double) * De); memset(tr, 0, sizeof(double) * Dr); memset(tt, 0, sizeof(double) * De);
            if (head_side) grad_triple_mag(p, nv, rv, tv, cneg, tt, tr, th); /* tt: the negative, th: the kept one */
            else grad_triple_mag(p, hv, rv, nv, cneg, th, tr, tt);
            const int64_t sk = head_side ? st : sh;
            for (int d = 0; d < De; ++d) {
                if (th[d] > mE[sk * De + d]) mE[sk * De + d] = th[d];
                if (tt[d] > mE[sn * De + d]) mE[sn * De + d] = tt[d];
            }
            for (int d = 0; d < Dr; ++d) if (tr[d] > mR[sr * Dr + d]) mR[sr * Dr + d] = tr[d];
            memset(th, 0, sizeof(double) * De); memset(tr, 0, sizeof(double) * Dr); memset(tt, 0, sizeof(double) * De);
        }
        if (use_split) {
            if (p->bf16_inputs) {
                /* the coefficient that multiplies the rounded operands in the backward products */
                if (p->model == KO_TRANSE_L2) {
                    double dist = p->gamma - fneg[j];
                    double wq = dist > 0 ? round_bf16(cneg / dist) : 0.0;
                    cneg = wq * dist;
                } else {
                    cneg = round_bf16(cneg);
                }
                for (int d = 0; d < De; ++d) nv[d] = round_bf16(nv[d]);
            }
            pair_grad(p, ov, nv, cneg, go, tt);
            add_rows(dE, sn, De, tt);
        } else if (head_side) {
            grad_triple(p, nv, rv, tv, cneg, th, tr, tt); /* (n, r, t) */
            add_rows(dE, sn, De, th); add_rows(dR, sr, Dr, tr); add_rows(dE, st, De, tt);
        } else {
            grad_triple(p, hv, rv, nv, cneg, th, tr, tt); /* (h, r, n) */
            add_rows(dE, sh, De, th); add_rows(dR, sr, Dr, tr); add_rows(dE, sn, De, tt);
        }
    }
    if (use_split) {
        memset(th, 0, sizeof(double) * De); memset(tr, 0, sizeof(double) * Dr);
        split_o_backward(p, head_side ? tv : hv, rv, go, th, tr);
        add_rows(dE, head_side ? st : sh, De, th); add_rows(dR, sr, Dr, tr);
    }
    return 0;
}

/* how many workers ko_loss_grad spreads the positives over: 1 unless this file was compiled with OpenMP */
int ko_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * h, r, t : [b] ids of the positive triples.   neg : [(b / chunk) * k] corrupting entity ids; positives
 * chunk*c .. chunk*(c+1)-1 share neg[c*k .. c*k+k-1]  (Sec. 3.3).
 * w_fixed : NULL, or [b*k] weights to use instead of computing them (finite-difference tests freeze them).
 * pos_score [b], neg_score [b*k], w_out [b*k] : outputs, each may be NULL.
 * dE / dR : NULL (no gradients wanted) or zero-initialised [n_slots * dim] accumulators; row s of dE
 * belongs to entity ent_ids[s] (ascending list), or to entity s when ent_ids == NULL.
 * aE / aR : NULL or accumulators of the same shape for the condition measure of grad_triple_mag.  With the
 *           ranking loss a pair whose margin term lies within 2e-5 * max(1, |f+|, |f-|) of the kink (fp32 scores
 *           may put it on the other side) adds 2^20 times what switching it on or off would change.
 * mE / mR : NULL or arrays of the same shape that receive, per element, the largest grad_triple_mag measure of a
 *           single (positive, negative) pair: how much one backward coefficient weighs in that element (the tests
 *           bound with it what a coefficient that rounds to the neighbouring bfloat16 value can change).
 * Returns 0, or -1 on bad arguments, -2 if an id has no slot, -3 if memory ran out.
 *
 * The parity oracle is this file compiled WITHOUT OpenMP: one worker takes the positives in order.  Compiled with
 * -fopenmp (the all-cores timing baseline) the positives are dealt to the threads in contiguous blocks, every
 * thread adds into accumulators of its own, and these are added up in thread order afterwards: the same terms in
 * another order of summation.
 */
int ko_loss_grad(const ko_params *p, const void *E, const void *R,
                 const int64_t *h, const int64_t *r, const int64_t *t, int64_t b,
                 const int64_t *neg, int64_t k, int64_t chunk, const double *w_fixed,
                 double *loss_out, double *pos_score, double *neg_score, double *w_out,
                 const int64_t *ent_ids, int64_t n_ent_slots, double *dE, double *aE,
                 const int64_t *rel_ids, int64_t n_rel_slots, double *dR, double *aR, double *mE, double *mR) {
    if (b <= 0 || chunk <= 0 || b % chunk != 0 || k < 0) return -1;
    if ((p->model == KO_COMPLEX || p->model == KO_ROTATE) && (p->ent_dim % 2)) return -1;
    if (p->model == KO_RESCAL && p->rel_dim != p->ent_dim * p->ent_dim) return -1;
    if (p->model == KO_TRANSR && p->rel_dim != p->ent_dim + p->ent_dim * p->ent_dim) return -1;
    if (p->model == KO_TRANSR && (p->bf16_inputs || p->split_form)) return -1; /* its pairs do not split into (o, n) */
    const int De = p->ent_dim, Dr = p->rel_dim;
    const ko_batch q = { p, E, R, h, r, t, neg, b, k, chunk, w_fixed, pos_score, neg_score, w_out,
                         ent_ids, rel_ids, n_ent_slots, n_rel_slots };
    int rc = 0;
    double total = 0.0;
#ifdef _OPENMP
    int nt = omp_get_max_threads();
    if ((int64_t)nt > b) nt = (int)b;
    if (nt > 1) {
        const size_t nE = (size_t)n_ent_slots * De, nR = (size_t)n_rel_slots * Dr;
        ko_acc *accs = calloc((size_t)nt, sizeof(ko_acc));
        int *rcs = calloc((size_t)nt, sizeof(int));
        if (!accs || !rcs) { free(accs); free(rcs); return -3; }
#pragma omp parallel num_threads(nt)
        {
            const int tid = omp_get_thread_num();
            ko_acc *a = &accs[tid];
            ko_scratch s;
            int ok = scratch_alloc(&s, De, Dr, k);
            if (dE) {
                a->dE = calloc(nE, sizeof(double)); a->dR = calloc(nR, sizeof(double));
                ok = ok && a->dE && a->dR;
                if (aE) { a->aE = calloc(nE, sizeof(double)); a->aR = calloc(nR, sizeof(double)); ok = ok && a->aE && a->aR; }
                if (mE && mR) { a->mE = calloc(nE, sizeof(double)); a->mR = calloc(nR, sizeof(double)); ok = ok && a->mE && a->mR; }
            }
            if (!ok) rcs[tid] = -3;
            const int64_t lo = b * tid / nt, hi = b * (tid + 1) / nt;
            for (int64_t i = lo; i < hi && rcs[tid] == 0; ++i) rcs[tid] = one_positive(&q, i, &s, a);
            scratch_free(&s);
        }
        for (int tid = 0; tid < nt; ++tid) {
            ko_acc *a = &accs[tid];
            if (rcs[tid] != 0 && rc == 0) rc = rcs[tid];
            total += a->total;
            if (a->dE && a->dR) {
                for (size_t x = 0; x < nE; ++x) dE[x] += a->dE[x];
                for (size_t x = 0; x < nR; ++x) dR[x] += a->dR[x];
            }
            if (a->aE && a->aR) {
                for (size_t x = 0; x < nE; ++x) aE[x] += a->aE[x];
                for (size_t x = 0; x < nR; ++x) aR[x] += a->aR[x];
            }
            if (a->mE && a->mR) {
                for (size_t x = 0; x < nE; ++x) if (a->mE[x] > mE[x]) mE[x] = a->mE[x];
                for (size_t x = 0; x < nR; ++x) if (a->mR[x] > mR[x]) mR[x] = a->mR[x];
            }
            free(a->dE); free(a->dR); free(a->aE); free(a->aR); free(a->mE); free(a->mR);
        }
        free(accs); free(rcs);
        if (loss_out) *loss_out = total;
        return rc;
    }
#endif
    ko_scratch s;
    if (!scratch_alloc(&s, De, Dr, k)) { scratch_free(&s); return -3; }
    ko_acc acc = { 0.0, dE, dR, aE, aR, mE, mR };
    for (int64_t i = 0; i < b && rc == 0; ++i) rc = one_positive(&q, i, &s, &acc);
    total = acc.total;
    if (loss_out) *loss_out = total;
    scratch_free(&s);
    return rc;
}

/* ------------------------------------------------------------------------------------------------ */
/* duplicates                                                                                         */

static int cmp_i64(const void *a, const void *b) {
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/* distinct values of keys[0..n) ascending in uniq, their multiplicities in cnt; returns how many */
int64_t ko_dedup(const int64_t *keys, int64_t n, int64_t *uniq, int64_t *cnt) {
    if (n <= 0) return 0;
    int64_t *tmp = malloc(sizeof(int64_t) * n);
    memcpy(tmp, keys, sizeof(int64_t) * n);
    qsort(tmp, n, sizeof(int64_t), cmp_i64);
    int64_t u = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (u > 0 && uniq[u - 1] == tmp[i]) cnt[u - 1] += 1;
        else { uniq[u] = tmp[i]; cnt[u] = 1; ++u; }
    }
    free(tmp);
    return u;
}

/* ------------------------------------------------------------------------------------------------ */
/* Adagrad                                                                                            */

/* rows ids[0..n) (or rows 0..n-1 when ids == NULL) of table/state, with gradient rows grad[s*dim ..].
 * rowwise == 0: element-wise state of the table's shape:  S_d += g_d^2 ;  x_d -= lr g_d / (sqrt(S_d) + eps)
 * rowwise != 0: one state value per row (state has n_rows floats):
 *               S += mean_d g_d^2 ;  x_d -= lr g_d / (sqrt(S) + eps)   (a row with zero gradient keeps its bits) */
void ko_adagrad_rows(float *table, float *state, const int64_t *ids, int64_t n, int dim, const double *grad,
                     double lr, double eps, int rowwise) {
    for (int64_t s = 0; s < n; ++s) {
        const int64_t row = ids ? ids[s] : s;
        float *th = table + row * (int64_t)dim, *st = state + row * (int64_t)dim;
        const double *g = grad + s * (int64_t)dim;
        if (rowwise) {
            double ms = 0.0;
            for (int d = 0; d < dim; ++d) ms += g[d] * g[d];
            ms /= (double)dim;
            const double S = (double)state[row] + ms;
            const double den = sqrt(S) + eps;
            for (int d = 0; d < dim; ++d) th[d] = (float)((double)th[d] - lr * g[d] / den);
            state[row] = (float)S;
            continue;
        }
        for (int d = 0; d < dim; ++d) {
            double S = (double)st[d] + g[d] * g[d];
            double x = (double)th[d] - lr * g[d] / (sqrt(S) + eps);
            st[d] = (float)S;
            th[d] = (float)x;
        }
    }
}

/*
 * One whole step on fp32 tables: loss, gradients, Adagrad.  dense != 0: gradients are accumulated in
 * arrays as large as the tables and every row is updated (rows with zero gradient come out bit-identical);
 * dense == 0: only the distinct rows that occur in the batch get a gradient row and an update.
 * Both give the same tables bit for bit (checked in the tests).
 */
int ko_train_step(const ko_params *p, float *E, float *SE, int64_t n_ent, float *R, float *SR, int64_t n_rel,
                  const int64_t *h, const int64_t *r, const int64_t *t, int64_t b,
                  const int64_t *neg, int64_t k, int64_t chunk, double lr, double eps, int dense, int rowwise,
                  double *loss_out, double *pos_score, double *neg_score,
                  int64_t *ent_ids_out, int64_t *n_ent_out, double *dE_out, double *aE_out,
                  int64_t *rel_ids_out, int64_t *n_rel_out, double *dR_out, double *aR_out,
                  double *mE_out, double *mR_out) {
    if (p->tables_f64) return -1;
    if (b <= 0 || chunk <= 0 || b % chunk != 0) return -1;
    const int64_t n_neg = (b / chunk) * k, n_keys = 2 * b + n_neg;
    for (int64_t i = 0; i < b; ++i)
        if (h[i] < 0 || h[i] >= n_ent || t[i] < 0 || t[i] >= n_ent || r[i] < 0 || r[i] >= n_rel) return -1;
    for (int64_t j = 0; j < n_neg; ++j) if (neg[j] < 0 || neg[j] >= n_ent) return -1;

    int64_t *ent_ids = NULL, *rel_ids = NULL, ue = n_ent, ur = n_rel;
    if (!dense) {
        int64_t *keys = malloc(sizeof(int64_t) * n_keys), *cnt = malloc(sizeof(int64_t) * n_keys);
        memcpy(keys, h, sizeof(int64_t) * b);
        memcpy(keys + b, t, sizeof(int64_t) * b);
        memcpy(keys + 2 * b, neg, sizeof(int64_t) * n_neg);
        ent_ids = malloc(sizeof(int64_t) * n_keys);
        ue = ko_dedup(keys, n_keys, ent_ids, cnt);
        rel_ids = malloc(sizeof(int64_t) * b);
        ur = ko_dedup(r, b, rel_ids, cnt);
        free(keys); free(cnt);
    }
    double *dE = calloc((size_t)ue * p->ent_dim, sizeof(double));
    double *dR = calloc((size_t)ur * p->rel_dim, sizeof(double));
    /* optional report for the tests (touched-rows mode only): ids, gradient rows, sums of |contribution| */
    const int report = !dense && ent_ids_out && dE_out && aE_out && rel_ids_out && dR_out && aR_out;
    if (report) {
        memset(aE_out, 0, sizeof(double) * (size_t)ue * p->ent_dim);
        memset(aR_out, 0, sizeof(double) * (size_t)ur * p->rel_dim);
        if (mE_out && mR_out) {
            memset(mE_out, 0, sizeof(double) * (size_t)ue * p->ent_dim);
            memset(mR_out, 0, sizeof(double) * (size_t)ur * p->rel_dim);
        }
    }
    int rc = (dE && dR) ? 0 : -3;
    if (rc == 0)
        rc = ko_loss_grad(p, E, R, h, r, t, b, neg, k, chunk, NULL, loss_out, pos_score, neg_score, NULL,
                          ent_ids, ue, dE, report ? aE_out : NULL, rel_ids, ur, dR, report ? aR_out : NULL,
                          report ? mE_out : NULL, report ? mR_out : NULL);
    if (rc == 0 && report) {
        memcpy(ent_ids_out, ent_ids, sizeof(int64_t) * ue); *n_ent_out = ue;
        memcpy(rel_ids_out, rel_ids, sizeof(int64_t) * ur); *n_rel_out = ur;
        memcpy(dE_out, dE, sizeof(double) * (size_t)ue * p->ent_dim);
        memcpy(dR_out, dR, sizeof(double) * (size_t)ur * p->rel_dim);
    }
    if (rc == 0) {
        ko_adagrad_rows(E, SE, ent_ids, ue, p->ent_dim, dE, lr, eps, rowwise);
        ko_adagrad_rows(R, SR, rel_ids, ur, p->rel_dim, dR, lr, eps, rowwise);
    }
    free(dE); free(dR); free(ent_ids); free(rel_ids);
    return rc;
}
