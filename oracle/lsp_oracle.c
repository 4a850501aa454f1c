/*
 * CPU oracle for the LSP compress / decompress-apply path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct loops in fp64.  It shares no code, header, table or
 * helper with the HIP library and must never be linked or called by the product path;
 * only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes (this repository's letters: G, W are m x n; r = subspace size;
 * d = nonzeros per projector row; the paper calls the subspace size "d" and the
 * nonzeros per row "r"):
 *
 *   compress          S = P^T G Q             -- Alg. 1, the "Compress on GPU and gradient
 *                                                offload" step; Alg. 3, the step that forms
 *                                                the projected gradient of a layer
 *   decompress-apply  W <- W - P S Q^T        -- Alg. 1, "Decompress, apply deltas on GPU";
 *                                                Alg. 3, the last step of the layer loop
 *   estimation bias   b = ||P P^T G Q Q^T - G||_F / ||G||_F
 *                                             -- Def. 2; the quantity MaybeUpdate in Alg. 1
 *                                                compares with its threshold alpha
 *   state re-projection  M <- (P^T P_prev) M (Q_prev^T Q),
 *                        V <- (P^T P_prev)^2 V (Q_prev^T Q)^2
 *                                             -- last two assignments of MaybeUpdate in Alg. 1:
 *                                                the optimiser's moments follow a change of
 *                                                projectors.  The squares are taken element by
 *                                                element (the second moment of a linear
 *                                                combination of independent terms weights their
 *                                                second moments with the squared coefficients,
 *                                                and V stays non-negative); a matrix square
 *                                                would do neither.
 *
 *   fitting gradient     dF/dP_val, dF/dQ_val for F = 1/2 ||P P^T G Q Q^T - G||_F^2
 *                                             -- the data term of the minimisation in MaybeUpdate
 *                                                (Alg. 1) / Eq. 2, squared and halved; the norm's own
 *                                                gradient is this one over ||b||_F, the regulariser is
 *                                                element-wise in the values and stays with the caller
 *
 * P (m x r) and Q (n x r) are (d,r)-sparse projectors in the sense of Def. 1: exactly d
 * stored entries per row, kept in ELL layout as idx[row][k] (int32 column in [0,r)) and
 * val[row][k] (fp32).  The dense view is  Phat[i][a] = sum over k with idx[i][k]==a of
 * val[i][k]  (duplicate columns in one row add; val == 0 entries are padding).
 * The learning-rate factor of Alg. 1 is taken to be folded into S by the CPU optimiser.
 * The weight expression in Table 2 (P^T S Q) is dimensionally impossible for P in
 * R^{m x r}; Eq. 1 and both algorithms use P S Q^T, which is what is computed here.
 *
 * Two forms are provided:
 *   *_dense   the definition written out literally on densified projectors, O(m n r^2);
 *             for tiny inputs only; it is what the working form is pinned against.
 *   working   associativity only:  T = G Q, S = P^T T;   U = P S, W' = W - U Q^T.
 *
 * Storage types: 0 = fp32, 1 = fp16 (IEEE binary16), 2 = bf16.  Every stored value is
 * widened exactly to fp64; results are produced in fp64 and, for W, additionally rounded
 * ONCE (nearest, ties to even) from fp64 to the storage type.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORA_F32 = 0, ORA_F16 = 1, ORA_BF16 = 2 };

/* ---------------------------------------------------------------- storage <-> fp64 */

static double f16_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);                 /* subnormal: f * 2^-10 * 2^-14 */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(f | 0x400), e - 25);    /* (1024+f) * 2^(e-15-10) */
    }
    return sign ? -v : v;
}

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double load_elem(const void *base, int64_t k, int dtype) {
    switch (dtype) {
        case ORA_F32:  return (double)((const float *)base)[k];
        case ORA_F16:  return f16_bits_to_double(((const uint16_t *)base)[k]);
        default:       return bf16_bits_to_double(((const uint16_t *)base)[k]);
    }
}

/* Round x (fp64) to a binary format with p significand bits (hidden bit included),
 * minimum normal exponent emin, maximum exponent emax; nearest, ties to even; gradual
 * underflow.  The result is returned as an fp64 that is exactly representable in the format
 * (or +-inf on overflow).  rint() rounds ties to even in the default rounding mode. */
static double round_to_format(double x, int p, int emin, int emax) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e = ilogb(x);
    if (e < emin) e = emin;
    double q = ldexp(1.0, e - (p - 1));            /* spacing of the format at this exponent */
    double y = rint(x / q) * q;
    double lim = ldexp(2.0 - ldexp(1.0, -(p - 1)), emax);   /* largest finite value */
    if (fabs(y) > lim) return x > 0 ? INFINITY : -INFINITY;
    return y;
}

static uint16_t double_to_f16_bits(double y) {     /* y must be exactly representable */
    uint16_t sign = signbit(y) ? 0x8000 : 0;
    double a = fabs(y);
    if (isnan(y)) return 0x7E00;
    if (isinf(y)) return sign | 0x7C00;
    if (a == 0.0) return sign;
    int e = ilogb(a);
    if (e < -14) {
        return sign | (uint16_t)llrint(ldexp(a, 24));
    }
    uint32_t mant = (uint32_t)llrint(ldexp(a, 10 - e));      /* in [1024, 2048) */
    return sign | (uint16_t)(((e + 15) << 10) | (mant & 0x3FF));
}

static uint16_t double_to_bf16_bits(double y) {    /* y must be exactly representable */
    float f = (float)y;                            /* exact: bf16 values are fp32 values */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if (isnan(y)) return 0x7FC0;
    return (uint16_t)(u >> 16);
}

static void store_rounded(void *base, int64_t k, int dtype, double x) {
    switch (dtype) {
        case ORA_F32:
            ((float *)base)[k] = (float)x;         /* one IEEE rounding fp64 -> fp32 (RNE) */
            break;
        case ORA_F16:
            ((uint16_t *)base)[k] = double_to_f16_bits(round_to_format(x, 11, -14, 15));
            break;
        default:
            ((uint16_t *)base)[k] = double_to_bf16_bits(round_to_format(x, 8, -126, 127));
            break;
    }
}

/* exposed so the tests can pin the rounding helpers against numpy's own conversions */
double lsp_oracle_round_to_storage(double x, int dtype) {
    if (dtype == ORA_F32) return (double)(float)x;
    if (dtype == ORA_F16) return round_to_format(x, 11, -14, 15);
    return round_to_format(x, 8, -126, 127);
}
double lsp_oracle_widen(const void *base, int64_t k, int dtype) { return load_elem(base, k, dtype); }

/* ---------------------------------------------------------------- definition, literal */

static double *densify(const int32_t *idx, const float *val, int64_t rows, int r, int d) {
    double *D = (double *)calloc((size_t)rows * (size_t)r, sizeof(double));
    if (!D) return NULL;
    for (int64_t i = 0; i < rows; ++i)
        for (int k = 0; k < d; ++k)
            D[i * r + idx[i * d + k]] += (double)val[i * d + k];
    return D;
}

/* S[a][b] = sum_i sum_j Phat[i][a] * G[i][j] * Qhat[j][b]   (compress step, written out) */
int lsp_oracle_compress_dense(const void *G, int dtype,
                              const int32_t *P_idx, const float *P_val,
                              const int32_t *Q_idx, const float *Q_val,
                              int64_t m, int64_t n, int r, int d, double *S) {
    double *Ph = densify(P_idx, P_val, m, r, d);
    double *Qh = densify(Q_idx, Q_val, n, r, d);
    if (!Ph || !Qh) { free(Ph); free(Qh); return -1; }
    for (int a = 0; a < r; ++a)
        for (int b = 0; b < r; ++b) {
            double acc = 0.0;
            for (int64_t i = 0; i < m; ++i)
                for (int64_t j = 0; j < n; ++j)
                    acc += Ph[i * r + a] * load_elem(G, i * n + j, dtype) * Qh[j * r + b];
            S[(int64_t)a * r + b] = acc;
        }
    free(Ph); free(Qh);
    return 0;
}

/* W'[i][j] = W[i][j] - sum_a sum_b Phat[i][a] * S[a][b] * Qhat[j][b]   (decompress-apply) */
int lsp_oracle_decompress_apply_dense(const void *W, int dtype, const float *S,
                                      const int32_t *P_idx, const float *P_val,
                                      const int32_t *Q_idx, const float *Q_val,
                                      int64_t m, int64_t n, int r, int d,
                                      double *Wprime, void *W_out) {
    double *Ph = densify(P_idx, P_val, m, r, d);
    double *Qh = densify(Q_idx, Q_val, n, r, d);
    if (!Ph || !Qh) { free(Ph); free(Qh); return -1; }
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double delta = 0.0;
            for (int a = 0; a < r; ++a)
                for (int b = 0; b < r; ++b)
                    delta += Ph[i * r + a] * (double)S[(int64_t)a * r + b] * Qh[j * r + b];
            double w = load_elem(W, i * n + j, dtype) - delta;
            if (Wprime) Wprime[i * n + j] = w;
            if (W_out) store_rounded(W_out, i * n + j, dtype, w);
        }
    free(Ph); free(Qh);
    return 0;
}

/* Def. 2 written out:  R = (Phat Phat^T) G (Qhat Qhat^T);  out[0] = sum (R - G)^2, out[1] = sum G^2.
 * The two projector products are formed first, as m x m and n x n matrices. */
int lsp_oracle_bias_dense(const void *G, int dtype,
                          const int32_t *P_idx, const float *P_val,
                          const int32_t *Q_idx, const float *Q_val,
                          int64_t m, int64_t n, int r, int d, double *out) {
    double *Ph = densify(P_idx, P_val, m, r, d);
    double *Qh = densify(Q_idx, Q_val, n, r, d);
    double *PP = (double *)calloc((size_t)(m * m), sizeof(double));
    double *QQ = (double *)calloc((size_t)(n * n), sizeof(double));
    double *A  = (double *)calloc((size_t)(m * n), sizeof(double));
    if (!Ph || !Qh || !PP || !QQ || !A) { free(Ph); free(Qh); free(PP); free(QQ); free(A); return -1; }
    for (int64_t i = 0; i < m; ++i)
        for (int64_t i2 = 0; i2 < m; ++i2)
            for (int a = 0; a < r; ++a) PP[i * m + i2] += Ph[i * r + a] * Ph[i2 * r + a];
    for (int64_t j = 0; j < n; ++j)
        for (int64_t j2 = 0; j2 < n; ++j2)
            for (int b = 0; b < r; ++b) QQ[j * n + j2] += Qh[j * r + b] * Qh[j2 * r + b];
    for (int64_t i = 0; i < m; ++i)                 /* A = (P P^T) G */
        for (int64_t j = 0; j < n; ++j)
            for (int64_t i2 = 0; i2 < m; ++i2) A[i * n + j] += PP[i * m + i2] * load_elem(G, i2 * n + j, dtype);
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < m; ++i)                 /* R = A (Q Q^T) */
        for (int64_t j = 0; j < n; ++j) {
            double rij = 0.0;
            for (int64_t j2 = 0; j2 < n; ++j2) rij += A[i * n + j2] * QQ[j2 * n + j];
            double g = load_elem(G, i * n + j, dtype);
            num += (rij - g) * (rij - g);
            den += g * g;
        }
    out[0] = num; out[1] = den;
    free(Ph); free(Qh); free(PP); free(QQ); free(A);
    return 0;
}

/* Optimiser-state re-projection, written out on densified projectors (all r x r, fp64):
 *   A = Phat^T Pprev_hat,  B = Qprev_hat^T Qhat,
 *   M_out = A M B,   V_out = (A o A) V (B o B)   with "o" the element-wise product.
 * M and V are fp32 inputs; M_out and V_out may alias nothing. */
int lsp_oracle_reproject(const int32_t *P_idx, const float *P_val,
                         const int32_t *Pp_idx, const float *Pp_val,
                         const int32_t *Q_idx, const float *Q_val,
                         const int32_t *Qp_idx, const float *Qp_val,
                         int64_t m, int64_t n, int r, int d,
                         const float *M, const float *V, double *M_out, double *V_out) {
    double *Ph = densify(P_idx, P_val, m, r, d), *Pp = densify(Pp_idx, Pp_val, m, r, d);
    double *Qh = densify(Q_idx, Q_val, n, r, d), *Qp = densify(Qp_idx, Qp_val, n, r, d);
    size_t rr = (size_t)r * (size_t)r;
    double *A = (double *)calloc(rr, sizeof(double)), *B = (double *)calloc(rr, sizeof(double));
    double *X = (double *)calloc(rr, sizeof(double)), *Y = (double *)calloc(rr, sizeof(double));
    int rc = -1;
    if (Ph && Pp && Qh && Qp && A && B && X && Y) {
        for (int a = 0; a < r; ++a)
            for (int b = 0; b < r; ++b) {
                double sa = 0.0, sb = 0.0;
                for (int64_t i = 0; i < m; ++i) sa += Ph[i * r + a] * Pp[i * r + b];     /* A = P^T P_prev */
                for (int64_t j = 0; j < n; ++j) sb += Qp[j * r + a] * Qh[j * r + b];     /* B = Q_prev^T Q */
                A[(size_t)a * r + b] = sa; B[(size_t)a * r + b] = sb;
            }
        for (int a = 0; a < r; ++a)
            for (int b = 0; b < r; ++b) {
                double x = 0.0, y = 0.0;
                for (int c = 0; c < r; ++c) {
                    double aac = A[(size_t)a * r + c];
                    x += aac * (double)M[(size_t)c * r + b];
                    y += aac * aac * (double)V[(size_t)c * r + b];
                }
                X[(size_t)a * r + b] = x; Y[(size_t)a * r + b] = y;
            }
        for (int a = 0; a < r; ++a)
            for (int b = 0; b < r; ++b) {
                double x = 0.0, y = 0.0;
                for (int c = 0; c < r; ++c) {
                    double bcb = B[(size_t)c * r + b];
                    x += X[(size_t)a * r + c] * bcb;
                    y += Y[(size_t)a * r + c] * bcb * bcb;
                }
                M_out[(size_t)a * r + b] = x; V_out[(size_t)a * r + b] = y;
            }
        rc = 0;
    }
    free(Ph); free(Pp); free(Qh); free(Qp); free(A); free(B); free(X); free(Y);
    return rc;
}

/* Gradient of the projector-fitting objective's data term with respect to the stored projector values
 * (the minimisation in MaybeUpdate, Alg. 1; Eq. 2):
 *     F(P, Q) = 1/2 || Phat Phat^T G Qhat Qhat^T - G ||_F^2        (half the squared norm of Def. 2's bias),
 *     gP[i][k] = dF / d P_val[i][k],   gQ[j][k] = dF / d Q_val[j][k].
 * A stored value val[i][k] enters Phat only through Phat[i][idx[i][k]] (linearly, duplicates add), so
 * gP[i][k] = dF / d Phat[i][idx[i][k]].  Written out on dense matrices, with A = Phat Phat^T (m x m),
 * B = Qhat Qhat^T (n x n) and R = A G B - G:
 *     dF = <R, dA G B> + <R, A G dB>,   dA = dPhat Phat^T + Phat dPhat^T,   dB likewise,
 * hence   dF/dPhat = (X + X^T) Phat  with X = R B G^T  (m x m),
 *         dF/dQhat = (Y + Y^T) Qhat  with Y = G^T A R  (n x n).
 * The paper's objective is ||b||_F + beta * regulariser; its data term is sqrt(2 F), whose gradient is
 * this one divided by ||b||_F, and the regulariser (whose exponents differ between Alg. 1 and Eq. 2) is an
 * element-wise function of the values: neither is part of this routine.  Tiny inputs only: O(m n (m + n)). */
int lsp_oracle_bias_grad_dense(const void *G, int dtype,
                               const int32_t *P_idx, const float *P_val,
                               const int32_t *Q_idx, const float *Q_val,
                               int64_t m, int64_t n, int r, int d, double *gP, double *gQ) {
    double *Ph = densify(P_idx, P_val, m, r, d);
    double *Qh = densify(Q_idx, Q_val, n, r, d);
    double *A  = (double *)calloc((size_t)(m * m), sizeof(double));
    double *B  = (double *)calloc((size_t)(n * n), sizeof(double));
    double *Gd = (double *)calloc((size_t)(m * n), sizeof(double));
    double *AG = (double *)calloc((size_t)(m * n), sizeof(double));      /* A G   */
    double *GB = (double *)calloc((size_t)(m * n), sizeof(double));      /* G B   */
    double *R  = (double *)calloc((size_t)(m * n), sizeof(double));      /* A G B - G */
    double *X  = (double *)calloc((size_t)(m * m), sizeof(double));      /* R (G B)^T */
    double *Y  = (double *)calloc((size_t)(n * n), sizeof(double));      /* (A G)^T R */
    int rc = -1;
    if (Ph && Qh && A && B && Gd && AG && GB && R && X && Y) {
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) Gd[i * n + j] = load_elem(G, i * n + j, dtype);
        for (int64_t i = 0; i < m; ++i)
            for (int64_t i2 = 0; i2 < m; ++i2)
                for (int a = 0; a < r; ++a) A[i * m + i2] += Ph[i * r + a] * Ph[i2 * r + a];
        for (int64_t j = 0; j < n; ++j)
            for (int64_t j2 = 0; j2 < n; ++j2)
                for (int b = 0; b < r; ++b) B[j * n + j2] += Qh[j * r + b] * Qh[j2 * r + b];
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                double ag = 0.0, gb = 0.0;
                for (int64_t i2 = 0; i2 < m; ++i2) ag += A[i * m + i2] * Gd[i2 * n + j];
                for (int64_t j2 = 0; j2 < n; ++j2) gb += Gd[i * n + j2] * B[j2 * n + j];
                AG[i * n + j] = ag; GB[i * n + j] = gb;
            }
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                double x = 0.0;
                for (int64_t j2 = 0; j2 < n; ++j2) x += AG[i * n + j2] * B[j2 * n + j];
                R[i * n + j] = x - Gd[i * n + j];
            }
        for (int64_t i = 0; i < m; ++i)
            for (int64_t i2 = 0; i2 < m; ++i2) {
                double x = 0.0;
                for (int64_t j = 0; j < n; ++j) x += R[i * n + j] * GB[i2 * n + j];
                X[i * m + i2] = x;
            }
        for (int64_t j = 0; j < n; ++j)
            for (int64_t j2 = 0; j2 < n; ++j2) {
                double y = 0.0;
                for (int64_t i = 0; i < m; ++i) y += AG[i * n + j] * R[i * n + j2];
                Y[j * n + j2] = y;
            }
        for (int64_t i = 0; i < m; ++i)
            for (int k = 0; k < d; ++k) {
                const int a = P_idx[i * d + k];
                double g = 0.0;
                for (int64_t i2 = 0; i2 < m; ++i2) g += (X[i * m + i2] + X[i2 * m + i]) * Ph[i2 * r + a];
                gP[i * d + k] = g;
            }
        for (int64_t j = 0; j < n; ++j)
            for (int k = 0; k < d; ++k) {
                const int b = Q_idx[j * d + k];
                double g = 0.0;
                for (int64_t j2 = 0; j2 < n; ++j2) g += (Y[j * n + j2] + Y[j2 * n + j]) * Qh[j2 * r + b];
                gQ[j * d + k] = g;
            }
        rc = 0;
    }
    free(Ph); free(Qh); free(A); free(B); free(Gd); free(AG); free(GB); free(R); free(X); free(Y);
    return rc;
}

/* ---------------------------------------------------------------- working form */

/* rows [i0, i1) of the compress sum, accumulated into S (which the caller zeroed).
 * Trow is scratch of r doubles.   T[i][:] = G[i][:] Q ;   S += P[i][:]^T T[i][:] */
static void compress_rows(const void *G, int dtype,
                          const int32_t *P_idx, const float *P_val,
                          const int32_t *Q_idx, const float *Q_val,
                          int64_t i0, int64_t i1, int64_t n, int r, int d,
                          double *Trow, double *S) {
    for (int64_t i = i0; i < i1; ++i) {
        for (int b = 0; b < r; ++b) Trow[b] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            double g = load_elem(G, i * n + j, dtype);
            for (int k = 0; k < d; ++k)
                Trow[Q_idx[j * d + k]] += g * (double)Q_val[j * d + k];
        }
        for (int k = 0; k < d; ++k) {
            double pv = (double)P_val[i * d + k];
            double *Srow = S + (int64_t)P_idx[i * d + k] * r;
            for (int b = 0; b < r; ++b) Srow[b] += pv * Trow[b];
        }
    }
}

/* S (r x r, fp64, overwritten) = P^T G Q */
int lsp_oracle_compress(const void *G, int dtype,
                        const int32_t *P_idx, const float *P_val,
                        const int32_t *Q_idx, const float *Q_val,
                        int64_t m, int64_t n, int r, int d, double *S) {
    double *Trow = (double *)malloc((size_t)r * sizeof(double));
    if (!Trow) return -1;
    memset(S, 0, (size_t)r * (size_t)r * sizeof(double));
    compress_rows(G, dtype, P_idx, P_val, Q_idx, Q_val, 0, m, n, r, d, Trow, S);
    free(Trow);
    return 0;
}

/* rows [i0, i1):  U[i][:] = P[i][:] S ;  W'[i][j] = W[i][j] - sum_k U[i][Q_idx[j][k]] Q_val[j][k] */
static void decompress_rows(const void *W, int dtype, const float *S,
                            const int32_t *P_idx, const float *P_val,
                            const int32_t *Q_idx, const float *Q_val,
                            int64_t i0, int64_t i1, int64_t n, int r, int d,
                            double *Urow, double *Wprime, void *W_out) {
    for (int64_t i = i0; i < i1; ++i) {
        for (int b = 0; b < r; ++b) Urow[b] = 0.0;
        for (int k = 0; k < d; ++k) {
            double pv = (double)P_val[i * d + k];
            const float *Srow = S + (int64_t)P_idx[i * d + k] * r;
            for (int b = 0; b < r; ++b) Urow[b] += pv * (double)Srow[b];
        }
        for (int64_t j = 0; j < n; ++j) {
            double delta = 0.0;
            for (int k = 0; k < d; ++k)
                delta += Urow[Q_idx[j * d + k]] * (double)Q_val[j * d + k];
            double w = load_elem(W, i * n + j, dtype) - delta;
            if (Wprime) Wprime[i * n + j] = w;
            if (W_out) store_rounded(W_out, i * n + j, dtype, w);
        }
    }
}

/* W' = W - P S Q^T.  Wprime (fp64, m x n) and/or W_out (storage type, m x n) may be NULL.
 * W itself is not modified. */
int lsp_oracle_decompress_apply(const void *W, int dtype, const float *S,
                                const int32_t *P_idx, const float *P_val,
                                const int32_t *Q_idx, const float *Q_val,
                                int64_t m, int64_t n, int r, int d,
                                double *Wprime, void *W_out) {
    double *Urow = (double *)malloc((size_t)r * sizeof(double));
    if (!Urow) return -1;
    decompress_rows(W, dtype, S, P_idx, P_val, Q_idx, Q_val, 0, m, n, r, d, Urow, Wprime, W_out);
    free(Urow);
    return 0;
}

/* Def. 2 by associativity:  S = P^T G Q (fp64, not rounded), then row by row U = P S,
 * R[i][j] = sum_k U[i][Q_idx[j][k]] Q_val[j][k];  out[0] = sum (R - G)^2, out[1] = sum G^2. */
int lsp_oracle_bias(const void *G, int dtype,
                    const int32_t *P_idx, const float *P_val,
                    const int32_t *Q_idx, const float *Q_val,
                    int64_t m, int64_t n, int r, int d, double *out) {
    double *S = (double *)malloc((size_t)r * (size_t)r * sizeof(double));
    double *row = (double *)malloc((size_t)r * sizeof(double));
    if (!S || !row) { free(S); free(row); return -1; }
    memset(S, 0, (size_t)r * (size_t)r * sizeof(double));
    compress_rows(G, dtype, P_idx, P_val, Q_idx, Q_val, 0, m, n, r, d, row, S);
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < m; ++i) {
        for (int b = 0; b < r; ++b) row[b] = 0.0;
        for (int k = 0; k < d; ++k) {
            double pv = (double)P_val[i * d + k];
            const double *Srow = S + (int64_t)P_idx[i * d + k] * r;
            for (int b = 0; b < r; ++b) row[b] += pv * Srow[b];
        }
        for (int64_t j = 0; j < n; ++j) {
            double rij = 0.0;
            for (int k = 0; k < d; ++k) rij += row[Q_idx[j * d + k]] * (double)Q_val[j * d + k];
            double g = load_elem(G, i * n + j, dtype);
            num += (rij - g) * (rij - g);
            den += g * g;
        }
    }
    out[0] = num; out[1] = den;
    free(S); free(row);
    return 0;
}

/* The same gradient by associativity, with sparse loops only (no m x m or n x n matrix):
 *     S = P^T G Q,   R = P S Q^T - G  (row by row),
 *     T_G = G Q,  T_R = R Q  (m x r);   Y_G = G^T P,  Y_R = R^T P  (n x r);   Z = P^T R Q = P^T T_R,
 *     dF/dPhat = T_R S^T + T_G Z^T,      dF/dQhat = Y_R S + Y_G Z,
 * read off at the stored positions.  (From the dense statement: X Phat = R B G^T Phat = (R Q)(Q^T G^T P) = T_R S^T and
 * X^T Phat = G B R^T Phat = (G Q)(Q^T R^T P) = T_G Z^T; the Q side is the mirror image.)
 * O(m n d + (m + n) d r) operations, fp64 throughout. */
int lsp_oracle_bias_grad(const void *G, int dtype,
                         const int32_t *P_idx, const float *P_val,
                         const int32_t *Q_idx, const float *Q_val,
                         int64_t m, int64_t n, int r, int d, double *gP, double *gQ) {
    const size_t rr = (size_t)r * (size_t)r;
    double *S  = (double *)calloc(rr, sizeof(double));
    double *Z  = (double *)calloc(rr, sizeof(double));
    double *TG = (double *)calloc((size_t)m * (size_t)r, sizeof(double));
    double *TR = (double *)calloc((size_t)m * (size_t)r, sizeof(double));
    double *YG = (double *)calloc((size_t)n * (size_t)r, sizeof(double));
    double *YR = (double *)calloc((size_t)n * (size_t)r, sizeof(double));
    double *row = (double *)malloc((size_t)r * sizeof(double));
    int rc = -1;
    if (S && Z && TG && TR && YG && YR && row) {
        compress_rows(G, dtype, P_idx, P_val, Q_idx, Q_val, 0, m, n, r, d, row, S);
        for (int64_t i = 0; i < m; ++i) {
            for (int b = 0; b < r; ++b) row[b] = 0.0;                     /* row i of U = P S */
            for (int k = 0; k < d; ++k) {
                const double pv = (double)P_val[i * d + k];
                const double *Srow = S + (int64_t)P_idx[i * d + k] * r;
                for (int b = 0; b < r; ++b) row[b] += pv * Srow[b];
            }
            for (int64_t j = 0; j < n; ++j) {
                double rij = 0.0;
                for (int k = 0; k < d; ++k) rij += row[Q_idx[j * d + k]] * (double)Q_val[j * d + k];
                const double g = load_elem(G, i * n + j, dtype);
                rij -= g;                                                 /* R[i][j] */
                for (int k = 0; k < d; ++k) {
                    const double qv = (double)Q_val[j * d + k];
                    TG[i * r + Q_idx[j * d + k]] += g * qv;
                    TR[i * r + Q_idx[j * d + k]] += rij * qv;
                }
                for (int k = 0; k < d; ++k) {
                    const double pv = (double)P_val[i * d + k];
                    YG[j * r + P_idx[i * d + k]] += g * pv;
                    YR[j * r + P_idx[i * d + k]] += rij * pv;
                }
            }
        }
        for (int64_t i = 0; i < m; ++i)                                   /* Z = P^T T_R */
            for (int k = 0; k < d; ++k) {
                const double pv = (double)P_val[i * d + k];
                double *Zrow = Z + (int64_t)P_idx[i * d + k] * r;
                for (int b = 0; b < r; ++b) Zrow[b] += pv * TR[i * r + b];
            }
        for (int64_t i = 0; i < m; ++i)
            for (int k = 0; k < d; ++k) {
                const int a = P_idx[i * d + k];
                double g = 0.0;
                for (int b = 0; b < r; ++b) g += TR[i * r + b] * S[(int64_t)a * r + b] + TG[i * r + b] * Z[(int64_t)a * r + b];
                gP[i * d + k] = g;
            }
        for (int64_t j = 0; j < n; ++j)
            for (int k = 0; k < d; ++k) {
                const int b = Q_idx[j * d + k];
                double g = 0.0;
                for (int a = 0; a < r; ++a) g += YR[j * r + a] * S[(int64_t)a * r + b] + YG[j * r + a] * Z[(int64_t)a * r + b];
                gQ[j * d + k] = g;
            }
        rc = 0;
    }
    free(S); free(Z); free(TG); free(TR); free(YG); free(YR); free(row);
    return rc;
}

/* Selected rows only (for sampled checks at sizes where all m rows would take too long):
 * out[t][j] = W'[rows[t]][j], fp64, nrows x n. */
int lsp_oracle_decompress_rows(const void *W, int dtype, const float *S,
                               const int32_t *P_idx, const float *P_val,
                               const int32_t *Q_idx, const float *Q_val,
                               int64_t m, int64_t n, int r, int d,
                               const int64_t *rows, int64_t nrows, double *out) {
    double *Urow = (double *)malloc((size_t)r * sizeof(double));
    if (!Urow) return -1;
    for (int64_t t = 0; t < nrows; ++t) {
        int64_t i = rows[t];
        if (i < 0 || i >= m) { free(Urow); return -2; }
        for (int b = 0; b < r; ++b) Urow[b] = 0.0;
        for (int k = 0; k < d; ++k) {
            double pv = (double)P_val[i * d + k];
            const float *Srow = S + (int64_t)P_idx[i * d + k] * r;
            for (int b = 0; b < r; ++b) Urow[b] += pv * (double)Srow[b];
        }
        for (int64_t j = 0; j < n; ++j) {
            double delta = 0.0;
            for (int k = 0; k < d; ++k)
                delta += Urow[Q_idx[j * d + k]] * (double)Q_val[j * d + k];
            out[t * n + j] = load_elem(W, i * n + j, dtype) - delta;
        }
    }
    free(Urow);
    return 0;
}

/* Selected entries of S only:  out[t] = S[a_t][b_t], by the definition restricted to the
 * rows of P that touch a_t and the rows of Q that touch b_t (no intermediate T). */
int lsp_oracle_compress_entries(const void *G, int dtype,
                                const int32_t *P_idx, const float *P_val,
                                const int32_t *Q_idx, const float *Q_val,
                                int64_t m, int64_t n, int r, int d,
                                const int32_t *ea, const int32_t *eb, int64_t nent, double *out) {
    (void)r;
    for (int64_t t = 0; t < nent; ++t) {
        int a = ea[t], b = eb[t];
        double acc = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            double pa = 0.0;
            for (int k = 0; k < d; ++k)
                if (P_idx[i * d + k] == a) pa += (double)P_val[i * d + k];
            if (pa == 0.0) continue;
            double rowsum = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                double qb = 0.0;
                for (int k = 0; k < d; ++k)
                    if (Q_idx[j * d + k] == b) qb += (double)Q_val[j * d + k];
                if (qb != 0.0) rowsum += load_elem(G, i * n + j, dtype) * qb;
            }
            acc += pa * rowsum;
        }
        out[t] = acc;
    }
    return 0;
}

/* ---------------------------------------------------------------- same loops, rows split over threads
 *
 * Used only to time the oracle on all host cores.  The arithmetic is the working form above,
 * unchanged: compress gives each thread a private S over a contiguous row range and adds the
 * private copies at the end; decompress gives each thread a disjoint row range. */
#include <pthread.h>

typedef struct {
    const void *X; int dtype; const float *S_in;
    const int32_t *P_idx; const float *P_val; const int32_t *Q_idx; const float *Q_val;
    int64_t i0, i1, n; int r, d;
    double *S_priv; double *Wprime; void *W_out; int rc;
} ora_job;

static void *compress_worker(void *arg) {
    ora_job *j = (ora_job *)arg;
    double *Trow = (double *)malloc((size_t)j->r * sizeof(double));
    if (!Trow) { j->rc = -1; return NULL; }
    compress_rows(j->X, j->dtype, j->P_idx, j->P_val, j->Q_idx, j->Q_val,
                  j->i0, j->i1, j->n, j->r, j->d, Trow, j->S_priv);
    free(Trow);
    j->rc = 0;
    return NULL;
}

static void *decompress_worker(void *arg) {
    ora_job *j = (ora_job *)arg;
    double *Urow = (double *)malloc((size_t)j->r * sizeof(double));
    if (!Urow) { j->rc = -1; return NULL; }
    decompress_rows(j->X, j->dtype, j->S_in, j->P_idx, j->P_val, j->Q_idx, j->Q_val,
                    j->i0, j->i1, j->n, j->r, j->d, Urow, j->Wprime, j->W_out);
    free(Urow);
    j->rc = 0;
    return NULL;
}

int lsp_oracle_compress_mt(const void *G, int dtype,
                           const int32_t *P_idx, const float *P_val,
                           const int32_t *Q_idx, const float *Q_val,
                           int64_t m, int64_t n, int r, int d, double *S, int nthreads) {
    if (nthreads < 1) nthreads = 1;
    if (nthreads > m) nthreads = (int)m;
    size_t rr = (size_t)r * (size_t)r;
    double *priv = (double *)calloc(rr * (size_t)nthreads, sizeof(double));
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    ora_job *jobs = (ora_job *)calloc((size_t)nthreads, sizeof(ora_job));
    if (!priv || !th || !jobs) { free(priv); free(th); free(jobs); return -1; }
    for (int t = 0; t < nthreads; ++t) {
        ora_job *j = &jobs[t];
        j->X = G; j->dtype = dtype; j->P_idx = P_idx; j->P_val = P_val; j->Q_idx = Q_idx; j->Q_val = Q_val;
        j->i0 = m * t / nthreads; j->i1 = m * (t + 1) / nthreads; j->n = n; j->r = r; j->d = d;
        j->S_priv = priv + rr * (size_t)t;
        pthread_create(&th[t], NULL, compress_worker, j);
    }
    int rc = 0;
    for (int t = 0; t < nthreads; ++t) { pthread_join(th[t], NULL); if (jobs[t].rc) rc = jobs[t].rc; }
    memset(S, 0, rr * sizeof(double));
    for (int t = 0; t < nthreads; ++t)
        for (size_t k = 0; k < rr; ++k) S[k] += priv[rr * (size_t)t + k];
    free(priv); free(th); free(jobs);
    return rc;
}

int lsp_oracle_decompress_apply_mt(const void *W, int dtype, const float *S,
                                   const int32_t *P_idx, const float *P_val,
                                   const int32_t *Q_idx, const float *Q_val,
                                   int64_t m, int64_t n, int r, int d,
                                   double *Wprime, void *W_out, int nthreads) {
    if (nthreads < 1) nthreads = 1;
    if (nthreads > m) nthreads = (int)m;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    ora_job *jobs = (ora_job *)calloc((size_t)nthreads, sizeof(ora_job));
    if (!th || !jobs) { free(th); free(jobs); return -1; }
    for (int t = 0; t < nthreads; ++t) {
        ora_job *j = &jobs[t];
        j->X = W; j->dtype = dtype; j->S_in = S;
        j->P_idx = P_idx; j->P_val = P_val; j->Q_idx = Q_idx; j->Q_val = Q_val;
        j->i0 = m * t / nthreads; j->i1 = m * (t + 1) / nthreads; j->n = n; j->r = r; j->d = d;
        j->Wprime = Wprime; j->W_out = W_out;
        pthread_create(&th[t], NULL, decompress_worker, j);
    }
    int rc = 0;
    for (int t = 0; t < nthreads; ++t) { pthread_join(th[t], NULL); if (jobs[t].rc) rc = jobs[t].rc; }
    free(th); free(jobs);
    return rc;
}
