/*
 * TEST INFRASTRUCTURE -- the CPU oracle for the structure2vec / deep-Q hot path.
 *
 * A plain, slow, float64 evaluation of what the method defines, written from the
 * paper (OpenGraphGym-MG, arXiv 2105.08764).  It exists to check the HIP library;
 * it shares no code with it and the product never calls it.  Only tests, the
 * smoke check and the bench's cpu_baseline leg may load this file.
 *
 * Parameter names use the structure2vec numbering of the library's interface.
 * The paper renumbers them; the correspondence is
 *     here    theta1 theta2 theta3 theta4 theta5 theta6 theta7
 *     paper   theta1 theta4 theta3 theta2 theta7 theta5 theta6
 * Matrices are row-major [out][in] and act on column vectors (y = theta * v).
 *
 * There is no blocking, fusion or algebraic shortcut: the embedding update of
 * Eq. (1) is evaluated edge by edge every round (including the edge-weight term,
 * which does not change between rounds), starting from a zero embedding as
 * Alg. 1 states.  OpenMP "parallel for" over nodes is the only parallelism.
 *
 * Pins (tests/test_oracle_*.py): edgeless and one-round closed forms, regular and
 * two-orbit graph recurrences, dense-adjacency brute force, the clip-free linear
 * regime against explicit matrix powers, permutation equivariance, batch ==
 * single graphs, selection against a lexicographic sort, gradients against
 * central finite differences.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double relu(double v) { return v > 0.0 ? v : 0.0; }

/* Whether a relu unit with pre-activation z passes its input.  d < 0: the definition (z > 0).
 * d = 0 / 1: the caller decides (oracle_loss_grad_decided: a float32 evaluation cannot tell the sign of
 * a pre-activation that lies within its own rounding of zero; a test may then ask for the gradient of
 * the branch that evaluation took). */
static inline int decided(double z, int d) { return d < 0 ? (z > 0.0) : (d != 0); }

/* y[p] = M[p][p] * v[p] */
static void matvec(int p, const double *M, const double *v, double *y) {
    for (int i = 0; i < p; ++i) {
        double acc = 0.0;
        for (int j = 0; j < p; ++j) acc += M[(size_t)i * p + j] * v[j];
        y[i] = acc;
    }
}

/* y[p] = M[p][p]^T * v[p] */
static void matvec_t(int p, const double *M, const double *v, double *y) {
    for (int j = 0; j < p; ++j) y[j] = 0.0;
    for (int i = 0; i < p; ++i)
        for (int j = 0; j < p; ++j) y[j] += M[(size_t)i * p + j] * v[i];
}

/*
 * One round of Eq. (1) for every node:
 *   mu_next[v] = relu(theta1 * x_v + theta2 * sum_{u in N(v)} mu[u]
 *                     + theta3 * sum_{u in N(v)} relu(theta4 * w(v,u)))
 * N(v) is exactly the stored entries of CSR row v.  w == NULL means all weights 1.
 * weighted != 0 takes the other reading of the aggregation step of Alg. 1 (a product with the
 * adjacency matrix that holds the weights): the second term becomes
 *   theta2 * sum_{u in N(v)} w(v,u) * mu[u].
 * If a_out / e_out are non-NULL the two neighbour sums are also stored ([n][p]).
 * force (NULL: none) holds one decision per unit, see decided(); on_out receives the decisions taken,
 * z_out the pre-activations and zs_out the summed magnitudes of their terms (each [n][p], optional).
 */
static void embed_round(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w, int weighted, int p,
                        const double *th1, const double *th2, const double *th3, const double *th4,
                        const double *x, const double *mu, double *mu_next, double *a_out, double *e_out,
                        const int8_t *force, uint8_t *on_out, double *z_out, double *zs_out) {
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * 4 * (size_t)p);
        double *e = a + p, *t2 = e + p, *t3 = t2 + p;
#pragma omp for schedule(dynamic, 256)
        for (int32_t v = 0; v < n; ++v) {
            for (int i = 0; i < p; ++i) { a[i] = 0.0; e[i] = 0.0; }
            for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
                const double *mu_u = mu + (size_t)colidx[j] * p;
                double wj = w ? w[j] : 1.0;
                double cj = weighted ? wj : 1.0;
                for (int i = 0; i < p; ++i) {
                    a[i] += cj * mu_u[i];
                    e[i] += relu(th4[i] * wj);
                }
            }
            matvec(p, th2, a, t2);
            matvec(p, th3, e, t3);
            for (int i = 0; i < p; ++i) {
                const double z = th1[i] * x[v] + t2[i] + t3[i];
                const int on = decided(z, force ? force[(size_t)v * p + i] : -1);
                mu_next[(size_t)v * p + i] = on ? z : 0.0;
                if (on_out) on_out[(size_t)v * p + i] = (uint8_t)on;
                if (z_out) z_out[(size_t)v * p + i] = z;
                if (zs_out) {
                    /* magnitude of what was summed into z: |theta1 x| + sum_j |theta2_ij a_j| + sum_j |theta3_ij e_j| */
                    double s = fabs(th1[i] * x[v]);
                    for (int j = 0; j < p; ++j) s += fabs(th2[(size_t)i * p + j] * a[j]) + fabs(th3[(size_t)i * p + j] * e[j]);
                    zs_out[(size_t)v * p + i] = s;
                }
            }
            if (a_out) memcpy(a_out + (size_t)v * p, a, sizeof(double) * p);
            if (e_out) memcpy(e_out + (size_t)v * p, e, sizeof(double) * p);
        }
        free(a);
    }
}

/*
 * Alg. 1 / Eq. (1): T rounds from mu^0 = 0.  mu_out is [n][p].  If mu_hist is
 * non-NULL it receives mu^1..mu^T as [T][n][p].
 */
int oracle_embed(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w, int32_t weighted,
                 int32_t p, int32_t T,
                 const double *th1, const double *th2, const double *th3, const double *th4, const double *x,
                 double *mu_out, double *mu_hist) {
    size_t np_ = (size_t)n * p;
    double *cur = (double *)calloc(np_ ? np_ : 1, sizeof(double));
    double *nxt = (double *)calloc(np_ ? np_ : 1, sizeof(double));
    if (!cur || !nxt) { free(cur); free(nxt); return -1; }
    for (int t = 0; t < T; ++t) {
        embed_round(n, rowptr, colidx, w, weighted, p, th1, th2, th3, th4, x, cur, nxt, NULL, NULL, NULL, NULL, NULL,
                    NULL);
        if (mu_hist) memcpy(mu_hist + (size_t)t * np_, nxt, sizeof(double) * np_);
        double *tmp = cur; cur = nxt; nxt = tmp;
    }
    memcpy(mu_out, cur, sizeof(double) * np_);
    free(cur); free(nxt);
    return 0;
}

/*
 * Eq. (2) / Alg. 2 for every node of every graph of a block-diagonal batch:
 *   g_b  = sum over ALL nodes of graph b of mu[v]
 *   Q_v  = theta5[0:p] . relu(theta6 * g_b) + theta5[p:2p] . relu(theta7 * mu[v])
 * graph_off is [G+1] node offsets (NULL when G == 1).  gsum_out is [G][p], q_out [n].
 */
int oracle_q(int32_t n, int32_t G, const int32_t *graph_off, int32_t p, const double *th5, const double *th6,
             const double *th7, const double *mu, double *gsum_out, double *q_out) {
    int32_t one[2] = {0, n};
    if (!graph_off) { graph_off = one; G = 1; }
    double *h = (double *)malloc(sizeof(double) * 2 * (size_t)p);
    for (int32_t b = 0; b < G; ++b) {
        double *g = gsum_out + (size_t)b * p;
        for (int i = 0; i < p; ++i) g[i] = 0.0;
        for (int32_t v = graph_off[b]; v < graph_off[b + 1]; ++v)
            for (int i = 0; i < p; ++i) g[i] += mu[(size_t)v * p + i];
        matvec(p, th6, g, h);
        double qa = 0.0;
        for (int i = 0; i < p; ++i) qa += th5[i] * relu(h[i]);
        for (int32_t v = graph_off[b]; v < graph_off[b + 1]; ++v) {
            matvec(p, th7, mu + (size_t)v * p, h + p);
            double qb = 0.0;
            for (int i = 0; i < p; ++i) qb += th5[p + i] * relu(h[p + i]);
            q_out[v] = qa + qb;
        }
    }
    free(h);
    return 0;
}

/*
 * Node selection (Alg. 3's argmax, and the top-d rule of Sec. 4.5.1 for k > 1).
 * Candidates are cand[v] != 0 when cand is given, else the nodes with x[v] == 0.
 * Per graph: candidates ordered by score descending, node index ascending on equal
 * scores; the first k are written.  idx_out/val_out are [G][k]; unused slots hold
 * -1 / -inf; count_out[b] = min(k, number of candidates of graph b).
 */
typedef struct { double q; int32_t v; } scored;
static int by_score_then_index(const void *a, const void *b) {
    const scored *sa = (const scored *)a, *sb = (const scored *)b;
    if (sa->q > sb->q) return -1;
    if (sa->q < sb->q) return 1;
    return (sa->v > sb->v) - (sa->v < sb->v);
}

int oracle_select(int32_t n, int32_t G, const int32_t *graph_off, const double *q, const double *x,
                  const uint8_t *cand, int32_t k, int32_t *idx_out, double *val_out, int32_t *count_out) {
    int32_t one[2] = {0, n};
    if (!graph_off) { graph_off = one; G = 1; }
    for (int32_t b = 0; b < G; ++b) {
        int32_t lo = graph_off[b], hi = graph_off[b + 1];
        scored *c = (scored *)malloc(sizeof(scored) * (size_t)(hi - lo + 1));
        int32_t m = 0;
        for (int32_t v = lo; v < hi; ++v) {
            int is_c = cand ? (cand[v] != 0) : (x[v] == 0.0);
            if (is_c) { c[m].q = q[v]; c[m].v = v; ++m; }
        }
        qsort(c, (size_t)m, sizeof(scored), by_score_then_index);
        int32_t take = m < k ? m : k;
        for (int32_t i = 0; i < k; ++i) {
            idx_out[(size_t)b * k + i] = i < take ? c[i].v : -1;
            val_out[(size_t)b * k + i] = i < take ? c[i].q : -INFINITY;
        }
        count_out[b] = take;
        free(c);
    }
    return 0;
}

/* Transpose of a CSR matrix by counting sort; the values w (NULL: none) follow their entries into
 * w_t.  No symmetry is assumed. */
static void csr_transpose(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w,
                          int32_t *rowptr_t, int32_t *colidx_t, double *w_t) {
    int32_t nnz = rowptr[n];
    for (int32_t v = 0; v <= n; ++v) rowptr_t[v] = 0;
    for (int32_t j = 0; j < nnz; ++j) rowptr_t[colidx[j] + 1]++;
    for (int32_t v = 0; v < n; ++v) rowptr_t[v + 1] += rowptr_t[v];
    int32_t *fill = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    memcpy(fill, rowptr_t, sizeof(int32_t) * (size_t)(n + 1));
    for (int32_t v = 0; v < n; ++v)
        for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
            int32_t at = fill[colidx[j]]++;
            colidx_t[at] = v;
            if (w && w_t) w_t[at] = w[j];
        }
    free(fill);
}

/*
 * Training loss and its gradient (the Train step of Alg. 4: forward = Alg. 1 then
 * Alg. 2, then back-propagation), for a minibatch of S states on one graph batch:
 *   L = (1/S) * sum_b (Q^{(b)}(action_b) - target_b)^2
 * with Q^{(b)} computed from x[b][.] by T rounds of Eq. (1) and Eq. (2).
 * Gradients are taken by reverse-mode differentiation of exactly those formulas;
 * relu'(0) = 0.  The adjoint of the neighbour sum uses the explicit transpose of
 * the CSR matrix (with its weights when weighted != 0, see embed_round).  States are
 * processed one at a time.
 * Outputs: loss_out[1], q_out[S] (the predicted Q of each action), and d1..d7 with
 * the shapes of theta1..theta7 (overwritten).
 */
static int loss_grad_impl(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w, int32_t weighted,
                          int32_t G,
                          const int32_t *graph_off, int32_t p, int32_t T, const double *th1, const double *th2,
                          const double *th3, const double *th4, const double *th5, const double *th6,
                          const double *th7, int32_t S, const double *x, const int32_t *action,
                          const double *target, double *loss_out, double *q_out, double *d1, double *d2,
                          double *d3, double *d4, double *d5, double *d6, double *d7,
                          const int8_t *force /*[S][T][n][p]*/, const int8_t *force_head /*[S][2][p]*/,
                          double *z_out /*[S][T][n][p]*/, double *zs_out /*[S][T][n][p]*/,
                          double *h_out /*[S][2][p]*/, double *hs_out /*[S][2][p]*/) {
    int32_t one[2] = {0, n};
    if (!graph_off) { graph_off = one; G = 1; }
    size_t np_ = (size_t)n * p, pp = (size_t)p * p;
    int32_t nnz = rowptr[n];
    memset(d1, 0, sizeof(double) * p); memset(d4, 0, sizeof(double) * p);
    memset(d5, 0, sizeof(double) * 2 * p);
    memset(d2, 0, sizeof(double) * pp); memset(d3, 0, sizeof(double) * pp);
    memset(d6, 0, sizeof(double) * pp); memset(d7, 0, sizeof(double) * pp);

    int32_t *rowptr_t = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int32_t *colidx_t = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
    if (!w) weighted = 0; /* all weights 1: both readings coincide */
    double *w_t = weighted ? (double *)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1)) : NULL;
    csr_transpose(n, rowptr, colidx, w, rowptr_t, colidx_t, w_t);

    /* mu[t] for t = 0..T, the two neighbour sums of the round that produced mu[t] */
    double *mu = (double *)calloc((size_t)(T + 1) * np_ + 1, sizeof(double));
    double *asum = (double *)malloc(sizeof(double) * ((size_t)(T + 1) * np_ + 1));
    double *esum = (double *)malloc(sizeof(double) * (np_ + 1));
    double *dmu = (double *)malloc(sizeof(double) * (np_ + 1));
    double *da = (double *)malloc(sizeof(double) * (np_ + 1));
    /* the decision of every relu unit of rounds 1..T (index t * n * p as for mu) */
    uint8_t *on = (uint8_t *)malloc((size_t)(T + 1) * np_ + 1);
    double *vec = (double *)malloc(sizeof(double) * 8 * (size_t)p);
    double *g = vec, *h1 = g + p, *h2 = h1 + p, *dh1 = h2 + p, *dh2 = dh1 + p, *dg = dh2 + p, *tmp = dg + p;
    if (!mu || !asum || !esum || !dmu || !da || !vec || !on || !rowptr_t || !colidx_t) return -1;

    double loss = 0.0;
    for (int32_t b = 0; b < S; ++b) {
        const double *xb = x + (size_t)b * n;
        memset(mu, 0, sizeof(double) * np_);
        for (int t = 1; t <= T; ++t) {
            const size_t at = ((size_t)b * T + (size_t)(t - 1)) * np_;   /* this (state, round) in the optional arrays */
            embed_round(n, rowptr, colidx, w, weighted, p, th1, th2, th3, th4, xb, mu + (size_t)(t - 1) * np_,
                        mu + (size_t)t * np_, asum + (size_t)t * np_, esum, force ? force + at : NULL,
                        on + (size_t)t * np_, z_out ? z_out + at : NULL, zs_out ? zs_out + at : NULL);
        }
        const double *muT = mu + (size_t)T * np_;
        int32_t act = action[b];
        int32_t gb = 0;
        if (act < 0 || act >= n) return -2;
        while (gb < G - 1 && act >= graph_off[gb + 1]) ++gb;
        int32_t lo = graph_off[gb], hi = graph_off[gb + 1];

        /* Eq. (2) at the action node */
        for (int i = 0; i < p; ++i) g[i] = 0.0;
        for (int32_t v = lo; v < hi; ++v)
            for (int i = 0; i < p; ++i) g[i] += muT[(size_t)v * p + i];
        matvec(p, th6, g, h1);
        matvec(p, th7, muT + (size_t)act * p, h2);
        /* decisions of the 2p relu units of Eq. (2) (p <= 128, checked by the entry points) */
        int on1[128], on2[128];
        for (int i = 0; i < p; ++i) {
            on1[i] = decided(h1[i], force_head ? force_head[((size_t)b * 2) * p + i] : -1);
            on2[i] = decided(h2[i], force_head ? force_head[((size_t)b * 2 + 1) * p + i] : -1);
            if (h_out) { h_out[((size_t)b * 2) * p + i] = h1[i]; h_out[((size_t)b * 2 + 1) * p + i] = h2[i]; }
            if (hs_out) {
                double s1 = 0.0, s2 = 0.0;
                for (int j = 0; j < p; ++j) {
                    s1 += fabs(th6[(size_t)i * p + j] * g[j]);
                    s2 += fabs(th7[(size_t)i * p + j] * muT[(size_t)act * p + j]);
                }
                hs_out[((size_t)b * 2) * p + i] = s1; hs_out[((size_t)b * 2 + 1) * p + i] = s2;
            }
        }
        double q = 0.0;
        for (int i = 0; i < p; ++i) q += th5[i] * (on1[i] ? h1[i] : 0.0) + th5[p + i] * (on2[i] ? h2[i] : 0.0);
        q_out[b] = q;
        double diff = q - target[b];
        loss += diff * diff / S;
        double dq = 2.0 * diff / S;

        /* Q-head backward */
        for (int i = 0; i < p; ++i) {
            d5[i] += dq * (on1[i] ? h1[i] : 0.0);
            d5[p + i] += dq * (on2[i] ? h2[i] : 0.0);
            dh1[i] = on1[i] ? dq * th5[i] : 0.0;
            dh2[i] = on2[i] ? dq * th5[p + i] : 0.0;
        }
        for (int i = 0; i < p; ++i)
            for (int j = 0; j < p; ++j) {
                d6[(size_t)i * p + j] += dh1[i] * g[j];
                d7[(size_t)i * p + j] += dh2[i] * muT[(size_t)act * p + j];
            }
        matvec_t(p, th6, dh1, dg);
        matvec_t(p, th7, dh2, tmp);
        memset(dmu, 0, sizeof(double) * np_);
        for (int32_t v = lo; v < hi; ++v)
            for (int i = 0; i < p; ++i) dmu[(size_t)v * p + i] = dg[i];
        for (int i = 0; i < p; ++i) dmu[(size_t)act * p + i] += tmp[i];

        /* rounds T..1 of Eq. (1), reversed */
        for (int t = T; t >= 1; --t) {
            const uint8_t *ont = on + (size_t)t * np_;
            const double *at = asum + (size_t)t * np_;
#pragma omp parallel
            {
                /* per-thread partial sums of the parameter gradients, added up at the end */
                double *loc = (double *)calloc(2 * pp + 4 * (size_t)p, sizeof(double));
                double *l2 = loc, *l3 = l2 + pp, *l1 = l3 + pp, *l4 = l1 + p, *ev = l4 + p, *dev = ev + p;
#pragma omp for schedule(dynamic, 256)
                for (int32_t v = 0; v < n; ++v) {
                    double *dz = dmu + (size_t)v * p; /* becomes d(pre-activation) in place */
                    int any = 0;
                    for (int i = 0; i < p; ++i) {
                        if (!ont[(size_t)v * p + i]) dz[i] = 0.0;
                        any |= dz[i] != 0.0;
                    }
                    double *dav = da + (size_t)v * p;
                    if (!any) { for (int i = 0; i < p; ++i) dav[i] = 0.0; continue; }
                    for (int i = 0; i < p; ++i) l1[i] += dz[i] * xb[v];
                    /* e_v does not depend on the round; recompute it edge by edge */
                    for (int i = 0; i < p; ++i) ev[i] = 0.0;
                    for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
                        double wj = w ? w[j] : 1.0;
                        for (int i = 0; i < p; ++i) ev[i] += relu(th4[i] * wj);
                    }
                    for (int i = 0; i < p; ++i)
                        for (int j = 0; j < p; ++j) {
                            l2[(size_t)i * p + j] += dz[i] * at[(size_t)v * p + j];
                            l3[(size_t)i * p + j] += dz[i] * ev[j];
                        }
                    matvec_t(p, th3, dz, dev);
                    for (int32_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
                        double wj = w ? w[j] : 1.0;
                        for (int i = 0; i < p; ++i)
                            if (th4[i] * wj > 0.0) l4[i] += dev[i] * wj;
                    }
                    matvec_t(p, th2, dz, dav);
                }
#pragma omp critical
                {
                    for (size_t i = 0; i < pp; ++i) { d2[i] += l2[i]; d3[i] += l3[i]; }
                    for (int i = 0; i < p; ++i) { d1[i] += l1[i]; d4[i] += l4[i]; }
                }
                free(loc);
            }
            /* adjoint of a_v = sum_{u in row v} c(v,u) mu[u], c = 1 or w:
             * dmu_prev[u] = sum_{v : u in row v} c(v,u) da[v] */
#pragma omp parallel for schedule(dynamic, 256)
            for (int32_t u = 0; u < n; ++u) {
                double *out = dmu + (size_t)u * p;
                for (int i = 0; i < p; ++i) out[i] = 0.0;
                for (int32_t j = rowptr_t[u]; j < rowptr_t[u + 1]; ++j) {
                    const double *src = da + (size_t)colidx_t[j] * p;
                    double cj = weighted ? w_t[j] : 1.0;
                    for (int i = 0; i < p; ++i) out[i] += cj * src[i];
                }
            }
        }
    }
    *loss_out = loss;
    free(mu); free(asum); free(esum); free(dmu); free(da); free(vec); free(on); free(rowptr_t); free(colidx_t); free(w_t);
    return 0;
}

int oracle_loss_grad(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w, int32_t weighted,
                     int32_t G,
                     const int32_t *graph_off, int32_t p, int32_t T, const double *th1, const double *th2,
                     const double *th3, const double *th4, const double *th5, const double *th6,
                     const double *th7, int32_t S, const double *x, const int32_t *action,
                     const double *target, double *loss_out, double *q_out, double *d1, double *d2,
                     double *d3, double *d4, double *d5, double *d6, double *d7) {
    if (p > 128) return -3;
    return loss_grad_impl(n, rowptr, colidx, w, weighted, G, graph_off, p, T, th1, th2, th3, th4, th5, th6, th7, S, x,
                          action, target, loss_out, q_out, d1, d2, d3, d4, d5, d6, d7, NULL, NULL, NULL, NULL, NULL,
                          NULL);
}

/*
 * The same loss and gradient with some relu decisions taken by the caller, and a report of every
 * pre-activation.  The gradient of Eq. (1) / Eq. (2) jumps where a pre-activation crosses zero; a float32
 * evaluation cannot resolve the sign of one that lies within float32 rounding of zero, and its gradient
 * is then that of the other branch.  A parity test reads the float32 path's decisions off its
 * activations, checks with z / zs from here that they differ from the definition's only where
 * |z| is within rounding of zero relative to zs, and asks for the gradient of that branch.
 *   force      [S][T][n][p] (NULL: none): -1 follow the sign of z, 0 / 1 unit off / on, for every unit of Eq. (1)
 *   force_head [S][2][p]    (NULL: none): the same for the units of Eq. (2): row 0 theta6 g, row 1 theta7 mu_a
 *   z_out, zs_out [S][T][n][p], h_out, hs_out [S][2][p] (each optional): the pre-activations and the
 *   summed magnitudes of their terms.
 * With force == NULL and force_head == NULL the results equal oracle_loss_grad's bit for bit.
 */
int oracle_loss_grad_decided(int32_t n, const int32_t *rowptr, const int32_t *colidx, const double *w,
                             int32_t weighted, int32_t G, const int32_t *graph_off, int32_t p, int32_t T,
                             const double *th1, const double *th2, const double *th3, const double *th4,
                             const double *th5, const double *th6, const double *th7, int32_t S, const double *x,
                             const int32_t *action, const double *target, double *loss_out, double *q_out,
                             double *d1, double *d2, double *d3, double *d4, double *d5, double *d6, double *d7,
                             const int8_t *force, const int8_t *force_head, double *z_out, double *zs_out,
                             double *h_out, double *hs_out) {
    if (p > 128) return -3;
    return loss_grad_impl(n, rowptr, colidx, w, weighted, G, graph_off, p, T, th1, th2, th3, th4, th5, th6, th7, S, x,
                          action, target, loss_out, q_out, d1, d2, d3, d4, d5, d6, d7, force, force_head, z_out,
                          zs_out, h_out, hs_out);
}

/* Plain gradient descent: theta <- theta - lr * grad (the optimiser of the benchmark's
 * training configuration; Sec. 4.5.2 repeats the step several times on one minibatch). */
int oracle_sgd(int64_t len, double *theta, const double *grad, double lr) {
    for (int64_t i = 0; i < len; ++i) theta[i] -= lr * grad[i];
    return 0;
}
