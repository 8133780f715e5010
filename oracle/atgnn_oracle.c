/*
 * CPU oracle for the attention-GNN graph convolution  O = SpMM(Softmax(SDDMM(Q, K, A)), V)
 * (Eq. 1 of Sec. 2.1) and its backward pass (Appendix B), for the three models of Sec. 5.1:
 * GT (dot-SDDMM), GAT (add-SDDMM) and AGNN (dot-SDDMM on L2-normalised features), plus GATv2, the
 * second member of the GAT family cited in Sec. 1, whose score is not a sum of two per-node scalars.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition written out as a single-threaded
 * loop over CSR rows in double precision.  It shares no code with the HIP library, is never called
 * by it, and may be used only from tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * Conventions (the graph is CSR by destination):
 *   row i = destination v;  N(i) = indices[indptr[i] .. indptr[i+1]) = its in-neighbours (sources) j;
 *   the softmax of Appendix A runs over N(i), i.e. over stored edges only (a missing edge is -inf,
 *   not 0); duplicates are separate terms; empty rows give O = 0, row_max = -inf, row_sum = 0.
 *   Node tensors are [N, H, D] row-major; heads are independent.
 *
 * Scores s_ij for edge i <- j, head h:
 *   GT   : scale * sum_d Q[i,h,d] K[j,h,d]
 *   GAT  : LeakyReLU(el[i,h] + er[j,h]),  el[v,h] = a_l[h,:].X[v,h,:],  er[v,h] = a_r[h,:].X[v,h,:]
 *   AGNN : beta * xhat[i,h,:].xhat[j,h,:],  xhat[v,h,:] = X[v,h,:] / max(||X[v,h,:]||_2, eps)   (beta = scale)
 *   GATv2: sum_d a[h,d] LeakyReLU(X[i,h,d] + K[j,h,d])   (X = destination-side, K = source-side projection;
 *          a = a_l; the non-linearity sits between the two linear maps, so the ranking of the neighbours
 *          depends on the destination)
 * Aggregated value rows: GT V, GAT X, AGNN X (the un-normalised features), GATv2 K.
 * Optional edge term (edge features entering the score, Sec. 1): bias[t,h] for CSR position t is added
 * to s_ij before the softmax; its gradient is dS of that edge.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ATGNN_GT = 0, ATGNN_GAT = 1, ATGNN_AGNN = 2, ATGNN_GATV2 = 3 };

typedef struct {
    int32_t model;
    int32_t H;
    int32_t D;
    double scale;     /* GT: score scale; AGNN: beta */
    double neg_slope; /* GAT LeakyReLU slope */
    double eps;       /* AGNN norm clamp */
} atgnn_layer;

/* Everything a score needs, precomputed per node where the model defines a per-node quantity. */
typedef struct {
    const atgnn_layer* L;
    int64_t N;
    const int32_t* indptr;
    const int32_t* indices;
    const double* X;   /* GT: Q; GAT: Wh; AGNN: h */
    const double* K;   /* GT keys; GATv2 source-side features */
    const double* Val; /* aggregated rows: GT V, GATv2 K, else X */
    const double* a;   /* GATv2 attention vector [H,D] */
    const double* bias; /* optional [nnz,H] additive edge term, NULL = none */
    double* el;        /* GAT [N,H] */
    double* er;        /* GAT [N,H] */
    double* nrm;       /* AGNN [N,H]: max(||x||, eps) */
    double* xhat;      /* AGNN [N,H,D] */
} ctx_t;

static double dot(const double* a, const double* b, int n) {
    double s = 0.0;
    for (int d = 0; d < n; ++d) s += a[d] * b[d];
    return s;
}

static int ctx_init(ctx_t* c, const atgnn_layer* L, int64_t N, const int32_t* indptr, const int32_t* indices,
                    const double* X, const double* K, const double* V, const double* a_l, const double* a_r) {
    const int H = L->H, D = L->D;
    memset(c, 0, sizeof(*c));
    c->L = L; c->N = N; c->indptr = indptr; c->indices = indices; c->X = X; c->K = K;
    c->Val = (L->model == ATGNN_GT) ? V : (L->model == ATGNN_GATV2 ? K : X);
    c->a = a_l;
    if (L->model == ATGNN_GAT) {
        c->el = (double*)malloc(sizeof(double) * (size_t)(N * H + 1));
        c->er = (double*)malloc(sizeof(double) * (size_t)(N * H + 1));
        if (!c->el || !c->er) return -1;
        for (int64_t v = 0; v < N; ++v)
            for (int h = 0; h < H; ++h) {
                const double* x = X + (v * H + h) * D;
                c->el[v * H + h] = dot(a_l + h * D, x, D);
                c->er[v * H + h] = dot(a_r + h * D, x, D);
            }
    } else if (L->model == ATGNN_AGNN) {
        c->nrm = (double*)malloc(sizeof(double) * (size_t)(N * H + 1));
        c->xhat = (double*)malloc(sizeof(double) * (size_t)(N * H * D + 1));
        if (!c->nrm || !c->xhat) return -1;
        for (int64_t v = 0; v < N; ++v)
            for (int h = 0; h < H; ++h) {
                const double* x = X + (v * H + h) * D;
                double n = sqrt(dot(x, x, D));
                if (n < L->eps) n = L->eps;
                c->nrm[v * H + h] = n;
                for (int d = 0; d < D; ++d) c->xhat[(v * H + h) * D + d] = x[d] / n;
            }
    }
    return 0;
}

static void ctx_free(ctx_t* c) {
    free(c->el); free(c->er); free(c->nrm); free(c->xhat);
}

/* pre-activation of GAT (needed again for the LeakyReLU derivative) */
static double gat_z(const ctx_t* c, int64_t i, int64_t j, int h) {
    return c->el[i * c->L->H + h] + c->er[j * c->L->H + h];
}

static double model_score(const ctx_t* c, int64_t i, int64_t j, int h);

/* score of the edge stored at CSR position t of row i */
static double score(const ctx_t* c, int64_t i, int64_t t, int h) {
    const double s = model_score(c, i, c->indices[t], h);
    return c->bias ? s + c->bias[t * c->L->H + h] : s;
}

static double model_score(const ctx_t* c, int64_t i, int64_t j, int h) {
    const int H = c->L->H, D = c->L->D;
    switch (c->L->model) {
    case ATGNN_GT:
        return c->L->scale * dot(c->X + (i * H + h) * D, c->K + (j * H + h) * D, D);
    case ATGNN_GAT: {
        double z = gat_z(c, i, j, h);
        return z > 0.0 ? z : c->L->neg_slope * z;
    }
    case ATGNN_GATV2: {
        double s = 0.0;
        for (int d = 0; d < D; ++d) {
            const double z = c->X[(i * H + h) * D + d] + c->K[(j * H + h) * D + d];
            s += c->a[h * D + d] * (z > 0.0 ? z : c->L->neg_slope * z);
        }
        return s;
    }
    default:
        return c->L->scale * dot(c->xhat + (i * H + h) * D, c->xhat + (j * H + h) * D, D);
    }
}

/* Edge softmax of one row and head, in the two rounds of Appendix A.  p has deg entries. */
static void row_softmax(const ctx_t* c, int64_t i, int h, double* p, double* zmax, double* zsum) {
    const int64_t b = c->indptr[i], e = c->indptr[i + 1];
    double m = -INFINITY, l = 0.0;
    for (int64_t t = b; t < e; ++t) { /* round 1: scores and their maximum */
        p[t - b] = score(c, i, t, h);
        if (p[t - b] > m) m = p[t - b];
    }
    for (int64_t t = b; t < e; ++t) { /* round 2: exponentials and their sum */
        p[t - b] = exp(p[t - b] - m);
        l += p[t - b];
    }
    for (int64_t t = b; t < e; ++t) p[t - b] /= l;
    *zmax = m; *zsum = l;
}

static int64_t max_degree(int64_t N, const int32_t* indptr) {
    int64_t m = 0;
    for (int64_t i = 0; i < N; ++i)
        if (indptr[i + 1] - indptr[i] > m) m = indptr[i + 1] - indptr[i];
    return m;
}

/*
 * Forward.  rows == NULL: all N rows; else only the n_rows listed rows are computed (the others are
 * left untouched).  O [N,H,D], row_max / row_sum [N,H] are full-size; P (optional, may be NULL) is
 * [nnz, H] and receives the normalised attention p_ij of every processed edge.
 */
int atgnn_oracle_forward(const atgnn_layer* L, int64_t N, const int32_t* indptr, const int32_t* indices,
                         const double* X, const double* K, const double* V, const double* a_l, const double* a_r,
                         const double* bias, int64_t n_rows, const int64_t* rows,
                         double* O, double* row_max, double* row_sum, double* P) {
    const int H = L->H, D = L->D;
    ctx_t c;
    if (ctx_init(&c, L, N, indptr, indices, X, K, V, a_l, a_r)) { ctx_free(&c); return -1; }
    c.bias = bias;
    double* p = (double*)malloc(sizeof(double) * (size_t)(max_degree(N, indptr) + 1));
    const int64_t count = rows ? n_rows : N;
    for (int64_t r = 0; r < count; ++r) {
        const int64_t i = rows ? rows[r] : r;
        const int64_t b = indptr[i], e = indptr[i + 1];
        for (int h = 0; h < H; ++h) {
            double m, l;
            double* o = O + (i * H + h) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            if (e == b) { row_max[i * H + h] = -INFINITY; row_sum[i * H + h] = 0.0; continue; }
            row_softmax(&c, i, h, p, &m, &l);
            for (int64_t t = b; t < e; ++t) {
                const double* val = c.Val + ((int64_t)indices[t] * H + h) * D;
                for (int d = 0; d < D; ++d) o[d] += p[t - b] * val[d];
                if (P) P[t * H + h] = p[t - b];
            }
            row_max[i * H + h] = m;
            row_sum[i * H + h] = l;
        }
    }
    free(p);
    ctx_free(&c);
    return 0;
}

/*
 * Backward, given G = dL/dO  [N,H,D].  Gradient arrays are full-size, zeroed here, and accumulated
 * over the processed rows (rows == NULL: all rows, which gives the complete gradient).  With a row
 * subset R the entries are complete for: dX[v] (query side) iff v in R; source-side terms of node v
 * iff every row that has v as a source is in R.  The per-node finalisation (GAT a_l/a_r terms, AGNN
 * normalisation) runs over all nodes on whatever has been accumulated; da_l, da_r, dscale are sums
 * over all processed rows.
 *
 *   dP_ij = G_i . Val_j                          (Appendix B, SpMM backward, sampled at the edges)
 *   dVal_j += p_ij G_i                           (Appendix B, P^T dO)
 *   dS_ij = p_ij (dP_ij - sum_k p_ik dP_ik)      (softmax backward; the sum is formed explicitly)
 *   GT   : dQ_i += scale dS_ij K_j ; dK_j += scale dS_ij Q_i     (Appendix B, SDDMM backward)
 *   GAT  : dz = dS_ij * (z > 0 ? 1 : neg_slope); d_el_i += dz; d_er_j += dz;
 *          dX_v += d_el_v a_l + d_er_v a_r;  da_l[h] = sum_v d_el[v,h] X[v,h,:];  da_r likewise
 *   AGNN : c = xhat_i . xhat_j; dbeta += dS_ij c; g_i += beta dS_ij xhat_j; g_j += beta dS_ij xhat_i;
 *          dX_v += (g_v - (g_v . xhat_v) xhat_v) / ||x_v||   (||x_v|| > eps), else g_v / eps
 *   GATv2: z_d = X_i,d + K_j,d; dz_d = dS_ij a_d (z_d > 0 ? 1 : neg_slope); dX_i += dz; dK_j += dz (on top of
 *          the value term p_ij G_i);  da_l[h,d] += dS_ij LeakyReLU(z_d)
 * dS_out (optional) [nnz,H] receives dS of every processed edge (= the gradient of the edge term).
 */
int atgnn_oracle_backward(const atgnn_layer* L, int64_t N, const int32_t* indptr, const int32_t* indices,
                          const double* X, const double* K, const double* V, const double* a_l, const double* a_r,
                          const double* bias, const double* G, int64_t n_rows, const int64_t* rows,
                          double* dX, double* dK, double* dV, double* da_l, double* da_r, double* dscale,
                          double* dS_out) {
    const int H = L->H, D = L->D;
    const size_t NHD = (size_t)N * H * D;
    ctx_t c;
    if (ctx_init(&c, L, N, indptr, indices, X, K, V, a_l, a_r)) { ctx_free(&c); return -1; }
    c.bias = bias;
    const int64_t md = max_degree(N, indptr);
    double* p = (double*)malloc(sizeof(double) * (size_t)(md + 1));
    double* dP = (double*)malloc(sizeof(double) * (size_t)(md + 1));
    double* d_el = NULL; double* d_er = NULL; double* g = NULL;
    double* dVal = (L->model == ATGNN_GT) ? dV : (L->model == ATGNN_GATV2 ? dK : dX);

    memset(dX, 0, sizeof(double) * NHD);
    if (L->model == ATGNN_GT) { memset(dK, 0, sizeof(double) * NHD); memset(dV, 0, sizeof(double) * NHD); }
    if (L->model == ATGNN_GAT) {
        d_el = (double*)calloc((size_t)N * H + 1, sizeof(double));
        d_er = (double*)calloc((size_t)N * H + 1, sizeof(double));
        memset(da_l, 0, sizeof(double) * H * D);
        memset(da_r, 0, sizeof(double) * H * D);
    }
    if (L->model == ATGNN_AGNN) { g = (double*)calloc(NHD + 1, sizeof(double)); *dscale = 0.0; }
    if (L->model == ATGNN_GATV2) { memset(dK, 0, sizeof(double) * NHD); memset(da_l, 0, sizeof(double) * H * D); }

    const int64_t count = rows ? n_rows : N;
    for (int64_t r = 0; r < count; ++r) {
        const int64_t i = rows ? rows[r] : r;
        const int64_t b = indptr[i], e = indptr[i + 1];
        if (e == b) continue;
        for (int h = 0; h < H; ++h) {
            double m, l, pdp = 0.0;
            const double* gi = G + (i * H + h) * D;
            row_softmax(&c, i, h, p, &m, &l);
            for (int64_t t = b; t < e; ++t) {
                const int64_t j = indices[t];
                dP[t - b] = dot(gi, c.Val + (j * H + h) * D, D);
                pdp += p[t - b] * dP[t - b];
                for (int d = 0; d < D; ++d) dVal[(j * H + h) * D + d] += p[t - b] * gi[d];
            }
            for (int64_t t = b; t < e; ++t) {
                const int64_t j = indices[t];
                const double dS = p[t - b] * (dP[t - b] - pdp);
                if (dS_out) dS_out[t * H + h] = dS;
                if (L->model == ATGNN_GT) {
                    for (int d = 0; d < D; ++d) {
                        dX[(i * H + h) * D + d] += L->scale * dS * K[(j * H + h) * D + d];
                        dK[(j * H + h) * D + d] += L->scale * dS * X[(i * H + h) * D + d];
                    }
                } else if (L->model == ATGNN_GAT) {
                    const double dz = dS * (gat_z(&c, i, j, h) > 0.0 ? 1.0 : L->neg_slope);
                    d_el[i * H + h] += dz;
                    d_er[j * H + h] += dz;
                } else if (L->model == ATGNN_GATV2) {
                    for (int d = 0; d < D; ++d) {
                        const double z = X[(i * H + h) * D + d] + K[(j * H + h) * D + d];
                        const double dz = dS * a_l[h * D + d] * (z > 0.0 ? 1.0 : L->neg_slope);
                        dX[(i * H + h) * D + d] += dz;
                        dK[(j * H + h) * D + d] += dz;
                        da_l[h * D + d] += dS * (z > 0.0 ? z : L->neg_slope * z);
                    }
                } else {
                    const double* xi = c.xhat + (i * H + h) * D;
                    const double* xj = c.xhat + (j * H + h) * D;
                    *dscale += dS * dot(xi, xj, D);
                    for (int d = 0; d < D; ++d) {
                        g[(i * H + h) * D + d] += L->scale * dS * xj[d];
                        g[(j * H + h) * D + d] += L->scale * dS * xi[d];
                    }
                }
            }
        }
    }

    if (L->model == ATGNN_GAT) {
        for (int64_t v = 0; v < N; ++v)
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d) {
                    dX[(v * H + h) * D + d] += d_el[v * H + h] * a_l[h * D + d] + d_er[v * H + h] * a_r[h * D + d];
                    da_l[h * D + d] += d_el[v * H + h] * X[(v * H + h) * D + d];
                    da_r[h * D + d] += d_er[v * H + h] * X[(v * H + h) * D + d];
                }
    }
    if (L->model == ATGNN_AGNN) {
        for (int64_t v = 0; v < N; ++v)
            for (int h = 0; h < H; ++h) {
                const double* gv = g + (v * H + h) * D;
                const double* xh = c.xhat + (v * H + h) * D;
                const double* x = X + (v * H + h) * D;
                double* out = dX + (v * H + h) * D;
                if (sqrt(dot(x, x, D)) > L->eps) {
                    const double proj = dot(gv, xh, D);
                    for (int d = 0; d < D; ++d) out[d] += (gv[d] - proj * xh[d]) / c.nrm[v * H + h];
                } else {
                    for (int d = 0; d < D; ++d) out[d] += gv[d] / L->eps;
                }
            }
    }
    free(p); free(dP); free(d_el); free(d_er); free(g);
    ctx_free(&c);
    return 0;
}
