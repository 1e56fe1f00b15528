/*
 * CPU oracle for normalized-adjacency message passing on a user-item graph.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the GPU library must compute.  Only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may call it; the product
 * path never does.  It shares no source, header, table or helper with the GPU
 * library.
 *
 * What is computed, and where the paper defines it:
 *   - A: n x n adjacency with A_ij > 0 iff (i,j) is an edge (Section 3,
 *     "Notation").  The graph is an undirected user-item graph: node u for
 *     user u, node n_users + i for item i; a distinct input pair (u,i) gives
 *     A[u][nu+i] = A[nu+i][u] = 1.  Repeated pairs are one edge.
 *   - A~ = A + I, D~ = D + I with D = diag(A 1), A^ = D~^-1/2 A~ D~^-1/2
 *     (Section 3, "Notation").
 *   - LightGCN propagation H(l+1) = A^ H(l) (Section 3.1, matrix form of the
 *     LightGCN update), K layers, K = number of sampled hops (Section 5).
 *   - Without the self-loop augmentation the same code evaluates the per-node
 *     LightGCN update, weights 1/(sqrt|N(u)| sqrt|N(i)|) (Section 3.1).
 *   - Backward: the transpose-Jacobian of the linear map, G(l) = A^T G(l+1)
 *     (Appendix A, the "GNN backprop" factor of the chain rule; Section 4.3.2,
 *     the J^T dL/dF_gnn terms of the multi-task gradient).  Written as a
 *     scatter over the forward CSR so that it is the transpose by construction
 *     and assumes no symmetry.
 *   - Layer combination of LightGCN, Y = 1/(L+1) sum_{l=0..L} H(l) (Section 3.1, the final
 *     representation as the mean of all layers), and the GFAE reconstruction loss with the
 *     identity decoder, L_ssl = ||X - Y||_F^2 (Section 4.2), with dL/dY = 2 (Y - X).
 *   - Weighted graphs (Section 3, "Notation": A_ij > 0 iff (i,j) in E, D = diag(A 1)): with real
 *     edge weights the same definitions give d~_i = 1 + sum_j A_ij and A^_ij = A~_ij / sqrt(d~_i d~_j),
 *     the self-loop weighing 1.  A pair given several times carries the largest of its weights.
 *   - GraphSAGE layer (Section 3.1): mean of the neighbours' rows, hbar_u = 1/|S(u)| sum_{v in S(u)} h_v
 *     with S(u) the node's neighbours in the given (sampled) graph, then
 *     h'_u = sigma(W . CONCAT(h_u, hbar_u)); sigma = ReLU here.
 *   - GradNorm task weighting (Section 4.3.1): G_i = || grad_{h(0)} (w_i L_i) ||_2, relative rates
 *     r_i = (L_i / L_i(0)) / mean_j (L_j / L_j(0)), meta-loss sum_i | G_i - Gbar r_i^gamma |, one
 *     gradient step on the weights and renormalisation to sum_i w_i = T.
 *   - Importance sampling of a multi-hop subgraph (Section 4.1, the sampling probability
 *     p(u->v) = w_uv^beta / sum_k w_uk^beta, at most k neighbours per node, depth L; Section 5,
 *     "Subgraph Sampling": fan-outs per hop).  A node with at most k neighbours (the diagonal entry of
 *     its row is not one) keeps all that have positive weight; otherwise k independent draws are made from the distribution and equal
 *     draws are one neighbour.  The distribution is held in integers (weights scaled to 2^24 at the
 *     row maximum) and the random numbers come from the counter-based generator Philox4x32-10
 *     (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC 2011), so that
 *     every decision is integer arithmetic.
 *   - Dense per-layer update Z = P W, H' = max(Z, 0): the update function psi of
 *     the generic message-passing layer with the W, sigma of the GraphSAGE
 *     layer (Section 3 and Section 3.1), and its backward.
 *
 * All floating point is IEEE double; sums run in CSR (ascending column) order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int32_t e2eg_oracle_max_threads(void) {
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

void e2eg_oracle_set_threads(int32_t t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

static int cmp_u64(const void* a, const void* b) {
    uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
    return (x > y) - (x < y);
}

/*
 * Structure of A~ (or of A when add_self_loops == 0) in canonical CSR:
 * rows in node order, columns strictly ascending.  Built the obvious way:
 * list every (row, col) entry, sort, drop repeats.
 * row_ptr has n+1 entries; col_idx has room for 2*n_edges + n entries.
 * Returns nnz, or -1 on an out-of-range id / allocation failure.
 */
int64_t e2eg_oracle_build_csr(int32_t n_users, int32_t n_items, int64_t n_edges,
                              const int32_t* users, const int32_t* items,
                              int32_t add_self_loops, int64_t* row_ptr, int32_t* col_idx) {
    int64_t n = (int64_t)n_users + n_items;
    int64_t cap = 2 * n_edges + (add_self_loops ? n : 0);
    uint64_t* key = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(cap > 0 ? cap : 1));
    if (!key) return -1;
    int64_t m = 0;
    for (int64_t e = 0; e < n_edges; ++e) {
        int64_t u = users[e], i = items[e];
        if (u < 0 || u >= n_users || i < 0 || i >= n_items) { free(key); return -1; }
        uint64_t a = (uint64_t)u, b = (uint64_t)(n_users + i);
        key[m++] = (a << 32) | b;   /* A[u][nu+i] */
        key[m++] = (b << 32) | a;   /* A[nu+i][u] */
    }
    if (add_self_loops)
        for (int64_t v = 0; v < n; ++v) key[m++] = ((uint64_t)v << 32) | (uint64_t)v;  /* + I */
    qsort(key, (size_t)m, sizeof(uint64_t), cmp_u64);
    int64_t nnz = 0;
    for (int64_t r = 0; r <= n; ++r) row_ptr[r] = 0;
    for (int64_t k = 0; k < m; ++k) {
        if (k > 0 && key[k] == key[k - 1]) continue;   /* repeated pair: one edge */
        col_idx[nnz++] = (int32_t)(key[k] & 0xffffffffu);
        row_ptr[(key[k] >> 32) + 1] += 1;
    }
    for (int64_t r = 0; r < n; ++r) row_ptr[r + 1] += row_ptr[r];
    free(key);
    return nnz;
}

/*
 * The same structure for the rows row_lo <= r < row_hi only (for graphs whose full entry list is
 * better not sorted in one piece): list every (row, col) entry whose row is in the range, sort,
 * drop repeats.  row_ptr_local has row_hi - row_lo + 1 entries and starts at 0; col_idx has room
 * for `cap` entries.  Returns the number of entries of the range (even when it exceeds cap, in
 * which case nothing is written beyond cap and the caller asks again), or -1 on an
 * out-of-range id / allocation failure.
 */
int64_t e2eg_oracle_build_csr_rows(int32_t n_users, int32_t n_items, int64_t n_edges, const int32_t* users,
                                   const int32_t* items, int32_t add_self_loops, int64_t row_lo, int64_t row_hi,
                                   int64_t* row_ptr_local, int32_t* col_idx, int64_t cap) {
    int64_t n = (int64_t)n_users + n_items;
    if (row_lo < 0 || row_hi > n || row_lo > row_hi) return -1;
    int64_t listed = 0;
    for (int64_t e = 0; e < n_edges; ++e) {
        int64_t u = users[e], i = items[e];
        if (u < 0 || u >= n_users || i < 0 || i >= n_items) return -1;
        listed += (u >= row_lo && u < row_hi) + (n_users + i >= row_lo && n_users + i < row_hi);
    }
    if (add_self_loops) listed += row_hi - row_lo;
    uint64_t* key = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(listed > 0 ? listed : 1));
    if (!key) return -1;
    int64_t m = 0;
    for (int64_t e = 0; e < n_edges; ++e) {
        uint64_t a = (uint64_t)users[e], b = (uint64_t)n_users + (uint64_t)items[e];
        if ((int64_t)a >= row_lo && (int64_t)a < row_hi) key[m++] = (a << 32) | b;   /* A[u][nu+i] */
        if ((int64_t)b >= row_lo && (int64_t)b < row_hi) key[m++] = (b << 32) | a;   /* A[nu+i][u] */
    }
    if (add_self_loops)
        for (int64_t v = row_lo; v < row_hi; ++v) key[m++] = ((uint64_t)v << 32) | (uint64_t)v;  /* + I */
    qsort(key, (size_t)m, sizeof(uint64_t), cmp_u64);
    int64_t nnz = 0;
    for (int64_t r = 0; r <= row_hi - row_lo; ++r) row_ptr_local[r] = 0;
    for (int64_t k = 0; k < m; ++k) {
        if (k > 0 && key[k] == key[k - 1]) continue;   /* repeated pair: one edge */
        if (nnz < cap) col_idx[nnz] = (int32_t)(key[k] & 0xffffffffu);
        ++nnz;
        row_ptr_local[(int64_t)(key[k] >> 32) - row_lo + 1] += 1;
    }
    for (int64_t r = 0; r < row_hi - row_lo; ++r) row_ptr_local[r + 1] += row_ptr_local[r];
    free(key);
    return nnz;
}

/* d~_i = sum_j A~_ij = number of stored entries in row i;  s_i = d~_i^-1/2 (0 for an
 * empty row, which can only occur without self-loops). */
void e2eg_oracle_normalize(int64_t n, const int64_t* row_ptr, int64_t* deg, double* dinv_sqrt) {
    for (int64_t i = 0; i < n; ++i) {
        int64_t d = row_ptr[i + 1] - row_ptr[i];
        deg[i] = d;
        dinv_sqrt[i] = d > 0 ? 1.0 / sqrt((double)d) : 0.0;
    }
}

/* A^_ij for a stored entry: A~_ij / sqrt(d~_i d~_j) with A~_ij = 1. */
static inline double a_hat(const int64_t* row_ptr, int64_t i, int64_t j) {
    double di = (double)(row_ptr[i + 1] - row_ptr[i]);
    double dj = (double)(row_ptr[j + 1] - row_ptr[j]);
    return 1.0 / sqrt(di * dj);
}

/* One layer, gather form:  Y_i = sum_j A^_ij X_j.   X, Y: [n][F] row-major doubles. */
void e2eg_oracle_propagate_layer(int64_t n, const int64_t* row_ptr, const int32_t* col_idx,
                                 int64_t F, const double* X, double* Y) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n; ++i) {
        double* y = Y + i * F;
        for (int64_t f = 0; f < F; ++f) y[f] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            double a = a_hat(row_ptr, i, j);
            const double* x = X + j * F;
            for (int64_t f = 0; f < F; ++f) y[f] += a * x[f];
        }
    }
}

/* Same, for a chosen list of rows only:  Y[r] = sum_j A^_{rows[r], j} X_j. */
void e2eg_oracle_propagate_rows(int64_t n_rows, const int64_t* rows, const int64_t* row_ptr,
                                const int32_t* col_idx, int64_t F, const double* X, double* Y) {
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t i = rows[r];
        double* y = Y + r * F;
        for (int64_t f = 0; f < F; ++f) y[f] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            double a = a_hat(row_ptr, i, j);
            const double* x = X + j * F;
            for (int64_t f = 0; f < F; ++f) y[f] += a * x[f];
        }
    }
}

/*
 * The backward's scatter (G_j += A^_ij Gnext_i for every stored (i, j): Appendix A, the "GNN backprop"
 * factor) restricted to chosen target nodes j and to the source rows row_lo <= i < row_lo + n_rows,
 * whose entries are given as a local CSR (row_ptr_local starting at 0).  deg[v] = d~_v for every node.
 * targets are ascending node ids; out[t] (n_targets x F) is ADDED to, so that calls over consecutive
 * row ranges build up (A^T Gnext)[targets].  No symmetry is assumed: an entry (i, j) feeds node j only.
 */
void e2eg_oracle_transposed_to_targets(int64_t row_lo, int64_t n_rows, const int64_t* row_ptr_local,
                                       const int32_t* col_idx_local, const int64_t* deg, int64_t F,
                                       const double* Gnext, int64_t n_targets, const int64_t* targets,
                                       double* out) {
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t i = row_lo + r;
        const double* g = Gnext + i * F;
        for (int64_t p = row_ptr_local[r]; p < row_ptr_local[r + 1]; ++p) {
            const int64_t j = col_idx_local[p];
            int64_t lo = 0, hi = n_targets;   /* is j a target? */
            while (lo < hi) {
                const int64_t mid = (lo + hi) / 2;
                if (targets[mid] < j) lo = mid + 1; else hi = mid;
            }
            if (lo == n_targets || targets[lo] != j) continue;
            const double a = 1.0 / sqrt((double)deg[i] * (double)deg[j]);
            double* o = out + lo * F;
            for (int64_t f = 0; f < F; ++f) o[f] += a * g[f];
        }
    }
}

/*
 * One layer of the backward, scatter form:  G_j += A^_ij Gnext_i for every stored (i,j),
 * i.e. G = A^T Gnext whatever the structure.  Threads split the feature columns, so every
 * element sees the same sequence of additions as in a single-threaded run.
 */
void e2eg_oracle_propagate_layer_transposed(int64_t n, const int64_t* row_ptr,
                                            const int32_t* col_idx, int64_t F,
                                            const double* Gnext, double* G) {
    int64_t nblk = (F + 7) / 8;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nblk; ++b) {
        int64_t f0 = b * 8, f1 = f0 + 8 < F ? f0 + 8 : F;
        for (int64_t i = 0; i < n; ++i)
            for (int64_t f = f0; f < f1; ++f) G[i * F + f] = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            const double* g = Gnext + i * F;
            for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
                int64_t j = col_idx[p];
                double a = a_hat(row_ptr, i, j);
                double* o = G + j * F;
                for (int64_t f = f0; f < f1; ++f) o[f] += a * g[f];
            }
        }
    }
}

/* Dense update:  Z = P W  ([n][Fin] x [Fin][Fout]),  H = relu ? max(Z, 0) : Z. */
void e2eg_oracle_transform_fwd(int64_t n, int64_t Fin, int64_t Fout, const double* P,
                               const double* W, int32_t relu, double* Z, double* H) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t o = 0; o < Fout; ++o) {
            double z = 0.0;
            for (int64_t c = 0; c < Fin; ++c) z += P[i * Fin + c] * W[c * Fout + o];
            Z[i * Fout + o] = z;
            H[i * Fout + o] = (relu && !(z > 0.0)) ? 0.0 : z;
        }
}

/*
 * Backward of the dense update.  dZ = gH * [mask > 0] when relu (mask: [n][Fout], the
 * caller passes Z or H; both have the same sign pattern), else dZ = gH.
 * dP = dZ W^T,  dW = P^T dZ.
 */
void e2eg_oracle_transform_bwd(int64_t n, int64_t Fin, int64_t Fout, const double* P,
                               const double* W, const double* mask, const double* gH,
                               int32_t relu, double* dP, double* dW) {
    double* dZ = (double*)malloc(sizeof(double) * (size_t)(n * Fout > 0 ? n * Fout : 1));
    for (int64_t k = 0; k < n * Fout; ++k) dZ[k] = (relu && !(mask[k] > 0.0)) ? 0.0 : gH[k];
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < Fin; ++c) {
            double s = 0.0;
            for (int64_t o = 0; o < Fout; ++o) s += dZ[i * Fout + o] * W[c * Fout + o];
            dP[i * Fin + c] = s;
        }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < Fin; ++c)
        for (int64_t o = 0; o < Fout; ++o) {
            double s = 0.0;
            for (int64_t i = 0; i < n; ++i) s += P[i * Fin + c] * dZ[i * Fout + o];
            dW[c * Fout + o] = s;
        }
    free(dZ);
}

/*
 * Layer combination (Section 3.1):  Y = 1/(K+1) * (H(0) + H(1) + ... + H(K)).
 * X0 = H(0) is [n][F]; layers holds H(1..K) back to back, each [n][F].
 */
void e2eg_oracle_readout_mean(int64_t n, int64_t F, int64_t K, const double* X0, const double* layers,
                              double* Y) {
    for (int64_t k = 0; k < n * F; ++k) {
        double s = X0[k];
        for (int64_t l = 0; l < K; ++l) s += layers[l * n * F + k];
        Y[k] = s / (double)(K + 1);
    }
}

/*
 * GFAE reconstruction loss with the identity decoder (Section 4.2):  L = ||X - Y||_F^2 = sum (X - Y)^2,
 * returned; if gY is not NULL it receives dL/dY = 2 (Y - X).
 */
double e2eg_oracle_gfae_loss(int64_t n, int64_t F, const double* X, const double* Y, double* gY) {
    double loss = 0.0;
    for (int64_t k = 0; k < n * F; ++k) {
        double d = X[k] - Y[k];
        loss += d * d;
        if (gY) gY[k] = 2.0 * (Y[k] - X[k]);
    }
    return loss;
}

/*
 * Mean aggregator of GraphSAGE (Section 3.1):  M_i = 1/|N(i)| * sum_{j in row i} X_j, the rows of
 * the CSR being the neighbour sets (built without self-loops); an empty row gives 0.
 */
void e2eg_oracle_mean_neighbours(int64_t n, const int64_t* row_ptr, const int32_t* col_idx, int64_t F,
                                 const double* X, double* M) {
    for (int64_t i = 0; i < n; ++i) {
        double* m = M + i * F;
        int64_t d = row_ptr[i + 1] - row_ptr[i];
        for (int64_t f = 0; f < F; ++f) m[f] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            const double* x = X + (int64_t)col_idx[p] * F;
            for (int64_t f = 0; f < F; ++f) m[f] += x[f];
        }
        if (d > 0)
            for (int64_t f = 0; f < F; ++f) m[f] /= (double)d;
    }
}

/*
 * Transpose of the mean aggregator, scatter form over the same CSR:  G_j += gM_i / |N(i)| for every
 * stored (i, j).  It is the transpose whatever the structure.
 */
void e2eg_oracle_mean_neighbours_transposed(int64_t n, const int64_t* row_ptr, const int32_t* col_idx,
                                            int64_t F, const double* gM, double* G) {
    for (int64_t k = 0; k < n * F; ++k) G[k] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t d = row_ptr[i + 1] - row_ptr[i];
        const double* g = gM + i * F;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            double* o = G + (int64_t)col_idx[p] * F;
            for (int64_t f = 0; f < F; ++f) o[f] += g[f] / (double)d;
        }
    }
}

/* 2-norms of the T column blocks of G ([n][T*F]): norms[t] = sqrt(sum_rows sum_{c in block t} G^2). */
void e2eg_oracle_block_norms(int64_t n, int64_t F, int64_t T, const double* G, double* norms) {
    for (int64_t t = 0; t < T; ++t) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i)
            for (int64_t f = 0; f < F; ++f) {
                double v = G[i * T * F + t * F + f];
                s += v * v;
            }
        norms[t] = sqrt(s);
    }
}

/*
 * One GradNorm step (Section 4.3.1).  gnorm[i] = || grad_{h(0)} L_i ||_2 (without the weight), so
 * G_i = w_i gnorm[i].  With the targets Gbar r_i^gamma held constant, d/dw_i of
 * sum_i | G_i - Gbar r_i^gamma | is sign(G_i - Gbar r_i^gamma) gnorm[i]; the weights take one step
 * of size lr against it, are kept positive (floor 1e-8) and rescaled to sum to T.
 * Returns the meta-loss at the weights given (before the step).
 */
double e2eg_oracle_gradnorm_step(int64_t T, const double* loss, const double* loss0, const double* gnorm,
                                 double gamma, double lr, double* w) {
    double Gbar = 0.0, rbar = 0.0, meta = 0.0, sum = 0.0;
    for (int64_t i = 0; i < T; ++i) {
        Gbar += w[i] * gnorm[i] / (double)T;
        rbar += loss[i] / loss0[i] / (double)T;
    }
    for (int64_t i = 0; i < T; ++i) {
        double G = w[i] * gnorm[i];
        double target = Gbar * pow(loss[i] / loss0[i] / rbar, gamma);
        double diff = G - target;
        meta += fabs(diff);
        double sgn = diff > 0.0 ? 1.0 : (diff < 0.0 ? -1.0 : 0.0);
        w[i] -= lr * sgn * gnorm[i];
    }
    for (int64_t i = 0; i < T; ++i) {
        if (w[i] < 1e-8) w[i] = 1e-8;
        sum += w[i];
    }
    for (int64_t i = 0; i < T; ++i) w[i] *= (double)T / sum;
    return meta;
}

/*
 * Values of the stored entries of a weighted A~ on the structure made by e2eg_oracle_build_csr:
 * val = 1 on the diagonal, the edge weight on (u, nu+i) and (nu+i, u); a pair listed several times
 * gets the largest of its weights.  Entries are found by scanning the row.
 */
void e2eg_oracle_edge_values(int32_t n_users, int64_t n_edges, const int32_t* users, const int32_t* items,
                             const double* weights, int64_t n, const int64_t* row_ptr, const int32_t* col_idx,
                             double* val) {
    for (int64_t i = 0; i < n; ++i)
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) val[p] = col_idx[p] == i ? 1.0 : 0.0;
    for (int64_t e = 0; e < n_edges; ++e) {
        int64_t a = users[e], b = (int64_t)n_users + items[e];
        for (int dir = 0; dir < 2; ++dir) {
            int64_t r = dir ? b : a, c = dir ? a : b;
            for (int64_t p = row_ptr[r]; p < row_ptr[r + 1]; ++p)
                if (col_idx[p] == c && weights[e] > val[p]) val[p] = weights[e];
        }
    }
}

/* d~_i = sum_j A~_ij with the stored values (Section 3: D~ = D + I, D = diag(A 1)). */
void e2eg_oracle_weighted_degrees(int64_t n, const int64_t* row_ptr, const double* val, double* deg) {
    for (int64_t i = 0; i < n; ++i) {
        double d = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) d += val[p];
        deg[i] = d;
    }
}

/* Y = A^ X with A^_ij = val_ij / sqrt(d~_i d~_j), d~ from the stored values (a row of zero sum gives 0). */
void e2eg_oracle_propagate_layer_weighted(int64_t n, const int64_t* row_ptr, const int32_t* col_idx,
                                          const double* val, const double* deg, int64_t F, const double* X,
                                          double* Y) {
    for (int64_t i = 0; i < n; ++i) {
        double* y = Y + i * F;
        for (int64_t f = 0; f < F; ++f) y[f] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            double den = sqrt(deg[i] * deg[j]);
            double a = den > 0.0 ? val[p] / den : 0.0;
            const double* x = X + j * F;
            for (int64_t f = 0; f < F; ++f) y[f] += a * x[f];
        }
    }
}

/* G = A^T Gnext for the weighted operator, scatter form over the same CSR. */
void e2eg_oracle_propagate_layer_weighted_transposed(int64_t n, const int64_t* row_ptr, const int32_t* col_idx,
                                                     const double* val, const double* deg, int64_t F,
                                                     const double* Gnext, double* G) {
    for (int64_t k = 0; k < n * F; ++k) G[k] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double* g = Gnext + i * F;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            double den = sqrt(deg[i] * deg[j]);
            double a = den > 0.0 ? val[p] / den : 0.0;
            double* o = G + j * F;
            for (int64_t f = 0; f < F; ++f) o[f] += a * g[f];
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Importance sampling (Section 4.1).
 * ------------------------------------------------------------------------------------------- */

/* Philox4x32-10 as published (SC 2011): ten rounds; a round multiplies words 0 and 2 of the counter
 * by two fixed odd constants, the high halves are mixed with the other two words and the key, the
 * low halves pass through; the key grows by two Weyl constants after every round. */
void e2eg_oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 64 random bits of draw t of node u at hop h under a 64-bit seed: counter (t, u, h, 0), key =
 * the two halves of the seed, words 0 (low) and 1 (high) of the output. */
static uint64_t draw_bits(uint64_t seed, uint32_t hop, uint32_t node, uint32_t t) {
    uint32_t ctr[4] = {t, node, hop, 0u}, key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)}, out[4];
    e2eg_oracle_philox4x32_10(ctr, key, out);
    return (uint64_t)out[0] | ((uint64_t)out[1] << 32);
}

/* w^beta for every stored entry (the numerator of the sampling probability). */
void e2eg_oracle_sampling_weights(int64_t nnz, const double* val, double beta, double* p) {
    for (int64_t e = 0; e < nnz; ++e) p[e] = val[e] > 0.0 ? pow(val[e], beta) : 0.0;
}

/* Integer form of one row's distribution, decided in single precision: q_e = floor(p_e / pmax * 2^24),
 * at least 1 where p_e > 0; the diagonal entry, entries that are not positive and entries that are
 * not finite get 0 (a node is not its own neighbour), and pmax is the largest usable p of the row. */
void e2eg_oracle_sampling_table(int64_t n, const int64_t* row_ptr, const int32_t* col_idx, const float* p,
                                uint64_t* q) {
    for (int64_t i = 0; i < n; ++i) {
        float pmax = 0.0f;
        for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e)
            if (col_idx[e] != i && p[e] > 0.0f && p[e] <= 3.402823466e38f && p[e] > pmax) pmax = p[e];
        for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            q[e] = 0;
            if (col_idx[e] != i && p[e] > 0.0f && p[e] <= 3.402823466e38f) {
                float scaled = floorf(p[e] / pmax * 16777216.0f);
                q[e] = scaled >= 1.0f ? (uint64_t)scaled : 1u;
            }
        }
    }
}

/*
 * Multi-hop sampling from `n_seeds` seed nodes with fan-out fanout[h] at hop h = 0..L-1.
 * hop_of[v] (output, [n]) = 0 if v is not in the subgraph, 1 for a seed, h + 2 for a node first
 * reached at hop h.  The frontier of hop 0 is the set of seeds, that of hop h + 1 the nodes first
 * reached at hop h; a frontier is walked in ascending node order, the draws of a node in order of
 * their index.  Every pick is written as (source node, picked neighbour, index of the stored entry);
 * returns the number of picks (never more than `cap` are written).
 */
int64_t e2eg_oracle_sample_subgraph(int64_t n, const int64_t* row_ptr, const int32_t* col_idx, const uint64_t* q,
                                    int64_t n_seeds, const int32_t* seeds, int32_t L, const int32_t* fanout,
                                    uint64_t seed, int32_t* hop_of, int32_t* src, int32_t* dst, int64_t* entry,
                                    int64_t cap) {
    int64_t picks = 0;
    for (int64_t v = 0; v < n; ++v) hop_of[v] = 0;
    for (int64_t s = 0; s < n_seeds; ++s) hop_of[seeds[s]] = 1;
    for (int32_t h = 0; h < L; ++h) {
        const int64_t k = fanout[h];
        for (int64_t u = 0; u < n; ++u) {
            if (hop_of[u] != h + 1) continue;
            const int64_t beg = row_ptr[u], end = row_ptr[u + 1];
            int64_t neighbours = 0;             /* stored entries other than the node itself */
            for (int64_t x = beg; x < end; ++x) neighbours += col_idx[x] != u;
            uint64_t total = 0;
            for (int64_t x = beg; x < end; ++x) total += q[x];
            /* at most k neighbours: every one that can be drawn at all, in stored order;
             * more: k independent draws, draw t from the random bits of (seed, hop, node, t) */
            const int64_t tries = neighbours <= k ? end - beg : k;
            for (int64_t t = 0; t < tries; ++t) {
                int64_t e = -1;
                if (neighbours <= k) {
                    if (q[beg + t] > 0) e = beg + t;
                } else if (total > 0) {
                    /* r uniform on [0, total): the high half of the 128-bit product bits * total */
                    uint64_t r = (uint64_t)(((unsigned __int128)draw_bits(seed, (uint32_t)h, (uint32_t)u, (uint32_t)t) * total) >> 64);
                    uint64_t acc = 0;
                    for (int64_t x = beg; x < end; ++x) {
                        acc += q[x];
                        if (acc > r) { e = x; break; }
                    }
                }
                if (e < 0) continue;
                const int32_t v = col_idx[e];
                if (hop_of[v] == 0) hop_of[v] = h + 2;
                if (picks < cap) { src[picks] = (int32_t)u; dst[picks] = v; entry[picks] = e; }
                ++picks;
            }
        }
    }
    return picks;
}
