/*
 * e2eg: normalized-adjacency message passing on a user-item interaction graph,
 * for AMD MI355X (gfx950).  C ABI of libe2eg.so.
 *
 * The operator (paper: Section 3, "Notation"): for an undirected graph with adjacency A
 * (A_ij > 0 iff (i,j) is an edge), A~ = A + I, D~ = D + I with D = diag(A 1), and
 *     A^ = D~^-1/2 A~ D~^-1/2 .
 * The path (Section 3.1, LightGCN in matrix form): H(l+1) = A^ H(l), l = 0..K-1, with K equal
 * to the number of sampled hops (Section 5), and its backward G(l) = A^T G(l+1) (Appendix A,
 * the "GNN backprop" factor; Section 4.3.2, the J^T dL/dF_gnn terms).  An optional dense
 * per-layer update H' = relu(P W) follows the generic message-passing layer's update function
 * psi and the W, sigma of the GraphSAGE layer (Section 3, Section 3.1).
 *
 * Conventions for every entry point
 *   - Nodes: users are 0 .. n_users-1, item i is node n_users + i; n = n_users + n_items.
 *   - All `d_` pointers are DEVICE pointers, all `h_` pointers HOST pointers.  The caller owns
 *     every buffer; the library allocates no device memory and keeps no state between calls.
 *     Inputs are never written.  Scratch memory is passed in as (ws, ws_bytes); the matching
 *     *_workspace_bytes() query is a pure host function.  Workspace must be 256-byte aligned.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Work is enqueued on it and the
 *     call returns without waiting, except e2eg_build_csr, which waits once to return nnz.
 *   - Feature matrices are row-major [n][F] with a leading dimension (in elements) >= F.
 *     dtype E2EG_F32: float.  dtype E2EG_BF16: bfloat16 bit patterns (uint16); arithmetic is
 *     fp32 and each stored layer is the fp32 result rounded to nearest-even once.  Between the
 *     layers of one call the next layer's input is kept in the workspace as d~^-1/2 H(l) in the
 *     storage type: the same fp32 result, scaled, with a rounding of its own (not the stored H(l)
 *     re-read), so a K-layer call and K one-layer calls agree to rounding, not bit for bit.
 *     F must be a multiple of 4 (fp32) or 8 (bf16), leading dimensions too, and base pointers
 *     16-byte aligned.
 *   - Return value: E2EG_OK or a negative E2EG_ERR_* code; e2eg_last_error() gives a
 *     thread-local message for the last failure on the calling thread.  Argument errors are
 *     found on the host before anything is enqueued.  No C++ exception crosses this boundary.
 */
#ifndef E2EG_H
#define E2EG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define E2EG_OK 0
#define E2EG_ERR_INVALID_ARG (-1) /* a size, flag, stride or alignment is not acceptable     */
#define E2EG_ERR_NULL_PTR (-2)    /* a required pointer is NULL                              */
#define E2EG_ERR_BAD_DTYPE (-3)   /* dtype is not one of E2EG_F32 / E2EG_BF16, or unsupported */
#define E2EG_ERR_CAPACITY (-4)    /* an output buffer is smaller than the result             */
#define E2EG_ERR_OVERFLOW (-5)    /* n or nnz would not fit in int32                         */
#define E2EG_ERR_WORKSPACE (-6)   /* ws is NULL, misaligned or smaller than the query says   */
#define E2EG_ERR_HIP (-7)         /* a HIP runtime call failed; see e2eg_last_error()        */
#define E2EG_ERR_BAD_INDEX (-8)   /* an input id is outside its range (found on the device)  */

#define E2EG_F32 0
#define E2EG_BF16 1

#define E2EG_ADD_SELF_LOOPS 1 /* build_csr flag bit 0: build A~ = A + I (else A itself) */

#define E2EG_AGG_SYM 0    /* D^-1/2 M D^-1/2 of the stored structure M (A^ when built with self-loops)  */
#define E2EG_AGG_MEAN 1   /* D^-1 M: the mean over each row's neighbours (0 for an empty row)          */
#define E2EG_AGG_MEAN_T 2 /* M D^-1: the transpose of E2EG_AGG_MEAN on a symmetric structure           */
#define E2EG_AGG_SUM 3    /* M itself: the plain neighbour sum                                          */

#define E2EG_TRANSFORM_FWD 0
#define E2EG_TRANSFORM_BWD 1

const char* e2eg_status_string(int32_t status);
const char* e2eg_last_error(void);
int32_t e2eg_version(void);

/* ------------------------------------------------------------------------------------------
 * e2eg_build_csr: structure of A~ = A + I (Section 3, "Notation") in CSR.
 *
 * Input: n_edges pairs (d_user_ids[e], d_item_ids[e]), user ids in [0, n_users), item ids in
 * [0, n_items), any order, repeats allowed (a repeated pair is one edge: A_ij > 0 iff (i,j) in E).
 * Each pair gives the two entries (u, n_users+i) and (n_users+i, u).  With E2EG_ADD_SELF_LOOPS
 * every node also gets its diagonal entry.
 * Output: d_row_ptr[n+1] (d_row_ptr[0] = 0) and d_col_idx[nnz], columns strictly ascending in
 * each row; *h_nnz_out = nnz.  col_capacity (entries) must be >= 2*n_edges + n (the bound
 * without knowing how many pairs repeat); fewer entries may be written.
 * Errors: OVERFLOW if n or 2*n_edges + n exceeds INT32_MAX; CAPACITY; WORKSPACE; BAD_INDEX if
 * an id is out of range (outputs are then unspecified).  Waits for the stream once.
 */
size_t e2eg_build_csr_workspace_bytes(int32_t n_users, int32_t n_items, int64_t n_edges);
int32_t e2eg_build_csr(int32_t n_users, int32_t n_items, int64_t n_edges,
                       const int32_t* d_user_ids, const int32_t* d_item_ids, int32_t flags,
                       int32_t* d_row_ptr, int32_t* d_col_idx, int64_t col_capacity,
                       int64_t* h_nnz_out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_normalize: D~ and D~^-1/2 (Section 3, "Notation"), plus the launch schedule.
 *
 * d_deg[i] = d~_i = sum_j A~_ij = d_row_ptr[i+1] - d_row_ptr[i]  (for a CSR built without
 * self-loops this is |N(i)|, the count the per-node LightGCN update of Section 3.1 uses);
 * d_dinv_sqrt[i] = (float)(1 / sqrt((double) d~_i)), and 0 for an empty row.
 * d_sched (sched_bytes >= e2eg_sched_bytes(n, nnz), 256-byte aligned) receives the row
 * schedule that e2eg_propagate_* read: rows cut into segments of bounded length so that
 * power-law rows spread over many wavefronts, the segments ordered by their first column
 * (d_col_idx is read for that).  Its content is private to the library and valid for this
 * (d_row_ptr, d_col_idx, n, nnz) only.  d_deg may be NULL.
 */
size_t e2eg_sched_bytes(int32_t n, int64_t nnz);
size_t e2eg_normalize_workspace_bytes(int32_t n, int64_t nnz);
int32_t e2eg_normalize(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                       const int32_t* d_col_idx, int32_t* d_deg, float* d_dinv_sqrt,
                       void* d_sched, size_t sched_bytes, void* ws, size_t ws_bytes, void* stream);

/* e2eg_sched_check_symmetric: may the transposed entry points (e2eg_propagate_bwd,
 * e2eg_propagate_weighted_bwd, e2eg_aggregate with E2EG_AGG_MEAN_T) run on this schedule?  They
 * apply the stored operator itself, which equals its transpose (Appendix A: the backward pass
 * multiplies by A^T) only when every stored entry (i, j) has its mirror (j, i) - and, on a weighted
 * graph, the same value there.  e2eg_normalize / e2eg_normalize_weighted test this while they build
 * the schedule and keep the answer in it; this call copies it to the host.  Waits for the stream
 * once.  Returns E2EG_OK if symmetric, E2EG_ERR_INVALID_ARG (with a message) if not.  Everything
 * e2eg_build_csr and e2eg_edge_weights produce is symmetric, so callers on that path need not ask.
 */
int32_t e2eg_sched_check_symmetric(const void* d_sched, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_propagate_fwd: H(l+1) = A^ H(l), l = 0..K-1, H(0) = X0 (Section 3.1, matrix form).
 *
 * (A^ H)_i = s_i * sum_{j in row i} s_j H_j with s = d_dinv_sqrt; accumulation in fp32.
 * d_X0 [n][F] (ldx).  d_Xout receives layers 1..K: layer l at d_Xout + (l-1)*layer_stride
 * elements, each [n][F] with leading dimension ldo.  layer_stride == 0 keeps only H(K) (written
 * at d_Xout); otherwise layer_stride >= n*ldo.  Every stored layer is written exactly once.
 * d_Xout must not overlap d_X0.  K >= 1.
 */
size_t e2eg_propagate_workspace_bytes(int32_t n, int64_t nnz, int32_t dtype, int32_t F, int32_t K);
int32_t e2eg_propagate_fwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                           const int32_t* d_col_idx, const float* d_dinv_sqrt,
                           const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                           const void* d_X0, int64_t ldx, void* d_Xout, int64_t ldo,
                           int64_t layer_stride, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_propagate_bwd: the transpose-Jacobian of e2eg_propagate_fwd (Appendix A, "GNN
 * backprop"; Section 4.3.2, J^T dL/dF_gnn).
 *
 * G(K) = d_gXK;  G(l) = A^T G(l+1) + D(l) for l = K-1 .. 0, where D(l) is the optional direct
 * gradient on layer l (a loss that reads intermediate layers), D(0) = 0; output d_gX0 = G(0).
 * d_gLayers == NULL means no direct terms; else layer l (1 <= l <= K-1) is at
 * d_gLayers + (l-1)*g_layer_stride elements with leading dimension ldg.
 * g_layer_stride == 0 means ONE array [n][F] (ldg) that is the direct term of every layer
 * l = 0 .. K-1, layer 0 included: the backward of a loss that reads all layers with equal weight
 * (the mean readout of e2eg_readout_mean, with d_gXK holding the same array for layer K).
 * The CSR must be structurally symmetric (everything e2eg_build_csr produces is), so that
 * A^T = A^ and the same row schedule serves.  e2eg_normalize finds out on the device and records it
 * in the schedule: on a schedule whose structure is not symmetric this call still returns E2EG_OK
 * (it reads nothing back) but every element of d_gX0 comes out NaN.  e2eg_sched_check_symmetric
 * gives the same verdict to the host as a status code.
 */
int32_t e2eg_propagate_bwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                           const int32_t* d_col_idx, const float* d_dinv_sqrt,
                           const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                           const void* d_gXK, int64_t ldg, const void* d_gLayers,
                           int64_t g_layer_stride, void* d_gX0, int64_t ldo, void* ws,
                           size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_aggregate: one neighbourhood aggregation  Y = S_out M S_in X (+ addend)  over the stored
 * structure M (d_row_ptr / d_col_idx and the schedule e2eg_normalize made for them), with diagonal
 * scales chosen by `mode` from the row lengths d_i:
 *   E2EG_AGG_MEAN   the mean aggregator of the GraphSAGE layer (Section 3.1),
 *                   hbar_u = 1/|S(u)| sum_{v in S(u)} h_v, with S(u) = row u of a structure built
 *                   WITHOUT self-loops (the sampled neighbours); an empty row gives 0;
 *   E2EG_AGG_MEAN_T its transpose, for the backward (the structure must be symmetric: on a schedule
 *                   that e2eg_normalize found not to be, the result is all NaN);
 *   E2EG_AGG_SYM    d_i^-1/2 d_j^-1/2 weights: one layer of e2eg_propagate_fwd;
 *   E2EG_AGG_SUM    no scaling.
 * d_X [n][F] (ldx) in, d_Y [n][F] (ldy) out, must not overlap; d_addend (may be NULL) [n][F]
 * (ld_add) is added to the result before it is stored (it may be d_Y's neighbour in a wider
 * array but must not overlap d_Y).  ldy > F lets the result land in one half of a CONCAT buffer.
 * fp32 accumulation, one rounding to the storage type.
 */
size_t e2eg_aggregate_workspace_bytes(int32_t n, int64_t nnz, int32_t dtype, int32_t F);
int32_t e2eg_aggregate(int32_t mode, int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                       const int32_t* d_col_idx, const void* d_sched, int32_t dtype, int32_t F,
                       const void* d_X, int64_t ldx, const void* d_addend, int64_t ld_add, void* d_Y,
                       int64_t ldy, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_layer_transform: the dense per-layer update (update function psi of the generic
 * message-passing layer with the W, sigma of the GraphSAGE layer; Section 3, Section 3.1).
 *
 * mode E2EG_TRANSFORM_FWD:  Z = P W, H = relu ? max(Z, 0) : Z.
 *     d_P [n][Fin] (ld Fin), d_W [Fin][Fout] row-major (input x output), d_H [n][Fout] out.
 *     d_gH, d_gP, d_gW are ignored.
 * mode E2EG_TRANSFORM_BWD:  dZ = relu ? d_gH * [H > 0] : d_gH;  dP = dZ W^T;  dW = P^T dZ.
 *     d_H is the forward output (its sign pattern is that of Z); d_gP [n][Fin] out;
 *     d_gW [Fin][Fout] fp32 out (overwritten, not accumulated).  d_gP or d_gW may be NULL
 *     to skip that product.
 * dtype E2EG_BF16 only (bf16 MFMA, fp32 accumulate); Fin and Fout multiples of 32, <= 256.
 * With d_P = CONCAT(h, hbar) ([n][2F], hbar written there by e2eg_aggregate) and d_W [2F][Fout]
 * this is the update of the GraphSAGE layer, h' = sigma(W . CONCAT(h, hbar)) (Section 3.1).
 */
size_t e2eg_layer_transform_workspace_bytes(int32_t mode, int32_t n, int32_t Fin, int32_t Fout,
                                            int32_t dtype);
int32_t e2eg_layer_transform(int32_t mode, int32_t n, int32_t Fin, int32_t Fout, int32_t dtype,
                             int32_t relu, const void* d_P, const void* d_W, void* d_H,
                             const void* d_gH, void* d_gP, float* d_gW, void* ws,
                             size_t ws_bytes, void* stream);

/* e2eg_layer_transform_noalloc: e2eg_layer_transform, argument for argument, without (ws, ws_bytes),
 * for callers that cannot allocate device memory or pass a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The partial weight-gradient
 * matrices of the backward mode go to a static device array inside the library instead, of
 * E2EG_TRANSFORM_STATIC_SCRATCH_BYTES (16 MiB) on every GPU the library runs on, held until the
 * process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 * Limit: e2eg_layer_transform_workspace_bytes(mode, n, Fin, Fout, dtype) must not exceed that size
 * (128 x 128 weights: any n; 256 x 256: n up to 8192), else E2EG_ERR_CAPACITY and nothing is
 * enqueued.  Results are those of e2eg_layer_transform bit for bit (same kernels, same order).
 * All calls on one GPU share the one array: two calls whose kernels may overlap on that GPU (different
 * streams, or threads) race on it; calls on one stream are ordered and safe.  The first call on each
 * device looks up the array's address and should be made outside graph capture.
 */
#define E2EG_TRANSFORM_STATIC_SCRATCH_BYTES (16u << 20)
int32_t e2eg_layer_transform_noalloc(int32_t mode, int32_t n, int32_t Fin, int32_t Fout, int32_t dtype,
                                     int32_t relu, const void* d_P, const void* d_W, void* d_H,
                                     const void* d_gH, void* d_gP, float* d_gW, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_readout_mean: layer combination of LightGCN (Section 3.1): the final representation is
 * the mean of all layers,  Y = 1/(K+1) * (H(0) + H(1) + ... + H(K)).
 *
 * d_X0 = H(0) [n][F] (ldx); d_layers holds H(1..K) as e2eg_propagate_fwd stores them with a
 * non-zero layer_stride: layer l at d_layers + (l-1)*layer_stride elements, leading dimension ld
 * (layer_stride is not looked at when K <= 1; d_layers may be NULL when K == 0).  d_Y [n][F] (ldy)
 * must not overlap the inputs.  fp32 arithmetic, one rounding to the storage type.
 */
int32_t e2eg_readout_mean(int32_t n, int32_t dtype, int32_t F, int32_t K, const void* d_X0, int64_t ldx,
                          const void* d_layers, int64_t ld, int64_t layer_stride, void* d_Y,
                          int64_t ldy, void* stream);

/* ------------------------------------------------------------------------------------------
 * e2eg_gfae_loss: the graph feature auto-encoder loss with the identity decoder (Section 4.2),
 *     L_ssl = || X - Y ||_F^2 ,
 * X the input features and Y the encoder output, and its gradient with respect to Y.
 *
 * *d_loss (a DEVICE double) receives the loss, summed in double in a fixed order (the value is
 * reproducible).  If d_gY is not NULL it receives grad_scale * dL/dY = grad_scale * 2 (Y - X) in
 * the storage type (ldg); grad_scale carries whatever constant factors follow (a task weight,
 * the 1/(K+1) of the mean readout).  d_gY must not overlap d_X or d_Y.  The gradient with respect
 * to X itself, when X is a trainable embedding, is the negative of the (unscaled) d_gY.
 */
size_t e2eg_gfae_loss_workspace_bytes(int32_t n, int32_t F);
int32_t e2eg_gfae_loss(int32_t n, int32_t dtype, int32_t F, const void* d_X, int64_t ldx, const void* d_Y,
                       int64_t ldy, double* d_loss, void* d_gY, int64_t ldg, float grad_scale, void* ws,
                       size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * GradNorm task weighting (Section 4.3.1).  The gradient norms are taken with respect to the
 * shared input features h(0): G_i = || grad_{h(0)} (w_i L_i) ||_2 = w_i || grad_{h(0)} L_i ||_2.
 *
 * e2eg_block_norms: the per-task gradients grad_{h(0)} L_i, i = 0..T-1, stand side by side as the
 * column blocks of d_G [n][T*F] (ld) - which is how one call of e2eg_propagate_bwd on T stacked
 * upstream gradients leaves them.  d_norms (DEVICE double[T]) receives the 2-norm of each block,
 * summed in double in a fixed order.  1 <= T <= 8.
 *
 * e2eg_gradnorm_step: host arithmetic on host arrays of length T.  With r_i = (L_i / L_i(0)) /
 * mean_j (L_j / L_j(0)) and Gbar = mean_i w_i gnorm_i, the meta-loss is sum_i |w_i gnorm_i - Gbar
 * r_i^gamma|; its derivative in w_i with the targets Gbar r_i^gamma held constant is
 * sign(w_i gnorm_i - Gbar r_i^gamma) gnorm_i.  h_w takes one step of size lr against it, is kept
 * positive (floor 1e-8) and rescaled so that sum_i w_i = T.  *h_meta_loss (may be NULL) receives the
 * meta-loss at the weights passed in.  Initial losses and weights must be positive.
 */
size_t e2eg_block_norms_workspace_bytes(int32_t n, int32_t F, int32_t T);
int32_t e2eg_block_norms(int32_t n, int32_t dtype, int32_t F, int32_t T, const void* d_G, int64_t ld,
                         double* d_norms, void* ws, size_t ws_bytes, void* stream);
int32_t e2eg_gradnorm_step(int32_t T, const double* h_loss, const double* h_loss0, const double* h_gnorm,
                           double gamma, double lr, double* h_w, double* h_meta_loss);

/* ------------------------------------------------------------------------------------------
 * Weighted graphs: A_ij is the strength of edge (i,j) instead of 1 (Section 3, "Notation": A is
 * nonnegative and A_ij > 0 marks an edge; D = diag(A 1), D~ = D + I, A^ = D~^-1/2 (A + I) D~^-1/2).
 * The structure is the one e2eg_build_csr makes (with E2EG_ADD_SELF_LOOPS); the values live in a
 * float array d_val[nnz] beside d_col_idx.
 *
 * e2eg_edge_weights: fills d_val for the CSR that e2eg_build_csr made from the same pairs:
 * 1 on every diagonal entry, d_weights[e] on the two entries of pair e; a pair listed several
 * times keeps the largest of its weights (the reading taken here: the structure already treats
 * repeats as one edge).  A weight that is not > 0 (NaN included) is ignored, and so is a pair whose
 * ids are out of range or that the CSR does not hold; an entry that no pair reaches stays 0.
 * Integer atomics only: the result does not depend on the order of the pairs.  Does not wait.
 *
 * e2eg_normalize_weighted: e2eg_normalize for such a graph.  d_deg[i] (may be NULL) = the number of
 * stored entries of row i; d_deg_w[i] (may be NULL) = d~_i = the sum of row i of d_val, added in
 * double in a fixed order; d_dinv_sqrt[i] = (float)(1 / sqrt(d~_i)), 0 where the sum is not positive.  d_sched needs e2eg_sched_weighted_bytes(n, nnz)
 * bytes: the unweighted schedule followed by the values in the library's own entry order.  Each
 * row must hold a column at most once (a repeat leaves one of the values out).  The workspace is
 * that of e2eg_normalize.
 *
 * e2eg_propagate_weighted_fwd / _bwd: e2eg_propagate_fwd / _bwd, argument for argument, on a
 * schedule made by e2eg_normalize_weighted; each gathered row is multiplied by its entry's value
 * (fp32 fused multiply-add).  The backward pass applies the same operator, so the values must
 * be symmetric, val(i,j) = val(j,i), which e2eg_edge_weights guarantees; e2eg_normalize_weighted
 * records whether they are, and the backward pass on a schedule where they are not returns all NaN
 * (see e2eg_propagate_bwd and e2eg_sched_check_symmetric).
 * Passing a schedule of the other kind to either family is an error the library cannot detect.
 */
int32_t e2eg_edge_weights(int32_t n_users, int32_t n_items, int64_t n_edges, const int32_t* d_user_ids,
                          const int32_t* d_item_ids, const float* d_weights, int64_t nnz,
                          const int32_t* d_row_ptr, const int32_t* d_col_idx, float* d_val, void* stream);
size_t e2eg_sched_weighted_bytes(int32_t n, int64_t nnz);
int32_t e2eg_normalize_weighted(int32_t n, int64_t nnz, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                                const float* d_val, int32_t* d_deg, float* d_deg_w, float* d_dinv_sqrt,
                                void* d_sched, size_t sched_bytes, void* ws, size_t ws_bytes, void* stream);
int32_t e2eg_propagate_weighted_fwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                    const int32_t* d_col_idx, const float* d_dinv_sqrt,
                                    const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                                    const void* d_X0, int64_t ldx, void* d_Xout, int64_t ldo,
                                    int64_t layer_stride, void* ws, size_t ws_bytes, void* stream);
int32_t e2eg_propagate_weighted_bwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                    const int32_t* d_col_idx, const float* d_dinv_sqrt,
                                    const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                                    const void* d_gXK, int64_t ldg, const void* d_gLayers,
                                    int64_t g_layer_stride, void* d_gX0, int64_t ldo, void* ws,
                                    size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Importance sampling of a multi-hop subgraph (Section 4.1: neighbour v of u is drawn with
 * probability w_uv^beta / sum_k w_uk^beta, at most k neighbours per node, depth L; Section 5,
 * "Subgraph Sampling": one fan-out per hop).  The parent graph is a CSR from e2eg_build_csr (users
 * are nodes [0, n_users), items the rest) with values as for the weighted path.  The result is the
 * step before the path: local (user, item) pairs ready for e2eg_build_csr.
 *
 * e2eg_sampling_weights: d_p[e] = d_val[e]^beta where d_val[e] > 0, else 0 (beta >= 0; beta = 1
 * copies, beta = 0 gives the uniform sampler).
 *
 * e2eg_sampler_prepare: the sampling table of a graph, made once per graph.  Each row's weights d_p
 * become integers, floor(p / pmax * 2^24) with pmax the row's largest usable weight, decided in fp32
 * with IEEE rounding, at least 1 where p > 0; the diagonal entry and entries that are not positive
 * and finite get 0 and are never drawn.  d_table (e2eg_sampler_table_bytes(nnz), 256-byte aligned)
 * receives their running sums over the whole CSR (nnz + 1 values of 64 bits).  The workspace
 * (e2eg_sampler_prepare_workspace_bytes(n, nnz)) holds the row maxima and the scan's partial sums.
 *
 * e2eg_sample_subgraph: hop h = 0..L-1 expands its frontier (hop 0: the distinct seeds; hop h+1:
 * the nodes first reached at hop h), each frontier node u with fan-out k = h_fanout[h] (HOST array):
 * a node with at most k neighbours (stored entries other than its own diagonal one) keeps every one
 * that can be drawn; otherwise k independent draws are made, draw t taking r = floor(bits * total / 2^64) with bits = words 0 (low) and 1 (high)
 * of Philox4x32-10 at counter (t, u, h, 0) under key (seed low half, seed high half), and picking the
 * first entry whose running sum within the row exceeds r.  Equal draws are kept as equal pairs
 * (e2eg_build_csr counts a repeated pair once).
 * Outputs: d_nodes = the global ids of the subgraph's nodes in ascending order (local id = position;
 * users come first); the picks in order (hop, frontier node ascending, draw) as local pairs
 * d_edge_users / d_edge_items (item ids counted from 0) and, if d_edge_w is not NULL, the value
 * d_val[entry] of each; h_counts (HOST int32[3]) = local users, local items, pairs.
 * node_capacity >= min(n, n_seeds + C) and edge_capacity >= C with C = e2eg_sample_capacity(...)
 * (the number of draws the fan-outs allow), else CAPACITY.  1 <= L <= 8, fan-outs in [1, 65536].
 * Errors: BAD_INDEX for a seed out of range or a stored entry that joins two users or two items
 * (outputs then unspecified).  Integer arithmetic only: the result depends on the inputs and the
 * seed alone.  Waits for the stream once, at the end.
 */
int32_t e2eg_sampling_weights(int64_t nnz, const float* d_val, float beta, float* d_p, void* stream);
size_t e2eg_sampler_table_bytes(int64_t nnz);
size_t e2eg_sampler_prepare_workspace_bytes(int32_t n, int64_t nnz);
int32_t e2eg_sampler_prepare(int32_t n, int64_t nnz, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                             const float* d_p, void* d_table, size_t table_bytes, void* ws, size_t ws_bytes,
                             void* stream);
int64_t e2eg_sample_capacity(int32_t n, int32_t n_seeds, int32_t L, const int32_t* h_fanout);
size_t e2eg_sample_subgraph_workspace_bytes(int32_t n, int32_t n_seeds, int32_t L, const int32_t* h_fanout);
int32_t e2eg_sample_subgraph(int32_t n_users, int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                             const int32_t* d_col_idx, const void* d_table, const float* d_val,
                             int32_t n_seeds, const int32_t* d_seeds, int32_t L, const int32_t* h_fanout,
                             uint64_t seed, int32_t* d_nodes, int64_t node_capacity, int32_t* d_edge_users,
                             int32_t* d_edge_items, float* d_edge_w, int64_t edge_capacity, int32_t* h_counts,
                             void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Measurement aid (not part of the path): per-launch duration of the neighbour-sum kernel, the
 * kernel that moves nearly all bytes of e2eg_propagate_*.  Between e2eg_profile_begin() and
 * e2eg_profile_end() every launch of that kernel made by the calling thread is bracketed by a
 * pair of HIP events on its own stream (up to `capacity` launches; later ones are not timed).
 * e2eg_profile_end() waits for the recorded events, writes up to h_capacity durations in
 * milliseconds (launch order) to h_ms, stores the number recorded in *h_count and switches
 * recording off.  Uses host memory and HIP events only.
 */
int32_t e2eg_profile_begin(int32_t capacity);
int32_t e2eg_profile_end(float* h_ms, int32_t h_capacity, int32_t* h_count);

/* Measurement aid: a plain streaming copy of nbytes device bytes (a multiple of 16, both pointers
 * 16-byte aligned, buffers must not overlap), one kernel (copy_bytes16) enqueued on `stream`.  It
 * reads nbytes and writes nbytes: the traffic of known size against which the profiler's HBM
 * byte counters are scaled. */
int32_t e2eg_profile_copy(void* d_dst, const void* d_src, size_t nbytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* E2EG_H */
