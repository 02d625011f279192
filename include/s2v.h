/*
 * s2v.h -- C interface of the MI355X (gfx950) structure2vec / deep-Q hot-path library.
 *
 * The library evaluates the policy model of OpenGraphGym-MG (arXiv 2105.08764) on one
 * GPU: the structure2vec graph embedding (Eq. 1 / Alg. 1), the action-evaluation
 * scores (Eq. 2 / Alg. 2), node selection (Alg. 3's argmax and the top-d rule of
 * Sec. 4.5.1), and the training step's backward pass and parameter update (the Train
 * function of Alg. 4, repeated as in Sec. 4.5.2).
 *
 * Parameter numbering.  This interface uses the structure2vec numbering; the paper
 * renumbers the same seven tensors:
 *     here    role                                   shape   paper's name
 *     theta1  weight of the node feature x_v         [p]     theta1
 *     theta2  weight of the neighbour-embedding sum  [p][p]  theta4
 *     theta3  outer weight of the edge term          [p][p]  theta3
 *     theta4  lift of the edge weight (inside relu)  [p]     theta2
 *     theta5  output vector of the score             [2p]    theta7
 *     theta6  weight of the graph sum in the score   [p][p]  theta5
 *     theta7  weight of the node's own embedding     [p][p]  theta6
 * 4p^2 + 4p values in total (Sec. 5.1 item 3).  Matrices are row-major [out][in] and
 * act on column vectors, y = theta * v, as Eq. 1 and Eq. 2 are written.
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller (allocated and freed by
 *     the caller) unless the comment says "host".  The structs themselves are host
 *     memory.  The library allocates no device memory: scratch space comes from the
 *     caller's workspace `ws`, sized by s2v_workspace_bytes.
 *   - Work is enqueued on the HIP stream given to s2v_create and the call returns
 *     without waiting for it; scalar results (loss, counts) are written to device memory.
 *     Four calls do wait for the stream: s2v_graph_prepare, s2v_workspace_bytes,
 *     s2v_mvc_inference and s2v_profile_end.  All others only enqueue kernels and
 *     device-to-device copies, so they may be recorded under HIP stream capture and replayed.
 *   - Every call returns an int32 status: S2V_OK or a negative S2V_ERR_* code.  Nothing
 *     throws, prints or exits.  A call that returns an error has enqueued nothing.
 *   - Layouts: x is [S][N]; embeddings are [N][S][p] (S states of one graph batch;
 *     S == 1 gives [N][p]); saved activations [T][N][S][p]; scores [S][N];
 *     graph sums [S][G][p].  N * S must be below 2^31.
 *   - Supported embedding sizes: p = 32 or 64.
 *   - Calls on one context must not overlap in time on different host threads, and two
 *     calls that share a workspace must run on the same stream.
 */
#ifndef S2V_H
#define S2V_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define S2V_OK 0
#define S2V_ERR_INVALID_ARG (-1)         /* null pointer, negative size, inconsistent shapes */
#define S2V_ERR_UNSUPPORTED (-2)         /* p not in {32, 64}; (G > 1 and k > 1) in selection */
#define S2V_ERR_WORKSPACE_TOO_SMALL (-3) /* ws_bytes below what s2v_workspace_bytes reports */
#define S2V_ERR_HIP (-4)                 /* a HIP call failed; see s2v_last_hip_error */
#define S2V_ERR_NO_DEVICE (-5)           /* no usable GPU in this process */
#define S2V_ERR_NOT_PREPARED (-6)        /* s2v_graph_prepare has not run for this graph + workspace */
#define S2V_ERR_TOO_LARGE (-7)           /* s2v_select_topk_noalloc: n_nodes or k beyond its fixed maximum */

typedef struct s2v_ctx s2v_ctx;

/*
 * A graph, or a block-diagonal batch of G independent graphs (the paper stacks B graphs,
 * Sec. 4.1; here they need not have equal size).  The adjacency matrix A of Sec. 4.1 is
 * held as a symmetric CSR pattern: every undirected edge {u,v} appears in row u and in
 * row v.  The neighbourhood N(v) of Eq. 1 is exactly the stored entries of row v.
 * Symmetry, sortedness and the absence of duplicates are the caller's promise; they are
 * not checked.  Column indices must lie in [0, n_nodes).
 */
typedef struct {
    int32_t n_nodes;          /* N >= 0 */
    int64_t nnz;              /* stored entries = 2 * undirected edges */
    const int32_t *rowptr;    /* device [N+1], rowptr[0] == 0, rowptr[N] == nnz */
    const int32_t *colidx;    /* device [nnz] */
    const float *w;           /* device [nnz] edge weights W(v,u) of Eq. 1, or NULL = all 1.0 */
    int32_t n_graphs;         /* G >= 1 */
    const int32_t *graph_off; /* device [G+1] ascending node offsets (0 .. N), or NULL when G == 1 */
    const int32_t *row_end;   /* device [N]: one past the last LIVE entry of each row, rowptr[v] <= row_end[v]
                                 <= rowptr[v+1], or NULL = every stored entry is live.  Used by the inference
                                 loop, whose rows shrink as nodes join the solution (s2v_residual_update). */
    int32_t state_residual;   /* non-zero: in s2v_embed_fwd / s2v_embed_bwd every state b lives on its OWN residual
                                 graph: the edges with an endpoint v that has x[b][v] != 0 are absent for that state
                                 (the sub-graphs the paper's Tuples2Graphs rebuilds for a training minibatch, Alg. 4);
                                 such nodes stay as isolated nodes.  Nothing is copied or edited: the states share
                                 this CSR.  Zero: all states use the stored graph as it is. */
    int32_t weighted_sum;     /* non-zero: the neighbour sum of Eq. 1 (second term) weights neighbour u of v by w(u, v),
                                 i.e. the aggregation step of Alg. 1 read as a product with the weighted adjacency
                                 matrix.  Zero (the default reading, Eq. 1 as printed): plain sum over neighbours.
                                 The edge term (third term of Eq. 1) uses w in both cases.  Applies to
                                 s2v_embed_fwd, s2v_embed_bwd and s2v_mvc_inference.  Needs w(u, v) == w(v, u). */
} s2v_graph;

/* The seven parameter tensors (device pointers), also used for their gradients. */
typedef struct {
    int32_t p;
    float *theta1; /* [p]    */
    float *theta2; /* [p][p] */
    float *theta3; /* [p][p] */
    float *theta4; /* [p]    */
    float *theta5; /* [2p]: [0:p] pairs with the graph term, [p:2p] with the node term */
    float *theta6; /* [p][p] */
    float *theta7; /* [p][p] */
} s2v_params;

/* Text for a status code (host string, never NULL). */
const char *s2v_status_str(int32_t status);

/*
 * Create a context bound to a HIP stream (`hip_stream` is a hipStream_t passed as void*;
 * NULL is the default stream) on the current device.  Host memory only.
 * Errors: S2V_ERR_INVALID_ARG (out == NULL), S2V_ERR_NO_DEVICE.
 */
int32_t s2v_create(void *hip_stream, s2v_ctx **out);
int32_t s2v_destroy(s2v_ctx *ctx);
/* hipError_t value of the last failed HIP call seen by this context (0 if none). */
int32_t s2v_last_hip_error(const s2v_ctx *ctx);

/*
 * Tuning knob of a context (no passage of the paper stands behind it: it is a property of this GPU's cache
 * hierarchy).  Embedding matrices [N][S][p] of at least `bytes` bytes (default 1.5 GiB) with S > 1 are
 * walked state by state instead of node by node (or row by row) in the rounds of Eq. 1 that read them, and
 * for S not a multiple of 16 in the reversed rounds that read rows as well, which keeps one state's rows in
 * the last-level cache.  The walks add their terms in different orders, so the last bits of the results
 * depend on which one is used; 0 forces the state-by-state walk.
 */
int32_t s2v_set_sliced_min_bytes(s2v_ctx *ctx, size_t bytes);

/*
 * Second tuning knob of a context (again a property of this GPU, not of the paper): when s2v_policy_select
 * runs the whole step as ONE kernel launch with one workgroup per graph.  That form needs every graph's
 * embedding to fit a compute unit's LDS and uses one compute unit per graph, so by default
 * (S2V_SINGLE_LAUNCH_AUTO) it is taken where it measured faster than the chain of launches: batches of at
 * least 64 graphs, graphs of at most half the LDS capacity, or p <= 32 with at least 4 graphs.
 * S2V_SINGLE_LAUNCH_ALWAYS takes it whenever the graphs fit, S2V_SINGLE_LAUNCH_NEVER never.
 * Errors: INVALID_ARG (NULL context, unknown mode).
 */
#define S2V_SINGLE_LAUNCH_AUTO 0
#define S2V_SINGLE_LAUNCH_ALWAYS 1
#define S2V_SINGLE_LAUNCH_NEVER 2
int32_t s2v_set_single_launch(s2v_ctx *ctx, int32_t mode);

/*
 * Bytes of workspace that every call below needs for this graph with embedding size p, T
 * rounds, S states and at most k_max selected nodes per call.  `training` non-zero includes
 * the scratch of s2v_embed_bwd and s2v_loss_grad (up to two [N][S][p] buffers, the relu-mask words and the
 * partial-gradient tables); leave it zero for inference.  `out` is a host pointer.
 * If ctx and g->rowptr are non-NULL the row lengths are read back from the device (the call
 * waits for the stream) and the buffers for long rows are sized exactly; with ctx == NULL or
 * rowptr == NULL only n_nodes, nnz and n_graphs are used and a safe upper bound is returned
 * (larger by up to nnz * S * p / 16 bytes).
 */
int32_t s2v_workspace_bytes(s2v_ctx *ctx, const s2v_graph *g, int32_t p, int32_t T, int32_t S,
                            int32_t k_max, int32_t training, size_t *out);

/*
 * One-time pass over a graph: the round-invariant part of Eq. 1's third term (Alg. 1
 * computes it once, before the layer loop).  Because relu(theta4_k * w) equals
 * relu(theta4_k) * max(w,0) + relu(-theta4_k) * max(-w,0), the sum over a row needs only
 * the two per-node scalars  s+_v = sum_u max(W(v,u),0)  and  s-_v = sum_u max(-W(v,u),0),
 * which are stored at the head of `ws` together with the reduction chunk table, the table of
 * long rows and, per row, the sum of s+ over the row's neighbours (what the neighbour sum of
 * round 2 comes to for a node none of whose neighbours is in the solution; used when the graph
 * has no row_end and no negative weight).  The head
 * of `ws` must stay untouched for as long as the graph is used with that workspace; the
 * other calls use the rest as scratch.  Reads graph_off back to the host, so this call
 * waits for the stream.  Call again if the graph's arrays change; a graph struct whose rowptr, colidx or w
 * pointer differs from the prepared one's is answered with S2V_ERR_NOT_PREPARED by the other calls.
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, HIP.
 */
int32_t s2v_graph_prepare(s2v_ctx *ctx, const s2v_graph *g, void *ws, size_t ws_bytes);

/*
 * Graph embedding, Eq. 1 / Alg. 1, for S states x[s][.] of the same graph batch:
 *   mu^0 = 0;  mu^{t+1}_v = relu(theta1 x_v + theta2 sum_{u in N(v)} mu^t_u
 *                                + theta3 sum_{u in N(v)} relu(theta4 W(v,u))),  t = 0..T-1.
 * The neighbour sum is unweighted, as Eq. 1 writes it.
 *   x        [S][N]  node feature (the partial-solution indicator S of Sec. 4.1; any float)
 *   mu_out   [N][S][p]  mu^T; may be NULL when mu_saved is given
 *   mu_saved [T][N][S][p] receives mu^1..mu^T (needed by s2v_embed_bwd), or NULL
 *   gsum     [S][G][p]  per-graph sum of mu^T over ALL nodes of the graph (Alg. 2 line 4),
 *                       or NULL to skip it
 * T >= 1, S >= 1.  Errors: INVALID_ARG, UNSUPPORTED, NOT_PREPARED, WORKSPACE_TOO_SMALL, HIP.
 */
int32_t s2v_embed_fwd(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                      int32_t S, float *mu_out, float *mu_saved, float *gsum, void *ws, size_t ws_bytes);

/*
 * Action-evaluation scores, Eq. 2 / Alg. 2, for EVERY node (candidates are filtered at
 * selection, not here):
 *   Q_v = theta5[0:p] . relu(theta6 g_b) + theta5[p:2p] . relu(theta7 mu_v),  b = graph of v.
 *   mu [N][S][p], gsum [S][G][p] (from s2v_embed_fwd), q [S][N] (output).
 * Errors: INVALID_ARG, UNSUPPORTED, NOT_PREPARED, WORKSPACE_TOO_SMALL, HIP.
 */
int32_t s2v_q_score(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *mu,
                    const float *gsum, int32_t S, float *q, void *ws, size_t ws_bytes);

/*
 * One policy evaluation (Alg. 3 lines 5-6: the embedding of Alg. 1, then the scores of Alg. 2 /
 * Eq. 2) in a single call: the same mu_out [N][S][p], gsum [S][G][p] and q [S][N] that
 * s2v_embed_fwd (without saved rounds) followed by s2v_q_score produce, all three required.
 * When the last embedding round runs row by row (S not a multiple of 16, T >= 2) the node term of
 * Eq. 2 is computed inside that round while the finished rows are still on chip, so the embedding
 * is not read a second time; otherwise the call is exactly the two calls in sequence.
 * Errors: as s2v_embed_fwd and s2v_q_score.
 */
int32_t s2v_policy_eval(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                        int32_t S, float *mu_out, float *gsum, float *q, void *ws, size_t ws_bytes);

/*
 * One step of Alg. 3 up to the choice of nodes (lines 5-7: embed, score, select) for ONE state in a single
 * call: s2v_policy_eval with S == 1 followed by s2v_select_topk on its scores, with the arguments of the
 * two (x [N], cand [N] bytes or NULL; mu_out [N][p], gsum [G][p], q [N], idx [G][k], val [G][k], count [G]:
 * all outputs required).  When every graph of the batch is small enough for its embedding to stay in the
 * on-chip memory of one compute unit (n_nodes of the largest graph times p at most 32768: 1024 nodes at
 * p = 32, 512 at p = 64), k <= 8 and the plain neighbour sum on the stored graph is asked for
 * (weighted_sum == 0, state_residual == 0), the whole step is ONE kernel launch with one workgroup per
 * graph: at those sizes the separate launches of the general path cost more than the arithmetic.  That
 * kernel adds a row's neighbours in another order than the general round kernels, so mu_out, gsum and q
 * then agree with s2v_policy_eval's up to float32 rounding (not bit for bit); given q, the selection is
 * the same exact function of the scores.  For any other shape the call IS the two calls in sequence.
 * Supported: (G >= 1, k == 1) and (G == 1, k >= 1).  Errors: as s2v_policy_eval and s2v_select_topk.
 */
int32_t s2v_policy_select(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x,
                          const uint8_t *cand, int32_t T, int32_t k, float *mu_out, float *gsum, float *q, int32_t *idx,
                          float *val, int32_t *count, void *ws, size_t ws_bytes);

/*
 * Node selection for one state: per graph, the k candidates with the highest scores,
 * ordered by score descending and node index ascending among equal scores (k == 1 is
 * the argmax of Alg. 3 line 7; k > 1 is the top-d selection of Sec. 4.5.1).
 *   q     [N] scores;  x [N] node feature
 *   cand  [N] bytes, non-zero = candidate (the set C of Sec. 4.1), or NULL = nodes with x == 0
 *   idx   [G][k] selected node ids (global numbering), -1 in unused slots
 *   val   [G][k] their scores, -inf in unused slots
 *   count [G]    min(k, number of candidates of the graph)
 * Scores must not be NaN; -0.0 and +0.0 compare equal.
 * Supported: (G >= 1, k == 1) and (G == 1, k >= 1); otherwise S2V_ERR_UNSUPPORTED.
 */
int32_t s2v_select_topk(s2v_ctx *ctx, const s2v_graph *g, const float *q, const float *x, const uint8_t *cand,
                        int32_t k, int32_t *idx, float *val, int32_t *count, void *ws, size_t ws_bytes);

/*
 * s2v_select_topk for callers that cannot allocate device memory or size a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same selection rule and outputs as
 * s2v_select_topk for ONE graph (G == 1): idx [k], val [k], count [1]; q, x [n_nodes], cand [n_nodes] bytes or NULL.
 * No graph struct, no workspace and no s2v_graph_prepare: the scratch of the selection kernels (chunk table,
 * per-chunk partial results, radix histograms, scan and sort buffers) lives in a fixed array of 5 MiB of
 * device memory inside the library, which every GPU this process creates a context on holds until the
 * process ends.  The call allocates and frees nothing, on the host or on the device.
 * Limits: n_nodes <= S2V_NOALLOC_MAX_NODES and k <= S2V_NOALLOC_MAX_K, else S2V_ERR_TOO_LARGE (nothing is
 * enqueued).  All contexts of one GPU share that GPU's array: two calls of this entry point that overlap in
 * time on the same GPU (different streams or contexts) race; calls on one stream are safe.  The context
 * must have been created with the GPU of its stream current.
 * Errors: INVALID_ARG, TOO_LARGE, HIP (also when the array's address could not be obtained in s2v_create).
 */
#define S2V_NOALLOC_MAX_NODES (1 << 22) /* 4 194 304 */
#define S2V_NOALLOC_MAX_K (1 << 18)     /* 262 144 */
int32_t s2v_select_topk_noalloc(s2v_ctx *ctx, int32_t n_nodes, const float *q, const float *x, const uint8_t *cand,
                                int32_t k, int32_t *idx, float *val, int32_t *count);

/*
 * Backward pass of the training step (Train of Alg. 4: forward = Alg. 1 then Alg. 2, then
 * back-propagation) for the squared loss averaged over the S states,
 *   L = (1/S) sum_b (Q^{(b)}(action_b) - target_b)^2,
 * through Eq. 2 at the action nodes and all T rounds of Eq. 1 (the adjoint of the
 * neighbour sum is the same sum because the pattern is symmetric).  relu'(0) = 0.
 *   mu_saved [T][N][S][p] and gsum [S][G][p] from s2v_embed_fwd with the same x, T, S
 *   action [S] node ids, target [S]
 *   loss   [1] output;  q_pred [S] output (Q of each action node), may be NULL
 *   grads  gradient of L w.r.t. theta1..theta7 (overwritten; grads->p must equal params->p)
 */
int32_t s2v_embed_bwd(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                      int32_t S, const float *mu_saved, const float *gsum, const int32_t *action,
                      const float *target, float *loss, float *q_pred, s2v_params *grads, void *ws,
                      size_t ws_bytes);

/*
 * Forward and backward pass of one training iteration in a single call (Train of Alg. 4 up to, not
 * including, the parameter update): the same loss, q_pred, grads and gsum, bit for bit, as
 * s2v_embed_fwd (with mu_saved, without mu_out) followed by s2v_embed_bwd.
 *   mu_saved [T][N][S][p] device scratch owned by the caller; its contents after the call are
 *            unspecified.  Knowing that the backward pass follows, the forward pass leaves out what that
 *            pass never reads when S == 16, G == 1, T >= 3 and state_residual == 0: the rows of round 1
 *            (the last reversed round works from per-node scalars) and all of mu^T except its relu mask
 *            (kept as one 64-bit word per (node, state) in the workspace), the action nodes' rows and the
 *            graph sums.  For any other shape the call is exactly the two calls in sequence.
 *   gsum     [S][G][p] output;  all other arguments as in s2v_embed_bwd.
 * The workspace must have been sized with training != 0.
 * Errors: as s2v_embed_fwd and s2v_embed_bwd.
 */
int32_t s2v_loss_grad(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                      int32_t S, float *mu_saved, float *gsum, const int32_t *action, const float *target,
                      float *loss, float *q_pred, s2v_params *grads, void *ws, size_t ws_bytes);

/* Plain gradient descent on all seven tensors: theta <- theta - lr * grad (Sec. 4.5.2 repeats
 * forward, backward and this update several times on one minibatch). */
int32_t s2v_sgd_step(s2v_ctx *ctx, s2v_params *params, const s2v_params *grads, float lr);

/*
 * Adam step on all seven tensors (the paper trains with Adam, Sec. 4.4; learning rate 1e-5 in
 * Sec. 6.1), with the usual bias correction: m, v are the first and second moment tensors
 * (device, updated in place, zero before the first step), step >= 1 is the step number.
 *   theta <- theta - lr / (1 - beta1^step) * m / (sqrt(v) / sqrt(1 - beta2^step) + eps)
 */
int32_t s2v_adam_step(s2v_ctx *ctx, s2v_params *params, const s2v_params *grads, s2v_params *m, s2v_params *v,
                      int32_t step, float lr, float beta1, float beta2, float eps);

/*
 * Deep-Q target values of a minibatch (Alg. 4: "compute a target value using the reward";
 * discount gamma = 0.9 in Sec. 6.1).  The paper does not define its reward, so it is an input:
 *   target[b] = reward[b] + gamma * max_{v in C'_b} q_next[b][v],   or reward[b] if C'_b is empty,
 * where q_next [S][N] are the scores of the NEXT states (s2v_embed_fwd + s2v_q_score on x_next) and
 * C'_b are the next state's candidates (cand_next [S][N] bytes, or NULL = nodes with x_next == 0)
 * inside the graph that holds action[b] (action [S]; may be NULL for a single graph).
 *   reward [S], target [S] (output).  Errors: INVALID_ARG, NOT_PREPARED, WORKSPACE_TOO_SMALL, HIP.
 */
int32_t s2v_q_target(s2v_ctx *ctx, const s2v_graph *g, const float *q_next, const float *x_next,
                     const uint8_t *cand_next, const int32_t *action, const float *reward, float gamma, int32_t S,
                     float *target, void *ws, size_t ws_bytes);

/*
 * State update of the inference loop, Alg. 3 lines 8-10, for a graph whose arrays the caller
 * owns as a MUTABLE copy (colidx, w and row_end are written through the const pointers of `g`;
 * g->row_end must be non-NULL, initially a copy of rowptr[1..N]):
 *   - the selected nodes sel_idx[G][k] (first sel_count[g] of each row) join the partial
 *     solution: x[v] = 1.  With sel_idx == NULL the whole state is rebuilt from x alone (a pass over
 *     every row); with a selection the update is incremental (only the rows next to the selected
 *     nodes are touched), so cand, stats, row_end and the arrays of `g` must then be the outcome of
 *     the previous call on this graph, the first of which was a full rebuild;
 *   - every edge with an endpoint in the solution (x != 0) is removed: rows shrink in place,
 *     keeping the order of the surviving entries; rows of solution nodes become empty;
 *   - s+ / s- in the workspace head are recomputed over the surviving entries, so the graph stays
 *     prepared for s2v_embed_fwd;
 *   - cand[v] = 1 for nodes outside the solution that still have an edge, else 0 (the set C);
 *   - stats[g] = {number of candidates, number of live stored entries} of graph g (device [G][2]).
 * The solution is a vertex cover of graph g exactly when stats[g][1] == 0.
 * Errors: INVALID_ARG, NOT_PREPARED, WORKSPACE_TOO_SMALL, HIP.
 */
int32_t s2v_residual_update(s2v_ctx *ctx, const s2v_graph *g, float *x, const int32_t *sel_idx,
                            const int32_t *sel_count, int32_t k, uint8_t *cand, int32_t *stats, void *ws,
                            size_t ws_bytes);

/*
 * The whole inference loop of Alg. 3 with the multiple-node selection of Sec. 4.5.1, for the
 * minimum-vertex-cover setting of the paper: repeat { embed (Eq. 1), score (Eq. 2), take the d best
 * candidates, update the state } until no edge is left or max_steps policy evaluations were made.
 * d = 1 when adaptive == 0; otherwise the 8/4/2/1 rule of s2v_adaptive_d on |C| and N (one graph
 * only; a batch with G > 1 always uses d = 1, each graph taking its own argmax per step).
 *   g        mutable graph copy as for s2v_residual_update, prepared with `ws`
 *   x        [N] in/out: the partial solution (0/1); on return a vertex cover unless max_steps hit
 *   buffers  mu [N][p], gsum [G][p], q [N], cand [N] bytes, sel_idx [G][8], sel_val [G][8],
 *            sel_count [G], stats [G][2]: device scratch owned by the caller
 *   steps_out, picked_out, live_out: host pointers; policy evaluations made, nodes added, live
 *            stored entries left (0 = complete cover)
 * Which d to use, whether an edge is left and the two counts are decided and kept on the device; the host
 * reads the state back once per block of steps (1, 2, 4, ... up to 64 steps, and never more than a sixteenth of
 * the candidates the largest graph has left), so the call waits for the stream a few times per solve, and a block that outlasts the solve still makes its (then ineffective) evaluations.
 * With the adaptive rule sel_idx / sel_val receive the eight best candidates of the last evaluation, of
 * which the first sel_count joined the solution.
 */
int32_t s2v_mvc_inference(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, float *x, int32_t T,
                          int32_t adaptive, int32_t max_steps, float *mu, float *gsum, float *q, uint8_t *cand,
                          int32_t *sel_idx, float *sel_val, int32_t *sel_count, int32_t *stats,
                          int32_t *steps_out, int64_t *picked_out, int64_t *live_out, void *ws, size_t ws_bytes);

/*
 * Optional live timing of the main kernels (for benchmarks; not part of the method).
 * Between s2v_profile_begin and s2v_profile_end the launches listed below are bracketed by HIP events on
 * the context's stream, up to max_launches spans in total.  Kinds:
 *   S2V_PROFILE_FWD_ROUND      rounds 3..T of Eq. 1 inside s2v_embed_fwd (neighbour rows read from memory)
 *   S2V_PROFILE_BWD_ROUND      a reversed round that gathers rows of dz (inside s2v_embed_bwd); for 16-state
 *                              blocks and T >= 4 the launch of round t = 3 also does round t = 2 on each tile
 *   S2V_PROFILE_FWD_ROUND2     round 2 of Eq. 1 (neighbour rows recomputed from per-node scalars)
 *   S2V_PROFILE_FWD_ROUND_Q    a last round with more fused into it: the node term of Eq. 2 (inside
 *                              s2v_policy_eval) or relu-mask words instead of its rows (inside s2v_loss_grad);
 *                              such a launch is not counted under S2V_PROFILE_FWD_ROUND
 *   S2V_PROFILE_BWD_ROUND_MASK the first reversed round (t = T), which gathers relu-mask words
 *   S2V_PROFILE_BWD_FIRST      the stand-alone last reversed round from per-node scalars (16-state blocks, T = 3)
 *   S2V_PROFILE_BWD_SEED       the kernel that forms dz^T's relu mask and its share of the parameter sums
 *   S2V_PROFILE_SELECT         all kernels of one s2v_select_topk call, as one span (the single launch of
 *                              s2v_policy_select on small graphs is counted here too)
 * s2v_profile_end waits for the stream and returns, per kind, the number of spans and the sum of their
 * durations in milliseconds (host arrays of S2V_PROFILE_KINDS elements).
 */
#define S2V_PROFILE_FWD_ROUND 0
#define S2V_PROFILE_BWD_ROUND 1
#define S2V_PROFILE_FWD_ROUND2 2
#define S2V_PROFILE_FWD_ROUND_Q 3
#define S2V_PROFILE_BWD_ROUND_MASK 4
#define S2V_PROFILE_BWD_FIRST 5
#define S2V_PROFILE_BWD_SEED 6
#define S2V_PROFILE_SELECT 7
#define S2V_PROFILE_KINDS 8
int32_t s2v_profile_begin(s2v_ctx *ctx, int32_t max_launches);
int32_t s2v_profile_end(s2v_ctx *ctx, int32_t *n_launches, float *total_ms);

/*
 * Read-only streaming probe (for benchmarks; not part of the method): loads every 16-byte word of the
 * device range [src, src + bytes) once, fully coalesced, and writes 4096 partial float sums to `out`
 * (device, 4096 floats).  Timed by the caller, it gives the rate at which this GPU streams memory that
 * is only read -- the ceiling to hold the gather rounds against.  src 16-byte aligned, bytes a multiple of 16.
 */
int32_t s2v_stream_read(s2v_ctx *ctx, const void *src, size_t bytes, float *out);

/*
 * Host helper: the adaptive number of nodes to select per policy evaluation (Sec. 4.5.1):
 * 8 if |C| > N/2, 4 if N/4 < |C| <= N/2, 2 if N/8 < |C| <= N/4, else 1.  Returns d >= 1.
 */
int32_t s2v_adaptive_d(int64_t n_candidates, int64_t n_nodes);

#ifdef __cplusplus
}
#endif
#endif /* S2V_H */
