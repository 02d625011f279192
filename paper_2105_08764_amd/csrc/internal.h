// Internal declarations shared by the translation units of libs2v.so.
// Host-side launchers only; every kernel lives in the .hip file that defines its launcher.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace s2v {

// Nodes per reduction chunk (graph sums, argmax partials).  A chunk never straddles two graphs.
constexpr int kChunkNodes = 1024;
// Workgroups of the backward round kernel: a fixed grid, so that the order in which
// per-workgroup partial gradients are summed does not depend on the device.
constexpr int kBwdGrid = 1024;
constexpr int kBwdHeadGrid = 1024;
// A workgroup of the reversed rounds folds its float32 accumulators (the p x p sum for dtheta2 and the column
// sums) into its partial rows every kBwdFlushTiles tiles, and the partial rows are kept as a compensated pair
// (row b: running sum, row kBwdGrid + b: the rounding remainders), so that no float accumulator ever takes
// more than kBwdFlushTiles * 16 terms however large the graph: with 10^6 nodes x 16 states a single running
// float32 sum per wave (62 500 terms) left the gradients ten times less accurate than on one state.
constexpr int kBwdFlushTiles = 32;
constexpr int kBwdRoundRows = 2 * kBwdGrid;   // partial rows per reversed round
// Blocks per state of the action-node fix-up of the backward pass (each adds one partial row).
constexpr int kFixSplit = 16;
// Elements per block of the selection scan / sort passes.
constexpr int kScanBlock = 2048;
constexpr int kSmallK = 8;         // top-k up to this k (the d of Sec. 4.5.1) takes the two-launch path
constexpr int kSortTile = 1024;
constexpr int kSortFusedMaxBlocks = 512;   // above this the sort uses separate count / scan / scatter kernels

constexpr size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Rows with more stored entries than kHubDegree are "hubs": their neighbour sums are formed ahead
// of the round kernel by many waves, each summing one segment of at most kHubSegment entries, so
// that no single wave ever walks a long row.
constexpr int kHubDegree = 256;
// (512: with 64-entry segments the partial sums of a graph whose rows are ALL long, the paper's ER(21 000, 0.15),
//  cost more to write and re-read than the gathers themselves: 0.79 ms per inference step against 0.54 ms)
constexpr int kHubSegment = 512;

struct HubTable {              // device pointers into the prepared head of the workspace
    int n_hubs, n_segs;
    const int32_t *hub_rows;     // [n_hubs] node ids, ascending
    const int32_t *hub_of;       // [N] (with n_hubs > 0) index of a long row's node in hub_rows
    int fold;                    // forward, one state: no combine pass; the round adds a long row's (few) segment sums itself
    const int32_t *hub_seg_off;  // [n_hubs+1] segments of hub h are [off[h], off[h+1])
    const int32_t *seg_row;      // [n_segs] node id of the segment's row
    const int32_t *seg_begin;    // [n_segs] first CSR entry of the segment
    const int32_t *seg_end;      // [n_segs] one past its last entry
};

struct ChunkTable {            // device pointers into the prepared head of the workspace
    int n_chunks;
    const int32_t *chunk_begin;      // [n_chunks] first node
    const int32_t *chunk_end;        // [n_chunks] one past the last node
    const int32_t *graph_chunk_off;  // [G+1] chunks of graph g are [off[g], off[g+1])
};

// Per-node scalar records.  Node v owns `ni` consecutive floats:
//   x_0[v] .. x_{S-1}[v],  then the edge sums s+ and s-,
// the sums stored once per node (all states live on the same graph: ss = 0) or once per state
// (per-state residual graphs: ss = 1).  ni is a multiple of 4; for S = 1 the record is the 16 bytes
// {x, s+, s-, pad}.
struct NodeInfo {
    const float *__restrict__ base;
    int ni;       // floats per node
    int S;
    int sp_off;   // offset of s+ (of state 0)
    int sn_off;   // offset of s- (of state 0)
    int ss;       // stride over states of s+ / s-: 0 or 1
    // S = 1 only, optional: compact[v] = s+ of v if its round-1 row is s+ relu(q+) (x = 0 and s- = 0), else NaN
    const float *__restrict__ compact;
    // S = 1 only, optional (static graph without negative weights): bit v of xbits = (x_v != 0), and the fourth
    // float of node v's record holds nbr_sp[v] = the sum of s+ over ALL neighbours of v (computed once per
    // graph).  The sum over the neighbours with x = 0 that round 2 needs is then nbr_sp[v] minus the s+ of
    // the few flagged neighbours, and the round reads a 4-byte table entry only for those.
    const unsigned *__restrict__ xbits;
    // The same idea for S a multiple of 16 (static graph, no negative weights, all states on the stored graph):
    // flags16[v * (S / 16) + k] has bit i set when x of node v in state 16 k + i is non-zero, and the first
    // spare float of node v's record (behind s-) holds nbr_sp[v].
    const unsigned short *__restrict__ flags16;
    __device__ __forceinline__ const float *node(int v) const { return base + (size_t)v * ni; }
    __device__ __forceinline__ float x(int v, int s) const { return node(v)[s]; }
    __device__ __forceinline__ float sp(int v, int s) const { return node(v)[sp_off + s * ss]; }
    __device__ __forceinline__ float sn(int v, int s) const { return node(v)[sn_off + s * ss]; }
    // {x, s+, s-} of (v, s)
    __device__ __forceinline__ float3 get(int v, int s) const {
        if (S == 1) {
            const float4 r = *reinterpret_cast<const float4 *>(base + (size_t)v * 4);
            return make_float3(r.x, r.y, r.z);
        }
        const float *r = node(v);
        return make_float3(r[s], r[sp_off + s * ss], r[sn_off + s * ss]);
    }
};

// Floats reserved per node for the records (an upper bound of both layouts) and the compact table.
inline int nodeinfo_stride(int S) { return 4 * S + 1; }
inline NodeInfo make_nodeinfo(const float *base, int S, bool per_state) {
    NodeInfo n;
    n.base = base;
    n.S = S;
    n.sp_off = S;
    n.sn_off = S + (per_state ? S : 1);
    n.ss = per_state ? 1 : 0;
    n.ni = (n.sn_off + (per_state ? S : 1) + 3) / 4 * 4;
    n.compact = nullptr;
    n.xbits = nullptr;
    n.flags16 = nullptr;
    return n;
}

// ---- forward (fwd_kernels.hip) ----
hipError_t launch_prepare_s(hipStream_t st, int N, const int32_t *rowptr, const int32_t *rowend, const float *w,
                            float *s_pos, float *s_neg, int32_t *neg_flag /*set to 1 if a weight is negative; may be NULL*/);
hipError_t launch_qvec(hipStream_t st, int p, const float *theta3, const float *theta4, float *qvec);
// x_res != NULL in the round launchers: per-state residual graphs (x_res is the caller's x [S][N]).
hipError_t launch_round1(hipStream_t st, int p, int N, int S, const NodeInfo &ni, const float *x_res, bool last,
                         const float *theta1, const float *qvec, float *mu_out);
hipError_t launch_stateinfo_residual(hipStream_t st, int N, int S, const HubTable &ht, const int32_t *rowptr,
                                     const int32_t *rowend, const int32_t *colidx, const float *w, const float *x,
                                     float *info /*written in the per-state layout of make_nodeinfo*/,
                                     float *compact /*[N], written when S == 1; may be NULL*/);
// upper bound of the embedding-round grid (also the number of partial rows of its fused graph sum)
#ifndef S2V_ROUND_GRID
#define S2V_ROUND_GRID (256 * 16)
#endif
constexpr int kRoundGridMax = S2V_ROUND_GRID;
int round_grid(long n_vrows);
// out[0..2] (zeroed by the caller) += {long rows, their segments, 1 if the row pointers are malformed}
hipError_t launch_row_stats(hipStream_t st, int N, long nnz, const int32_t *rowptr, int32_t *out);
hipError_t launch_nodeinfo(hipStream_t st, int N, int S, const float *x, const float *s_pos, const float *s_neg,
                           float *info /*written in the shared-sums layout of make_nodeinfo*/,
                           float *compact /*[N], written when S == 1; may be NULL*/,
                           const float *nbr_sp = nullptr /*[N]: goes into the records' first spare float (S == 1 or S % 16 == 0)*/,
                           unsigned long long *xbits = nullptr /*S == 1: [ceil(N/64)], bit v = (x_v != 0);
                                                                 S % 16 == 0: [N][S/16] 16-bit words, see NodeInfo::flags16*/,
                           int p = 0, const float *theta3 = nullptr, const float *theta4 = nullptr,
                           float *qvec = nullptr /*non-NULL: also q+- = theta3 relu(+-theta4), as launch_qvec writes it*/);
// nbr_sp[v] = sum of s_pos over the live entries of row v (0 for rows longer than kHubDegree, which never use it)
// nbr_spw: the same with each neighbour weighted by its edge weight (w == NULL: equal to nbr_sp)
hipError_t launch_prepare_nbr(hipStream_t st, int N, const int32_t *rowptr, const int32_t *rowend, const int32_t *colidx,
                              const float *w, const float *s_pos, float *nbr_sp, float *nbr_spw);
// Neighbour sums of the hub rows: hub_sum[h][S][p] = sum over the row of hub h of src[u][s][:]
// (mask != NULL: counts of set relu-mask bits instead; else src == NULL: the round-1 rows
// recomputed from info).  partial is [n_segs][S][p] scratch.
hipError_t launch_hub_sums(hipStream_t st, int p, int S, const HubTable &ht, const int32_t *rowend,
                           const int32_t *colidx, const float *wagg, const float *src,
                           const NodeInfo &ni, const float *theta1, const float *qvec,
                           const unsigned long long *mask, float *partial, float *hub_sum);
// Eq. 2's node term fused into the last embedding round (row mode): q == NULL switches it off.
struct QHead {
    const float *theta5;
    const float *theta7;
    float *q;   // [S][N], receives theta5[p:2p] . relu(theta7 mu[v][s])
};
// Mask output of the last embedding round of a fused training pass (node mode, S == 16, one graph):
// words == NULL switches it off.
struct MaskOut {
    unsigned long long *words;   // [N*S]: bit j of word (v, s) = (mu^T[v][s][j] > 0)
    const int32_t *action;       // [S]: the rows of these nodes are still written to mu_out
};
// whether launch_round honours a QHead for this S (else the caller runs the separate node-term kernel)
inline bool round_fuses_qnode(int S, int T) { return (S % 16) != 0 || T >= 3; }
hipError_t launch_qfinish(hipStream_t st, int N, int S, int G, const int32_t *graph_off, const float *qa, float *q);
hipError_t launch_hub_combine(hipStream_t st, int L, const HubTable &ht, const float *partial, float *hub_sum);
hipError_t launch_round(hipStream_t st, int p, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                        const int32_t *colidx, const float *wagg /*NULL: unweighted neighbour sum*/, const float *mu_in,
                        float *mu_out, const NodeInfo &ni, const float *theta1,
                        const float *theta2, const float *qvec, bool from_scalars, float *gpart, const HubTable &ht,
                        const float *hub_sum, const float *x_res, bool last, const QHead &qh,
                        const MaskOut &mo = MaskOut{nullptr, nullptr},
                        bool by_state = false /*visit the rows state by state (see k_round) where that applies*/);
hipError_t launch_gsum_from_round(hipStream_t st, int p, int S, int rows, const float *partial, float *gsum);
hipError_t launch_gsum(hipStream_t st, int p, int N, int S, int G, const ChunkTable &ct, const float *mu,
                       float *partial /*[n_chunks][S*p]*/, float *gsum /*[S][G][p]*/);
hipError_t launch_qa(hipStream_t st, int p, int S, int G, const float *theta5, const float *theta6, const float *gsum,
                     float *qa /*[S][G]*/);
hipError_t launch_qnode(hipStream_t st, int p, int N, int S, int G, const int32_t *graph_off, const float *theta5,
                        const float *theta7, const float *mu, const float *qa, float *q /*[S][N]*/);

// read-only streaming probe (benchmarks): out receives 4096 floats
hipError_t launch_stream_read(hipStream_t st, const void *src, size_t bytes, float *out);

// ---- state update of the inference loop (residual_kernels.hip) ----
struct UpdateState;   // (loop_util.h)
// what the end of a step of the inference loop needs beyond the selection's outputs (see loop_control)
struct StepEnd {
    int N;
    bool adaptive;
    unsigned long long *counters;
    const UpdateState *update;
};
hipError_t launch_residual_update(hipStream_t st, int N, const UpdateState &u, int32_t *colidx, float *w,
                                  const int32_t *sel_idx /*[G][k] or NULL: full pass*/, const int32_t *sel_count,
                                  bool begun = false);
hipError_t launch_zero_i32(hipStream_t st, long n, int32_t *p);
hipError_t launch_loop_control(hipStream_t st, int N, bool adaptive, int32_t *sel_count,
                               unsigned long long *counters /*[2]: evaluations that mattered, nodes added*/,
                               const int32_t *sel_idx /*[G][k]*/, const UpdateState &u);

// ---- one launch per step of Alg. 3 on small graphs (small_kernels.hip) ----
// floats of LDS that hold one graph's embedding: a graph qualifies when n_nodes * p does not exceed it
constexpr int kSmallLdsFloats = 32768;
// LDS bytes per workgroup the kernel needs (its static arrays, rounded up)
constexpr size_t kSmallLdsBytes = 160 * 1024;
struct SmallPolicyArgs {
    int N, G, T, k;                       // k: nodes to select per graph (with idx != NULL)
    const int32_t *graph_off;             // [G+1] or NULL (one graph)
    const int32_t *rowptr, *rowend, *colidx;
    const float *x, *s_pos, *s_neg;       // [N] each
    const uint8_t *cand;                  // [N] or NULL (candidates: x == 0)
    const float *theta1, *theta2, *theta3, *theta4, *theta5, *theta6, *theta7;
    float *agg;                           // [N][p] scratch: the neighbour sums of the current round
    float *mu_out, *gsum, *q;             // [N][p], [G][p], [N]
    int32_t *idx;                         // [G][k] or NULL: no selection
    float *val;                           // [G][k]
    int32_t *count;                       // [G]
};
hipError_t launch_small_policy(hipStream_t st, int p, const SmallPolicyArgs &a);

// ---- selection (select_kernels.hip) ----
struct SelectScratch {
    float *part_val;    // [n_chunks][kSmallK]
    int32_t *part_idx;  // [n_chunks][kSmallK]
    uint32_t *hist;     // [4][256]
    uint32_t *state;    // [16]
    uint32_t *blk;      // [2][n_scan_blocks][2]
    uint32_t *keys[2];  // [k] each
    int32_t *ids[2];    // [k] each
    uint32_t *sort_cnt; // [n_sort_blocks][256] ([256][n_sort_blocks] with more than kSortFusedMaxBlocks tiles)
};
hipError_t launch_chunk_table_single(hipStream_t st, int N, int n_chunks, int32_t *chunk_begin, int32_t *chunk_end,
                                     int32_t *graph_chunk_off /*[2]*/);
hipError_t launch_argmax(hipStream_t st, int N, int G, const ChunkTable &ct, const float *q, const float *x,
                         const uint8_t *cand, const SelectScratch &sc, int32_t *idx, float *val, int32_t *count);
hipError_t launch_q_target(hipStream_t st, int N, int S, int G, const int32_t *graph_off, const ChunkTable &ct,
                           const float *q_next, const float *x_next, const uint8_t *cand_next, const int32_t *action,
                           const float *reward, float gamma, float *part_val /*[S][n_chunks]*/,
                           int32_t *part_idx /*[S][n_chunks]*/, float *target);
hipError_t launch_smallk(hipStream_t st, const ChunkTable &ct, const float *q, const float *x, const uint8_t *cand,
                         int k /*2..kSmallK, one graph*/, const SelectScratch &sc, int32_t *idx, float *val, int32_t *count);
// gsum stage 2 + graph term of Eq. 2 + q = qa + node term + first selection stage in one launch, then the second
// selection stage (one state, one graph, n_chunks >= 1, 1 <= k <= kSmallK, few partial rows)
constexpr int kTailMaxRows = 256;
hipError_t launch_tail_select(hipStream_t st, int p, int rows, int k, const float *gpart /*[rows][p]*/,
                              const float *theta5, const float *theta6, float *gsum /*[p]*/,
                              float *q /*[N]: in the node term, out Eq. 2*/, const float *x, const uint8_t *cand,
                              const ChunkTable &ct, const SelectScratch &sc, int32_t *idx, float *val, int32_t *count,
                              const StepEnd *end = nullptr /*non-NULL: the selection's last launch also takes the
                                                             step's decisions and begins the state update*/);
hipError_t launch_topk(hipStream_t st, int N, const float *q, const float *x, const uint8_t *cand, int k,
                       const SelectScratch &sc, int32_t *idx, float *val, int32_t *count);

// ---- backward (bwd_kernels.hip) ----
struct BwdScratch {
    float *dg;          // [S][p]   theta6^T dh1 : gradient w.r.t. the graph sum
    float *da;          // [S][p]   theta7^T dh2 : extra gradient at the action node
    int32_t *glo;       // [S] first node of the action's graph
    int32_t *ghi;       // [S] one past its last node
    float *head_part;   // [S][2p + 2*p*p + 1]  per-state partials of dtheta5, dtheta6, dtheta7, loss
    float *dz[2];       // [N][S][p] each
    unsigned long long *maskT;  // [N][S] relu mask of mu^T
    float *dc_part;     // [dc_rows][3][p]   partial sums of x*dz, s+ * dz, s- * dz
    float *d2_part;     // [d2_rows][p][p]   partial sums of G (x) mu
    float *dvec;        // [3][p] reduced dtheta1, dq+, dq-
    float *red_tmp;     // [ceil(max rows / 64)][max(3p, p*p)] second level of the final reductions
    float *rec;         // per-node scalar records (see NodeInfo), nodeinfo_stride(S) floats per node
};
hipError_t launch_bwd_head(hipStream_t st, int p, int N, int S, int G, const int32_t *graph_off, const float *theta5,
                           const float *theta6, const float *theta7, const float *muT, const float *gsum,
                           const int32_t *action, const float *target, const BwdScratch &sc, float *q_pred);
hipError_t launch_bwd_head_reduce(hipStream_t st, int p, int S, const BwdScratch &sc, float *loss, float *d5, float *d6,
                                  float *d7);
hipError_t launch_bwd_maskT(hipStream_t st, int p, int N, int S, const float *muT, const NodeInfo &ni, const float *x_res,
                            const int32_t *action, const BwdScratch &sc, unsigned long long *mask /*[N][S] or NULL*/,
                            float *dc_part /*[kBwdHeadGrid][3][p]*/,
                            bool words_ready = false /*mask already holds the words: read them, not muT*/);
// maskT != NULL selects the first reversed round (t = T), which reads relu-mask words instead of dz_in.
// Asks launch_bwd_round (node mode, rows in memory) to do the round after it as well, in its scalar form.
struct BwdFuse {
    const float *theta1;
    const float *qvec;
    const float *hub_sum4;   // [n_hubs][4][S][p], from launch_hub_sums_grad
    bool has_neg;
};
hipError_t launch_bwd_round(hipStream_t st, int p, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                            const int32_t *colidx, const float *wagg, const float *dz_in,
                            const unsigned long long *maskT, const BwdScratch &sc,
                            const float *mu_prev, float *dz_out /*may be NULL*/, const NodeInfo &ni, const float *theta2,
                            float *dc_part /*[kBwdRoundRows][3][p]*/, float *d2_part /*[kBwdRoundRows][p][p]*/,
                            const HubTable &ht, const float *hub_sum, const BwdFuse *fuse /*may be NULL*/,
                            bool by_state = false /*row mode, rows in memory: walk the rows state by state*/);
// The last reversed round (t = 2) from the scalars: node mode (S a multiple of 16) and T >= 3 only.
hipError_t launch_bwd_first(hipStream_t st, int p, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                            const int32_t *colidx, const float *wagg, const float *dz_in /*dz^2 [N][S][p]*/,
                            const NodeInfo &ni, bool has_neg, const float *theta1, const float *theta2,
                            const float *qvec, float *dc_part /*[kBwdRoundRows][3][p]*/,
                            float *d2_part /*[kBwdRoundRows][p][p]*/, const HubTable &ht,
                            const float *hub_sum4 /*[n_hubs][4][S][p]*/);
hipError_t launch_hub_sums_grad(hipStream_t st, int p, int S, const HubTable &ht, const int32_t *rowend,
                                const int32_t *colidx, const float *wagg, const NodeInfo &ni, bool has_neg,
                                const float *theta1, const float *qvec, float *partial4 /*[n_segs][4][S][p]*/,
                                float *hub_sum4 /*[n_hubs][4][S][p]*/);
hipError_t launch_bwd_action_fix(hipStream_t st, int p, int S, const int32_t *rowptr, const int32_t *rowend,
                                 const int32_t *colidx, const float *wagg,
                                 const int32_t *action, const unsigned long long *maskT, const BwdScratch &sc,
                                 const float *theta2, const float *mu_prev, float *dz_out /*may be NULL*/,
                                 const NodeInfo &ni, float *dc_part /*[S*kFixSplit][3][p]*/,
                                 float *d2_part /*[S*kFixSplit][p][p]*/);
hipError_t launch_bwd_finish(hipStream_t st, int p, int dc_rows, int d2_rows, const BwdScratch &sc, const float *theta3,
                             const float *theta4, float *d1, float *d2, float *d3, float *d4);
hipError_t launch_sgd(hipStream_t st, int p, float *const theta[7], const float *const grad[7], float lr);
hipError_t launch_adam(hipStream_t st, int p, float *const theta[7], const float *const grad[7], float *const m[7],
                       float *const v[7], float lr, float b1, float b2, float eps, float bias1, float bias2_sqrt);

}  // namespace s2v
