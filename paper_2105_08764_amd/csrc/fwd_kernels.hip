// Forward kernels: graph preparation, the embedding rounds of Eq. 1 / Alg. 1, the per-graph
// embedding sum (Alg. 2 lines 4-5) and the scores of Eq. 2 / Alg. 2.
#include "device_util.h"
#include "internal.h"
#include "reduce_util.h"

namespace s2v {

// ------------------------------------------------------------------------------------------
// Graph preparation: s+_v = sum_u max(W(v,u), 0), s-_v = sum_u max(-W(v,u), 0).
// With these, the third term of Eq. 1 is  s+_v * theta3 relu(theta4) + s-_v * theta3 relu(-theta4),
// the same for every round (Alg. 1 computes it before the layer loop).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_prepare_s(int N, const int32_t *__restrict__ rowptr,
                                                   const int32_t *__restrict__ rowend,
                                                   const float *__restrict__ w, float *__restrict__ s_pos,
                                                   float *__restrict__ s_neg, int32_t *__restrict__ neg_flag) {
    for (int v = blockIdx.x * blockDim.x + threadIdx.x; v < N; v += gridDim.x * blockDim.x) {
        const int b = rowptr[v], e = rowend[v];
        double sp = 0.0, sn = 0.0;
        if (w) {
            for (int j = b; j < e; ++j) {
                const float wj = w[j];
                sp += (double)fmaxf(wj, 0.f);
                sn += (double)fmaxf(-wj, 0.f);
            }
        } else {
            sp = (double)(e - b);
        }
        s_pos[v] = (float)sp;
        s_neg[v] = (float)sn;
        if (neg_flag && sn > 0.0) atomicOr(neg_flag, 1);   // the graph has a negative weight
    }
}

hipError_t launch_prepare_s(hipStream_t st, int N, const int32_t *rowptr, const int32_t *rowend, const float *w,
                            float *s_pos, float *s_neg, int32_t *neg_flag) {
    if (N == 0) return hipSuccess;
    const int grid = min((N + 255) / 256, 65536);
    k_prepare_s<<<grid, 256, 0, st>>>(N, rowptr, rowend, w, s_pos, s_neg, neg_flag);
    return hipGetLastError();
}

// nbr_sp[v] = sum_{u in N(v)} s+_u: what the neighbour sum of round 2 comes to when no neighbour is in the
// solution (then mu^1_u = s+_u relu(q+) for every u).  Rows beyond kHubDegree go through the long-row
// pre-pass and never use it.
// (sixteen lanes per row: the row's entries are read in coalesced pieces; double accumulators, added in a fixed
//  order, so the rounded result does not depend on the launch)
__global__ __launch_bounds__(256) void k_prepare_nbr(int N, const int32_t *__restrict__ rowptr,
                                                     const int32_t *__restrict__ rowend,
                                                     const int32_t *__restrict__ colidx,
                                                     const float *__restrict__ w,
                                                     const float *__restrict__ s_pos, float *__restrict__ nbr_sp,
                                                     float *__restrict__ nbr_spw) {
    const int sub = threadIdx.x & 15;
    const long groups = ((long)gridDim.x * blockDim.x) >> 4;
    const long n_iter = (N + groups - 1) / groups;   // every lane makes the same number of steps (shuffles below)
    for (long it = 0; it < n_iter; ++it) {
        const long v = it * groups + (((long)blockIdx.x * blockDim.x + threadIdx.x) >> 4);
        const bool in = v < N;
        const int b = in ? rowptr[v] : 0, e = in ? rowend[v] : 0;
        double a = 0.0, aw = 0.0;   // aw: each neighbour weighted by its edge (the weighted neighbour sum)
        if (e - b <= kHubDegree)
            for (int j = b + sub; j < e; j += 16) {
                const double sp = (double)s_pos[colidx[j]];
                a += sp;
                if (w) aw += (double)w[j] * sp;
            }
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            a += __shfl_xor(a, m);
            aw += __shfl_xor(aw, m);
        }
        if (in && sub == 0) {
            nbr_sp[v] = (float)a;
            nbr_spw[v] = w ? (float)aw : (float)a;
        }
    }
}

hipError_t launch_prepare_nbr(hipStream_t st, int N, const int32_t *rowptr, const int32_t *rowend, const int32_t *colidx,
                              const float *w, const float *s_pos, float *nbr_sp, float *nbr_spw) {
    if (N == 0) return hipSuccess;
    k_prepare_nbr<<<(int)min(((long)N * 16 + 255) / 256, (long)65536), 256, 0, st>>>(N, rowptr, rowend, colidx, w, s_pos, nbr_sp,
                                                                                  nbr_spw);
    return hipGetLastError();
}

// Row statistics of a CSR graph, so that the host need not read the row pointers back for a graph without
// long rows: out[0] = rows longer than kHubDegree, out[1] = their segments of kHubSegment entries,
// out[2] = 1 when the row pointers are not a non-decreasing sequence from 0 to nnz.  out starts at zero.
__global__ __launch_bounds__(256) void k_row_stats(int N, long nnz, const int32_t *__restrict__ rowptr,
                                                   int32_t *__restrict__ out) {
    int hubs = 0, segs = 0, bad = 0;
    for (int v = blockIdx.x * 256 + threadIdx.x; v < N; v += gridDim.x * 256) {
        const int a = rowptr[v], b = rowptr[v + 1];
        if (b < a) bad = 1;
        if (v == 0 && a != 0) bad = 1;
        if (v == N - 1 && (long)b != nnz) bad = 1;
        const int d = b - a;
        if (d > kHubDegree) {
            ++hubs;
            segs += (d + kHubSegment - 1) / kHubSegment;
        }
    }
    if (hubs) atomicAdd(&out[0], hubs);
    if (segs) atomicAdd(&out[1], segs);
    if (bad) atomicOr(&out[2], 1);
}

hipError_t launch_row_stats(hipStream_t st, int N, long nnz, const int32_t *rowptr, int32_t *out) {
    if (N == 0) return hipSuccess;
    k_row_stats<<<min((N + 255) / 256, 4096), 256, 0, st>>>(N, nnz, rowptr, out);
    return hipGetLastError();
}

// q+ = theta3 relu(theta4), q- = theta3 relu(-theta4)   (two p-vectors, qvec = [q+ ; q-])
__global__ void k_qvec(int p, const float *__restrict__ theta3, const float *__restrict__ theta4,
                       float *__restrict__ qvec) {
    const int i = threadIdx.x;
    if (i >= 2 * p) return;
    // (the same double accumulation in the same order as the copy inside k_nodeinfo: identical bits)
    const bool neg = i >= p;
    const int r = neg ? i - p : i;
    double acc = 0.0;
    for (int j = 0; j < p; ++j) {
        const float t4 = theta4[j];
        acc += (double)theta3[r * p + j] * (double)fmaxf(neg ? -t4 : t4, 0.f);
    }
    qvec[i] = (float)acc;
}

hipError_t launch_qvec(hipStream_t st, int p, const float *theta3, const float *theta4, float *qvec) {
    k_qvec<<<1, 128, 0, st>>>(p, theta3, theta4, qvec);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Round 1: mu^0 = 0 (Alg. 1), so mu^1_v = relu(theta1 x_v + s+_v q+ + s-_v q-): no neighbour sum.
// One thread per float4 of the [N][S][p] output; the scalars come from the node records.
// x_res != NULL (per-state residual graphs): a row whose node is in that state's solution is an
// isolated node; its embedding is relu(theta1 x) in the final round and is stored as zero in
// every earlier round, so that nobody's neighbour sum sees it.
// ------------------------------------------------------------------------------------------
template <int P>
__global__ __launch_bounds__(256) void k_round1(long n_vrows, int N, int S, NodeInfo ni,
                                                const float *__restrict__ x_res, int last,
                                                const float *__restrict__ theta1, const float *__restrict__ qvec,
                                                float *__restrict__ mu_out) {
    constexpr int LPR = P / 4;
    // the grid stride is a multiple of LPR, so a thread keeps its four columns: constants in registers
    const int c = (int)(threadIdx.x % LPR) * 4;
    const float4 t1 = ld4(theta1 + c), qp = ld4(qvec + c), qn = ld4(qvec + P + c);
    const long rows_per_step = (long)gridDim.x * blockDim.x / LPR;
    for (long r = ((long)blockIdx.x * blockDim.x + threadIdx.x) / LPR; r < n_vrows; r += rows_per_step) {
        const int v = (int)r / S, s = (int)r - v * S;   // n_vrows < 2^31: 32-bit division
        const float3 q = ni.get(v, s);
        float xs = q.x;
        const float sp = q.y, sn = q.z;
        float keep = 1.f;
        if (x_res) {
            const float xo = x_res[(size_t)s * N + v];
            if (xo != 0.f) { xs = xo; keep = last ? 1.f : 0.f; }
        }
        float4 o = mu1_row(xs, sp, sn, t1, qp, qn);
        o.x *= keep; o.y *= keep; o.z *= keep; o.w *= keep;
        st4(mu_out + (size_t)r * P + c, o);
    }
}

hipError_t launch_round1(hipStream_t st, int p, int N, int S, const NodeInfo &ni, const float *x_res, bool last,
                         const float *theta1, const float *qvec, float *mu_out) {
    const long n_vrows = (long)N * S;
    if (n_vrows == 0) return hipSuccess;
    const long total = n_vrows * (p / 4);
    const int grid = (int)min((total + 255) / 256, (long)(256 * 32));
    if (p == 32) k_round1<32><<<grid, 256, 0, st>>>(n_vrows, N, S, ni, x_res, last ? 1 : 0, theta1, qvec, mu_out);
    else k_round1<64><<<grid, 256, 0, st>>>(n_vrows, N, S, ni, x_res, last ? 1 : 0, theta1, qvec, mu_out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// The scalar records (see NodeInfo) when all states share the graph: per node the S values of x,
// then s+ and s- once.  A neighbour's record is all the second round needs (see Mu1Row), and
// every kernel reads its own rows' scalars here.
// ------------------------------------------------------------------------------------------
// q+- of one output row i (i < p: q+, else q-), accumulated in double and rounded once: q+- multiply every
// node's edge sums, so an error here moves every pre-activation of the graph the same way
__device__ __forceinline__ float qvec_entry(int p, int i, const float *__restrict__ theta3,
                                            const float *__restrict__ theta4) {
    const bool neg = i >= p;
    const int r = neg ? i - p : i;
    double acc = 0.0;
    for (int j = 0; j < p; ++j) {
        const float t4 = theta4[j];
        acc += (double)theta3[r * p + j] * (double)fmaxf(neg ? -t4 : t4, 0.f);
    }
    return (float)acc;
}

// (qvec != NULL: the last workgroup does not take part in the records; it forms q+- instead, which saves the
//  launch of k_qvec where a round follows at once)
__global__ __launch_bounds__(256) void k_nodeinfo(int N, int S, int ni, const float *__restrict__ x,
                                                  const float *__restrict__ s_pos, const float *__restrict__ s_neg,
                                                  float *__restrict__ info, float *__restrict__ compact,
                                                  const float *__restrict__ nbr_sp, int p,
                                                  const float *__restrict__ theta3, const float *__restrict__ theta4,
                                                  float *__restrict__ qvec, int work_blocks) {
    if (qvec && (int)blockIdx.x == work_blocks) {
        if ((int)threadIdx.x < 2 * p) qvec[threadIdx.x] = qvec_entry(p, threadIdx.x, theta3, theta4);
        return;
    }
    const long total = (long)N * ni;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)work_blocks * 256) {
        const int v = (int)(i / ni), c = (int)(i - (long)v * ni);
        float o = 0.f;
        if (c < S) o = x[(size_t)c * N + v];
        else if (c == S) o = s_pos[v];
        else if (c == S + 1) o = s_neg[v];
        else if (nbr_sp && c == S + 2) o = nbr_sp[v];   // (the record's first spare float)
        info[i] = o;
        // S = 1: s+ alone for a node whose round-1 row is s+ relu(q+), NaN for any other node
        if (compact && c == 0) compact[v] = (o == 0.f && s_neg[v] == 0.f) ? s_pos[v] : __int_as_float(0x7fc00000);
    }
}

// bit v of bits = (x[v] != 0); one 64-bit word per wave and step
__global__ __launch_bounds__(256) void k_xbits(int N, const float *__restrict__ x, unsigned long long *__restrict__ bits) {
    const int n_words = (N + 63) / 64;
    const int lane = threadIdx.x & 63;
    for (int wd = blockIdx.x * 4 + (threadIdx.x >> 6); wd < n_words; wd += gridDim.x * 4) {   // wave-uniform
        const int v = wd * 64 + lane;
        const unsigned long long b = __builtin_amdgcn_ballot_w64(v < N && x[v] != 0.f);
        if (lane == 0) bits[wd] = b;
    }
}

// flags[v * nb + k]: bit i = (x[16 k + i][v] != 0), nb = S / 16
__global__ __launch_bounds__(256) void k_flags16(int N, int nb, const float *__restrict__ x,
                                                 unsigned short *__restrict__ flags) {
    const long total = (long)N * nb;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int k = (int)(i / N), v = (int)(i - (long)k * N);    // consecutive threads: consecutive nodes
        unsigned f = 0u;
#pragma unroll
        for (int b = 0; b < 16; ++b) f |= (x[(size_t)(16 * k + b) * N + v] != 0.f ? 1u : 0u) << b;
        flags[(size_t)v * nb + k] = (unsigned short)f;
    }
}

hipError_t launch_nodeinfo(hipStream_t st, int N, int S, const float *x, const float *s_pos, const float *s_neg,
                           float *info, float *compact, const float *nbr_sp, unsigned long long *xbits, int p,
                           const float *theta3, const float *theta4, float *qvec) {
    if (N == 0) return qvec ? launch_qvec(st, p, theta3, theta4, qvec) : hipSuccess;
    const int ni = make_nodeinfo(info, S, false).ni;
    const long total = (long)N * ni;
    const int work_blocks = (int)min((total + 255) / 256, (long)65535);
    k_nodeinfo<<<work_blocks + (qvec ? 1 : 0), 256, 0, st>>>(N, S, ni, x, s_pos, s_neg, info, S == 1 ? compact : nullptr,
                                                             (S == 1 || S % 16 == 0) ? nbr_sp : nullptr, p, theta3,
                                                             theta4, qvec, work_blocks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !xbits) return e;
    if (S % 16 == 0) {
        const long total = (long)N * (S / 16);
        k_flags16<<<(int)min((total + 255) / 256, (long)65536), 256, 0, st>>>(N, S / 16, x,
                                                                             reinterpret_cast<unsigned short *>(xbits));
        return hipGetLastError();
    }
    if (S != 1) return e;
    const int n_words = (N + 63) / 64;
    k_xbits<<<min((n_words + 3) / 4, 16384), 256, 0, st>>>(N, x, xbits);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Records for per-state residual graphs (what the paper's Tuples2Graphs builds explicitly, Alg. 4):
// in state s every edge with an endpoint in that state's solution (x_s != 0) is absent.  So for a
// solution node all three scalars of that state are zero (isolated, and its recomputed round-1 row
// is zero for its neighbours); any other node keeps x (= 0) and gets
//   s+ = sum max(w, 0),  s- = sum max(-w, 0)   over its neighbours u with x_s[u] == 0.
// Pass 1 copies x into the records and clears the sums, pass 2 writes the sums of ordinary rows
// (one thread per (v, s); a neighbour is in the solution when its x in the records is non-zero),
// pass 3 those of the long rows (one wave per (long row, s)), pass 4 clears x of the solution nodes.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_stateinfo_x(int N, int S, int ni, const float *__restrict__ x,
                                                     float *__restrict__ info) {
    const long total = (long)N * ni;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int v = (int)(i / ni), c = (int)(i - (long)v * ni);
        info[i] = c < S ? x[(size_t)c * N + v] : 0.f;
    }
}

__global__ __launch_bounds__(256) void k_stateinfo_sums(int N, int S, int ni, const int32_t *__restrict__ rowptr,
                                                        const int32_t *__restrict__ rowend,
                                                        const int32_t *__restrict__ colidx, const float *__restrict__ w,
                                                        float *__restrict__ info) {
    const long total = (long)N * S;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int v = (int)i / S, s = (int)i - v * S;   // N * S < 2^31: 32-bit division
        const int b = rowptr[v], e = rowend[v];
        float *mine = info + (size_t)v * ni;
        if (e - b > kHubDegree || mine[s] != 0.f) continue;   // long rows: pass 3; solution nodes keep zero sums
        double sp = 0.0, sn = 0.0;
        for (int j = b; j < e; ++j) {
            if (info[(size_t)colidx[j] * ni + s] != 0.f) continue;   // neighbour in the solution
            const float wj = w ? w[j] : 1.f;
            sp += (double)fmaxf(wj, 0.f);
            sn += (double)fmaxf(-wj, 0.f);
        }
        mine[S + s] = (float)sp;
        mine[2 * S + s] = (float)sn;
    }
}

__global__ __launch_bounds__(256) void k_stateinfo_hubs(int S, int ni, HubTable ht, const int32_t *__restrict__ rowptr,
                                                        const int32_t *__restrict__ rowend,
                                                        const int32_t *__restrict__ colidx, const float *__restrict__ w,
                                                        float *__restrict__ info) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long items = (long)ht.n_hubs * S;
    for (long it = (long)blockIdx.x * 4 + wave; it < items; it += (long)gridDim.x * 4) {
        const int h = (int)(it / S), s = (int)(it - (long)h * S);
        const int v = ht.hub_rows[h];
        const int b = rowptr[v], e = rowend[v];
        float *mine = info + (size_t)v * ni;
        if (e - b <= kHubDegree || mine[s] != 0.f) continue;   // wave-uniform
        double sp = 0.0, sn = 0.0;
        for (int j = b + lane; j < e; j += 64) {
            if (info[(size_t)colidx[j] * ni + s] != 0.f) continue;
            const float wj = w ? w[j] : 1.f;
            sp += (double)fmaxf(wj, 0.f);
            sn += (double)fmaxf(-wj, 0.f);
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            sp += __shfl_xor(sp, m);
            sn += __shfl_xor(sn, m);
        }
        if (lane == 0) {
            mine[S + s] = (float)sp;
            mine[2 * S + s] = (float)sn;
        }
    }
}

__global__ __launch_bounds__(256) void k_stateinfo_clear_x(int N, int S, int ni, float *__restrict__ info,
                                                           float *__restrict__ compact) {
    const long total = (long)N * S;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int v = (int)i / S, s = (int)i - v * S;   // N * S < 2^31: 32-bit division
        float *mine = info + (size_t)v * ni;
        mine[s] = 0.f;   // a live node has x = 0 already, a solution node gets it now
        // S = 1 (see k_nodeinfo): x is 0 for every node here
        if (compact) compact[v] = mine[2] == 0.f ? mine[1] : __int_as_float(0x7fc00000);
    }
}

hipError_t launch_stateinfo_residual(hipStream_t st, int N, int S, const HubTable &ht, const int32_t *rowptr,
                                     const int32_t *rowend, const int32_t *colidx, const float *w, const float *x,
                                     float *info, float *compact) {
    if (N == 0) return hipSuccess;
    const int ni = make_nodeinfo(info, S, true).ni;
    const long total = (long)N * S;
    const int grid = (int)min((total + 255) / 256, (long)65536);
    k_stateinfo_x<<<(int)min(((long)N * ni + 255) / 256, (long)65536), 256, 0, st>>>(N, S, ni, x, info);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_stateinfo_sums<<<grid, 256, 0, st>>>(N, S, ni, rowptr, rowend, colidx, w, info);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ht.n_hubs > 0) {
        const long items = (long)ht.n_hubs * S;
        k_stateinfo_hubs<<<(int)min((items + 3) / 4, (long)65536), 256, 0, st>>>(S, ni, ht, rowptr, rowend, colidx, w,
                                                                                 info);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    k_stateinfo_clear_x<<<grid, 256, 0, st>>>(N, S, ni, info, S == 1 ? compact : nullptr);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Rounds 2..T of Eq. 1, fused: neighbour sum (CSR gather of p-float rows), theta2 product on
// the matrix cores, the round-invariant terms, relu.  The matrix being updated is viewed as
// [N*S][p]: row r = (node v = r / S, state s = r % S); the neighbours of row r are the rows
// (u, s) for u in N(v).  A wave owns 16 consecutive rows at a time: it gathers their sums into
// its own LDS tile, multiplies the tile by theta2 and writes the 16 output rows.
//   NODE: S is a multiple of 16, so a tile is 16 states of one node (contiguous 1 KB loads).
//   MU1 : this is round 2; the neighbours' round-1 rows are recomputed from their records instead of read.
//   GSUM: also emit this workgroup's column sums of the output, the first stage of the graph sum of
//         Alg. 2 line 4 (one graph only): gpart[blockIdx.x][P] for S == 1; in node mode with S == 16
//         every tile holds the same 16 states, so the sums are kept per state: gpart[blockIdx.x][16][P].
//   W   : the neighbour sum weights each neighbour by its entry of wagg (the reading of the
//         aggregation step of Alg. 1 as a product with the weighted adjacency).
//   QN  : this is the last round and Eq. 2 follows: also emit the node term of Q,
//         theta5[p:2p] . relu(theta7 mu_v), for every output row (row mode only).  The product with
//         theta7 runs on the matrix cores while the wave's next gather is already the bottleneck.
//   VAR = kRoundMaskOut (MO below): the last round of a training pass whose backward follows in the same call (node mode): of the
//         output only the relu mask is kept, one 64-bit word per (node, state) with bit j = entry j
//         positive, plus the rows of the action nodes (Eq. 2 is evaluated there) and whatever GSUM asks for.
//         The backward pass needs nothing else of mu^T, so its N*S*p floats are neither written nor read.
//   VAR = kRoundByState: row mode with the rows visited state by state (see the tile loop); a variant of
//         its own so that it shows under its own name in profiles.
// ------------------------------------------------------------------------------------------
//   VAR = kRoundFlags: node mode of round 2 when the flag words are there (info.flags16): the gather from the
//         records and its staging area in LDS are left out, which lets a fourth workgroup onto a compute unit.
constexpr int kRoundPlain = 0, kRoundMaskOut = 1, kRoundByState = 2, kRoundFlags = 3;
template <int P, bool NODE, bool MU1, bool GSUM, bool W, bool QN, int VAR = kRoundPlain>
#ifndef S2V_ROUND_OCC
#define S2V_ROUND_OCC 4
#endif
#ifndef S2V_ROUND2_OCC
#define S2V_ROUND2_OCC 4
#endif
// (node-mode round 2 also holds the record staging area in LDS: three workgroups per CU)
__global__ __launch_bounds__(kThreads, MU1 ? ((NODE && VAR != kRoundFlags) ? 3 : S2V_ROUND2_OCC) : S2V_ROUND_OCC) void k_round(int n_vrows, int S, const int32_t *__restrict__ rowptr,
                                                    const int32_t *__restrict__ rowend,
                                                    const int32_t *__restrict__ colidx,
                                                    const float *__restrict__ wagg,
                                                    const float *__restrict__ mu_in, float *__restrict__ mu_out,
                                                    NodeInfo info,
                                                    const float *__restrict__ theta1,
                                                    const float *__restrict__ theta2,
                                                    const float *__restrict__ qvec, float *__restrict__ gpart,
                                                    HubTable ht, const float *__restrict__ hub_sum,
                                                    const float *__restrict__ x_res, int N, int last, QHead qh,
                                                    MaskOut mo) {
    using G = Geo<P>;
    constexpr bool MO = VAR == kRoundMaskOut, SLICED = VAR == kRoundByState, FL = VAR == kRoundFlags;
    static_assert(!FL || (NODE && MU1), "the flag-word variant is node mode of round 2");
    static_assert(!SLICED || (!NODE && !MU1 && !GSUM && !QN), "the state-by-state order is a plain row-mode variant");
    static_assert(!(QN && NODE && MU1), "in node mode the node term of Q is fused into rounds that read rows");
    static_assert(!MO || (NODE && !MU1 && !QN), "mask output is a node-mode variant of the rounds that read rows");
    __shared__ __attribute__((aligned(16))) float lds[kWaves][kTileRows * G::STRIDE];
    __shared__ __attribute__((aligned(16))) float lds_b[P * G::STRIDE];   // theta2, the B operand
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *tile = lds[wave];
    const int li = lane % G::LPR;
    const int jl = lane & 15, gl = lane >> 4;

    // theta1, q+, q- of the epilogue live in LDS, not in registers, while a tile is gathered
    __shared__ float lds_c[3 * P];
    // staging area of the record gather (node mode of round 2 only)
    __shared__ __attribute__((aligned(16))) float rec_stage[(NODE && MU1 && !FL) ? kWaves * kRecStageFloats : 4];
    stage_matrix_lds<P>(lds_b, theta2, false);
    for (int i = threadIdx.x; i < 3 * P; i += kThreads) lds_c[i] = i < P ? theta1[i] : qvec[i - P];
    __syncthreads();
    constexpr int CS = NODE ? 4 : 1;   // node mode keeps the four tile rows of a lane apart (they are states)
    float csum[G::CB][CS];
#pragma unroll
    for (int cb = 0; cb < G::CB; ++cb)
#pragma unroll
        for (int k = 0; k < CS; ++k) csum[cb][k] = 0.f;
    Mu1Row mu1;
    if (MU1) {
        mu1.ni = info;
        mu1.s = 0;
        mu1.t1 = ld4(theta1 + 4 * li);
        mu1.qp = ld4(qvec + 4 * li);
        mu1.qn = ld4(qvec + P + 4 * li);
    }

    const size_t row_stride = (size_t)S * P;
    // Row mode visits the rows either in memory order (16 consecutive rows per tile) or, sliced, state by
    // state: tile row i is then (node v0 + i, state st), so that the launch works through one state's
    // N rows of p floats at a time (a working set S times smaller than the whole matrix).
    const int tps = (N + kWgRows - 1) / kWgRows;   // tiles per state when sliced
    const int n_tiles = SLICED ? tps * S : (n_vrows + kWgRows - 1) / kWgRows;
    // Node mode of round 2: a tile is one node with a handful of neighbours, and row range -> column indices ->
    // flag words -> records is a chain of four dependent trips to memory.  The row range and the first column
    // indices of the wave's NEXT tile are fetched while the current one is worked on.
    constexpr bool PF = NODE && MU1;
    int pf_b = 0, pf_e = 0, pf_cols = 0;
    if (PF) {
        const int r0 = blockIdx.x * kWgRows + wave * kTileRows;
        if ((int)blockIdx.x < n_tiles && r0 < n_vrows) {
            const int v0 = r0 / S;
            pf_b = rowptr[v0];
            pf_e = rowend[v0];
            pf_cols = (lane < min(64, pf_e - pf_b)) ? colidx[pf_b + lane] : 0;
        }
    }
    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        int r0, r_step, n_here;
        if (SLICED) {
            const int st = t / tps;
            const int v0 = (t - st * tps) * kWgRows + wave * kTileRows;
            r0 = v0 * S + st;
            r_step = S;
            n_here = N - v0;
        } else {
            r0 = t * kWgRows + wave * kTileRows;
            r_step = 1;
            n_here = n_vrows - r0;
        }
        // lane i (mod 16) carries the metadata of tile row i
        const int r = r0 + jl * r_step;
        const bool valid = jl < n_here;
        const int v = valid ? r / S : 0;
        const int s = valid ? r - v * S : 0;
        const int rb = PF ? pf_b : (valid ? rowptr[v] : 0);
        const int re = PF ? pf_e : (valid ? rowend[v] : 0);
        const int cols_first = pf_cols;
        int nx_b = 0, nx_e = 0;
        bool nx_ok = false;
        if (PF) {
            const int tn = t + gridDim.x, r0n = tn * kWgRows + wave * kTileRows;
            nx_ok = tn < n_tiles && r0n < n_vrows;
            if (nx_ok) {
                const int vn = r0n / S;
                nx_b = rowptr[vn];
                nx_e = rowend[vn];
            }
        }
        const float3 mine = valid ? info.get(v, s) : make_float3(0.f, 0.f, 0.f);
        const float sp = mine.y, sn = mine.z;
        float xs = mine.x;
        // Per-state residual graphs: a row whose node is in its state's solution is an isolated node.
        // Its record is zero (so it adds nothing to its neighbours); here it gets relu(theta1 x) in the
        // final round and zero before, whatever its (ignored) neighbour sum is.
        float keep = 1.f, cut = 1.f;     // cut = 0 drops the neighbour term of such a row
        if (x_res && valid) {
            const float xo = x_res[(size_t)s * N + v];
            if (xo != 0.f) { xs = xo; cut = 0.f; keep = last ? 1.f : 0.f; }
        }

        if (NODE) {
            // one node, 16 states: s0 = state of tile row 0
            const int b = __builtin_amdgcn_readfirstlane(rb), e = __builtin_amdgcn_readfirstlane(re);
            const int s0 = __builtin_amdgcn_readfirstlane(s);
            NodeAcc<P> acc;
            if (e - b > kHubDegree) {
                const int h = hub_index(ht, __builtin_amdgcn_readfirstlane(v));
                acc = load_node_block<P>(hub_sum + ((size_t)h * S + s0) * P, lane);
                store_node_block<P>(tile, acc, lane);
            } else if (MU1 && (FL || info.flags16)) {
                // flag words and the row's total instead of the neighbours' records
                gather_node_tile_flags<P, W>(tile, info, s0, lds_c, colidx, b, e, lane,
                                             info.node(__builtin_amdgcn_readfirstlane(v))[info.sn_off + 1], wagg,
                                             cols_first, PF);
            } else if (MU1 && !FL) {
                // the gather from the records works in the state-major lane layout
                acc = gather_node_block_mu1<P, W>(info, s0, theta1, qvec, colidx, wagg, b, e, lane,
                                                  rec_stage + ((NODE && MU1 && !FL) ? wave * kRecStageFloats : 0));
                store_node_block_sm<P>(tile, acc, lane);
            } else if (!MU1) {
                acc = gather_node_block<P, W>(mu_in, row_stride, (size_t)s0 * P, colidx, wagg, b, e, lane);
                store_node_block<P>(tile, acc, lane);
            }
            if (PF) {
                // the next tile's first column indices (its row range has arrived by now)
                pf_cols = (nx_ok && lane < min(64, nx_e - nx_b)) ? colidx[nx_b + lane] : 0;
                pf_b = nx_b;
                pf_e = nx_e;
            }
        } else {
            // The long rows of the tile first: their sums are ready in hub_sum, and all lanes fetch
            // them together (each lane looks up its own row, then RPI rows per wave-wide load).
            const bool long_mine = re - rb > kHubDegree;
            if (__builtin_amdgcn_ballot_w64(long_mine) != 0ull) {
                const int h_mine = long_mine ? hub_index(ht, v) : -1;
                constexpr int RPI = G::NPL, NC = 16 / RPI;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int i = c * RPI + lane / G::LPR;
                    const int hi = __shfl(h_mine, i), si = __shfl(s, i);
                    if (hi >= 0) {
                        float4 a;
                        if (ht.fold) {
                            // (hub_sum holds the segment sums: added here in segment order, as k_hub_combine would)
                            a = make_float4(0.f, 0.f, 0.f, 0.f);
                            for (int seg = ht.hub_seg_off[hi]; seg < ht.hub_seg_off[hi + 1]; ++seg)
                                a = add4(a, ld4(hub_sum + ((size_t)seg * S + si) * P + 4 * li));
                        } else {
                            a = ld4(hub_sum + ((size_t)hi * S + si) * P + 4 * li);
                        }
                        st4(tile + i * G::STRIDE + 4 * li, a);
                    }
                }
            }
            if (MU1 && S == 1 && (!W || info.xbits)) {
                // single state, round 2: one lane per neighbour, the whole tile's records in flight
                if (info.xbits)
                    gather_tile_mu1_single<P, 2, W>(tile, info.base, nullptr, info.xbits, lds_c, colidx, rb, re, kHubDegree,
                                                    lane, valid ? info.base[(size_t)v * 4 + 3] : 0.f, wagg);
                else if (W) {}
                else if (info.compact)
                    gather_tile_mu1_levels<P, 1>(tile, info.base, info.compact, lds_c, colidx, rb, re, kHubDegree, lane);
                else
                    gather_tile_mu1_levels<P, 0>(tile, info.base, nullptr, lds_c, colidx, rb, re, kHubDegree, lane);
            } else if (MU1 && S > 1) {
                // several states, round 2: the same with the general records
                gather_tile_mu1_rows<P, W>(tile, info, s, lds_c, colidx, wagg, rb, re, kHubDegree, lane);
            } else {
            int b_next = __builtin_amdgcn_readlane(rb, 0), e_next = __builtin_amdgcn_readlane(re, 0);
            int cols_next = (lane < min(64, e_next - b_next)) ? colidx[b_next + lane] : 0;
#pragma unroll 1
            for (int i = 0; i < kTileRows; ++i) {
                const int b = b_next, e = e_next;
                const int cols = cols_next;
                const int si = __builtin_amdgcn_readlane(s, i);   // (i is wave-uniform)
                if (i + 1 < kTileRows) {
                    b_next = __builtin_amdgcn_readlane(rb, i + 1);
                    e_next = __builtin_amdgcn_readlane(re, i + 1);
                    // long rows need no indices here
                    cols_next = (e_next - b_next <= kHubDegree && lane < min(64, e_next - b_next)) ? colidx[b_next + lane] : 0;
                }
                if (e - b > kHubDegree) continue;   // stored by the pass above
                float4 a;
                if (MU1) {
                    if (S == 1) {
                        const float4 rp = make_float4(fmaxf(mu1.qp.x, 0.f), fmaxf(mu1.qp.y, 0.f), fmaxf(mu1.qp.z, 0.f),
                                                      fmaxf(mu1.qp.w, 0.f));
                        a = gather_row_sum_mu1_single<P, W>(info.base, mu1.t1, mu1.qp, mu1.qn, rp, colidx, wagg, b, e,
                                                            cols, lane);
                    } else {
                        mu1.s = si;
                        a = gather_row_sum<P, W>(mu1, colidx, wagg, b, e, cols, lane);
                    }
                } else {
                    const MemRow mem{mu_in, row_stride, (size_t)si * P + 4 * li};
                    a = gather_row_sum<P, W>(mem, colidx, wagg, b, e, cols, lane);
                }
                if (lane < G::LPR) st4(tile + i * G::STRIDE + 4 * lane, a);
            }
            }
        }
        __builtin_amdgcn_wave_barrier();
        const Frag<P> afrag = load_a_frag_lds<P>(tile, lane);
        __builtin_amdgcn_wave_barrier();
        f32x4 acc[G::CB];
#pragma unroll
        for (int cb = 0; cb < G::CB; ++cb) {
            acc[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
            acc[cb] = mfma_tile<P>(afrag, load_b_frag_lds<P>(lds_b, cb, lane), acc[cb]);
        }
        // lane (jl, gl) holds rows 4*gl + rr, columns 16*cb + jl
        float t1[G::CB], qp[G::CB], qn[G::CB];
#pragma unroll
        for (int cb = 0; cb < G::CB; ++cb) {
            t1[cb] = lds_c[16 * cb + jl];
            qp[cb] = lds_c[P + 16 * cb + jl];
            qn[cb] = lds_c[2 * P + 16 * cb + jl];
        }
        if constexpr (MO) {
            // (node mode: the tile is one node's 16 states, all of them real rows, or lies past the end)
            if (r0 < n_vrows) {
                const int vt = __builtin_amdgcn_readfirstlane(v);
                // is this node the action node of one of its 16 states?  Then its rows are written as usual.
                const bool hit = mo.action[s] == vt;   // lane jl looks at state s0 + jl
                const bool rows_out = __builtin_amdgcn_ballot_w64(hit) != 0ull;
                unsigned long long word = 0ull;   // lane st < 16: the mask word of state s0 + st
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int i = 4 * gl + rr;
                    const float xi = __shfl(xs, i), spi = __shfl(sp, i), sni = __shfl(sn, i);
                    float *out = mu_out + (size_t)(r0 + i) * P + jl;
#pragma unroll
                    for (int cb = 0; cb < G::CB; ++cb) {
                        const float o = fmaxf(__fmaf_rn(sni, qn[cb], __fmaf_rn(spi, qp[cb], __fmaf_rn(xi, t1[cb], acc[cb][rr]))), 0.f);
                        if (rows_out) out[16 * cb] = o;
                        if (GSUM) csum[cb][rr] += o;
                        // lane (jl, gl) answered for state 4*gl + rr, column 16*cb + jl
                        const unsigned long long bal = __builtin_amdgcn_ballot_w64(o > 0.f);
                        if ((lane & 3) == rr)
                            word |= ((bal >> (16 * ((lane >> 2) & 3))) & 0xFFFFull) << (16 * cb);
                    }
                }
                if (lane < 16) mo.words[(size_t)r0 + lane] = word;
            }
        } else {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int i = 4 * gl + rr;
            const float xi = __shfl(xs, i), spi = __shfl(sp, i), sni = __shfl(sn, i);
            const float keepi = __shfl(keep, i), cuti = __shfl(cut, i);
            const int ro = r0 + i * r_step;
            if (i < n_here) {
                float *out = mu_out + (size_t)ro * P + jl;
#pragma unroll
                for (int cb = 0; cb < G::CB; ++cb) {
                    // (the order of the fused multiply-adds is spelled out: the mask-output variant above must
                    //  reproduce these values bit for bit)
                    const float o = keepi * fmaxf(__fmaf_rn(sni, qn[cb], __fmaf_rn(spi, qp[cb],
                                                  __fmaf_rn(xi, t1[cb], cuti * acc[cb][rr]))), 0.f);
                    out[16 * cb] = o;
                    if (GSUM) csum[cb][NODE ? rr : 0] += o;
                    if (QN) tile[i * G::STRIDE + 16 * cb + jl] = o;
                }
            }
        }
        }
        if (QN) {
            // the finished tile (rows past the end hold stale values, never written out) times theta7
            __builtin_amdgcn_wave_barrier();
            const Frag<P> ofrag = load_a_frag_lds<P>(tile, lane);
            __builtin_amdgcn_wave_barrier();
            float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int cb = 0; cb < G::CB; ++cb) {
                f32x4 h = (f32x4){0.f, 0.f, 0.f, 0.f};
                h = mfma_tile<P>(ofrag, load_b_frag_rows<P>(qh.theta7, cb, lane), h);
                const float t5 = qh.theta5[P + 16 * cb + jl];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) part[rr] += t5 * fmaxf(h[rr], 0.f);
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
#pragma unroll
                for (int m = 1; m < 16; m <<= 1) part[rr] += __shfl_xor(part[rr], m);
            }
            if (jl == 0) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int ro = r0 + (4 * gl + rr) * r_step;
                    if (4 * gl + rr < n_here) {
                        const int vo = ro / S, so = ro - vo * S;
                        qh.q[(size_t)so * N + vo] = part[rr];
                    }
                }
            }
        }
    }
    if (GSUM) {
        // column sums of everything this workgroup wrote: lanes with equal jl, then the four waves
        __syncthreads();
        float *red = &lds[0][0];
        if (NODE) {
            // lane (jl, gl) holds states 4*gl + k, columns 16*cb + jl: only the four waves are left to add
#pragma unroll
            for (int cb = 0; cb < G::CB; ++cb)
#pragma unroll
                for (int k = 0; k < CS; ++k) red[(wave * 16 + 4 * gl + k) * P + 16 * cb + jl] = csum[cb][k];
            __syncthreads();
            for (int el = threadIdx.x; el < 16 * P; el += kThreads)
                gpart[(size_t)blockIdx.x * 16 * P + el] =
                    (red[el] + red[16 * P + el]) + (red[2 * 16 * P + el] + red[3 * 16 * P + el]);
        } else {
#pragma unroll
            for (int cb = 0; cb < G::CB; ++cb) {
                float c0 = csum[cb][0];
                c0 += __shfl_xor(c0, 16);
                c0 += __shfl_xor(c0, 32);
                if (gl == 0) red[wave * P + 16 * cb + jl] = c0;
            }
            __syncthreads();
            if (threadIdx.x < P)
                gpart[(size_t)blockIdx.x * P + threadIdx.x] =
                    (red[threadIdx.x] + red[P + threadIdx.x]) + (red[2 * P + threadIdx.x] + red[3 * P + threadIdx.x]);
        }
    }
}

int round_grid(long n_vrows) {
    const long n_tiles = (n_vrows + kWgRows - 1) / kWgRows;
    return (int)min(n_tiles, (long)kRoundGridMax);
}

template <int P>
static hipError_t launch_round_p(hipStream_t st, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                                 const int32_t *colidx, const float *wagg,
                                 const float *mu_in, float *mu_out, const NodeInfo &info, const float *theta1,
                                 const float *theta2, const float *qvec, bool from_scalars, float *gpart,
                                 const HubTable &ht, const float *hub_sum, const float *x_res, bool last,
                                 const QHead &qh, const MaskOut &mo, bool by_state) {
    const long n_vrows = (long)N * S;
    const int grid = round_grid(n_vrows);
    // (sliced: the caller asks for the state-by-state row order; it applies to the rounds that read rows
    //  and have no fused extras, and replaces node mode there)
    const bool sliced = by_state && S > 1 && !from_scalars && !gpart && !mo.words && !qh.q;
    const bool node = (S % 16) == 0 && !sliced;
#define S2V_LAUNCH_ROUND_Q(NODE, MU1, GSUM, WW, QQ)                                                                   \
    k_round<P, NODE, MU1, GSUM, WW, QQ><<<grid, kThreads, 0, st>>>((int)n_vrows, S, rowptr, rowend, colidx, wagg, mu_in,  \
                                                                   mu_out, info, theta1, theta2, qvec, gpart, ht,         \
                                                                   hub_sum, x_res, N, last ? 1 : 0, qh, mo)
#define S2V_LAUNCH_ROUND_W(NODE, MU1, GSUM, WW)                            \
    do {                                                                   \
        if (!(NODE && MU1) && qh.q) S2V_LAUNCH_ROUND_Q(NODE, MU1, GSUM, WW, !(NODE && MU1)); \
        else S2V_LAUNCH_ROUND_Q(NODE, MU1, GSUM, WW, false);               \
    } while (0)
#define S2V_LAUNCH_ROUND(NODE, MU1, GSUM)                \
    do {                                                 \
        if (wagg) S2V_LAUNCH_ROUND_W(NODE, MU1, GSUM, true); \
        else S2V_LAUNCH_ROUND_W(NODE, MU1, GSUM, false);     \
    } while (0)
    if (mo.words) {
        // checked by the caller: node mode, rows read from memory, fused graph sum, no per-state residuals
        if (!node || from_scalars || !gpart || x_res) return hipErrorInvalidValue;
        if (wagg)
            k_round<P, true, false, true, true, false, kRoundMaskOut><<<grid, kThreads, 0, st>>>(
                (int)n_vrows, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, gpart, ht,
                hub_sum, x_res, N, 1, qh, mo);
        else
            k_round<P, true, false, true, false, false, kRoundMaskOut><<<grid, kThreads, 0, st>>>(
                (int)n_vrows, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, gpart, ht,
                hub_sum, x_res, N, 1, qh, mo);
        return hipGetLastError();
    }
    if (sliced) {
        if (wagg)
            k_round<P, false, false, false, true, false, kRoundByState><<<grid, kThreads, 0, st>>>(
                (int)n_vrows, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, gpart, ht,
                hub_sum, x_res, N, last ? 1 : 0, qh, mo);
        else
            k_round<P, false, false, false, false, false, kRoundByState><<<grid, kThreads, 0, st>>>(
                (int)n_vrows, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, gpart, ht,
                hub_sum, x_res, N, last ? 1 : 0, qh, mo);
        return hipGetLastError();
    }
    if (node && from_scalars && info.flags16 && !qh.q) {
#define S2V_LAUNCH_ROUND_FL(GSUM, WW)                                                                                  \
    k_round<P, true, true, GSUM, WW, false, kRoundFlags><<<grid, kThreads, 0, st>>>(                                   \
        (int)n_vrows, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, gpart, ht, hub_sum, \
        x_res, N, last ? 1 : 0, qh, mo)
        if (gpart) { if (wagg) S2V_LAUNCH_ROUND_FL(true, true); else S2V_LAUNCH_ROUND_FL(true, false); }
        else { if (wagg) S2V_LAUNCH_ROUND_FL(false, true); else S2V_LAUNCH_ROUND_FL(false, false); }
#undef S2V_LAUNCH_ROUND_FL
    } else if (node && gpart) {
        if (from_scalars) S2V_LAUNCH_ROUND(true, true, true);
        else S2V_LAUNCH_ROUND(true, false, true);
    } else if (node) {
        if (from_scalars) S2V_LAUNCH_ROUND(true, true, false);
        else S2V_LAUNCH_ROUND(true, false, false);
    } else if (gpart) {
        if (from_scalars) S2V_LAUNCH_ROUND(false, true, true);
        else S2V_LAUNCH_ROUND(false, false, true);
    } else {
        if (from_scalars) S2V_LAUNCH_ROUND(false, true, false);
        else S2V_LAUNCH_ROUND(false, false, false);
    }
#undef S2V_LAUNCH_ROUND
#undef S2V_LAUNCH_ROUND_W
#undef S2V_LAUNCH_ROUND_Q
    return hipGetLastError();
}

// gpart != NULL asks for the fused column sums (only legal for a single graph and S == 1 or S == 16).
hipError_t launch_round(hipStream_t st, int p, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                        const int32_t *colidx, const float *wagg, const float *mu_in, float *mu_out, const NodeInfo &info,
                        const float *theta1,
                        const float *theta2, const float *qvec, bool from_scalars, float *gpart, const HubTable &ht,
                        const float *hub_sum, const float *x_res, bool last, const QHead &qh, const MaskOut &mo,
                        bool by_state) {
    if ((long)N * S == 0) return hipSuccess;
    if (p == 32)
        return launch_round_p<32>(st, N, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, from_scalars,
                                  gpart, ht, hub_sum, x_res, last, qh, mo, by_state);
    return launch_round_p<64>(st, N, S, rowptr, rowend, colidx, wagg, mu_in, mu_out, info, theta1, theta2, qvec, from_scalars, gpart,
                              ht, hub_sum, x_res, last, qh, mo, by_state);
}

// ------------------------------------------------------------------------------------------
// Hub pre-pass.  Stage A: one wave per (segment, block of rows of that node) sums at most
// kHubDegree neighbour rows with the same gather code as the round kernel.  Stage B adds the
// segment partials of each hub in segment order.
// ------------------------------------------------------------------------------------------
template <int P, bool NODE, int SRC, bool W>   // SRC: 0 rows in memory, 1 round-1 rows from scalars, 2 relu-mask bits
__global__ __launch_bounds__(kThreads) void k_hub_partial(int S, HubTable ht,
                                                          const int32_t *__restrict__ rowend,
                                                          const int32_t *__restrict__ colidx,
                                                          const float *__restrict__ wagg,
                                                          const float *__restrict__ src,
                                                          NodeInfo info,
                                                          const float *__restrict__ theta1,
                                                          const float *__restrict__ qvec,
                                                          const unsigned long long *__restrict__ mask,
                                                          float *__restrict__ partial) {
    using G = Geo<P>;
    __shared__ __attribute__((aligned(16))) unsigned bits_stage[(NODE && SRC == 2) ? kWaves * kBitsStageBytes / 4 : 4];
    __shared__ __attribute__((aligned(16))) float rec_stage[(NODE && SRC == 1) ? kWaves * kRecStageFloats : 4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane % G::LPR;
    const int bpn = NODE ? S / 16 : S;  // blocks per node
    const long items = (long)ht.n_segs * bpn;
    for (long item = (long)blockIdx.x * kWaves + wave; item < items; item += (long)gridDim.x * kWaves) {
        const int seg = (int)(item / bpn), blk = (int)(item - (long)seg * bpn);
        // a segment covers stored entries of one row; entries past the row's live end do not count
        const int b = ht.seg_begin[seg], e = min(ht.seg_end[seg], rowend[ht.seg_row[seg]]);
        if (NODE) {
            const int s0 = blk * 16;
            NodeAcc<P> acc;
            if (SRC == 1)
                acc = gather_node_block_mu1<P, W>(info, s0, theta1, qvec, colidx, wagg, b, e, lane,
                                                  rec_stage + ((NODE && SRC == 1) ? wave * kRecStageFloats : 0));
            else if (SRC == 2)
                acc = W ? gather_node_block_bits_w<P>(mask, S, s0, colidx, wagg, b, e, lane)
                        : gather_node_block_bits<P>(mask, S, s0, colidx, b, e, lane,
                                                    bits_stage + (NODE && SRC == 2 ? wave * (kBitsStageBytes / 4) : 0));
            else acc = gather_node_block<P, W>(src, (size_t)S * P, (size_t)s0 * P, colidx, wagg, b, e, lane);
            float *out = partial + ((size_t)seg * S + s0) * P;
            if (SRC == 1) {
                write_node_block_sm<P>(out, acc, lane);   // gathered in the state-major lane layout
            } else {
#pragma unroll
                for (int c = 0; c < 16 / G::NPL; ++c) st4(out + c * G::NPL * P + 4 * lane, acc.a[c]);
            }
        } else {
            const int s = blk;
            if (SRC == 1 && S == 1) {
                // single state: one lane per neighbour, the whole segment's loads in flight at once
                const int j = lane % P;
                const float v1 = gather_segment_mu1_lanes<P, W>(info.base, theta1[j], qvec[j], qvec[P + j], colidx, wagg, b,
                                                                e, lane);
                if (lane < P) partial[(size_t)seg * P + lane] = v1;
                continue;
            }
            const int cols = (lane < min(64, e - b)) ? colidx[b + lane] : 0;
            float4 a;
            if (SRC == 1) {
                const float4 t1 = ld4(theta1 + 4 * li), qp = ld4(qvec + 4 * li), qn = ld4(qvec + P + 4 * li);
                if (S == 1) {
                    // single state: neighbours with x = 0 and s- = 0 are summed as scalars
                    const float4 rp = make_float4(fmaxf(qp.x, 0.f), fmaxf(qp.y, 0.f), fmaxf(qp.z, 0.f), fmaxf(qp.w, 0.f));
                    a = gather_row_sum_mu1_single<P, W>(info.base, t1, qp, qn, rp, colidx, wagg, b, e, cols, lane);
                } else {
                    Mu1Row mu1{info, s, t1, qp, qn};
                    a = gather_row_sum<P, W>(mu1, colidx, wagg, b, e, cols, lane);
                }
            } else if (SRC == 2) {
                const BitsRow bits{mask, S, s, 4 * li};
                a = gather_row_sum<P, W>(bits, colidx, wagg, b, e, cols, lane);
            } else {
                const MemRow mem{src, (size_t)S * P, (size_t)s * P + 4 * li};
                a = gather_row_sum<P, W>(mem, colidx, wagg, b, e, cols, lane);
            }
            if (lane < G::LPR) st4(partial + ((size_t)seg * S + s) * P + 4 * lane, a);
        }
    }
}

__global__ __launch_bounds__(256) void k_hub_combine(int L, HubTable ht, const float *__restrict__ partial,
                                                     float *__restrict__ hub_sum) {
    const long total = (long)ht.n_hubs * L;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int h = (int)(i / L), c = (int)(i - (long)h * L);
        float acc = 0.f;
        for (int seg = ht.hub_seg_off[h]; seg < ht.hub_seg_off[h + 1]; ++seg) acc += partial[(size_t)seg * L + c];
        hub_sum[i] = acc;
    }
}

// hub_sum[h][c] = sum over the segments of hub h, in segment order, of partial[seg][c]  (c < L)
hipError_t launch_hub_combine(hipStream_t st, int L, const HubTable &ht, const float *partial, float *hub_sum) {
    const long total = (long)ht.n_hubs * L;
    if (total == 0) return hipSuccess;
    k_hub_combine<<<(int)min((total + 255) / 256, (long)65536), 256, 0, st>>>(L, ht, partial, hub_sum);
    return hipGetLastError();
}

hipError_t launch_hub_sums(hipStream_t st, int p, int S, const HubTable &ht, const int32_t *rowend,
                           const int32_t *colidx, const float *wagg, const float *src,
                           const NodeInfo &info, const float *theta1, const float *qvec,
                           const unsigned long long *mask, float *partial, float *hub_sum) {
    if (ht.n_hubs == 0) return hipSuccess;
    const bool node = (S % 16) == 0;
    const int kind = mask ? 2 : (src ? 0 : 1);
    // every long row a single segment: the segment sums ARE the row sums (segment h belongs to long row h),
    // so they are written where the row sums go and the pass that adds a row's segments is not launched
    const bool single = ht.n_segs == ht.n_hubs;
    if (single) partial = hub_sum;
    // (ht.fold: the caller's round kernel adds the segments; the caller passes the segment sums on as hub_sum)
    const bool no_combine = single || ht.fold != 0;
    const long items = (long)ht.n_segs * (node ? S / 16 : S);
    const int grid = (int)min((items + kWaves - 1) / kWaves, (long)65536);
#define S2V_LAUNCH_HUB_W(PP, NODE, SRC, WW)                                                                       \
    k_hub_partial<PP, NODE, SRC, WW><<<grid, kThreads, 0, st>>>(S, ht, rowend, colidx, wagg, src, info, theta1, qvec, \
                                                                mask, partial)
#define S2V_LAUNCH_HUB(PP, NODE, SRC)                   \
    do {                                                \
        if (wagg) S2V_LAUNCH_HUB_W(PP, NODE, SRC, true);    \
        else S2V_LAUNCH_HUB_W(PP, NODE, SRC, false);        \
    } while (0)
#define S2V_LAUNCH_HUB_P(PP)                                                                           \
    do {                                                                                               \
        if (node) {                                                                                    \
            if (kind == 0) S2V_LAUNCH_HUB(PP, true, 0); else if (kind == 1) S2V_LAUNCH_HUB(PP, true, 1);   \
            else S2V_LAUNCH_HUB(PP, true, 2);                                                          \
        } else {                                                                                       \
            if (kind == 0) S2V_LAUNCH_HUB(PP, false, 0); else if (kind == 1) S2V_LAUNCH_HUB(PP, false, 1); \
            else S2V_LAUNCH_HUB(PP, false, 2);                                                         \
        }                                                                                              \
    } while (0)
    if (p == 32) S2V_LAUNCH_HUB_P(32); else S2V_LAUNCH_HUB_P(64);
#undef S2V_LAUNCH_HUB_P
#undef S2V_LAUNCH_HUB
#undef S2V_LAUNCH_HUB_W
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || no_combine) return err;
    return launch_hub_combine(st, S * p, ht, partial, hub_sum);
}

// ------------------------------------------------------------------------------------------
// Per-graph sum of the final embedding (Alg. 2 lines 4-5), deterministic two stages:
// stage 1 sums each chunk of <= kChunkNodes nodes (a chunk lies inside one graph) column by
// column; stage 2 adds the chunk partials of each graph in chunk order, in double.
// The matrix is [N][L] with L = S*p columns.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_gsum_stage1(int L, const int32_t *__restrict__ chunk_begin,
                                                     const int32_t *__restrict__ chunk_end,
                                                     const float *__restrict__ mu, float *__restrict__ partial) {
    __shared__ float red[256];
    const int c = blockIdx.x;
    const int vb = chunk_begin[c], ve = chunk_end[c];
    const int tid = threadIdx.x;
    if (L >= 256) {
        for (int col = tid; col < L; col += 256) {
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
            int v = vb;
            for (; v + 4 <= ve; v += 4) {
                a0 += mu[(size_t)v * L + col];
                a1 += mu[(size_t)(v + 1) * L + col];
                a2 += mu[(size_t)(v + 2) * L + col];
                a3 += mu[(size_t)(v + 3) * L + col];
            }
            for (; v < ve; ++v) a0 += mu[(size_t)v * L + col];
            partial[(size_t)c * L + col] = (a0 + a1) + (a2 + a3);
        }
    } else {
        // L in {32, 64, 128}: 256 / L row groups, combined through LDS in group order
        const int groups = 256 / L;
        const int col = tid % L, grp = tid / L;
        float a0 = 0.f, a1 = 0.f;
        if (grp < groups) {
            int v = vb + grp;
            for (; v + groups < ve; v += 2 * groups) {
                a0 += mu[(size_t)v * L + col];
                a1 += mu[(size_t)(v + groups) * L + col];
            }
            if (v < ve) a0 += mu[(size_t)v * L + col];
        }
        red[tid] = a0 + a1;
        __syncthreads();
        if (grp == 0) {
            float s = red[col];
            for (int g = 1; g < groups; ++g) s += red[g * L + col];
            partial[(size_t)c * L + col] = s;
        }
    }
}

// Stage 2: per (graph, column) add the partial rows [row_begin, row_end) of that graph.  A block
// owns 16 columns; its 64 row lanes take rows round-robin (double accumulators, four loads in
// flight each) and are combined through LDS in lane order, so the result does not depend on timing.
__global__ __launch_bounds__(1024) void k_gsum_stage2(int p, int S, int G, const int32_t *__restrict__ graph_row_off,
                                                     int rows_if_single, const float *__restrict__ partial,
                                                     float *__restrict__ gsum) {
    __shared__ double red[64][17];
    const int L = S * p;
    const int blocks_per_graph = L / 16;
    const int g = blockIdx.x / blocks_per_graph;
    const int col = (blockIdx.x - g * blocks_per_graph) * 16 + (threadIdx.x & 15);
    const int rb = graph_row_off ? graph_row_off[g] : 0;
    const int re = graph_row_off ? graph_row_off[g + 1] : rows_if_single;
    const double acc = gsum_stage2_cols(L, col, rb, re, partial, red);
    if ((threadIdx.x >> 4) == 0) {
        const int s = col / p, j = col - s * p;
        gsum[((size_t)s * G + g) * p + j] = (float)acc;
    }
}

hipError_t launch_gsum(hipStream_t st, int p, int N, int S, int G, const ChunkTable &ct, const float *mu, float *partial,
                       float *gsum) {
    (void)N;
    const int L = S * p;
    if (ct.n_chunks > 0) {
        k_gsum_stage1<<<ct.n_chunks, 256, 0, st>>>(L, ct.chunk_begin, ct.chunk_end, mu, partial);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    k_gsum_stage2<<<G * (L / 16), 1024, 0, st>>>(p, S, G, ct.graph_chunk_off, 0, partial, gsum);
    return hipGetLastError();
}

// Second stage alone, over `rows` partial rows of S * p floats written by the last embedding round
// (one graph; S == 1 or S == 16).
hipError_t launch_gsum_from_round(hipStream_t st, int p, int S, int rows, const float *partial, float *gsum) {
    k_gsum_stage2<<<S * p / 16, 1024, 0, st>>>(p, S, 1, nullptr, rows, partial, gsum);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Eq. 2, graph term: qa[s][g] = theta5[0:p] . relu(theta6 gsum[s][g])   (one block per (s, g))
// ------------------------------------------------------------------------------------------
__global__ void k_qa(int p, const float *__restrict__ theta5, const float *__restrict__ theta6,
                     const float *__restrict__ gsum, float *__restrict__ qa) {
    __shared__ float gs[128];
    __shared__ float red[128];
    const int b = blockIdx.x;
    const float v = qa_value(p, theta5, theta6, gsum + (size_t)b * p, gs, red);
    if (threadIdx.x == 0) qa[b] = v;
}

hipError_t launch_qa(hipStream_t st, int p, int S, int G, const float *theta5, const float *theta6, const float *gsum,
                     float *qa) {
    k_qa<<<S * G, 128, 0, st>>>(p, theta5, theta6, gsum, qa);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Eq. 2, node term + sum: q[s][v] = qa[s][graph(v)] + theta5[p:2p] . relu(theta7 mu[v][s])
// Same 16-row wave tiles as the embedding round; the A operand comes straight from mu, theta7 is
// staged in LDS.  Streaming and latency-bound: four workgroups per CU, each wave two tiles ahead.
// ------------------------------------------------------------------------------------------
// The node term is already in q (written by the last embedding round): add the graph term.
__global__ __launch_bounds__(256) void k_qfinish(int N, int S, int G, const int32_t *__restrict__ graph_off,
                                                 const float *__restrict__ qa, float *__restrict__ q) {
    const long total = (long)N * S;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int s = (int)(i / N), v = (int)(i - (long)s * N);
        int g = 0;
        if (G > 1) {  // last graph whose offset is <= v
            int lo = 0, hi = G;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (graph_off[mid] <= v) lo = mid; else hi = mid;
            }
            g = lo;
        }
        q[i] = qa[(size_t)s * G + g] + q[i];
    }
}

hipError_t launch_qfinish(hipStream_t st, int N, int S, int G, const int32_t *graph_off, const float *qa, float *q) {
    const long total = (long)N * S;
    if (total == 0) return hipSuccess;
    k_qfinish<<<(int)min((total + 255) / 256, (long)8192), 256, 0, st>>>(N, S, G, graph_off, qa, q);
    return hipGetLastError();
}

template <int P>
__global__ __launch_bounds__(kThreads, 4) void k_qnode(int n_vrows, int N, int S, int G,
                                                    const int32_t *__restrict__ graph_off,
                                                    const float *__restrict__ theta5,
                                                    const float *__restrict__ theta7, const float *__restrict__ mu,
                                                    const float *__restrict__ qa, float *__restrict__ q) {
    using Ge = Geo<P>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int jl = lane & 15, gl = lane >> 4;
    __shared__ __attribute__((aligned(16))) float lds[kWaves][kTileRows * Ge::STRIDE];
    __shared__ __attribute__((aligned(16))) float lds_b[P * Ge::STRIDE];   // theta7, the B operand
    stage_matrix_lds<P>(lds_b, theta7, false);
    __syncthreads();
    float t5[Ge::CB];
#pragma unroll
    for (int cb = 0; cb < Ge::CB; ++cb) t5[cb] = theta5[P + 16 * cb + jl];
    // The wave's 16 x P tile is 16 contiguous rows: fetch it with fully coalesced float4 loads (two
    // tiles ahead of the arithmetic) and turn it into matrix-core fragments through LDS.
    float *tile = lds[wave];
    constexpr int MV = (kTileRows * Ge::LPR) / 64;
    const int n_tiles = (n_vrows + kWgRows - 1) / kWgRows;
    float4 cur[MV], nxt[MV];
    auto fetch = [&](int t, float4 *dst) {
        const int r0 = t * kWgRows + wave * kTileRows;
#pragma unroll
        for (int c = 0; c < MV; ++c) {
            const int f = c * 64 + lane, row = f / Ge::LPR, col4 = f % Ge::LPR;
            dst[c] = (t < n_tiles && r0 + row < n_vrows) ? ld4(mu + (size_t)(r0 + row) * P + 4 * col4)
                                                         : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    fetch(blockIdx.x, cur);
    fetch(blockIdx.x + gridDim.x, nxt);
    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int r0 = t * kWgRows + wave * kTileRows;
#pragma unroll
        for (int c = 0; c < MV; ++c) {
            const int f = c * 64 + lane;
            st4(tile + (f / Ge::LPR) * Ge::STRIDE + 4 * (f % Ge::LPR), cur[c]);
            cur[c] = nxt[c];
        }
        fetch(t + 2 * gridDim.x, nxt);
        __builtin_amdgcn_wave_barrier();
        const Frag<P> afrag = load_a_frag_lds<P>(tile, lane);
        __builtin_amdgcn_wave_barrier();
        if (r0 >= n_vrows) continue;
        float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cb = 0; cb < Ge::CB; ++cb) {
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
            acc = mfma_tile<P>(afrag, load_b_frag_lds<P>(lds_b, cb, lane), acc);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) part[rr] += t5[cb] * fmaxf(acc[rr], 0.f);
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
#pragma unroll
            for (int m = 1; m < 16; m <<= 1) part[rr] += __shfl_xor(part[rr], m);
        }
        if (jl == 0) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = r0 + 4 * gl + rr;
                if (r < n_vrows) {
                    const int v = r / S, s = r - v * S;
                    int g = 0;
                    if (G > 1) {  // last graph whose offset is <= v
                        int lo = 0, hi = G;
                        while (hi - lo > 1) {
                            const int mid = (lo + hi) >> 1;
                            if (graph_off[mid] <= v) lo = mid; else hi = mid;
                        }
                        g = lo;
                    }
                    q[(size_t)s * N + v] = qa[(size_t)s * G + g] + part[rr];
                }
            }
        }
    }
}

hipError_t launch_qnode(hipStream_t st, int p, int N, int S, int G, const int32_t *graph_off, const float *theta5,
                        const float *theta7, const float *mu, const float *qa, float *q) {
    const long n_vrows = (long)N * S;
    if (n_vrows == 0) return hipSuccess;
    const long n_tiles = (n_vrows + kWgRows - 1) / kWgRows;
    const int grid = (int)min(n_tiles, (long)(256 * 16));
    if (p == 32) k_qnode<32><<<grid, kThreads, 0, st>>>((int)n_vrows, N, S, G, graph_off, theta5, theta7, mu, qa, q);
    else k_qnode<64><<<grid, kThreads, 0, st>>>((int)n_vrows, N, S, G, graph_off, theta5, theta7, mu, qa, q);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Read-only streaming probe for benchmarks: every 16-byte word of [src, src + bytes) is loaded once,
// fully coalesced, and folded into one float per workgroup (so the loads cannot be dropped).  Gives the
// rate at which this GPU streams memory it only reads, the comparable ceiling for the gather rounds.
// ------------------------------------------------------------------------------------------
constexpr int kStreamReadGrid = 256 * 16;
__global__ __launch_bounds__(256) void k_stream_read(const float4 *__restrict__ src, size_t n16, float *__restrict__ out) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a, c = a, d = a;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const float4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        a = add4(a, v0); b = add4(b, v1); c = add4(c, v2); d = add4(d, v3);
    }
    for (; i < n16; i += stride) a = add4(a, src[i]);
    a = add4(add4(a, b), add4(c, d));
    float s = (a.x + a.y) + (a.z + a.w);
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m);
    __shared__ float red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

hipError_t launch_stream_read(hipStream_t st, const void *src, size_t bytes, float *out /*[kStreamReadGrid]*/) {
    k_stream_read<<<kStreamReadGrid, 256, 0, st>>>(static_cast<const float4 *>(src), bytes / 16, out);
    return hipGetLastError();
}

}  // namespace s2v
