// State update of the inference loop (Alg. 3 lines 8-10): add the selected nodes to the partial
// solution, remove the edges connected to them, and recompute the candidate set.  The graph is a
// mutable CSR copy whose rows shrink in place: row v keeps its start rowptr[v] and gets a live
// end rowend[v]; entries whose neighbour joined the solution are squeezed out (order kept), and
// the rows of solution nodes become empty.  The round-invariant edge sums s+ / s- are refreshed
// in the same pass, so no new graph preparation is needed between steps.
#include "internal.h"

namespace s2v {

__global__ __launch_bounds__(256) void k_mark_selected(int total, int k, const int32_t *__restrict__ idx,
                                                       const int32_t *__restrict__ count, float *__restrict__ x) {
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        const int g = i / k, j = i - g * k;
        if (j < count[g]) {
            const int v = idx[i];
            if (v >= 0) x[v] = 1.f;
        }
    }
}

__global__ void k_zero_stats(int n, int32_t *__restrict__ stats) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) stats[i] = 0;
}

// Squeeze the entries of row v whose neighbour is in the solution out of the row (one wave; the
// order of the survivors is kept), refresh s+ / s- over the survivors, and return the new length.
// A row of a solution node becomes empty.  Every lane returns the same value.
__device__ __forceinline__ int filter_row(int v, int lane, const int32_t *__restrict__ rowptr,
                                          int32_t *__restrict__ rowend, int32_t *__restrict__ colidx,
                                          float *__restrict__ w, const float *__restrict__ x,
                                          float *__restrict__ s_pos, float *__restrict__ s_neg) {
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int b = rowptr[v], e = rowend[v];
    int out = 0;
    double sp = 0.0, sn = 0.0;
    if (x[v] == 0.f) {
        for (int base = b; base < e; base += 64) {
            const int i = base + lane;
            const bool have = i < e;
            const int c = have ? colidx[i] : 0;
            const float ww = have ? (w ? w[i] : 1.f) : 0.f;
            const bool keep = have && x[c] == 0.f;
            const unsigned long long m = __ballot(keep);
            if (keep) {
                const int pos = b + out + __popcll(m & lt);   // never beyond the entry just read
                colidx[pos] = c;
                if (w) w[pos] = ww;
                sp += (double)fmaxf(ww, 0.f);
                sn += (double)fmaxf(-ww, 0.f);
            }
            out += __popcll(m);
        }
#pragma unroll
        for (int mm = 1; mm < 64; mm <<= 1) {
            sp += __shfl_xor(sp, mm);
            sn += __shfl_xor(sn, mm);
        }
    }
    if (lane == 0) {
        rowend[v] = b + out;
        s_pos[v] = (float)sp;
        s_neg[v] = (float)sn;
    }
    return out;
}

__device__ __forceinline__ int graph_of(int G, const int32_t *__restrict__ graph_off, int v) {
    if (G == 1) return 0;
    int lo = 0, hi = G;   // last graph whose offset is <= v
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (graph_off[mid] <= v) lo = mid; else hi = mid;
    }
    return lo;
}

// Full pass: one wave per row.  stats[g] = {candidates, live stored entries} of graph g (integer atomics).
__global__ __launch_bounds__(256) void k_residual_rows(int N, const int32_t *__restrict__ rowptr,
                                                       int32_t *__restrict__ rowend, int32_t *__restrict__ colidx,
                                                       float *__restrict__ w, const float *__restrict__ x,
                                                       float *__restrict__ s_pos, float *__restrict__ s_neg,
                                                       uint8_t *__restrict__ cand, int G,
                                                       const int32_t *__restrict__ graph_off,
                                                       int32_t *__restrict__ stats) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int my_cand = 0, my_live = 0;  // per-wave totals (single graph)
    for (int v = blockIdx.x * 4 + wave; v < N; v += gridDim.x * 4) {
        const int out = filter_row(v, lane, rowptr, rowend, colidx, w, x, s_pos, s_neg);
        if (lane == 0) {
            const bool is_cand = out > 0;   // a solution node's row is empty
            cand[v] = is_cand ? 1 : 0;
            if (G == 1) {
                my_cand += is_cand ? 1 : 0;
                my_live += out;
            } else if (out > 0) {
                const int g = graph_of(G, graph_off, v);
                atomicAdd(&stats[2 * g], 1);
                atomicAdd(&stats[2 * g + 1], out);
            }
        }
    }
    if (G == 1 && lane == 0 && (my_cand | my_live)) {
        atomicAdd(&stats[0], my_cand);
        atomicAdd(&stats[1], my_live);
    }
}

// ---- incremental update: only the rows next to the newly selected nodes change ------------------
// Step 1 (one wave per selected node v): list v and every live neighbour of v, each row once
// (`touched` is a per-node flag, test-and-set).  list[0] is the list length.
__global__ __launch_bounds__(256) void k_touch_rows(int total, int k, const int32_t *__restrict__ idx,
                                                    const int32_t *__restrict__ count,
                                                    const int32_t *__restrict__ rowptr,
                                                    const int32_t *__restrict__ rowend,
                                                    const int32_t *__restrict__ colidx, int32_t *__restrict__ touched,
                                                    int32_t *__restrict__ list) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = blockIdx.x * 4 + wave; i < total; i += gridDim.x * 4) {
        const int g = i / k, j = i - g * k;
        if (j >= count[g]) continue;
        const int v = idx[i];
        if (v < 0) continue;
        if (lane == 0 && atomicExch(&touched[v], 1) == 0) list[1 + atomicAdd(&list[0], 1)] = v;
        for (int e = rowptr[v] + lane; e < rowend[v]; e += 64) {
            const int u = colidx[e];
            if (atomicExch(&touched[u], 1) == 0) list[1 + atomicAdd(&list[0], 1)] = u;
        }
    }
}

// Step 2 (one wave per listed row): filter the row and move the counters by the change.  The
// outcome of a row does not depend on the order in which rows are processed.
__global__ __launch_bounds__(256) void k_refilter_rows(const int32_t *__restrict__ rowptr, int32_t *__restrict__ rowend,
                                                       int32_t *__restrict__ colidx, float *__restrict__ w,
                                                       const float *__restrict__ x, float *__restrict__ s_pos,
                                                       float *__restrict__ s_neg, uint8_t *__restrict__ cand, int G,
                                                       const int32_t *__restrict__ graph_off,
                                                       int32_t *__restrict__ stats, int32_t *__restrict__ touched,
                                                       const int32_t *__restrict__ list) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = list[0];
    for (int i = blockIdx.x * 4 + wave; i < n; i += gridDim.x * 4) {
        const int v = list[1 + i];
        const int old_len = rowend[v] - rowptr[v];
        const int old_cand = cand[v];
        const int out = filter_row(v, lane, rowptr, rowend, colidx, w, x, s_pos, s_neg);
        if (lane == 0) {
            const int new_cand = out > 0 ? 1 : 0;
            cand[v] = (uint8_t)new_cand;
            touched[v] = 0;
            const int g = graph_of(G, graph_off, v);
            if (new_cand != old_cand) atomicAdd(&stats[2 * g], new_cand - old_cand);
            if (out != old_len) atomicAdd(&stats[2 * g + 1], out - old_len);
        }
    }
}

__global__ void k_reset_list(int32_t *__restrict__ list) {
    if (threadIdx.x == 0) list[0] = 0;
}

__global__ __launch_bounds__(256) void k_zero_i32(long n, int32_t *__restrict__ p) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) p[i] = 0;
}

hipError_t launch_zero_i32(hipStream_t st, long n, int32_t *p) {
    if (n <= 0) return hipSuccess;
    k_zero_i32<<<(int)min((n + 255) / 256, (long)4096), 256, 0, st>>>(n, p);
    return hipGetLastError();
}

// The decisions of one step of the loop of Alg. 3, taken on the device so that the host need not read anything
// back between steps.  stats holds {candidates, live stored entries} per graph as the last state update left
// them (the state this step's scores were computed on); sel_count holds how many nodes the selection found per
// graph (it asked for the largest d of the rule).  For one graph and the adaptive rule of Sec. 4.5.1, d follows
// from the candidate count and the count is cut to d (the selection is ordered, so its first d entries are the
// top-d); when no edge is left anywhere the counts become zero and the state update that follows changes nothing.
// counters[0] += 1 when an edge was left (a policy evaluation that mattered), counters[1] += nodes added.
// The same launch also does the first two steps of the state update that follows: the selected nodes join the
// solution (x = 1, as k_mark_selected) and the work list of the incremental update is emptied (as k_reset_list).
__global__ __launch_bounds__(256) void k_loop_control(int G, int N, int adaptive, const int32_t *__restrict__ stats,
                                                      int32_t *__restrict__ sel_count,
                                                      unsigned long long *__restrict__ counters, int k,
                                                      const int32_t *__restrict__ sel_idx, float *__restrict__ x,
                                                      int32_t *__restrict__ list) {
    __shared__ unsigned long long s_live, s_picked;
    if (threadIdx.x == 0) { s_live = 0ull; s_picked = 0ull; }
    __syncthreads();
    unsigned long long live = 0ull;
    for (int b = threadIdx.x; b < G; b += 256) live += (unsigned long long)stats[2 * b + 1];
    if (live) atomicAdd(&s_live, live);
    __syncthreads();
    const bool going = s_live > 0ull;
    int d = 1;
    if (adaptive && G == 1) {
        const long long c = stats[0];
        d = 2 * c > N ? 8 : (4 * c > N ? 4 : (8 * c > N ? 2 : 1));
    }
    unsigned long long picked = 0ull;
    for (int b = threadIdx.x; b < G; b += 256) {
        const int c = going ? min(sel_count[b], d) : 0;
        sel_count[b] = c;
        picked += (unsigned long long)c;
    }
    if (picked) atomicAdd(&s_picked, picked);
    __syncthreads();
    if (threadIdx.x == 0 && going) {
        counters[0] += 1ull;
        counters[1] += s_picked;
    }
    if (threadIdx.x == 0) list[0] = 0;
    // (this block wrote the counts: after the barrier above every thread sees them)
    for (int i = threadIdx.x; i < G * k; i += 256) {
        const int g = i / k, j = i - g * k;
        if (j < sel_count[g]) {
            const int v = sel_idx[i];
            if (v >= 0) x[v] = 1.f;
        }
    }
}

hipError_t launch_loop_control(hipStream_t st, int G, int N, bool adaptive, const int32_t *stats, int32_t *sel_count,
                               unsigned long long *counters, int k, const int32_t *sel_idx, float *x, int32_t *list) {
    k_loop_control<<<1, 256, 0, st>>>(G, N, adaptive ? 1 : 0, stats, sel_count, counters, k, sel_idx, x, list);
    return hipGetLastError();
}

// sel_idx == NULL: full pass over every row (state from x alone).  Otherwise incremental: cand, stats,
// rowend and s+- must be the outcome of the previous call; only rows next to the selection change.
hipError_t launch_residual_update(hipStream_t st, int N, int G, const int32_t *graph_off, const int32_t *rowptr,
                                  int32_t *rowend, int32_t *colidx, float *w, float *x, const int32_t *sel_idx,
                                  const int32_t *sel_count, int k, float *s_pos, float *s_neg, uint8_t *cand,
                                  int32_t *stats, int32_t *touched, int32_t *list, bool marked) {
    hipError_t e;
    if (sel_idx && k > 0) {
        const int total = G * k;
        if (!marked) {   // (marked: launch_loop_control has set x and emptied the list already)
            k_mark_selected<<<min((total + 255) / 256, 1024), 256, 0, st>>>(total, k, sel_idx, sel_count, x);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            k_reset_list<<<1, 64, 0, st>>>(list);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        k_touch_rows<<<min((total + 3) / 4, 1024), 256, 0, st>>>(total, k, sel_idx, sel_count, rowptr, rowend, colidx,
                                                                touched, list);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        k_refilter_rows<<<1024, 256, 0, st>>>(rowptr, rowend, colidx, w, x, s_pos, s_neg, cand, G, graph_off, stats,
                                              touched, list);
        return hipGetLastError();
    }
    k_zero_stats<<<1, 256, 0, st>>>(2 * G, stats);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (N > 0) {
        const int grid = min((N + 3) / 4, 256 * 32);
        k_residual_rows<<<grid, 256, 0, st>>>(N, rowptr, rowend, colidx, w, x, s_pos, s_neg, cand, G, graph_off, stats);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace s2v
