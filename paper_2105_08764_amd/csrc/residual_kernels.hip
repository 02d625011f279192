// State update of the inference loop (Alg. 3 lines 8-10): add the selected nodes to the partial
// solution, remove the edges connected to them, and recompute the candidate set.  The graph is a
// mutable CSR copy whose rows shrink in place: row v keeps its start rowptr[v] and gets a live
// end rowend[v]; entries whose neighbour joined the solution are squeezed out (order kept), and
// the rows of solution nodes become empty.  The round-invariant edge sums s+ / s- are refreshed
// in the same pass, so no new graph preparation is needed between steps.
#include "internal.h"
#include "loop_util.h"

namespace s2v {

__global__ void k_zero_stats(int n, int32_t *__restrict__ stats) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) stats[i] = 0;
}

// Squeeze the entries of row v whose neighbour is in the solution out of the row (one wave; the
// order of the survivors is kept), refresh s+ / s- over the survivors, and return the new length.
// A row of a solution node becomes empty.  Every lane returns the same value.
// The row is taken in batches of four 64-entry chunks whose loads (entries, then the neighbours' x) are issued
// together: two trips to memory per 256 entries.  Survivors are written at or below the place they were read
// from, and a batch is read completely before any of its survivors is written, so the squeeze works in place.
__device__ __forceinline__ int filter_row(int v, int lane, const int32_t *__restrict__ rowptr,
                                          int32_t *__restrict__ rowend, int32_t *__restrict__ colidx,
                                          float *__restrict__ w, const float *__restrict__ x,
                                          float *__restrict__ s_pos, float *__restrict__ s_neg,
                                          float *rec = nullptr, float *compact = nullptr) {
    constexpr int B = 4;
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int b = rowptr[v], e = rowend[v];
    int out = 0;
    double sp = 0.0, sn = 0.0;
    if (x[v] == 0.f) {
        for (int base = b; base < e; base += 64 * B) {
            int c[B];
            float ww[B], xc[B];
#pragma unroll
            for (int k = 0; k < B; ++k) {
                const int i = base + 64 * k + lane;
                const bool have = i < e;
                c[k] = have ? colidx[i] : -1;
                ww[k] = have ? (w ? w[i] : 1.f) : 0.f;
            }
#pragma unroll
            for (int k = 0; k < B; ++k) xc[k] = c[k] >= 0 ? x[c[k]] : 1.f;
#pragma unroll
            for (int k = 0; k < B; ++k) {
                const bool keep = c[k] >= 0 && xc[k] == 0.f;
                const unsigned long long m = __ballot(keep);
                if (keep) {
                    const int pos = b + out + __popcll(m & lt);   // never beyond the entry just read
                    colidx[pos] = c[k];
                    if (w) w[pos] = ww[k];
                    sp += (double)fmaxf(ww[k], 0.f);
                    sn += (double)fmaxf(-ww[k], 0.f);
                }
                out += __popcll(m);
            }
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
        refresh_record(rec, compact, v, x[v], (float)sp, (float)sn);
    }
    return out;
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
// First half (begin_update): the selected nodes join the solution and their rows become empty; the stored entries
// of such a row stay in place and touched[v] = -(its old length).
__global__ __launch_bounds__(256) void k_begin_update(UpdateState u, const int32_t *__restrict__ sel_idx,
                                                      const int32_t *__restrict__ sel_count) {
    begin_update(u, sel_idx, sel_count, blockIdx.x * 256 + threadIdx.x, gridDim.x * 256);
    if (blockIdx.x == 0 && threadIdx.x == 0) u.epoch[0] += 1;
}

// Second half: blockIdx.y walks the selected nodes, the waves of the blocks along x the entries their rows had.
// Each neighbour u outside the solution is filtered once per update: the first wave to stamp touched[u] with the
// update's number does it (a solution node's row is empty already, and its touched word holds a length).
// The outcome of a row does not depend on the order in which rows are processed; the counters move by the change.
__global__ __launch_bounds__(256) void k_refilter_neighbours(int total, int k, const int32_t *__restrict__ sel_idx,
                                                             const int32_t *__restrict__ sel_count,
                                                             const int32_t *__restrict__ rowptr,
                                                             int32_t *__restrict__ rowend, int32_t *__restrict__ colidx,
                                                             float *__restrict__ w, const float *__restrict__ x,
                                                             float *__restrict__ s_pos, float *__restrict__ s_neg,
                                                             uint8_t *__restrict__ cand, int G,
                                                             const int32_t *__restrict__ graph_off,
                                                             int32_t *__restrict__ stats, int32_t *__restrict__ touched,
                                                             const int32_t *__restrict__ epoch, float *rec,
                                                             float *compact, const int32_t *__restrict__ jobs) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ep = epoch[0];
    for (int i = blockIdx.y; i < total; i += gridDim.y) {
        int b, len;
        if (jobs) {   // (the first half listed first entry and old length of every selected entry's row)
            b = jobs[2 * i];
            len = jobs[2 * i + 1];
        } else {
            const int g = i / k, j = i - g * k;
            if (j >= sel_count[g]) continue;
            const int v = sel_idx[i];
            if (v < 0) continue;
            len = -touched[v];
            b = rowptr[v];
        }
        if (len <= 0) continue;   // (the node had no live entry when it joined)
        for (int t = blockIdx.x * 4 + wave; t < len; t += gridDim.x * 4) {
            const int u = colidx[b + t];
            if (x[u] != 0.f) continue;
            int first = 0;
            if (lane == 0) first = atomicExch(&touched[u], ep) != ep ? 1 : 0;
            if (!__shfl(first, 0)) continue;
            const int old_len = rowend[u] - rowptr[u];
            const int old_cand = cand[u];
            const int out = filter_row(u, lane, rowptr, rowend, colidx, w, x, s_pos, s_neg, rec, compact);
            if (lane == 0) {
                const int new_cand = out > 0 ? 1 : 0;
                cand[u] = (uint8_t)new_cand;
                const int gg = graph_of(G, graph_off, u);
                if (new_cand != old_cand) atomicAdd(&stats[2 * gg], new_cand - old_cand);
                if (out != old_len) atomicAdd(&stats[2 * gg + 1], out - old_len);
            }
        }
    }
}

__global__ __launch_bounds__(256) void k_zero_i32(long n, int32_t *__restrict__ p) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) p[i] = 0;
}

hipError_t launch_zero_i32(hipStream_t st, long n, int32_t *p) {
    if (n <= 0) return hipSuccess;
    k_zero_i32<<<(int)min((n + 255) / 256, (long)4096), 256, 0, st>>>(n, p);
    return hipGetLastError();
}

// The decisions of one step of the loop and the first half of the state update that follows (see loop_util.h).
__global__ __launch_bounds__(256) void k_loop_control(int N, int adaptive, int32_t *__restrict__ sel_count,
                                                      unsigned long long *__restrict__ counters,
                                                      const int32_t *__restrict__ sel_idx, UpdateState u) {
    __shared__ unsigned long long s_live, s_picked;
    loop_control(N, adaptive, sel_count, counters, sel_idx, u, &s_live, &s_picked);
}

hipError_t launch_loop_control(hipStream_t st, int N, bool adaptive, int32_t *sel_count, unsigned long long *counters,
                               const int32_t *sel_idx, const UpdateState &u) {
    k_loop_control<<<1, 256, 0, st>>>(N, adaptive ? 1 : 0, sel_count, counters, sel_idx, u);
    return hipGetLastError();
}

// sel_idx == NULL: full pass over every row (state from x alone).  Otherwise incremental: cand, stats,
// rowend and s+- must be the outcome of the previous call; only rows next to the selection change.
// begun: launch_loop_control (or a kernel that runs loop_control) has done the first half already.
hipError_t launch_residual_update(hipStream_t st, int N, const UpdateState &u, int32_t *colidx, float *w,
                                  const int32_t *sel_idx, const int32_t *sel_count, bool begun) {
    hipError_t e;
    if (sel_idx && u.k > 0) {
        if (!begun) {
            k_begin_update<<<min((u.total + 255) / 256, 64), 256, 0, st>>>(u, sel_idx, sel_count);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        const int gy = min(u.total, 1024);
        const int gx = max(1, min(1024 / gy, (N + 3) / 4));
        k_refilter_neighbours<<<dim3(gx, gy), 256, 0, st>>>(u.total, u.k, sel_idx, sel_count, u.rowptr, u.rowend, colidx, w,
                                                           u.x, u.s_pos, u.s_neg, u.cand, u.G, u.graph_off, u.stats,
                                                           u.touched, u.epoch, u.rec, u.compact,
                                                           (u.jobs && u.total <= kUpdateJobs) ? u.jobs : nullptr);
        return hipGetLastError();
    }
    k_zero_stats<<<1, 256, 0, st>>>(2 * u.G, u.stats);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (N > 0) {
        const int grid = min((N + 3) / 4, 256 * 32);
        k_residual_rows<<<grid, 256, 0, st>>>(N, u.rowptr, u.rowend, colidx, w, u.x, u.s_pos, u.s_neg, u.cand, u.G,
                                              u.graph_off, u.stats);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace s2v
