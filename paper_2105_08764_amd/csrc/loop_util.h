// The end of one step of the loop of Alg. 3 as device functions, so that the kernel that finishes the selection
// can take the step's decisions and start the state update in the same launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2v {

__device__ __forceinline__ int graph_of(int G, const int32_t *__restrict__ graph_off, int v) {
    if (G == 1) return 0;
    int lo = 0, hi = G;   // last graph whose offset is <= v
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (graph_off[mid] <= v) lo = mid; else hi = mid;
    }
    return lo;
}

// What the incremental state update needs to know and change (Alg. 3 lines 8-10 on the mutable CSR copy).
struct UpdateState {
    int G, total, k;                     // total = G * k entries of sel_idx
    const int32_t *graph_off;
    const int32_t *rowptr;
    int32_t *rowend;
    float *x, *s_pos, *s_neg;
    uint8_t *cand;
    int32_t *stats;                      // [G][2]: candidates, live stored entries
    int32_t *touched;                    // [N]: > 0 the update that last filtered the row; < 0 see begin_update
    int32_t *epoch;                      // [1]: number of updates so far
    // optional (inside the inference loop): the single-state node records {x, s+, s-, 0} [N][4] and the table
    // compact[v] = s+ of a node with x = 0 and s- = 0, NaN for any other, kept current for the rows that change
    float *rec, *compact;
    // [kUpdateJobs][2]: first entry and old length of the row of selected entry i (written for every i when
    // total <= kUpdateJobs), so that the second half finds a row's entries with one load
    int32_t *jobs;
};
constexpr int kUpdateJobs = 64;

// The record of node v after its x, s+ or s- changed.
__device__ __forceinline__ void refresh_record(float *rec, float *compact, int v, float xv, float sp, float sn) {
    if (!rec) return;
    rec[(size_t)v * 4 + 0] = xv;
    rec[(size_t)v * 4 + 1] = sp;
    rec[(size_t)v * 4 + 2] = sn;
    if (compact) compact[v] = (xv == 0.f && sn == 0.f) ? sp : __int_as_float(0x7fc00000);
}

// First half of the incremental state update, by the threads [tid, tid + stride, ...) of one or more workgroups:
// every selected node joins the solution (x = 1) and its row becomes empty.  The row's stored entries stay where
// they are, and touched[v] = -(the length it had): the second half (k_refilter_neighbours) walks them to find
// the rows that lose an entry.  A node listed twice is emptied once (the exchange on its row end decides).
__device__ __forceinline__ void begin_update(const UpdateState &u, const int32_t *sel_idx, const int32_t *sel_count,
                                             int tid, int stride) {
    const bool list_jobs = u.jobs && u.total <= kUpdateJobs;
    for (int i = tid; i < u.total; i += stride) {
        const int g = i / u.k, j = i - g * u.k;
        int b = 0, len = 0;
        const int v = j < sel_count[g] ? sel_idx[i] : -1;
        if (v >= 0) {
            u.x[v] = 1.f;
            refresh_record(u.rec, u.compact, v, 1.f, 0.f, 0.f);   // (a solution node has no live entry: both sums are zero)
            b = u.rowptr[v];
            len = atomicExch(&u.rowend[v], b) - b;
            if (len > 0) {
                u.touched[v] = -len;
                u.s_pos[v] = 0.f;
                u.s_neg[v] = 0.f;
                const int gg = graph_of(u.G, u.graph_off, v);
                if (u.cand[v]) atomicAdd(&u.stats[2 * gg], -1);
                u.cand[v] = 0;
                atomicAdd(&u.stats[2 * gg + 1], -len);
            }
        }
        if (list_jobs) {
            u.jobs[2 * i] = b;
            u.jobs[2 * i + 1] = len > 0 ? len : 0;
        }
    }
}

// The decisions of one step, taken on the device so that the host need not read anything back between steps; by
// one workgroup of 256 threads.  stats holds {candidates, live stored entries} per graph as the last state update
// left them (the state this step's scores were computed on); sel_count holds how many nodes the selection found
// per graph (it asked for the largest d of the rule).  For one graph and the adaptive rule of Sec. 4.5.1, d
// follows from the candidate count and the count is cut to d (the selection is ordered, so its first d entries
// are the top-d); when no edge is left anywhere the counts become zero and the state update that follows changes
// nothing.  counters[0] += 1 when an edge was left (a policy evaluation that mattered), counters[1] += nodes
// added.  Then the first half of the state update (begin_update) and the update counter.
// s_live, s_picked: LDS, one word each.  Starts with a barrier (the caller may just have written sel_count).
// (no __restrict__ here: a caller may have written sel_idx and sel_count through pointers of its own)
__device__ __forceinline__ void loop_control(int N, int adaptive, int32_t *sel_count, unsigned long long *counters,
                                             const int32_t *sel_idx, const UpdateState &u,
                                             unsigned long long *s_live, unsigned long long *s_picked) {
    const int G = u.G;
    if (threadIdx.x == 0) { *s_live = 0ull; *s_picked = 0ull; }
    __syncthreads();
    unsigned long long live = 0ull;
    for (int b = threadIdx.x; b < G; b += 256) live += (unsigned long long)u.stats[2 * b + 1];
    if (live) atomicAdd(s_live, live);
    int d = 1;
    if (adaptive && G == 1) {
        const long long c = u.stats[0];
        d = 2 * c > N ? 8 : (4 * c > N ? 4 : (8 * c > N ? 2 : 1));
    }
    __syncthreads();
    const bool going = *s_live > 0ull;
    unsigned long long picked = 0ull;
    for (int b = threadIdx.x; b < G; b += 256) {
        const int c = going ? min(sel_count[b], d) : 0;
        sel_count[b] = c;
        picked += (unsigned long long)c;
    }
    if (picked) atomicAdd(s_picked, picked);
    __syncthreads();   // (this workgroup wrote the counts and read the statistics: both are settled from here on)
    if (threadIdx.x == 0 && going) {
        counters[0] += 1ull;
        counters[1] += *s_picked;
    }
    begin_update(u, sel_idx, sel_count, threadIdx.x, 256);
    if (threadIdx.x == 0) u.epoch[0] += 1;
}

}  // namespace s2v
