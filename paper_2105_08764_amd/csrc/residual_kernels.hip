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

// One wave per row.  stats[g] = {candidates, live stored entries} of graph g (integer atomics).
__global__ __launch_bounds__(256) void k_residual_rows(int N, const int32_t *__restrict__ rowptr,
                                                       int32_t *__restrict__ rowend, int32_t *__restrict__ colidx,
                                                       float *__restrict__ w, const float *__restrict__ x,
                                                       float *__restrict__ s_pos, float *__restrict__ s_neg,
                                                       uint8_t *__restrict__ cand, int G,
                                                       const int32_t *__restrict__ graph_off,
                                                       int32_t *__restrict__ stats) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int my_cand = 0, my_live = 0;  // per-wave totals (single graph)
    for (int v = blockIdx.x * 4 + wave; v < N; v += gridDim.x * 4) {
        const int b = rowptr[v], e = rowend[v];
        const bool in_solution = x[v] != 0.f;
        int out = 0;
        double sp = 0.0, sn = 0.0;
        if (!in_solution) {
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
            const bool is_cand = !in_solution && out > 0;
            cand[v] = is_cand ? 1 : 0;
            if (G == 1) {
                my_cand += is_cand ? 1 : 0;
                my_live += out;
            } else if (out > 0) {
                int lo = 0, hi = G;   // last graph whose offset is <= v
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (graph_off[mid] <= v) lo = mid; else hi = mid;
                }
                if (is_cand) atomicAdd(&stats[2 * lo], 1);
                atomicAdd(&stats[2 * lo + 1], out);
            }
        }
    }
    if (G == 1 && lane == 0 && (my_cand | my_live)) {
        atomicAdd(&stats[0], my_cand);
        atomicAdd(&stats[1], my_live);
    }
}

hipError_t launch_residual_update(hipStream_t st, int N, int G, const int32_t *graph_off, const int32_t *rowptr,
                                  int32_t *rowend, int32_t *colidx, float *w, float *x, const int32_t *sel_idx,
                                  const int32_t *sel_count, int k, float *s_pos, float *s_neg, uint8_t *cand,
                                  int32_t *stats) {
    if (sel_idx && k > 0) {
        const int total = G * k;
        k_mark_selected<<<min((total + 255) / 256, 1024), 256, 0, st>>>(total, k, sel_idx, sel_count, x);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    k_zero_stats<<<1, 256, 0, st>>>(2 * G, stats);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (N > 0) {
        const int grid = min((N + 3) / 4, 256 * 32);
        k_residual_rows<<<grid, 256, 0, st>>>(N, rowptr, rowend, colidx, w, x, s_pos, s_neg, cand, G, graph_off, stats);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace s2v
