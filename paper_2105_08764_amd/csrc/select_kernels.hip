// Node selection: masked per-graph argmax (Alg. 3 line 7) and top-k of one graph
// (the top-d selection of Sec. 4.5.1).  Order: score descending, node index ascending on
// equal scores.  All results are exact functions of the float32 scores: no atomics on floats,
// integer atomics only for histogram counts.
#include <limits.h>

#include "internal.h"
#include "loop_util.h"
#include "reduce_util.h"
#include "select_util.h"

namespace s2v {

__device__ __forceinline__ void block_best(float &val, int &idx, float *sval, int *sidx) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const float v2 = __shfl_xor(val, m);
        const int i2 = __shfl_xor(idx, m);
        take_better(val, idx, v2, i2);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sval[wave] = val; sidx[wave] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) take_better(val, idx, sval[w], sidx[w]);
    }
}

// The best (val, idx) of a wave, returned to every lane.
__device__ __forceinline__ void wave_best(float &val, int &idx) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const float v2 = __shfl_xor(val, m);
        const int i2 = __shfl_xor(idx, m);
        take_better(val, idx, v2, i2);
    }
}

// The k best of the (at most two) candidates every lane of ONE wave holds, in order, without a barrier: k times
// the wave's best of what is left.  (v0, i0), (v1, i1): the lane's candidates, idx INT_MAX = none; node indices
// are distinct, so the winner's owner knows itself by the index.  out(it, val, idx) is called by every lane with
// the it-th pick (idx INT_MAX from the first pick that does not exist on; the loop stops there).
// Returns the number of picks.
template <class Out>
__device__ __forceinline__ int wave_topk(float v0, int i0, float v1, int i1, int k, Out out) {
    int found = 0;
    for (int it = 0; it < k; ++it) {
        float val = v0;
        int idx = i0;
        take_better(val, idx, v1, i1);
        if (i0 == INT_MAX) { val = v1; idx = i1; }
        if (idx == INT_MAX) val = -INFINITY;
        wave_best(val, idx);
        out(it, val, idx);
        if (idx == INT_MAX) break;
        if (i0 == idx) { i0 = INT_MAX; v0 = -INFINITY; }
        if (i1 == idx) { i1 = INT_MAX; v1 = -INFINITY; }
        ++found;
    }
    return found;
}

__global__ __launch_bounds__(256) void k_argmax_stage1(const int32_t *__restrict__ chunk_begin,
                                                       const int32_t *__restrict__ chunk_end,
                                                       const float *__restrict__ q, const float *__restrict__ x,
                                                       const uint8_t *__restrict__ cand,
                                                       float *__restrict__ part_val, int32_t *__restrict__ part_idx) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    const int c = blockIdx.x;
    const int vb = chunk_begin[c], ve = chunk_end[c];
    float val = -INFINITY;
    int idx = INT_MAX;
    for (int v = vb + threadIdx.x; v < ve; v += 256)
        if (is_candidate(x, cand, v)) take_better(val, idx, q[v], v);
    block_best(val, idx, sval, sidx);
    if (threadIdx.x == 0) { part_val[c] = val; part_idx[c] = idx; }
}

// Second stage of the argmax of graph g, by one workgroup of 256 threads.  sval, sidx: LDS, 4 entries each.
__device__ __forceinline__ void argmax_stage2(int g, const int32_t *graph_chunk_off, const float *part_val,
                                              const int32_t *part_idx, int32_t *idx_out, float *val_out, int32_t *count,
                                              float *sval, int *sidx) {
    float val = -INFINITY;
    int idx = INT_MAX;
    for (int c = graph_chunk_off[g] + threadIdx.x; c < graph_chunk_off[g + 1]; c += 256)
        take_better(val, idx, part_val[c], part_idx[c]);
    block_best(val, idx, sval, sidx);
    if (threadIdx.x == 0) {
        const bool any = idx != INT_MAX;
        idx_out[g] = any ? idx : -1;
        val_out[g] = any ? val : -INFINITY;
        count[g] = any ? 1 : 0;
    }
}

__global__ __launch_bounds__(256) void k_argmax_stage2(const int32_t *__restrict__ graph_chunk_off,
                                                       const float *__restrict__ part_val,
                                                       const int32_t *__restrict__ part_idx,
                                                       int32_t *__restrict__ idx_out, float *__restrict__ val_out,
                                                       int32_t *__restrict__ count) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    argmax_stage2(blockIdx.x, graph_chunk_off, part_val, part_idx, idx_out, val_out, count, sval, sidx);
}

hipError_t launch_argmax(hipStream_t st, int N, int G, const ChunkTable &ct, const float *q, const float *x,
                         const uint8_t *cand, const SelectScratch &sc, int32_t *idx, float *val, int32_t *count) {
    (void)N;
    if (ct.n_chunks > 0) {
        k_argmax_stage1<<<ct.n_chunks, 256, 0, st>>>(ct.chunk_begin, ct.chunk_end, q, x, cand, sc.part_val, sc.part_idx);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    k_argmax_stage2<<<G, 256, 0, st>>>(ct.graph_chunk_off, sc.part_val, sc.part_idx, idx, val, count);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Top-k for the small k of the adaptive rule of Sec. 4.5.1 (d = 2, 4, 8; here any 2 <= k <=
// kSmallK): two launches instead of the radix chain.  The order (score descending, index
// ascending) is total, so "the next best" is "the best entry that the last pick beats": stage 1
// finds the k best candidates of every chunk that way, stage 2 the k best of those.
// ------------------------------------------------------------------------------------------

// Broadcasts thread 0's (val, idx) after block_best to the whole workgroup.
__device__ __forceinline__ void share_best(float &val, int &idx, float *sval, int *sidx) {
    __syncthreads();
    if (threadIdx.x == 0) { sval[0] = val; sidx[0] = idx; }
    __syncthreads();
    val = sval[0];
    idx = sidx[0];
    __syncthreads();
}

__global__ __launch_bounds__(256) void k_smallk_stage1(int k, const int32_t *__restrict__ chunk_begin,
                                                       const int32_t *__restrict__ chunk_end,
                                                       const float *__restrict__ q, const float *__restrict__ x,
                                                       const uint8_t *__restrict__ cand,
                                                       float *__restrict__ part_val, int32_t *__restrict__ part_idx) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    const int c = blockIdx.x;
    const int vb = chunk_begin[c], ve = chunk_end[c];
    // this thread's (at most kChunkNodes / 256) candidates
    float mv[kChunkNodes / 256];
    int mi[kChunkNodes / 256];
#pragma unroll
    for (int i = 0; i < kChunkNodes / 256; ++i) {
        const int v = vb + threadIdx.x + 256 * i;
        const bool ok = v < ve && is_candidate(x, cand, v);
        mv[i] = ok ? q[v] : -INFINITY;
        mi[i] = ok ? v : INT_MAX;
    }
    float lv = INFINITY;
    int lidx = -1;
    for (int it = 0; it < k; ++it) {
        float val = -INFINITY;
        int idx = INT_MAX;
#pragma unroll
        for (int i = 0; i < kChunkNodes / 256; ++i)
            if (mi[i] != INT_MAX && beats(lv, lidx, mv[i], mi[i])) take_better(val, idx, mv[i], mi[i]);
        block_best(val, idx, sval, sidx);
        share_best(val, idx, sval, sidx);
        if (threadIdx.x == 0) { part_val[(size_t)c * kSmallK + it] = val; part_idx[(size_t)c * kSmallK + it] = idx; }
        lv = val;
        lidx = idx;
        if (idx == INT_MAX) {   // the chunk has no further candidate (uniform: every thread holds the same pick)
            for (int r = it + 1 + threadIdx.x; r < k; r += 256) {
                part_val[(size_t)c * kSmallK + r] = -INFINITY;
                part_idx[(size_t)c * kSmallK + r] = INT_MAX;
            }
            break;
        }
    }
}

// Second stage of the top-k (k <= kSmallK) of one graph, by one workgroup of 256 threads.
__device__ __forceinline__ void smallk_stage2(int k, int n_chunks, const float *part_val, const int32_t *part_idx,
                                              int32_t *idx_out, float *val_out, int32_t *count, float *sval, int *sidx) {
    if (n_chunks * kSmallK <= 128) {
        // few chunks (a graph of up to 16 384 nodes): the first wave alone, two listed picks per lane, no barrier
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            auto slot = [&](int sl, float &v, int &i) {
                const int c = sl / kSmallK, r = sl - c * kSmallK;
                const bool have = c < n_chunks && r < k;   // (a chunk's list is padded with INT_MAX behind its last pick)
                i = have ? part_idx[(size_t)c * kSmallK + r] : INT_MAX;
                v = (have && i != INT_MAX) ? part_val[(size_t)c * kSmallK + r] : -INFINITY;
            };
            float v0, v1;
            int i0, i1;
            slot(lane, v0, i0);
            slot(lane + 64, v1, i1);
            const int found = wave_topk(v0, i0, v1, i1, k, [&](int it, float val, int idx) {
                if (lane == 0 && idx != INT_MAX) { idx_out[it] = idx; val_out[it] = val + 0.0f; }
            });
            for (int r = found + lane; r < k; r += 64) { idx_out[r] = -1; val_out[r] = -INFINITY; }
            if (lane == 0) count[0] = found;
        }
        return;
    }
    float lv = INFINITY;
    int lidx = -1;
    int found = 0;
    for (int it = 0; it < k; ++it) {
        float val = -INFINITY;
        int idx = INT_MAX;
        for (int c = threadIdx.x; c < n_chunks; c += 256) {
            // a chunk's picks are in order: the first one the last pick beats is its best remaining
            for (int r = 0; r < k; ++r) {
                const int pi = part_idx[(size_t)c * kSmallK + r];
                if (pi == INT_MAX) break;
                const float pv = part_val[(size_t)c * kSmallK + r];
                if (beats(lv, lidx, pv, pi)) { take_better(val, idx, pv, pi); break; }
            }
        }
        block_best(val, idx, sval, sidx);
        share_best(val, idx, sval, sidx);
        if (idx == INT_MAX) break;
        if (threadIdx.x == 0) { idx_out[it] = idx; val_out[it] = val + 0.0f; }
        lv = val;
        lidx = idx;
        ++found;
    }
    for (int r = found + threadIdx.x; r < k; r += 256) { idx_out[r] = -1; val_out[r] = -INFINITY; }
    if (threadIdx.x == 0) count[0] = found;
}

__global__ __launch_bounds__(256) void k_smallk_stage2(int k, int n_chunks, const float *__restrict__ part_val,
                                                       const int32_t *__restrict__ part_idx,
                                                       int32_t *__restrict__ idx_out, float *__restrict__ val_out,
                                                       int32_t *__restrict__ count) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    smallk_stage2(k, n_chunks, part_val, part_idx, idx_out, val_out, count, sval, sidx);
}

// The last launch of a step of the loop on one graph: second stage of the selection, then the step's decisions
// and the first half of the state update (loop_control).
__global__ __launch_bounds__(256) void k_step_end(int k, int n_chunks, const int32_t *graph_chunk_off,
                                                  const float *part_val, const int32_t *part_idx, int32_t *idx_out,
                                                  float *val_out, int32_t *count, int N, int adaptive,
                                                  unsigned long long *counters, UpdateState u) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    __shared__ unsigned long long s_live, s_picked;
    if (k == 1) argmax_stage2(0, graph_chunk_off, part_val, part_idx, idx_out, val_out, count, sval, sidx);
    else smallk_stage2(k, n_chunks, part_val, part_idx, idx_out, val_out, count, sval, sidx);
    loop_control(N, adaptive, count, counters, idx_out, u, &s_live, &s_picked);
}

hipError_t launch_smallk(hipStream_t st, const ChunkTable &ct, const float *q, const float *x, const uint8_t *cand,
                         int k, const SelectScratch &sc, int32_t *idx, float *val, int32_t *count) {
    if (ct.n_chunks > 0) {
        k_smallk_stage1<<<ct.n_chunks, 256, 0, st>>>(k, ct.chunk_begin, ct.chunk_end, q, x, cand, sc.part_val, sc.part_idx);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    k_smallk_stage2<<<1, 256, 0, st>>>(k, ct.n_chunks, sc.part_val, sc.part_idx, idx, val, count);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Deep-Q target of the training step (Alg. 4, "compute a target value using the reward"):
//   target[b] = reward[b] + gamma * max over the candidates v of the next state b, inside the graph
//   of action[b], of q_next[b][v];   target[b] = reward[b] when that state has no candidate left.
// Same two-stage (chunk, graph) maximum as the argmax, once per state.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_target_stage1(int N, int n_chunks, const int32_t *__restrict__ chunk_begin,
                                                       const int32_t *__restrict__ chunk_end,
                                                       const float *__restrict__ q, const float *__restrict__ x,
                                                       const uint8_t *__restrict__ cand,
                                                       float *__restrict__ part_val, int32_t *__restrict__ part_idx) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    const int c = blockIdx.x, s = blockIdx.y;
    const size_t off = (size_t)s * N;
    const int vb = chunk_begin[c], ve = chunk_end[c];
    float val = -INFINITY;
    int idx = INT_MAX;
    for (int v = vb + threadIdx.x; v < ve; v += 256)
        if (is_candidate(x + off, cand ? cand + off : nullptr, v)) take_better(val, idx, q[off + v], v);
    block_best(val, idx, sval, sidx);
    if (threadIdx.x == 0) { part_val[(size_t)s * n_chunks + c] = val; part_idx[(size_t)s * n_chunks + c] = idx; }
}

__global__ __launch_bounds__(256) void k_target_stage2(int G, int n_chunks, const int32_t *__restrict__ graph_off,
                                                       const int32_t *__restrict__ graph_chunk_off,
                                                       const int32_t *__restrict__ action,
                                                       const float *__restrict__ reward, float gamma,
                                                       const float *__restrict__ part_val,
                                                       const int32_t *__restrict__ part_idx,
                                                       float *__restrict__ target) {
    __shared__ float sval[4];
    __shared__ int sidx[4];
    const int s = blockIdx.x;
    int g = 0;
    if (G > 1) {   // last graph whose offset is <= the action node
        const int a = action[s];
        int lo = 0, hi = G;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (graph_off[mid] <= a) lo = mid; else hi = mid;
        }
        g = lo;
    }
    float val = -INFINITY;
    int idx = INT_MAX;
    for (int c = graph_chunk_off[g] + threadIdx.x; c < graph_chunk_off[g + 1]; c += 256)
        take_better(val, idx, part_val[(size_t)s * n_chunks + c], part_idx[(size_t)s * n_chunks + c]);
    block_best(val, idx, sval, sidx);
    if (threadIdx.x == 0) target[s] = idx != INT_MAX ? reward[s] + gamma * val : reward[s];
}

hipError_t launch_q_target(hipStream_t st, int N, int S, int G, const int32_t *graph_off, const ChunkTable &ct,
                           const float *q_next, const float *x_next, const uint8_t *cand_next, const int32_t *action,
                           const float *reward, float gamma, float *part_val, int32_t *part_idx, float *target) {
    if (ct.n_chunks > 0) {
        k_target_stage1<<<dim3(ct.n_chunks, S), 256, 0, st>>>(N, ct.n_chunks, ct.chunk_begin, ct.chunk_end, q_next, x_next,
                                                            cand_next, part_val, part_idx);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    k_target_stage2<<<S, 256, 0, st>>>(G, ct.n_chunks, graph_off, ct.graph_chunk_off, action, reward, gamma, part_val,
                                       part_idx, target);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Top-k of one graph.
//  1. radix select: four 8-bit histogram passes from the top byte find the k-th largest key tau
//     and how many keys equal to tau are still needed (`need`).  No kernel of its own picks the
//     digit between two passes: every workgroup of the next kernel re-derives it from the finished
//     histograms (topk_resolve, a 256-bin suffix scan by one wave);
//  2. index-ordered compaction of {key > tau} and the first `need` nodes with key == tau;
//  3. stable LSD radix sort of the selected (<= k) entries by key descending; stability keeps
//     equal scores in ascending node index.
// state (written by the scan kernel of step 2 for the kernels after it):
//   [0] tau, [1] need, [2] number of candidates, [3] 1 if candidates < k (take all),
//   [4] count = min(k, candidates)
// ------------------------------------------------------------------------------------------
__global__ void k_topk_init(uint32_t *__restrict__ hist, uint32_t *__restrict__ state) {
    for (int i = threadIdx.x; i < 4 * 256; i += blockDim.x) hist[i] = 0;
    if (threadIdx.x < 16) state[threadIdx.x] = 0u;
}

struct TopkSel {
    uint32_t prefix;    // the digits fixed so far, in place
    uint32_t k_rem;     // entries still to find among the keys that match the prefix
    uint32_t total;     // number of candidates (known after pass 0)
    uint32_t take_all;  // fewer candidates than k
};

// The selection state after `passes` finished histogram passes.  Called by all threads of a
// workgroup (blockDim.x >= 64); wave 0 computes, `sh` is 4 words of shared memory.
__device__ __forceinline__ TopkSel topk_resolve(const uint32_t *__restrict__ hist, uint32_t k, int passes,
                                                uint32_t *sh) {
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        uint32_t prefix = 0, k_rem = k, total = 0, take_all = 0;
        for (int p = 0; p < passes; ++p) {
            const uint4 hv = *reinterpret_cast<const uint4 *>(hist + p * 256 + 4 * lane);   // bins 4l .. 4l+3
            const uint32_t mine = hv.x + hv.y + hv.z + hv.w;
            uint32_t suf = mine;                                 // sum over the bins of lanes >= l
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) {
                const uint32_t t = __shfl_down(suf, m);
                if (lane + m < 64) suf += t;
            }
            if (p == 0) {
                total = __shfl(suf, 0);
                if (total < k_rem) { take_all = 1; break; }
            }
            // the digit is the largest d with (sum of bins >= d) >= k_rem; it lies in the highest lane
            // whose suffix sum reaches k_rem
            const unsigned long long reach = __ballot(suf >= k_rem) | 1ull;
            const int ls = 63 - __clzll(reach);
            uint32_t cum = suf - mine;                           // bins above this lane's four
            int d = 0;
            if (cum + hv.w >= k_rem) d = 3;
            else if (cum + hv.w + hv.z >= k_rem) { d = 2; cum += hv.w; }
            else if (cum + hv.w + hv.z + hv.y >= k_rem) { d = 1; cum += hv.w + hv.z; }
            else cum += hv.w + hv.z + hv.y;
            const uint32_t digit = (uint32_t)__shfl(4 * lane + d, ls);
            const uint32_t above = __shfl(cum, ls);
            prefix |= digit << (24 - 8 * p);
            k_rem -= above;
        }
        if (lane == 0) { sh[0] = prefix; sh[1] = k_rem; sh[2] = total; sh[3] = take_all; }
    }
    __syncthreads();
    TopkSel r;
    r.prefix = sh[0]; r.k_rem = sh[1]; r.total = sh[2]; r.take_all = sh[3];
    return r;
}

// One count into a shared-memory histogram per active lane, with the lanes that share the digit
// of the first active lane combined into a single add (twice): scores that agree in their leading
// bytes would otherwise serialise on one bin.  Must be called by whole waves.
__device__ __forceinline__ void hist_add(uint32_t *h, bool active, uint32_t digit) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const unsigned long long act = __ballot(active);
        if (act == 0ull) return;
        const int leader = __ffsll((long long)act) - 1;
        const uint32_t d0 = (uint32_t)__shfl((int)digit, leader);
        const bool same = active && digit == d0;
        const unsigned long long grp = __ballot(same);
        if (lane == leader) atomicAdd(&h[d0], (uint32_t)__popcll(grp));
        if (same) active = false;
    }
    if (active) atomicAdd(&h[digit], 1u);
}

__global__ __launch_bounds__(256) void k_topk_hist(int N, int pass, uint32_t k, const float *__restrict__ q,
                                                   const float *__restrict__ x, const uint8_t *__restrict__ cand,
                                                   uint32_t *__restrict__ hist) {
    __shared__ uint32_t h[256];
    __shared__ uint32_t sel_sh[4];
    h[threadIdx.x] = 0;
    const TopkSel sel = topk_resolve(hist, k, pass, sel_sh);     // includes the barrier after h[] = 0
    if (sel.take_all) return;
    const int shift = 24 - 8 * pass;
    const uint32_t mask_hi = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    // four independent elements per thread and step; few workgroups, because each ends with up to 256
    // adds to the same global bins
    for (int base = blockIdx.x * 1024; base < N; base += gridDim.x * 1024) {
        bool active[4];
        uint32_t key[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int v = base + j * 256 + threadIdx.x;
            active[j] = v < N && is_candidate(x, cand, v);
            key[j] = active[j] ? score_key(q[v]) : 0u;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            hist_add(h, active[j] && (key[j] & mask_hi) == sel.prefix, (key[j] >> shift) & 255u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&hist[pass * 256 + threadIdx.x], h[threadIdx.x]);
}

// flags of one node: bit 0 = key > tau (or any candidate when taking all), bit 1 = key == tau
__device__ __forceinline__ uint32_t sel_flags(const float *__restrict__ q, const float *__restrict__ x,
                                              const uint8_t *__restrict__ cand, int v, uint32_t tau, bool take_all,
                                              uint32_t &key) {
    if (!is_candidate(x, cand, v)) return 0;
    key = score_key(q[v]);
    if (take_all || key > tau) return 1u;
    return key == tau ? 2u : 0u;
}

__global__ __launch_bounds__(256) void k_topk_scan1(int N, uint32_t k, const float *__restrict__ q,
                                                    const float *__restrict__ x, const uint8_t *__restrict__ cand,
                                                    const uint32_t *__restrict__ hist, uint32_t *__restrict__ blk) {
    __shared__ uint32_t sg[4], se[4];
    __shared__ uint32_t sel_sh[4];
    const TopkSel sel = topk_resolve(hist, k, 4, sel_sh);
    const uint32_t tau = sel.prefix;
    const bool take_all = sel.take_all != 0;
    const int base = blockIdx.x * kScanBlock + threadIdx.x * 8;
    uint32_t gt = 0, eq = 0, key;
    for (int i = 0; i < 8; ++i) {
        const int v = base + i;
        if (v < N) {
            const uint32_t f = sel_flags(q, x, cand, v, tau, take_all, key);
            gt += f & 1u;
            eq += f >> 1;
        }
    }
    for (int m = 1; m < 64; m <<= 1) { gt += __shfl_xor(gt, m); eq += __shfl_xor(eq, m); }
    if ((threadIdx.x & 63) == 0) { sg[threadIdx.x >> 6] = gt; se[threadIdx.x >> 6] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk[2 * blockIdx.x] = sg[0] + sg[1] + sg[2] + sg[3];
        blk[2 * blockIdx.x + 1] = se[0] + se[1] + se[2] + se[3];
    }
}

// exclusive scan of the per-block (gt, eq) pairs, single workgroup; also publishes the selection
// state for the kernels that follow
__global__ __launch_bounds__(256) void k_topk_scan2(int n_blk, uint32_t k, const uint32_t *__restrict__ hist,
                                                    const uint32_t *__restrict__ blk, uint32_t *__restrict__ blk_scan,
                                                    uint32_t *__restrict__ state, int32_t *__restrict__ count) {
    __shared__ uint32_t sg[256], se[256];
    __shared__ uint32_t sel_sh[4];
    const int tid = threadIdx.x;
    const TopkSel sel = topk_resolve(hist, k, 4, sel_sh);
    if (tid == 0) {
        const uint32_t n_sel = sel.take_all ? sel.total : k;
        state[0] = sel.prefix;
        state[1] = sel.k_rem;
        state[2] = sel.total;
        state[3] = sel.take_all;
        state[4] = n_sel;
        count[0] = (int32_t)n_sel;
    }
    const int per = (n_blk + 255) / 256;
    const int b0 = tid * per, b1 = min(n_blk, b0 + per);
    uint32_t gt = 0, eq = 0;
    for (int b = b0; b < b1; ++b) { gt += blk[2 * b]; eq += blk[2 * b + 1]; }
    sg[tid] = gt; se[tid] = eq;
    __syncthreads();
    if (tid == 0) {
        uint32_t cg = 0, ce = 0;
        for (int i = 0; i < 256; ++i) {
            const uint32_t tg = sg[i], te = se[i];
            sg[i] = cg; se[i] = ce;
            cg += tg; ce += te;
        }
    }
    __syncthreads();
    gt = sg[tid]; eq = se[tid];
    for (int b = b0; b < b1; ++b) {
        blk_scan[2 * b] = gt; blk_scan[2 * b + 1] = eq;
        gt += blk[2 * b]; eq += blk[2 * b + 1];
    }
}

__global__ __launch_bounds__(256) void k_topk_scan3(int N, const float *__restrict__ q, const float *__restrict__ x,
                                                    const uint8_t *__restrict__ cand,
                                                    const uint32_t *__restrict__ state,
                                                    const uint32_t *__restrict__ blk_scan,
                                                    uint32_t *__restrict__ keys, int32_t *__restrict__ ids) {
    __shared__ uint32_t sg[4], se[4];
    const uint32_t tau = state[0];
    const bool take_all = state[3] != 0;
    const uint32_t need = take_all ? 0u : state[1];
    const int base = blockIdx.x * kScanBlock + threadIdx.x * 8;
    uint32_t f[8], key[8];
    uint32_t gt = 0, eq = 0;
    for (int i = 0; i < 8; ++i) {
        const int v = base + i;
        key[i] = 0;
        f[i] = v < N ? sel_flags(q, x, cand, v, tau, take_all, key[i]) : 0u;
        gt += f[i] & 1u;
        eq += f[i] >> 1;
    }
    // exclusive prefix over the threads of the block: inclusive wave scan, then wave bases
    uint32_t ig = gt, ie = eq;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int m = 1; m < 64; m <<= 1) {
        const uint32_t tg = __shfl_up(ig, m), te = __shfl_up(ie, m);
        if (lane >= m) { ig += tg; ie += te; }
    }
    if (lane == 63) { sg[wave] = ig; se[wave] = ie; }
    __syncthreads();
    uint32_t pg = blk_scan[2 * blockIdx.x] + ig - gt, pe = blk_scan[2 * blockIdx.x + 1] + ie - eq;
    for (int w = 0; w < wave; ++w) { pg += sg[w]; pe += se[w]; }
    for (int i = 0; i < 8; ++i) {
        if (f[i] & 1u) {
            const uint32_t pos = pg + min(pe, need);
            keys[pos] = key[i]; ids[pos] = base + i;
            ++pg;
        } else if (f[i] & 2u) {
            if (pe < need) {
                const uint32_t pos = pg + pe;
                keys[pos] = key[i]; ids[pos] = base + i;
            }
            ++pe;
        }
    }
}

// ---- stable LSD radix sort of n = state[4] (key, id) pairs by key descending, 8 bits per pass ----
__global__ __launch_bounds__(64) void k_sort_hist(int pass, int n_blk, const uint32_t *__restrict__ state,
                                                  const uint32_t *__restrict__ keys, uint32_t *__restrict__ cnt) {
    __shared__ uint32_t h[256];
    const int n = (int)state[4];
    for (int i = threadIdx.x; i < 256; i += 64) h[i] = 0;
    __syncthreads();
    const int b = blockIdx.x * kSortTile, e = min(n, b + kSortTile);
    for (int i = b + threadIdx.x; i < e; i += 64) atomicAdd(&h[((~keys[i]) >> (8 * pass)) & 255u], 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < 256; d += 64) cnt[(size_t)d * n_blk + blockIdx.x] = h[d];
}

__global__ __launch_bounds__(256) void k_sort_scan(int n_blk, uint32_t *__restrict__ cnt) {
    __shared__ uint32_t tot[256];
    const int d = threadIdx.x;
    uint32_t s = 0;
    for (int b = 0; b < n_blk; ++b) s += cnt[(size_t)d * n_blk + b];
    tot[d] = s;
    __syncthreads();
    if (d == 0) {
        uint32_t c = 0;
        for (int i = 0; i < 256; ++i) { const uint32_t t = tot[i]; tot[i] = c; c += t; }
    }
    __syncthreads();
    s = tot[d];
    for (int b = 0; b < n_blk; ++b) {
        const uint32_t t = cnt[(size_t)d * n_blk + b];
        cnt[(size_t)d * n_blk + b] = s;
        s += t;
    }
}

__global__ __launch_bounds__(64) void k_sort_scatter(int pass, int n_blk, const uint32_t *__restrict__ state,
                                                     const uint32_t *__restrict__ keys_in,
                                                     const int32_t *__restrict__ ids_in,
                                                     const uint32_t *__restrict__ cnt, uint32_t *__restrict__ keys_out,
                                                     int32_t *__restrict__ ids_out) {
    __shared__ uint32_t base[256];
    const int n = (int)state[4];
    const int lane = threadIdx.x;
    for (int d = lane; d < 256; d += 64) base[d] = cnt[(size_t)d * n_blk + blockIdx.x];
    __syncthreads();
    const int b = blockIdx.x * kSortTile, e = min(n, b + kSortTile);
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    for (int i0 = b; i0 < e; i0 += 64) {
        const int i = i0 + lane;
        const bool valid = i < e;
        const uint32_t key = valid ? keys_in[i] : 0u;
        const int32_t id = valid ? ids_in[i] : 0;
        const uint32_t digit = ((~key) >> (8 * pass)) & 255u;
        uint64_t m = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool on = (digit >> bit) & 1u;
            const uint64_t bm = __ballot(on);
            m &= on ? bm : ~bm;
        }
        uint32_t pos = 0;
        if (valid) pos = base[digit] + (uint32_t)__popcll(m & lt_mask);
        __syncthreads();
        if (valid) {
            keys_out[pos] = key;
            ids_out[pos] = id;
            if ((m >> lane) == 1ull) base[digit] += (uint32_t)__popcll(m);  // highest lane of its digit group
        }
        __syncthreads();
    }
}

// ---- the same sort with fewer launches, for up to kSortFusedMaxBlocks tiles --------------------
// The count table is [tile][256].  k_sort_count writes the plain counts of digit p per tile;
// k_sort_pass derives its scatter offsets from them inside every workgroup (the per-digit totals
// and the part of the tiles before its own: the scan kernel folded in).  The last pass writes the
// result arrays directly.
__global__ __launch_bounds__(64) void k_sort_count(int pass, const uint32_t *__restrict__ state,
                                                   const uint32_t *__restrict__ keys, uint32_t *__restrict__ cnt) {
    __shared__ uint32_t h[256];
    const int n = (int)state[4];
    for (int i = threadIdx.x; i < 256; i += 64) h[i] = 0;
    __syncthreads();
    const int b = blockIdx.x * kSortTile, e = min(n, b + kSortTile);
    for (int i = b + threadIdx.x; i < e; i += 64) atomicAdd(&h[((~keys[i]) >> (8 * pass)) & 255u], 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < 256; d += 64) cnt[(size_t)blockIdx.x * 256 + d] = h[d];
}

__global__ __launch_bounds__(64) void k_sort_pass(int pass, int n_blk, int k, const uint32_t *__restrict__ state,
                                                  const uint32_t *__restrict__ keys_in,
                                                  const int32_t *__restrict__ ids_in,
                                                  const uint32_t *__restrict__ cnt_cur, uint32_t *__restrict__ keys_out,
                                                  int32_t *__restrict__ ids_out, int32_t *__restrict__ idx /*last pass*/,
                                                  float *__restrict__ val /*last pass*/) {
    __shared__ uint32_t base[256];
    const int n = (int)state[4];
    const int lane = threadIdx.x;
    // digits 4*lane .. 4*lane+3: totals over all tiles and over the tiles before this one
    uint4 tot = make_uint4(0, 0, 0, 0), bef = make_uint4(0, 0, 0, 0);
#pragma unroll 8
    for (int t = 0; t < n_blk; ++t) {
        const uint4 c = *reinterpret_cast<const uint4 *>(cnt_cur + (size_t)t * 256 + 4 * lane);
        tot.x += c.x; tot.y += c.y; tot.z += c.z; tot.w += c.w;
        if (t < (int)blockIdx.x) { bef.x += c.x; bef.y += c.y; bef.z += c.z; bef.w += c.w; }
    }
    const uint32_t mine = tot.x + tot.y + tot.z + tot.w;
    uint32_t incl = mine;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const uint32_t t = __shfl_up(incl, m);
        if (lane >= m) incl += t;
    }
    const uint32_t excl = incl - mine;
    base[4 * lane] = excl + bef.x;
    base[4 * lane + 1] = excl + tot.x + bef.y;
    base[4 * lane + 2] = excl + tot.x + tot.y + bef.z;
    base[4 * lane + 3] = excl + tot.x + tot.y + tot.z + bef.w;
    __syncthreads();
    const int b = blockIdx.x * kSortTile, e = min(n, b + kSortTile);
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    // The workgroup is ONE wave: its LDS operations execute in program order for all lanes, so the
    // running offsets in base[] need no workgroup barrier (which would also wait for every store of
    // the step to land); the entries of the next step are fetched while this one is placed.
    uint32_t key_next = (b + lane < e) ? keys_in[b + lane] : 0u;
    int32_t id_next = (b + lane < e) ? ids_in[b + lane] : 0;
    for (int i0 = b; i0 < e; i0 += 64) {
        const bool valid = i0 + lane < e;
        const uint32_t key = key_next;
        const int32_t id = id_next;
        if (i0 + 64 < e) {
            const int i = i0 + 64 + lane;
            key_next = i < e ? keys_in[i] : 0u;
            id_next = i < e ? ids_in[i] : 0;
        }
        const uint32_t digit = ((~key) >> (8 * pass)) & 255u;
        uint64_t m = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool on = (digit >> bit) & 1u;
            const uint64_t bm = __ballot(on);
            m &= on ? bm : ~bm;
        }
        uint32_t pos = 0;
        if (valid) pos = base[digit] + (uint32_t)__popcll(m & lt_mask);
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            if (idx) {
                idx[pos] = id;
                val[pos] = key_score(key);
            } else {
                keys_out[pos] = key;
                ids_out[pos] = id;
            }
            if ((m >> lane) == 1ull) base[digit] += (uint32_t)__popcll(m);  // highest lane of its digit group
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (idx) {   // result slots beyond the selected count
        for (int i = max(b, n) + lane; i < min(k, b + kSortTile); i += 64) {
            idx[i] = -1;
            val[i] = -INFINITY;
        }
    }
}

__global__ __launch_bounds__(256) void k_topk_write(int k, const uint32_t *__restrict__ state,
                                                    const uint32_t *__restrict__ keys, const int32_t *__restrict__ ids,
                                                    int32_t *__restrict__ idx, float *__restrict__ val) {
    const int n = (int)state[4];
    for (int i = blockIdx.x * 256 + threadIdx.x; i < k; i += gridDim.x * 256) {
        idx[i] = i < n ? ids[i] : -1;
        val[i] = i < n ? key_score(keys[i]) : -INFINITY;
    }
}

// ------------------------------------------------------------------------------------------
// The tail of a policy evaluation and the first stage of the selection in one launch, for one state of one
// small graph (few partial rows): what k_gsum_stage2, k_qa, k_qfinish and k_argmax_stage1 / k_smallk_stage1
// do in four.  Every workgroup (one per chunk of kChunkNodes nodes, 1024 threads) adds the partial rows of
// the graph sum and forms the graph term of Eq. 2 for itself -- the same device functions as the stand-alone
// kernels, so the same bits --, completes the scores of its chunk (q = qa + node term) and finds the chunk's
// k best candidates.  The second stage of the selection follows as usual.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_tail_select1(int p, int rows, int k, const float *__restrict__ gpart,
                                                       const float *__restrict__ theta5,
                                                       const float *__restrict__ theta6, float *__restrict__ gsum,
                                                       float *__restrict__ q, const float *__restrict__ x,
                                                       const uint8_t *__restrict__ cand,
                                                       const int32_t *__restrict__ chunk_begin,
                                                       const int32_t *__restrict__ chunk_end,
                                                       float *__restrict__ part_val, int32_t *__restrict__ part_idx) {
    __shared__ double red[64][17];
    __shared__ float gsv[128], gs[128], redf[128];
    __shared__ float wv[16][kSmallK];   // the waves' picks
    __shared__ int wi[16][kSmallK];
    const int tid = threadIdx.x;
    for (int cb = 0; cb < p / 16; ++cb) {
        const int col = 16 * cb + (tid & 15);
        const double acc = gsum_stage2_cols(p, col, 0, rows, gpart, red);
        if ((tid >> 4) == 0) gsv[col] = (float)acc;
    }
    __syncthreads();
    if (blockIdx.x == 0 && tid < p) gsum[tid] = gsv[tid];
    const float qa = qa_value(p, theta5, theta6, gsv, gs, redf);
    const int c = blockIdx.x;
    const int vb = chunk_begin[c], ve = chunk_end[c];
    const int v = vb + tid;                                  // kChunkNodes == blockDim.x: one node per thread
    float myv = -INFINITY;
    int myi = INT_MAX;
    if (v < ve) {
        const float qv = qa + q[v];
        q[v] = qv;
        if (is_candidate(x, cand, v)) { myv = qv; myi = v; }
    }
    // the chunk's k best: every wave picks the k best of its 64 nodes (no barrier), then the first wave picks the
    // k best of those 16 x k (two per lane); the order rule makes the outcome the same as any other way of picking
    const int wave = tid >> 6, lane = tid & 63;
    wave_topk(myv, myi, -INFINITY, INT_MAX, k, [&](int it, float val, int idx) {
        if (lane == 0) { wv[wave][it] = val; wi[wave][it] = idx; }
    });
    __syncthreads();
    if (wave == 0) {
        // candidate slot s of the 16 x kSmallK table: wave s / kSmallK... laid out [wave][pick]; lane l takes slots l and l + 64
        auto slot = [&](int sl, float &v, int &i) {
            const int w = sl / kSmallK, r = sl - w * kSmallK;
            const bool have = r < k;
            // (a wave stops at its first missing pick: the slots behind it hold nothing valid)
            i = have ? wi[w][r] : INT_MAX;
            v = have ? wv[w][r] : -INFINITY;
        };
        float v0, v1;
        int i0, i1;
        slot(lane, v0, i0);
        slot(lane + 64, v1, i1);
        // a wave's list ends at its first INT_MAX: mask what lies behind it
        {
            const int w0 = lane / kSmallK, r0 = lane - w0 * kSmallK;
            for (int r = 0; r < r0; ++r) if (r < k && wi[w0][r] == INT_MAX) { i0 = INT_MAX; v0 = -INFINITY; }
            const int w1 = (lane + 64) / kSmallK, r1 = (lane + 64) - w1 * kSmallK;
            for (int r = 0; r < r1; ++r) if (r < k && wi[w1][r] == INT_MAX) { i1 = INT_MAX; v1 = -INFINITY; }
        }
        const int found = wave_topk(v0, i0, v1, i1, k, [&](int it, float val, int idx) {
            // same layout of the partial results as k_argmax_stage1 (k == 1) and k_smallk_stage1 (k > 1)
            const size_t at = k == 1 ? (size_t)c : (size_t)c * kSmallK + it;
            if (lane == 0) { part_val[at] = val; part_idx[at] = idx; }
        });
        if (k > 1)
            for (int r = found + 1 + lane; r < k; r += 64) {   // (slot `found` holds the end mark already)
                part_val[(size_t)c * kSmallK + r] = -INFINITY;
                part_idx[(size_t)c * kSmallK + r] = INT_MAX;
            }
    }
}

hipError_t launch_tail_select(hipStream_t st, int p, int rows, int k, const float *gpart, const float *theta5,
                              const float *theta6, float *gsum, float *q, const float *x, const uint8_t *cand,
                              const ChunkTable &ct, const SelectScratch &sc, int32_t *idx, float *val, int32_t *count,
                              const StepEnd *end) {
    static_assert(kChunkNodes == 1024, "k_tail_select1 takes one node per thread");
    k_tail_select1<<<ct.n_chunks, 1024, 0, st>>>(p, rows, k, gpart, theta5, theta6, gsum, q, x, cand, ct.chunk_begin,
                                                 ct.chunk_end, sc.part_val, sc.part_idx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (end)
        k_step_end<<<1, 256, 0, st>>>(k, ct.n_chunks, ct.graph_chunk_off, sc.part_val, sc.part_idx, idx, val, count, end->N,
                                      end->adaptive ? 1 : 0, end->counters, *end->update);
    else if (k == 1) k_argmax_stage2<<<1, 256, 0, st>>>(ct.graph_chunk_off, sc.part_val, sc.part_idx, idx, val, count);
    else k_smallk_stage2<<<1, 256, 0, st>>>(k, ct.n_chunks, sc.part_val, sc.part_idx, idx, val, count);
    return hipGetLastError();
}

// The reduction chunk table of ONE graph of N nodes (what s2v_graph_prepare builds on the host for a
// prepared graph), written on the device: chunk c covers nodes [c * kChunkNodes, min(N, (c + 1) * kChunkNodes)).
__global__ __launch_bounds__(256) void k_chunk_table_single(int N, int n_chunks, int32_t *__restrict__ chunk_begin,
                                                            int32_t *__restrict__ chunk_end,
                                                            int32_t *__restrict__ graph_chunk_off) {
    for (int c = blockIdx.x * 256 + threadIdx.x; c < n_chunks; c += gridDim.x * 256) {
        chunk_begin[c] = c * kChunkNodes;
        chunk_end[c] = min(N, (c + 1) * kChunkNodes);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        graph_chunk_off[0] = 0;
        graph_chunk_off[1] = n_chunks;
    }
}

hipError_t launch_chunk_table_single(hipStream_t st, int N, int n_chunks, int32_t *chunk_begin, int32_t *chunk_end,
                                     int32_t *graph_chunk_off) {
    k_chunk_table_single<<<max(1, min((n_chunks + 255) / 256, 64)), 256, 0, st>>>(N, n_chunks, chunk_begin, chunk_end,
                                                                                  graph_chunk_off);
    return hipGetLastError();
}

#define S2V_CHECK_LAUNCH()                         \
    do {                                           \
        hipError_t e_ = hipGetLastError();         \
        if (e_ != hipSuccess) return e_;           \
    } while (0)

hipError_t launch_topk(hipStream_t st, int N, const float *q, const float *x, const uint8_t *cand, int k,
                       const SelectScratch &sc, int32_t *idx, float *val, int32_t *count) {
    k_topk_init<<<1, 256, 0, st>>>(sc.hist, sc.state);
    S2V_CHECK_LAUNCH();
    const int n_scan_blk = (N + kScanBlock - 1) / kScanBlock;
    uint32_t *blk = sc.blk, *blk_scan = sc.blk + 2 * (size_t)n_scan_blk;
    const uint32_t ku = (uint32_t)k;
    if (N > 0) {
        const int hist_grid = min((N + 1023) / 1024, 512);
        for (int pass = 0; pass < 4; ++pass) {
            k_topk_hist<<<hist_grid, 256, 0, st>>>(N, pass, ku, q, x, cand, sc.hist);
            S2V_CHECK_LAUNCH();
        }
        k_topk_scan1<<<n_scan_blk, 256, 0, st>>>(N, ku, q, x, cand, sc.hist, blk);
        S2V_CHECK_LAUNCH();
    }
    k_topk_scan2<<<1, 256, 0, st>>>(n_scan_blk, ku, sc.hist, blk, blk_scan, sc.state, count);
    S2V_CHECK_LAUNCH();
    if (N == 0) {
        k_topk_write<<<min((k + 255) / 256, 1024), 256, 0, st>>>(k, sc.state, sc.keys[0], sc.ids[0], idx, val);
        return hipGetLastError();
    }
    k_topk_scan3<<<n_scan_blk, 256, 0, st>>>(N, q, x, cand, sc.state, blk_scan, sc.keys[0], sc.ids[0]);
    S2V_CHECK_LAUNCH();
    const int n_sort_blk = (k + kSortTile - 1) / kSortTile;
    if (n_sort_blk <= kSortFusedMaxBlocks) {
        for (int pass = 0; pass < 4; ++pass) {
            const int a = pass & 1, b = a ^ 1;
            const bool last = pass == 3;
            k_sort_count<<<n_sort_blk, 64, 0, st>>>(pass, sc.state, sc.keys[a], sc.sort_cnt);
            S2V_CHECK_LAUNCH();
            k_sort_pass<<<n_sort_blk, 64, 0, st>>>(pass, n_sort_blk, k, sc.state, sc.keys[a], sc.ids[a], sc.sort_cnt,
                                                   sc.keys[b], sc.ids[b], last ? idx : nullptr, last ? val : nullptr);
            S2V_CHECK_LAUNCH();
        }
        return hipGetLastError();
    }
    for (int pass = 0; pass < 4; ++pass) {
        const int a = pass & 1, b = a ^ 1;
        k_sort_hist<<<n_sort_blk, 64, 0, st>>>(pass, n_sort_blk, sc.state, sc.keys[a], sc.sort_cnt);
        S2V_CHECK_LAUNCH();
        k_sort_scan<<<1, 256, 0, st>>>(n_sort_blk, sc.sort_cnt);
        S2V_CHECK_LAUNCH();
        k_sort_scatter<<<n_sort_blk, 64, 0, st>>>(pass, n_sort_blk, sc.state, sc.keys[a], sc.ids[a], sc.sort_cnt,
                                                  sc.keys[b], sc.ids[b]);
        S2V_CHECK_LAUNCH();
    }
    k_topk_write<<<min((k + 255) / 256, 1024), 256, 0, st>>>(k, sc.state, sc.keys[0], sc.ids[0], idx, val);
    return hipGetLastError();
}

}  // namespace s2v
