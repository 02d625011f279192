// One launch for a whole step of Alg. 3 (lines 5-7: embed, score, select) on small graphs.
//
// When a graph's embedding matrix fits the LDS of one compute unit (n * p <= 32768 floats: 1024 nodes at
// p = 32, 512 at p = 64), one workgroup of 16 waves runs the whole evaluation for that graph: all T rounds
// of Eq. 1, the graph sum and the scores of Eq. 2, and the masked argmax / top-d selection, with
// workgroup barriers where the general path has kernel boundaries.  A block-diagonal batch takes one
// workgroup per graph, so the graphs of a batch run side by side on different compute units.
// The previous round's embedding lives in LDS, so the neighbour gathers are LDS reads (tens of cycles)
// instead of L2 reads (hundreds): at these sizes the general path is bound by launch and memory latency,
// not by bytes.  Per round:
//   gather : a group of p/4 lanes per row walks the row's neighbours and adds their rows from LDS
//            (4 or 8 rows per wave at once); the sums of a wave's tiles stay in registers;
//   dense  : after a barrier (everybody has read the old rows), each 16-row tile of sums is brought into the
//            operand layout by lane shuffles and multiplied by theta2 on the matrix cores (same product and
//            epilogue as the general round kernel), relu, result written over the old rows in LDS.
// Global memory sees the column indices, the per-node scalars, the parameters and the outputs, nothing else.
#include <limits.h>

#include "device_util.h"
#include "internal.h"
#include "select_util.h"

namespace s2v {

constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / 64;

template <int P>
struct SmallGeo {
    static constexpr int MAXN = kSmallLdsFloats / P;   // nodes per graph
};

// best (val, idx) of the workgroup's 1024 threads, returned to every thread
__device__ __forceinline__ void small_block_best(float &val, int &idx, float *sval, int *sidx) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const float v2 = __shfl_xor(val, m);
        const int i2 = __shfl_xor(idx, m);
        take_better(val, idx, v2, i2);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) { sval[wave] = val; sidx[wave] = idx; }
    __syncthreads();
    val = sval[0];
    idx = sidx[0];
#pragma unroll
    for (int w = 1; w < kSmallWaves; ++w) take_better(val, idx, sval[w], sidx[w]);
}

template <int P>
__global__ __launch_bounds__(kSmallThreads) void k_small_policy(SmallPolicyArgs a) {
    using G = Geo<P>;
    constexpr int MAXN = SmallGeo<P>::MAXN, LPR = G::LPR, NPL = G::NPL, KS = G::KS, CB = G::CB;
    constexpr int NB = kTileRows / NPL;                       // row batches per 16-row tile
    constexpr int TPW = MAXN / kTileRows / kSmallWaves;       // tiles per wave (4 at p = 32, 2 at p = 64)
    __shared__ __attribute__((aligned(16))) float cur[MAXN * P];            // the embedding of the previous round
    __shared__ __attribute__((aligned(16))) float lds_b[P * G::STRIDE];     // theta2, the B operand
    __shared__ __attribute__((aligned(16))) float lds_c[4 * P];             // theta1, q+, q-, theta4
    __shared__ int rb[MAXN], re[MAXN];                                      // live range of every row
    __shared__ float red[kSmallThreads];                                    // reductions, then the scores
    __shared__ float gs[P];
    __shared__ float sval[kSmallWaves];
    __shared__ int sidx[kSmallWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x;
    const int lo = a.graph_off ? a.graph_off[g] : 0;
    const int hi = a.graph_off ? a.graph_off[g + 1] : a.N;
    const int n = hi - lo;   // <= MAXN (checked on the host)
    const int jl = lane & 15, gl = lane >> 4;
    const int gq = lane / LPR, li = lane % LPR;

    // the scalars of "my" row of each of this wave's tiles (lane jl <-> tile row jl), fetched once
    float xs[TPW], sp[TPW], sn[TPW];
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int row = (wave + kSmallWaves * j) * kTileRows + jl;
        xs[j] = row < n ? a.x[lo + row] : 0.f;
        sp[j] = row < n ? a.s_pos[lo + row] : 0.f;
        sn[j] = row < n ? a.s_neg[lo + row] : 0.f;
    }
    stage_matrix_lds<P>(lds_b, a.theta2, false);
    if (tid < P) {
        lds_c[tid] = a.theta1[tid];
        lds_c[3 * P + tid] = a.theta4[tid];
    }
    for (int r = tid; r < n; r += kSmallThreads) {
        rb[r] = a.rowptr[lo + r];
        re[r] = a.rowend[lo + r];
    }
    // q+ = theta3 relu(theta4), q- = theta3 relu(-theta4): eight lanes per output, each with an eighth of the
    // row of theta3 (vector loads issued before the barrier), partial sums in double, added in a fixed order
    constexpr int QL = 8, QF = P / QL;   // lanes per output, floats per lane
    const int q_out = tid / QL, q_part = tid % QL;
    float q_t3[QF];
    if (q_out < 2 * P) {
#pragma unroll
        for (int c = 0; c < QF / 4; ++c) {
            const float4 v4 = ld4(a.theta3 + (q_out % P) * P + q_part * QF + 4 * c);
            q_t3[4 * c] = v4.x; q_t3[4 * c + 1] = v4.y; q_t3[4 * c + 2] = v4.z; q_t3[4 * c + 3] = v4.w;
        }
    }
    __syncthreads();
    {
        const bool neg = q_out >= P;
        double acc = 0.0;
        if (q_out < 2 * P) {
#pragma unroll
            for (int c = 0; c < QF; ++c) {
                const float t4 = lds_c[3 * P + q_part * QF + c];
                acc += (double)q_t3[c] * (double)fmaxf(neg ? -t4 : t4, 0.f);
            }
        }
#pragma unroll
        for (int m = 1; m < QL; m <<= 1) acc += __shfl_xor(acc, m);
        if (q_out < 2 * P && q_part == 0) lds_c[P + q_out] = (float)acc;
    }
    __syncthreads();

    // ---- round 1: mu^0 = 0, so mu^1 = relu(theta1 x + s+ q+ + s- q-) ----
    for (int f = tid; f < n * LPR; f += kSmallThreads) {
        const int r = f / LPR, c = 4 * (f % LPR);
        const int v = lo + r;
        const float4 o = mu1_row(a.x[v], a.s_pos[v], a.s_neg[v], ld4(lds_c + c), ld4(lds_c + P + c), ld4(lds_c + 2 * P + c));
        st4(cur + r * P + c, o);
        if (a.T == 1) st4(a.mu_out + (size_t)v * P + c, o);
    }
    __syncthreads();

    const int n_tiles = (n + kTileRows - 1) / kTileRows;
    for (int t = 2; t <= a.T; ++t) {
        // ---- gather: a_v = sum over the live entries of row v of cur[u], kept in registers ----
        // batch (j, bb) = rows (wave + 16 j) * 16 + bb * NPL + gq of tile j; a group of LPR lanes per row
        float4 accb[TPW][NB];
        int b0[TPW][NB], e0[TPW][NB], idx0[TPW][NB], idx1[TPW][NB];
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int bb = 0; bb < NB; ++bb) {
                const int r = (wave + kSmallWaves * j) * kTileRows + bb * NPL + gq;
                const bool ok = r < n;
                b0[j][bb] = ok ? rb[r] : 0;
                e0[j][bb] = ok ? re[r] : 0;
                // the first 2 LPR column indices of every batch are requested before any of them is used
                idx0[j][bb] = (b0[j][bb] + li < e0[j][bb]) ? a.colidx[b0[j][bb] + li] : -1;
                idx1[j][bb] = (b0[j][bb] + LPR + li < e0[j][bb]) ? a.colidx[b0[j][bb] + LPR + li] : -1;   // second chunk
            }
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int bb = 0; bb < NB; ++bb) {
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                int base = b0[j][bb], idx = idx0[j][bb];
                const int e = e0[j][bb];
                while (true) {
                    // entries base .. base + LPR - 1 of this group's row: lane li holds the index of entry base + li
                    // Four entries per step, their four LDS reads in flight together; as many steps as the longest
                    // of the wave's rows has entries left in this chunk.  Entry k of each group's chunk reaches the
                    // group's lanes through a lane read per group (the scalar unit, not a cross-lane LDS operation) when
                    // a wave holds four groups.
                    const int left = e - base;
#pragma unroll
                    for (int k0 = 0; k0 < LPR; k0 += 4) {
                        if (__builtin_amdgcn_ballot_w64(k0 < left) == 0ull) break;   // wave-uniform
                        int u[4];
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) {
                            if constexpr (NPL <= 4) {
                                u[kk] = -1;
#pragma unroll
                                for (int gg = 0; gg < NPL; ++gg) {
                                    const int ug = __builtin_amdgcn_readlane(idx, gg * LPR + k0 + kk);
                                    u[kk] = gq == gg ? ug : u[kk];
                                }
                            } else {
                                u[kk] = __shfl(idx, gq * LPR + k0 + kk);   // (eight groups: one shuffle is cheaper)
                            }
                        }
                        float4 v[4];
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk)
                            v[kk] = u[kk] >= 0 ? ld4(cur + (u[kk] - lo) * P + 4 * li) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) acc = add4(acc, v[kk]);
                    }
                    base += LPR;
                    if (__builtin_amdgcn_ballot_w64(base < e) == 0ull) break;   // wave-uniform
                    if (base == b0[j][bb] + LPR) idx = idx1[j][bb];             // (uniform: every group is at its second chunk)
                    else idx = (base + li < e) ? a.colidx[base + li] : -1;
                }
                accb[j][bb] = acc;
            }
        __syncthreads();   // every wave has read what it needs of cur: the tiles may be overwritten
        // ---- dense: mu^t = relu(theta2 a + theta1 x + s+ q+ + s- q-) ----
        const bool last = t == a.T;
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int ti = wave + kSmallWaves * j;
            if (ti >= n_tiles) break;   // wave-uniform
            const int r0 = ti * kTileRows;
            // From the gather layout (lane (gq, li) of batch bb: row bb * NPL + gq, columns 4 li ..) to the operand
            // layout of the matrix instruction (lane (jl, gl): row jl, columns gl * KS ..): lane shuffles.
            Frag<P> af;
            const int src_bb = jl / NPL;
#pragma unroll
            for (int c = 0; c < KS / 4; ++c) {
                const int src = (jl % NPL) * LPR + gl * (KS / 4) + c;
                float4 pick = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int bb = 0; bb < NB; ++bb) {
                    const float4 v4 = make_float4(__shfl(accb[j][bb].x, src), __shfl(accb[j][bb].y, src),
                                                  __shfl(accb[j][bb].z, src), __shfl(accb[j][bb].w, src));
                    if (bb == src_bb) pick = v4;
                }
                af.v[4 * c] = pick.x; af.v[4 * c + 1] = pick.y; af.v[4 * c + 2] = pick.z; af.v[4 * c + 3] = pick.w;
            }
            f32x4 acc[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                acc[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
                acc[cb] = mfma_tile<P>(af, load_b_frag_lds<P>(lds_b, cb, lane), acc[cb]);
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int i = 4 * gl + rr;
                const float xi = __shfl(xs[j], i), spi = __shfl(sp[j], i), sni = __shfl(sn[j], i);
                if (r0 + i < n) {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        const int col = 16 * cb + jl;
                        const float o = fmaxf(__fmaf_rn(sni, lds_c[2 * P + col], __fmaf_rn(spi, lds_c[P + col],
                                              __fmaf_rn(xi, lds_c[col], acc[cb][rr]))), 0.f);
                        cur[(r0 + i) * P + col] = o;
                        if (last) a.mu_out[(size_t)(lo + r0 + i) * P + col] = o;
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- graph sum (Alg. 2 line 4): slices of rows per thread, then the slices in order ----
    // (meanwhile: theta6 for the graph term, eight lanes per output as above, requested ahead)
    float q_t6[QF];
    if (q_out < P) {
#pragma unroll
        for (int c = 0; c < QF / 4; ++c) {
            const float4 v4 = ld4(a.theta6 + q_out * P + q_part * QF + 4 * c);
            q_t6[4 * c] = v4.x; q_t6[4 * c + 1] = v4.y; q_t6[4 * c + 2] = v4.z; q_t6[4 * c + 3] = v4.w;
        }
    }
    {
        constexpr int SL = kSmallThreads / P;
        const int jc = tid % P, s = tid / P;
        float acc = 0.f;
        for (int r = s; r < n; r += SL) acc += cur[r * P + jc];
        red[tid] = acc;
        __syncthreads();
        if (tid < P) {
            double sum = 0.0;
            for (int k = 0; k < SL; ++k) sum += (double)red[k * P + tid];
            gs[tid] = (float)sum;
            a.gsum[(size_t)g * P + tid] = (float)sum;
        }
        __syncthreads();
    }
    // ---- graph term of Eq. 2: qa = theta5[0:p] . relu(theta6 g) ----
    {
        double h = 0.0;
        if (q_out < P) {
#pragma unroll
            for (int c = 0; c < QF; ++c) h += (double)q_t6[c] * (double)gs[q_part * QF + c];
        }
#pragma unroll
        for (int m = 1; m < QL; m <<= 1) h += __shfl_xor(h, m);
        __syncthreads();
        if (q_out < P && q_part == 0) red[128 + q_out] = a.theta5[q_out] * fmaxf((float)h, 0.f);
        __syncthreads();
        const float term = tid < P ? red[128 + tid] : 0.f;
        if (tid < 128) red[tid] = term;
        __syncthreads();
        for (int w = 64; w >= 1; w >>= 1) {
            if (tid < w) red[tid] += red[tid + w];
            __syncthreads();
        }
    }
    const float qa = red[0];
    __syncthreads();
    // ---- node term of Eq. 2 for every node: theta5[p:2p] . relu(theta7 mu_v), tiles on the matrix cores ----
    for (int ti = wave; ti < n_tiles; ti += kSmallWaves) {
        const int r0 = ti * kTileRows;
        const int row = r0 + jl;
        Frag<P> af;
#pragma unroll
        for (int c = 0; c < KS / 4; ++c) {
            const float4 v4 = row < n ? ld4(cur + row * P + gl * KS + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
            af.v[4 * c] = v4.x; af.v[4 * c + 1] = v4.y; af.v[4 * c + 2] = v4.z; af.v[4 * c + 3] = v4.w;
        }
        float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            f32x4 h = (f32x4){0.f, 0.f, 0.f, 0.f};
            h = mfma_tile<P>(af, load_b_frag_rows<P>(a.theta7, cb, lane), h);
            const float t5 = a.theta5[P + 16 * cb + jl];
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
                const int rq = r0 + 4 * gl + rr;
                if (rq < n) {
                    const float qv = qa + part[rr];
                    red[rq] = qv;                       // (n <= MAXN <= 1024 floats of `red`)
                    a.q[lo + rq] = qv;
                }
            }
        }
    }
    __syncthreads();
    if (!a.idx) return;
    // ---- selection (Alg. 3 line 7, Sec. 4.5.1): the k best candidates, score descending, index ascending ----
    // one node per thread; "the next best" is the best entry that the last pick beats
    const bool mine = tid < n && is_candidate(a.x, a.cand, lo + tid);
    const float myv = mine ? red[tid] : -INFINITY;
    const int myi = mine ? lo + tid : INT_MAX;
    float lv = INFINITY;
    int lidx = -1, found = 0;
    for (int it = 0; it < a.k; ++it) {
        float val = -INFINITY;
        int idx = INT_MAX;
        if (myi != INT_MAX && beats(lv, lidx, myv, myi)) { val = myv; idx = myi; }
        small_block_best(val, idx, sval, sidx);
        if (idx == INT_MAX) break;   // uniform: no candidate left
        if (tid == 0) {
            a.idx[(size_t)g * a.k + it] = idx;
            a.val[(size_t)g * a.k + it] = val + 0.0f;
        }
        lv = val;
        lidx = idx;
        ++found;
    }
    for (int r = found + tid; r < a.k; r += kSmallThreads) {
        a.idx[(size_t)g * a.k + r] = -1;
        a.val[(size_t)g * a.k + r] = -INFINITY;
    }
    if (tid == 0) a.count[g] = found;
}

hipError_t launch_small_policy(hipStream_t st, int p, const SmallPolicyArgs &a) {
    if (a.G <= 0) return hipSuccess;
    if (p == 32) k_small_policy<32><<<a.G, kSmallThreads, 0, st>>>(a);
    else k_small_policy<64><<<a.G, kSmallThreads, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace s2v
