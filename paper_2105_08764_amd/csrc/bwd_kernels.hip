// Backward pass of the training step (Train of Alg. 4): reverse-mode differentiation of the
// squared loss through Eq. 2 at the action nodes and through all T rounds of Eq. 1, and the
// plain gradient-descent update (repeated per minibatch as in Sec. 4.5.2).
//
// Notation (state b, node v, round t):  z^t_v = c_v + theta2 a^{t-1}_v,  a^{t-1}_v = sum_{u in N(v)} mu^{t-1}_u,
// mu^t = relu(z^t),  c_v = theta1 x_v + s+_v q+ + s-_v q-,  q+- = theta3 relu(+-theta4).
//   dz^t     = dmu^t (.) [mu^t > 0]
//   G_u      = sum_{v in N(u)} dz^t_v             (adjoint of the neighbour sum; the pattern is symmetric)
//   dtheta2 += sum_u G_u mu^{t-1}_u^T
//   dmu^{t-1}_u = theta2^T G_u
//   dtheta1 = sum_t sum_v x_v dz^t_v,  dq+- = sum_t sum_v s+-_v dz^t_v
//   dtheta3 = dq+ relu(theta4)^T + dq- relu(-theta4)^T
//   dtheta4 = [theta4 > 0] (.) theta3^T dq+  -  [theta4 < 0] (.) theta3^T dq-
// Every reduction is a fixed tree over a fixed grid: results do not vary from run to run.
#include "device_util.h"
#include "internal.h"

namespace s2v {

// ------------------------------------------------------------------------------------------
// Head: Eq. 2 at the action node of each state, the loss, and the gradients that do not need
// the graph: per-state partials of dtheta5/6/7 and the two vectors that seed dmu^T:
//   dg = theta6^T dh1 (goes to every node of the action's graph), da = theta7^T dh2 (action node only).
// One workgroup of 128 threads per state.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void k_bwd_head(int p, int N, int S, int G, const int32_t *__restrict__ graph_off,
                                                  const float *__restrict__ theta5, const float *__restrict__ theta6,
                                                  const float *__restrict__ theta7, const float *__restrict__ muT,
                                                  const float *__restrict__ gsum, const int32_t *__restrict__ action,
                                                  const float *__restrict__ target, float *__restrict__ dg,
                                                  float *__restrict__ da, int32_t *__restrict__ glo,
                                                  int32_t *__restrict__ ghi, float *__restrict__ head_part,
                                                  float *__restrict__ q_pred) {
    __shared__ float g[128], m[128], dh1[128], dh2[128], red[128];
    const int b = blockIdx.x, i = threadIdx.x;
    const int a = action[b];
    int gi = 0, lo = 0, hi = N;
    if (G > 1) {
        int l = 0, h = G;
        while (h - l > 1) {
            const int mid = (l + h) >> 1;
            if (graph_off[mid] <= a) l = mid; else h = mid;
        }
        gi = l; lo = graph_off[gi]; hi = graph_off[gi + 1];
    }
    if (i < p) {
        g[i] = gsum[((size_t)b * G + gi) * p + i];
        m[i] = muT[((size_t)a * S + b) * p + i];
    }
    __syncthreads();
    float h1 = 0.f, h2 = 0.f, r1 = 0.f, r2 = 0.f, term = 0.f;
    if (i < p) {
        // the 2p pre-activations of Eq. 2 in double, rounded once: each of these relu units carries a large
        // share of the state's gradient, and the work is 2 p^2 operations per state
        double a1 = 0.0, a2 = 0.0;
        for (int j = 0; j < p; ++j) {
            a1 += (double)theta6[i * p + j] * (double)g[j];
            a2 += (double)theta7[i * p + j] * (double)m[j];
        }
        h1 = (float)a1;
        h2 = (float)a2;
        r1 = fmaxf(h1, 0.f);
        r2 = fmaxf(h2, 0.f);
        term = theta5[i] * r1 + theta5[p + i] * r2;
    }
    red[i] = term;
    __syncthreads();
    for (int w = 64; w >= 1; w >>= 1) {
        if (i < w) red[i] += red[i + w];
        __syncthreads();
    }
    const float q = red[0];
    const float diff = q - target[b];
    const float dq = 2.f * diff / (float)S;
    float *part = head_part + (size_t)b * (2 * p + 2 * p * p + 1);
    if (i < p) {
        part[i] = dq * r1;
        part[p + i] = dq * r2;
        dh1[i] = h1 > 0.f ? dq * theta5[i] : 0.f;
        dh2[i] = h2 > 0.f ? dq * theta5[p + i] : 0.f;
    }
    if (i == 0) {
        part[2 * p + 2 * p * p] = diff * diff / (float)S;
        glo[b] = lo; ghi[b] = hi;
        if (q_pred) q_pred[b] = q;
    }
    __syncthreads();
    float *p6 = part + 2 * p, *p7 = p6 + p * p;
    for (int e = i; e < p * p; e += 128) {
        const int r = e / p, c = e - r * p;
        p6[e] = dh1[r] * g[c];
        p7[e] = dh2[r] * m[c];
    }
    if (i < p) {
        float s6 = 0.f, s7 = 0.f;
        for (int r = 0; r < p; ++r) {
            s6 += theta6[r * p + i] * dh1[r];
            s7 += theta7[r * p + i] * dh2[r];
        }
        dg[(size_t)b * p + i] = s6;
        da[(size_t)b * p + i] = s7;
    }
}

hipError_t launch_bwd_head(hipStream_t st, int p, int N, int S, int G, const int32_t *graph_off, const float *theta5,
                           const float *theta6, const float *theta7, const float *muT, const float *gsum,
                           const int32_t *action, const float *target, const BwdScratch &sc, float *q_pred) {
    k_bwd_head<<<S, 128, 0, st>>>(p, N, S, G, graph_off, theta5, theta6, theta7, muT, gsum, action, target, sc.dg, sc.da,
                                  sc.glo, sc.ghi, sc.head_part, q_pred);
    return hipGetLastError();
}

// Sum the per-state partials over the S states in state order: dtheta5, dtheta6, dtheta7, loss.
__global__ __launch_bounds__(256) void k_bwd_head_reduce(int p, int S, const float *__restrict__ head_part,
                                                         float *__restrict__ loss, float *__restrict__ d5,
                                                         float *__restrict__ d6, float *__restrict__ d7) {
    const int width = 2 * p + 2 * p * p + 1;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= width) return;
    double acc = 0.0;
    for (int b = 0; b < S; ++b) acc += (double)head_part[(size_t)b * width + e];
    const float out = (float)acc;
    if (e < 2 * p) d5[e] = out;
    else if (e < 2 * p + p * p) d6[e - 2 * p] = out;
    else if (e < 2 * p + 2 * p * p) d7[e - 2 * p - p * p] = out;
    else loss[0] = out;
}

hipError_t launch_bwd_head_reduce(hipStream_t st, int p, int S, const BwdScratch &sc, float *loss, float *d5, float *d6,
                                  float *d7) {
    const int width = 2 * p + 2 * p * p + 1;
    k_bwd_head_reduce<<<(width + 255) / 256, 256, 0, st>>>(p, S, sc.head_part, loss, d5, d6, d7);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Last-round seed.  dz^T[v][s] = (dg[s] if v is in the action's graph, + da[s] if v is the action
// node) (.) [mu^T[v][s] > 0] is never written out: this kernel streams mu^T once, stores only the
// relu mask (one 64-bit word per (node, state), bit j = entry j positive; skipped when T == 1) and
// adds dz^T's share of sum x dz, sum s+ dz, sum s- dz.  Fixed grid, each workgroup owns a
// contiguous block of rows; thread = (row slot, float4 column).
//   WORDS: the mask words are already there (the forward pass of the same call left them instead of
//          mu^T): they are read in place of mu^T, by the same threads in the same order, so the sums
//          come out bit for bit as from mu^T itself.
// ------------------------------------------------------------------------------------------
template <int P, bool WORDS>
__global__ __launch_bounds__(256) void k_bwd_maskT(long n_vrows, int N, int S, const float *__restrict__ muT,
                                                   NodeInfo ni, const float *__restrict__ x_res,
                                                   const int32_t *__restrict__ action,
                                                   const float *__restrict__ dg, const float *__restrict__ da,
                                                   const int32_t *__restrict__ glo, const int32_t *__restrict__ ghi,
                                                   unsigned long long *__restrict__ mask,
                                                   float *__restrict__ dc_part) {
    constexpr int LPR = P / 4, SLOTS = 256 / LPR;
    __shared__ float red[3][SLOTS][P];
    // per-state constants of up to kStatesInLds states, fetched once per workgroup
    constexpr int kStatesInLds = 32;
    __shared__ __attribute__((aligned(16))) float s_dg[kStatesInLds][P], s_da[kStatesInLds][P];
    __shared__ int s_glo[kStatesInLds], s_ghi[kStatesInLds], s_act[kStatesInLds];
    const bool cached = S <= kStatesInLds;
    if (cached) {
        for (int i = threadIdx.x; i < S * P; i += 256) { s_dg[i / P][i % P] = dg[i]; s_da[i / P][i % P] = da[i]; }
        for (int i = threadIdx.x; i < S; i += 256) { s_glo[i] = glo[i]; s_ghi[i] = ghi[i]; s_act[i] = action[i]; }
    }
    __syncthreads();
    const int c4 = threadIdx.x % LPR, slot = threadIdx.x / LPR;
    const long per = (n_vrows + gridDim.x - 1) / gridDim.x;
    const long r_begin = (long)blockIdx.x * per, r_end = min(n_vrows, r_begin + per);
    float4 ax = make_float4(0.f, 0.f, 0.f, 0.f), ap = ax, an = ax;
    // All lanes of a wave run the same number of iterations (the shuffles below need that); four
    // rows per thread and step keep four independent loads in flight.
    constexpr int U = 4;
    // (node, state) of this thread's current row, advanced by SLOTS rows at a time without a division
    const int step_v = SLOTS / S, step_s = SLOTS - step_v * S;
    int v_cur = (int)((r_begin + slot) / S), s_cur = (int)((r_begin + slot) - (long)v_cur * S);
    for (long rbase = r_begin; rbase < r_end; rbase += U * SLOTS) {
        float4 mu[U];
        int vk[U], sk[U];
        float3 rec[U];
        float xres[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const long r = rbase + k * SLOTS + slot;
            vk[k] = v_cur;
            sk[k] = s_cur;
            v_cur += step_v;
            s_cur += step_s;
            if (s_cur >= S) { s_cur -= S; ++v_cur; }
            // the row's scalars are requested together with its data: one trip to memory per step
            rec[k] = r < r_end ? ni.get(vk[k], sk[k]) : make_float3(0.f, 0.f, 0.f);
            xres[k] = (x_res && r < r_end) ? x_res[(size_t)sk[k] * N + vk[k]] : 0.f;
            if (WORDS) {
                // only the signs matter below: 1 where the bit is set
                const unsigned nib = r < r_end ? (unsigned)(mask[r] >> (4 * c4)) & 15u : 0u;
                mu[k] = make_float4((float)(nib & 1u), (float)((nib >> 1) & 1u), (float)((nib >> 2) & 1u),
                                    (float)((nib >> 3) & 1u));
            } else {
                mu[k] = r < r_end ? ld4(muT + (size_t)r * P + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const long r = rbase + k * SLOTS + slot;
            const bool valid = r < r_end;
            unsigned long long word = 0ull;
            const int v = vk[k], s = sk[k];
            if (valid) {
                float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
                if (cached) {
                    if (v >= s_glo[s] && v < s_ghi[s]) d = ld4(&s_dg[s][4 * c4]);
                    if (v == s_act[s]) d = add4(d, ld4(&s_da[s][4 * c4]));
                } else {
                    if (v >= glo[s] && v < ghi[s]) d = ld4(dg + (size_t)s * P + 4 * c4);
                    if (v == action[s]) d = add4(d, ld4(da + (size_t)s * P + 4 * c4));
                }
                d.x = mu[k].x > 0.f ? d.x : 0.f;
                d.y = mu[k].y > 0.f ? d.y : 0.f;
                d.z = mu[k].z > 0.f ? d.z : 0.f;
                d.w = mu[k].w > 0.f ? d.w : 0.f;
                const unsigned nib = (mu[k].x > 0.f ? 1u : 0u) | (mu[k].y > 0.f ? 2u : 0u) |
                                     (mu[k].z > 0.f ? 4u : 0u) | (mu[k].w > 0.f ? 8u : 0u);
                word = (unsigned long long)nib << (4 * c4);
                const float3 q = rec[k];
                float xs = q.x;
                const float sp = q.y, sn = q.z;
                if (x_res) {
                    // per-state residual graphs: a solution node is isolated; it still feeds dtheta1 through
                    // the graph sum, but its mask word is zero so that no neighbour gathers from it
                    const float xo = xres[k];
                    if (xo != 0.f) { xs = xo; word = 0ull; }
                }
                ax.x += xs * d.x; ax.y += xs * d.y; ax.z += xs * d.z; ax.w += xs * d.w;
                ap.x += sp * d.x; ap.y += sp * d.y; ap.z += sp * d.z; ap.w += sp * d.w;
                an.x += sn * d.x; an.y += sn * d.y; an.z += sn * d.z; an.w += sn * d.w;
            }
            if (mask && !WORDS) {
                // OR the nibbles of the LPR lanes that share a row
#pragma unroll
                for (int m = 1; m < LPR; m <<= 1) word |= __shfl_xor(word, m);
                if (valid && c4 == 0) mask[r] = word;
            }
        }
    }
    st4(&red[0][slot][4 * c4], ax);
    st4(&red[1][slot][4 * c4], ap);
    st4(&red[2][slot][4 * c4], an);
    __syncthreads();
    for (int e = threadIdx.x; e < 3 * P; e += 256) {
        const int c = e / P, j = e - c * P;
        float s = 0.f;
        for (int k = 0; k < SLOTS; ++k) s += red[c][k][j];
        dc_part[(size_t)blockIdx.x * 3 * P + e] = s;
    }
}

hipError_t launch_bwd_maskT(hipStream_t st, int p, int N, int S, const float *muT, const NodeInfo &ni, const float *x_res,
                            const int32_t *action, const BwdScratch &sc, unsigned long long *mask, float *dc_part,
                            bool words_ready) {
    const long n_vrows = (long)N * S;
    if (words_ready && (!mask || x_res)) return hipErrorInvalidValue;
#define S2V_LAUNCH_MASKT(P, WORDS)                                                                                 \
    k_bwd_maskT<P, WORDS><<<kBwdHeadGrid, 256, 0, st>>>(n_vrows, N, S, muT, ni, x_res, action, sc.dg, sc.da, sc.glo, \
                                                        sc.ghi, mask, dc_part)
    if (p == 32) {
        if (words_ready) S2V_LAUNCH_MASKT(32, true);
        else S2V_LAUNCH_MASKT(32, false);
    } else {
        if (words_ready) S2V_LAUNCH_MASKT(64, true);
        else S2V_LAUNCH_MASKT(64, false);
    }
#undef S2V_LAUNCH_MASKT
    return hipGetLastError();
}

// *hi + *lo += v without losing the rounding error of the addition (the exact remainder of h + v goes to lo).
// first: the pair is uninitialised and becomes (v, 0).
__device__ __forceinline__ void comp_add(float *hi, float *lo, float v, bool first) {
    if (first) {
        *hi = v;
        *lo = 0.f;
        return;
    }
    const float h = *hi;
    const float s = h + v;
    const float bb = s - h;
    const float err = (h - (s - bb)) + (v - bb);
    *hi = s;
    *lo = *lo + err;
}

// ------------------------------------------------------------------------------------------
// One reversed round t (T >= t >= 2), fused: G = A dz^t (same gathers as the forward round),
// dtheta2 partial += G^T mu^{t-1}, dz^{t-1} = (G theta2) (.) [mu^{t-1} > 0], and this round's share
// of sum x dz^{t-1}, sum s+- dz^{t-1}.  Wave tiles of 16 rows of the [N*S][p] matrices; the
// p x p accumulator of dtheta2 stays in registers over all tiles of the wave.
//   NODE: S is a multiple of 16 (a tile is 16 states of one node).
//   MASK: this is round t = T.  dz^T is not in memory; apart from the action node's own term
//         (added afterwards by k_bwd_action_fix, the round being linear in dz^T) it equals
//         dg[s] (.) [mu^T > 0] on the nodes of the action's graph, so G_u = dg[s] (.) (number of
//         neighbours of u whose mask bit is set): the gather reads 8-byte mask words, not rows.
//   dz_out may be NULL (t == 2: dz^1 is needed for the sums only).
//   FUSE (node mode, not the mask round; used for t = 3): the round t = 2 that would follow is done here,
//         tile by tile, in its scalar form (see k_bwd_first): the tile's dz^2 is still on chip, so it is
//         neither written nor read back, and its contributions go into the SAME dtheta2 and column-sum
//         accumulators (the parameter gradients are sums over the rounds anyway).  NEG as in k_bwd_first.
// ------------------------------------------------------------------------------------------
struct FirstFuse {
    const float *theta1;
    const float *qvec;
    const float *hub_sum4;   // [n_hubs][4][S][P]
};

#ifndef S2V_BWD_MASK_OCC
#define S2V_BWD_MASK_OCC 2
#endif
template <int P, bool NODE, bool MASK, bool W, bool FUSE, bool NEG, bool FLAGS = false>   // W: weighted neighbour sum (symmetric weights wagg)
__global__ __launch_bounds__(kThreads, (NODE && MASK) ? S2V_BWD_MASK_OCC : 2) void k_bwd_round(
    int n_vrows, int S, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ rowend,
    const int32_t *__restrict__ colidx, const float *__restrict__ wagg, const float *__restrict__ dz_in, const unsigned long long *__restrict__ maskT, const float *__restrict__ dg,
    const int32_t *__restrict__ glo, const int32_t *__restrict__ ghi, const float *__restrict__ mu_prev,
    float *__restrict__ dz_out, NodeInfo ni, const float *__restrict__ theta2,
    float *__restrict__ dc_part,
    float *__restrict__ d2_part, HubTable ht, const float *__restrict__ hub_sum, FirstFuse ff, int by_state) {
    // by_state (row mode only): tile row i is (node v0 + i, state st), the launch works through one state's rows
    // at a time, as the forward rounds do for large matrices (the sums do not depend on the order of the tiles)
    using Ge = Geo<P>;
    constexpr int CB = Ge::CB, STRIDE = Ge::STRIDE;
    constexpr int TILE_F = kTileRows * STRIDE;
    static_assert(kWaves * TILE_F >= kWaves * 16 * P, "tile area is reused for the final reductions");
    static_assert(!FUSE || (NODE && !MASK), "the fused last round needs node mode and dz in memory");
    // second tile per wave and record staging of the fused last round
    __shared__ __attribute__((aligned(16))) float lds_a[FUSE ? kWaves * TILE_F : 4];
    __shared__ __attribute__((aligned(16))) float rec_stage[(FUSE && !FLAGS) ? kWaves * kRecStageFloats : 4];
    __shared__ __attribute__((aligned(16))) float lds[kWaves * TILE_F];
    // staging area of the mask-word gather (node mode of the MASK round only)
    __shared__ __attribute__((aligned(16))) unsigned bits_stage[(NODE && MASK) ? kWaves * kBitsStageBytes / 4 : 4];
    __shared__ __attribute__((aligned(16))) float lds_b[P * STRIDE];   // theta2^T: B operand of G theta2
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *tile_g = lds + wave * TILE_F;
    const int li = lane % Ge::LPR;
    const int jl = lane & 15, gl = lane >> 4;

    stage_matrix_lds<P>(lds_b, theta2, true);
    // MASK: the per-state constants (dg and the node range of the action's graph) of up to kMaskStatesLds states
    // live in LDS: a load from memory inside the tile loop would have to wait for the prefetches issued before it
    constexpr int kMaskStatesLds = 32;
    __shared__ __attribute__((aligned(16))) float s_dg[MASK ? kMaskStatesLds * P : 4];
    __shared__ int s_glo[MASK ? kMaskStatesLds : 1], s_ghi[MASK ? kMaskStatesLds : 1];
    const bool dg_lds = MASK && S <= kMaskStatesLds;
    if (dg_lds) {
        for (int i = threadIdx.x; i < S * P; i += kThreads) s_dg[MASK ? i : 0] = dg[i];
        for (int i = threadIdx.x; i < S; i += kThreads) { s_glo[MASK ? i : 0] = glo[i]; s_ghi[MASK ? i : 0] = ghi[i]; }
    }
    __syncthreads();
    auto in_range = [&](int node, int st) {
        return dg_lds ? (node >= s_glo[MASK ? st : 0] && node < s_ghi[MASK ? st : 0]) : (node >= glo[st] && node < ghi[st]);
    };
    auto dg_at = [&](int st, int col) {
        return dg_lds ? ld4(s_dg + (MASK ? st * P + col : 0)) : ld4(dg + (size_t)st * P + col);
    };

    f32x4 d2acc[CB][CB];
#pragma unroll
    for (int ib = 0; ib < CB; ++ib)
#pragma unroll
        for (int jb = 0; jb < CB; ++jb) d2acc[ib][jb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float cx[CB], cp[CB], cn[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) cx[cb] = cp[cb] = cn[cb] = 0.f;
    // column sums of the fused last round (columns 4 * li .. of this lane)
    float4 fx4 = make_float4(0.f, 0.f, 0.f, 0.f), fp4 = fx4, fn4 = fx4;
    // FLAGS: that round works from flag words and the rows' totals (see gather_node_tile_flags_grad); its
    // sums are kept per column lane % P
    static_assert(!FLAGS || (FUSE && !NEG), "flag words: no negative weight");
    float fxj = 0.f, fpj = 0.f, t1j = 0.f, qpj = 0.f;
    if (FLAGS) {
        t1j = ff.theta1[lane % P];
        qpj = ff.qvec[lane % P];
    }

    const size_t row_stride = (size_t)S * P;
    const bool sliced = !NODE && by_state != 0;
    const int n_nodes = n_vrows / S;
    const int tps = (n_nodes + kWgRows - 1) / kWgRows;   // tiles per state when sliced
    const int n_tiles = sliced ? tps * S : (n_vrows + kWgRows - 1) / kWgRows;
    // Node mode: a tile is one node, and the row range and first column indices of the wave's NEXT tile
    // are fetched while the current one is worked on (rowptr -> colidx -> data is a chain of three
    // dependent trips to memory otherwise).
    int pf_b = 0, pf_e = 0, pf_cols = 0;
    if (NODE) {
        const int r0 = blockIdx.x * kWgRows + wave * kTileRows;
        if ((int)blockIdx.x < n_tiles && r0 < n_vrows) {
            const int v0 = r0 / S;
            pf_b = rowptr[v0];
            pf_e = rowend[v0];
            pf_cols = (lane < min(64, pf_e - pf_b)) ? colidx[pf_b + lane] : 0;
        }
    }
    // The mask round does little per tile besides its two matrix products: there the next tile's mu^{t-1}
    // (4 KB, needed first thing) is fetched a tile ahead as well.
    constexpr bool PFM = NODE && MASK;
    // ... and so are the mask words of the next tile's first 32 neighbours, which takes the row ranges three
    // tiles and the column indices two tiles ahead: tile t (pf_*, pw), t + G (q1_*), t + 2G (q2_*).
    constexpr bool PFW = PFM && !W;
    int q1_b = 0, q1_e = 0, q1_cols = 0, q2_b = 0, q2_e = 0;
    unsigned long long pw[PFW ? 8 : 1];
    auto tile_range = [&](int tile, int &b, int &e) {
        const int r0x = tile * kWgRows + wave * kTileRows;
        b = 0;
        e = 0;
        if (tile < n_tiles && r0x < n_vrows) {
            const int vx = r0x / S;
            b = rowptr[vx];
            e = rowend[vx];
        }
    };
    auto tile_words = [&](int tile, int b, int e, int cols, unsigned long long *w) {
        // in the load layout of gather_node_block_bits: lane = (neighbour slot lane / 16, state lane % 16)
        const int r0x = tile * kWgRows + wave * kTileRows;
        const bool ok = tile < n_tiles && r0x < n_vrows && e > b && e - b <= kHubDegree;   // wave-uniform
        const int s0x = ok ? r0x - (r0x / S) * S : 0;
        const int m = min(32, e - b);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int u = __shfl(cols, max(0, min(4 * k + (lane >> 4), m - 1)));
            w[k] = ok ? maskT[(size_t)u * S + s0x + (lane & 15)] : 0ull;
        }
    };
    if (PFW) {
        const int G = (int)gridDim.x;
        tile_range((int)blockIdx.x + G, q1_b, q1_e);
        tile_range((int)blockIdx.x + 2 * G, q2_b, q2_e);
        q1_cols = (lane < min(64, q1_e - q1_b)) ? colidx[q1_b + lane] : 0;
        tile_words((int)blockIdx.x, pf_b, pf_e, pf_cols, pw);
    }
    float mpn[PFM ? CB : 1][4];
    if (PFM) {
        const int r0 = blockIdx.x * kWgRows + wave * kTileRows;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int ro = r0 + 4 * gl + k;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                mpn[PFM ? cb : 0][k] = ((int)blockIdx.x < n_tiles && ro < n_vrows) ? mu_prev[(size_t)ro * P + 16 * cb + jl] : 0.f;
        }
    }
    // ---- workgroup reductions, fixed order over the four waves: the accumulators go into this workgroup's
    // partial rows (compensated pair: row blockIdx.x and row kBwdGrid + blockIdx.x) and start again at zero ----
    int n_flushed = 0;
    auto flush = [&](bool first) {
        __syncthreads();
        // dtheta2: in 16-row slabs of the p x p matrix (one ib at a time) to bound LDS use
#pragma unroll
        for (int ib = 0; ib < CB; ++ib) {
            float *slab = lds + wave * (16 * P);
#pragma unroll
            for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    slab[(4 * gl + rr) * P + 16 * jb + jl] = d2acc[ib][jb][rr];
                    d2acc[ib][jb][rr] = 0.f;
                }
            __syncthreads();
            for (int e = threadIdx.x; e < 16 * P; e += kThreads) {
                const float sum = (lds[e] + lds[16 * P + e]) + (lds[2 * 16 * P + e] + lds[3 * 16 * P + e]);
                const size_t at = (size_t)blockIdx.x * P * P + (size_t)ib * 16 * P + e;
                comp_add(d2_part + at, d2_part + (size_t)kBwdGrid * P * P + at, sum, first);
            }
            __syncthreads();
        }
        // sum x dz, sum s+ dz, sum s- dz: lanes with equal jl first, then waves
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            cx[cb] += __shfl_xor(cx[cb], 16); cx[cb] += __shfl_xor(cx[cb], 32);
            cp[cb] += __shfl_xor(cp[cb], 16); cp[cb] += __shfl_xor(cp[cb], 32);
            cn[cb] += __shfl_xor(cn[cb], 16); cn[cb] += __shfl_xor(cn[cb], 32);
        }
        if (gl == 0) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                lds[(wave * 3 + 0) * P + 16 * cb + jl] = cx[cb];
                lds[(wave * 3 + 1) * P + 16 * cb + jl] = cp[cb];
                lds[(wave * 3 + 2) * P + 16 * cb + jl] = cn[cb];
            }
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) cx[cb] = cp[cb] = cn[cb] = 0.f;
        if (FUSE) {
            // the fused round's sums: lanes with equal li, then into the same slots of this wave
            constexpr int LPR = Ge::LPR;
#pragma unroll
            for (int m = LPR; m < 64; m <<= 1) {
                fx4.x += __shfl_xor(fx4.x, m); fx4.y += __shfl_xor(fx4.y, m); fx4.z += __shfl_xor(fx4.z, m); fx4.w += __shfl_xor(fx4.w, m);
                fp4.x += __shfl_xor(fp4.x, m); fp4.y += __shfl_xor(fp4.y, m); fp4.z += __shfl_xor(fp4.z, m); fp4.w += __shfl_xor(fp4.w, m);
                fn4.x += __shfl_xor(fn4.x, m); fn4.y += __shfl_xor(fn4.y, m); fn4.z += __shfl_xor(fn4.z, m); fn4.w += __shfl_xor(fn4.w, m);
            }
            __builtin_amdgcn_wave_barrier();
            if (lane < LPR) {
                float *px = lds + (wave * 3 + 0) * P + 4 * lane, *pp = lds + (wave * 3 + 1) * P + 4 * lane;
                float *pn = lds + (wave * 3 + 2) * P + 4 * lane;
                st4(px, add4(ld4(px), fx4));
                st4(pp, add4(ld4(pp), fp4));
                st4(pn, add4(ld4(pn), fn4));
            }
            if (FLAGS) {
                __builtin_amdgcn_wave_barrier();
                if (lane < P) {
                    lds[(wave * 3 + 0) * P + lane] += fxj;
                    lds[(wave * 3 + 1) * P + lane] += fpj;
                }
            }
            fx4 = fp4 = fn4 = make_float4(0.f, 0.f, 0.f, 0.f);
            fxj = fpj = 0.f;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < 3 * P; e += kThreads) {
            const float sum = (lds[e] + lds[3 * P + e]) + (lds[2 * 3 * P + e] + lds[3 * 3 * P + e]);
            const size_t at = (size_t)blockIdx.x * 3 * P + e;
            comp_add(dc_part + at, dc_part + (size_t)kBwdGrid * 3 * P + at, sum, first);
        }
        __syncthreads();   // the tile area is free again
        ++n_flushed;
    };

    int it = 0;
    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x, ++it) {
        // (every wave of the workgroup makes the same number of iterations: the barriers inside are safe)
        if (it > 0 && it % kBwdFlushTiles == 0) flush(n_flushed == 0);
        int r0 = t * kWgRows + wave * kTileRows, r_step = 1, n_here = n_vrows - r0;
        if (sliced) {
            const int st = t / tps;
            const int v0 = (t - st * tps) * kWgRows + wave * kTileRows;
            r0 = v0 * S + st;
            r_step = S;
            n_here = n_nodes - v0;
        }
        const int r = r0 + jl * r_step;
        const bool valid = jl < n_here;
        const int v = valid ? r / S : 0;
        const int s = valid ? r - v * S : 0;
        const int rb = NODE ? pf_b : (valid ? rowptr[v] : 0);
        const int re = NODE ? pf_e : (valid ? rowend[v] : 0);
        const int cols_first = pf_cols;
        int nx_b = 0, nx_e = 0;
        bool nx_ok = false;
        unsigned long long nw[PFW ? 8 : 1];
        int q2_cols = 0, q3_b = 0, q3_e = 0;
        if (PFW) {
            // everything the tiles behind this one need next, issued before this tile's work
            const int G = (int)gridDim.x;
            const int r0n = (t + G) * kWgRows + wave * kTileRows;
            nx_ok = t + G < n_tiles && r0n < n_vrows;
            nx_b = q1_b;
            nx_e = q1_e;
            tile_words(t + G, q1_b, q1_e, q1_cols, nw);
            q2_cols = (lane < min(64, q2_e - q2_b)) ? colidx[q2_b + lane] : 0;
            tile_range(t + 3 * G, q3_b, q3_e);
        } else if (NODE) {
            const int tn = t + gridDim.x, r0n = tn * kWgRows + wave * kTileRows;
            nx_ok = tn < n_tiles && r0n < n_vrows;
            if (nx_ok) {
                const int vn = r0n / S;
                nx_b = rowptr[vn];
                nx_e = rowend[vn];
            }
        }
        const float3 mine = valid ? ni.get(v, s) : make_float3(0.f, 0.f, 0.f);
        const float xs = mine.x, sp = mine.y, sn = mine.z;
        // MASK: rows outside the action's graph receive nothing from the broadcast part of dz^T
        const bool in_graph = MASK ? (valid && in_range(v, s)) : true;

        // mu^{t-1} in the layout of the matrix-core result (row 4*gl + k, column 16*cb + jl): it is the
        // relu mask of this tile's output AND the B operand of the dtheta2 update.  Rows past the end: 0.
        float mp[CB][4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int ro = r0 + (4 * gl + k) * r_step;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                if (PFM) mp[cb][k] = mpn[PFM ? cb : 0][k];
                else mp[cb][k] = 4 * gl + k < n_here ? mu_prev[(size_t)ro * P + 16 * cb + jl] : 0.f;
            }
        }
        if (PFM) {
            const int r0n = (t + (int)gridDim.x) * kWgRows + wave * kTileRows;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ro = r0n + 4 * gl + k;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    mpn[PFM ? cb : 0][k] = (nx_ok && ro < n_vrows) ? mu_prev[(size_t)ro * P + 16 * cb + jl] : 0.f;
            }
        }

        if (NODE) {
            const int b = __builtin_amdgcn_readfirstlane(rb), e = __builtin_amdgcn_readfirstlane(re);
            const int s0 = __builtin_amdgcn_readfirstlane(s);
            NodeAcc<P> ga;
            if (e - b > kHubDegree) {
                const int h = hub_index(ht, __builtin_amdgcn_readfirstlane(v));
                ga = load_node_block<P>(hub_sum + ((size_t)h * S + s0) * P, lane);
            } else if (MASK) {
                ga = W ? gather_node_block_bits_w<P>(maskT, S, s0, colidx, wagg, b, e, lane)
                       : gather_node_block_bits<P>(maskT, S, s0, colidx, b, e, lane,
                                                   bits_stage + (NODE && MASK ? wave * (kBitsStageBytes / 4) : 0),
                                                   cols_first, true, PFW ? pw : nullptr);
            } else {
                ga = gather_node_block<P, W>(dz_in, row_stride, (size_t)s0 * P, colidx, wagg, b, e, lane);
            }
            if (PFW) {
                pf_b = q1_b; pf_e = q1_e; pf_cols = q1_cols;
#pragma unroll
                for (int k = 0; k < 8; ++k) pw[PFW ? k : 0] = nw[PFW ? k : 0];
                q1_b = q2_b; q1_e = q2_e; q1_cols = q2_cols;
                q2_b = q3_b; q2_e = q3_e;
            } else {
                // the next tile's first column indices (its row range has arrived by now)
                pf_cols = (nx_ok && lane < min(64, nx_e - nx_b)) ? colidx[nx_b + lane] : 0;
                pf_b = nx_b;
                pf_e = nx_e;
            }
            if (MASK) {
                // counts -> G: times dg of this lane's state and columns (the node is wave-uniform)
                constexpr int RPI = Ge::NPL, NC = 16 / RPI;
                const int vn = __builtin_amdgcn_readfirstlane(v);
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int sl = s0 + c * RPI + lane / Ge::LPR;      // this lane's state for block c
                    const bool ing = in_range(vn, sl);
                    const float4 d = dg_at(sl, 4 * li);
                    ga.a[c].x = ing ? ga.a[c].x * d.x : 0.f;
                    ga.a[c].y = ing ? ga.a[c].y * d.y : 0.f;
                    ga.a[c].z = ing ? ga.a[c].z * d.z : 0.f;
                    ga.a[c].w = ing ? ga.a[c].w * d.w : 0.f;
                }
            }
            store_node_block<P>(tile_g, ga, lane);
        } else if constexpr (MASK) {
            // row mode of the mask round: the long rows' sums are ready; the others by one lane per stored entry
            if (__builtin_amdgcn_ballot_w64(re - rb > kHubDegree) != 0ull) {
#pragma unroll 1
                for (int i = 0; i < kTileRows; ++i) {
                    if (__builtin_amdgcn_readlane(re, i) - __builtin_amdgcn_readlane(rb, i) <= kHubDegree) continue;
                    const int si = __builtin_amdgcn_readlane(s, i);
                    const int h = hub_index(ht, __builtin_amdgcn_readlane(v, i));
                    const bool ing = __builtin_amdgcn_readlane((int)in_graph, i) != 0;
                    float4 a = ld4(hub_sum + ((size_t)h * S + si) * P + 4 * li);
                    const float4 d = dg_at(si, 4 * li);
                    a.x = ing ? a.x * d.x : 0.f;
                    a.y = ing ? a.y * d.y : 0.f;
                    a.z = ing ? a.z * d.z : 0.f;
                    a.w = ing ? a.w * d.w : 0.f;
                    if (lane < Ge::LPR) st4(tile_g + i * STRIDE + 4 * lane, a);
                }
            }
            auto dg_col = [&](int st, int col) { return dg_lds ? s_dg[MASK ? st * P + col : 0] : dg[(size_t)st * P + col]; };
            gather_tile_bits_rows<P, W>(tile_g, maskT, S, s, in_graph, dg_col, colidx, wagg, rb, re, kHubDegree, lane);
        } else {
            // row mode, rows of dz^t in memory: the rows two at a time; two short rows share one trip to memory
            auto first_cols = [&](int b, int e) {
                return (e - b <= kHubDegree && lane < min(64, e - b)) ? colidx[b + lane] : 0;
            };
            int nb0 = __builtin_amdgcn_readlane(rb, 0), ne0 = __builtin_amdgcn_readlane(re, 0);
            int nb1 = __builtin_amdgcn_readlane(rb, 1), ne1 = __builtin_amdgcn_readlane(re, 1);
            int nc0 = first_cols(nb0, ne0), nc1 = first_cols(nb1, ne1);
#pragma unroll 1
            for (int i = 0; i < kTileRows; i += 2) {
                const int b0 = nb0, e0 = ne0, c0 = nc0, b1 = nb1, e1 = ne1, c1 = nc1;
                if (i + 2 < kTileRows) {
                    nb0 = __builtin_amdgcn_readlane(rb, i + 2); ne0 = __builtin_amdgcn_readlane(re, i + 2);
                    nb1 = __builtin_amdgcn_readlane(rb, i + 3); ne1 = __builtin_amdgcn_readlane(re, i + 3);
                    nc0 = first_cols(nb0, ne0);
                    nc1 = first_cols(nb1, ne1);
                }
                const int s0 = __builtin_amdgcn_readlane(s, i), s1 = __builtin_amdgcn_readlane(s, i + 1);
                const MemRow mem0{dz_in, row_stride, (size_t)s0 * P + 4 * li}, mem1{dz_in, row_stride, (size_t)s1 * P + 4 * li};
                float4 a0, a1;
                if (e0 - b0 <= 4 * Ge::NPL && e1 - b1 <= 4 * Ge::NPL) {
                    gather_row_sum_pair<P, W>(mem0, mem1, wagg, b0, e0, c0, b1, e1, c1, lane, a0, a1);
                } else {
                    if (e0 - b0 > kHubDegree) a0 = ld4(hub_sum + ((size_t)hub_index(ht, __builtin_amdgcn_readlane(v, i)) * S + s0) * P + 4 * li);
                    else a0 = gather_row_sum<P, W>(mem0, colidx, wagg, b0, e0, c0, lane);
                    if (e1 - b1 > kHubDegree) a1 = ld4(hub_sum + ((size_t)hub_index(ht, __builtin_amdgcn_readlane(v, i + 1)) * S + s1) * P + 4 * li);
                    else a1 = gather_row_sum<P, W>(mem1, colidx, wagg, b1, e1, c1, lane);
                }
                if (lane < Ge::LPR) {
                    st4(tile_g + i * STRIDE + 4 * lane, a0);
                    st4(tile_g + (i + 1) * STRIDE + 4 * lane, a1);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();

        // dmu^{t-1} = G theta2, masked by mu^{t-1} > 0
        const Frag<P> afrag = load_a_frag_lds<P>(tile_g, lane);
        f32x4 acc[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            acc[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
            acc[cb] = mfma_tile<P>(afrag, load_b_frag_lds<P>(lds_b, cb, lane), acc[cb]);
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int i = 4 * gl + rr;
            const float xi = __shfl(xs, i), spi = __shfl(sp, i), sni = __shfl(sn, i);
            const int ro = r0 + i * r_step;
            if (i < n_here) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const float d = mp[cb][rr] > 0.f ? acc[cb][rr] : 0.f;
                    if (dz_out) dz_out[(size_t)ro * P + 16 * cb + jl] = d;
                    cx[cb] += xi * d; cp[cb] += spi * d; cn[cb] += sni * d;
                    if (FUSE) acc[cb][rr] = d;
                }
            } else if (FUSE) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) acc[cb][rr] = 0.f;
            }
        }

        // dtheta2[i][j] += sum_r G[r][i] mu^{t-1}[r][j]: 16x16 blocks, k runs over the 16 tile rows
        // (lane group gl takes row 4*gl + ks at k-step ks); rows past the end are zero in both operands.
#pragma unroll
        for (int ib = 0; ib < CB; ++ib) {
            float a2[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) a2[ks] = tile_g[(4 * gl + ks) * STRIDE + 16 * ib + jl];
#pragma unroll
            for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    d2acc[ib][jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[ks], mp[jb][ks], d2acc[ib][jb], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();

        if (FUSE && r0 < n_vrows) {
            // ---- the round after this one, for the same node (scalar form, see k_bwd_first) ----
            constexpr int LPR = Ge::LPR, NC = 16 / Ge::NPL;
            float *tile_a = lds_a + (FUSE ? wave * TILE_F : 0);
            const int vf = r0 / S, s0f = r0 - vf * S;
            const int bf = __builtin_amdgcn_readfirstlane(rb), ef = __builtin_amdgcn_readfirstlane(re);
            // this tile's dz^{t-1} (masked, rows 4 * gl + rr, columns 16 * cb + jl) becomes the tile
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) tile_g[(4 * gl + rr) * STRIDE + 16 * cb + jl] = acc[cb][rr];
            NodeAcc4<P> g4;
            float cx16[FLAGS ? 16 : 1], cp16[FLAGS ? 16 : 1];
            if constexpr (FLAGS) {
                if (ef - bf > kHubDegree) {
                    // the long row's four sums, plain [4][S][P] blocks: a into the tile, cx and cp by column
                    const int h = hub_index(ht, vf);
                    const float *hb = ff.hub_sum4 + ((size_t)h * 4 * S + s0f) * P + (lane % P);
#pragma unroll
                    for (int st = 0; st < 16; ++st) {
                        if (lane < P) tile_a[st * STRIDE + lane] = hb[(size_t)st * P];
                        cx16[st] = hb[((size_t)S + st) * P];
                        cp16[st] = hb[(2 * (size_t)S + st) * P];
                    }
                } else {
                    gather_node_tile_flags_grad<P, W>(tile_a, cx16, cp16, ni, s0f, t1j, qpj, colidx, bf, ef, lane,
                                                      ni.node(vf)[ni.sn_off + 1], wagg);
                }
            } else if (ef - bf > kHubDegree) {
                const int h = hub_index(ht, vf);
                const float *hb = ff.hub_sum4 + ((size_t)h * 4 * S + s0f) * P;
                g4.a = load_node_block_sm<P>(hb, lane);
                g4.cx = load_node_block_sm<P>(hb + (size_t)S * P, lane);
                g4.cp = load_node_block_sm<P>(hb + 2 * (size_t)S * P, lane);
                g4.cn = load_node_block_sm<P>(hb + 3 * (size_t)S * P, lane);
            } else {
                g4 = gather_node_block_mu1_grad<P, W, NEG>(ni, s0f, ff.theta1, ff.qvec, colidx, wagg, bf, ef, lane,
                                                           rec_stage + ((FUSE && !FLAGS) ? wave * kRecStageFloats : 0));
            }
            if constexpr (!FLAGS) store_node_block_sm<P>(tile_a, g4.a, lane);
            __builtin_amdgcn_wave_barrier();
            // e = dz^{t-1} theta2 ; dtheta2 += dz^{t-1}^T a
            const Frag<P> ffrag = load_a_frag_lds<P>(tile_g, lane);
            f32x4 eacc[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                eacc[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
                eacc[cb] = mfma_tile<P>(ffrag, load_b_frag_lds<P>(lds_b, cb, lane), eacc[cb]);
            }
            float ya[CB][4];
#pragma unroll
            for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) ya[jb][ks] = tile_a[(4 * gl + ks) * STRIDE + 16 * jb + jl];
#pragma unroll
            for (int ib = 0; ib < CB; ++ib) {
                float a2[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) a2[ks] = tile_g[(4 * gl + ks) * STRIDE + 16 * ib + jl];
#pragma unroll
                for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        d2acc[ib][jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[ks], ya[jb][ks], d2acc[ib][jb], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) tile_g[(4 * gl + rr) * STRIDE + 16 * cb + jl] = eacc[cb][rr];
            __builtin_amdgcn_wave_barrier();
            if constexpr (FLAGS) {
                if (lane < P) {
#pragma unroll
                    for (int st = 0; st < 16; ++st) {
                        const float ev = tile_g[st * STRIDE + lane];
                        fxj = fmaf(ev, cx16[st], fxj);
                        fpj = fmaf(ev, cp16[st], fpj);
                    }
                }
            } else
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 e4 = ld4(tile_g + (NC * (lane / LPR) + c) * STRIDE + 4 * li);
                fx4.x = fmaf(e4.x, g4.cx.a[c].x, fx4.x); fx4.y = fmaf(e4.y, g4.cx.a[c].y, fx4.y);
                fx4.z = fmaf(e4.z, g4.cx.a[c].z, fx4.z); fx4.w = fmaf(e4.w, g4.cx.a[c].w, fx4.w);
                fp4.x = fmaf(e4.x, g4.cp.a[c].x, fp4.x); fp4.y = fmaf(e4.y, g4.cp.a[c].y, fp4.y);
                fp4.z = fmaf(e4.z, g4.cp.a[c].z, fp4.z); fp4.w = fmaf(e4.w, g4.cp.a[c].w, fp4.w);
                if (NEG) {
                    fn4.x = fmaf(e4.x, g4.cn.a[c].x, fn4.x); fn4.y = fmaf(e4.y, g4.cn.a[c].y, fn4.y);
                    fn4.z = fmaf(e4.z, g4.cn.a[c].z, fn4.z); fn4.w = fmaf(e4.w, g4.cn.a[c].w, fn4.w);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }

    flush(n_flushed == 0);
}

hipError_t launch_bwd_round(hipStream_t st, int p, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                            const int32_t *colidx, const float *wagg, const float *dz_in,
                            const unsigned long long *maskT, const BwdScratch &sc,
                            const float *mu_prev, float *dz_out, const NodeInfo &ni, const float *theta2,
                            float *dc_part, float *d2_part, const HubTable &ht, const float *hub_sum,
                            const BwdFuse *fuse, bool by_state) {
    const long n_vrows = (long)N * S;
    const int bs = (by_state && S % 16 != 0 && S > 1 && !maskT) ? 1 : 0;
    const bool node = (S % 16) == 0, mask = maskT != nullptr;
    const bool do_fuse = fuse != nullptr && node && !mask;
    const bool neg = do_fuse && fuse->has_neg;
    FirstFuse ff{nullptr, nullptr, nullptr};
    if (do_fuse) ff = FirstFuse{fuse->theta1, fuse->qvec, fuse->hub_sum4};
#define S2V_LAUNCH_BWD_F(PP, NODE, MASK, WW, FF, NN)                                                                   \
    k_bwd_round<PP, NODE, MASK, WW, FF, NN><<<kBwdGrid, kThreads, 0, st>>>((int)n_vrows, S, rowptr, rowend, colidx, wagg, \
                                                                           dz_in, maskT, sc.dg, sc.glo, sc.ghi, mu_prev,  \
                                                                           dz_out, ni, theta2, dc_part, d2_part, ht,       \
                                                                           hub_sum, ff, bs)
#define S2V_LAUNCH_BWD_W(PP, NODE, MASK, WW)                                                   \
    do {                                                                                       \
        if (NODE && !MASK && do_fuse) {                                                        \
            if (neg) S2V_LAUNCH_BWD_F(PP, NODE, MASK, WW, (NODE && !MASK), true);              \
            else if (ni.flags16)                                                               \
                k_bwd_round<PP, NODE, MASK, WW, (NODE && !MASK), false, (NODE && !MASK)>           \
                    <<<kBwdGrid, kThreads, 0, st>>>((int)n_vrows, S, rowptr, rowend, colidx, wagg, dz_in, maskT, sc.dg,   \
                                                    sc.glo, sc.ghi, mu_prev, dz_out, ni, theta2, dc_part, d2_part, ht,    \
                                                    hub_sum, ff, bs);                                                     \
            else S2V_LAUNCH_BWD_F(PP, NODE, MASK, WW, (NODE && !MASK), false);                 \
        } else S2V_LAUNCH_BWD_F(PP, NODE, MASK, WW, false, false);                             \
    } while (0)
#define S2V_LAUNCH_BWD(PP, NODE, MASK)                    \
    do {                                                  \
        if (wagg) S2V_LAUNCH_BWD_W(PP, NODE, MASK, true);     \
        else S2V_LAUNCH_BWD_W(PP, NODE, MASK, false);         \
    } while (0)
#define S2V_LAUNCH_BWD_P(PP)                                                                          \
    do {                                                                                              \
        if (node) { if (mask) S2V_LAUNCH_BWD(PP, true, true); else S2V_LAUNCH_BWD(PP, true, false); }  \
        else { if (mask) S2V_LAUNCH_BWD(PP, false, true); else S2V_LAUNCH_BWD(PP, false, false); }     \
    } while (0)
    if (p == 32) S2V_LAUNCH_BWD_P(32); else S2V_LAUNCH_BWD_P(64);
#undef S2V_LAUNCH_BWD_P
#undef S2V_LAUNCH_BWD
#undef S2V_LAUNCH_BWD_W
#undef S2V_LAUNCH_BWD_F
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// The last reversed round (t = 2), taken from the scalars instead of gathering dz^2.
// What the round must deliver is only sums over the nodes (dz^1 is never needed as a matrix):
//   dtheta2[i][j] += sum_u G_u[i] mu^1_u[j],   sum_u x_u dz^1_u,  sum_u s+-_u dz^1_u,
//   with G = A dz^2 and dz^1_u = (theta2^T G_u) (.) [mu^1_u > 0].
// Moving the (symmetric) adjacency to the other factor,
//   sum_u G_u[i] mu^1_u[j]      = sum_v dz^2_v[i] a_v[j],         a_v  = sum_{u in N(v)} mu^1_u,
//   sum_u x_u dz^1_u[j]         = sum_v e_v[j] cx_v[j],           e_v  = theta2^T dz^2_v,
//                                                                 cx_v = sum_{u in N(v)} x_u [mu^1_u > 0],
// (likewise with s+ and s-), and mu^1_u is a function of the three scalars of u.  So the kernel
// STREAMS dz^2 once and gathers the neighbours' scalars (80 bytes per neighbour at S = 16, see
// gather_node_block_mu1_grad) where the generic round gathers 4 KB rows of dz^2 and reads mu^1.
// Used for T >= 3 only: when t = 2 is also the first reversed round (T = 2), dz^2 = dz^T is not in
// memory and the mask-word round is cheaper than recomputing masks from the scalars.
// NODE (S a multiple of 16): a wave owns one node's 16-state block at a time.  Otherwise (row mode, any S) a
// tile is 16 consecutive rows (node, state): e = dz^2 theta2 is formed first and kept as a tile, then
// gather_tile_mu1_grad_rows walks the sixteen rows' entries (one lane per stored entry) and each row's cx, cp,
// cn meet its row of e at once; the sums are held per column (lane % P).  hub_sum4 holds the four sums of
// the long rows as [hub][4][S][P] in both modes.
// ------------------------------------------------------------------------------------------
// FLAGS: the four sums come from flag words and the rows' totals (gather_node_tile_flags_grad) instead of the
// neighbours' records; they are then held per column (lane % P), not in the state-major layout.
template <int P, bool W, bool NEG, bool FLAGS = false, bool NODE = true>
__global__ __launch_bounds__(kThreads, 2) void k_bwd_first(
    int n_vrows, int S, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ rowend,
    const int32_t *__restrict__ colidx, const float *__restrict__ wagg, const float *__restrict__ dz_in,
    NodeInfo ni, const float *__restrict__ theta1, const float *__restrict__ theta2,
    const float *__restrict__ qvec, float *__restrict__ dc_part, float *__restrict__ d2_part, HubTable ht,
    const float *__restrict__ hub_sum4) {
    using Ge = Geo<P>;
    constexpr int CB = Ge::CB, STRIDE = Ge::STRIDE, LPR = Ge::LPR, RPI = Ge::NPL, NC = 16 / RPI;
    constexpr int TILE_F = kTileRows * STRIDE;
    static_assert(2 * kWaves * TILE_F >= kWaves * 16 * P, "tile area is reused for the final reductions");
    static_assert(!FLAGS || !NEG, "flag words: no negative weight");
    static_assert(!FLAGS || NODE, "flag words: node mode");
    constexpr int NT = NODE ? 2 : 3;
    __shared__ __attribute__((aligned(16))) float lds[NT * kWaves * TILE_F];   // per wave: dz^2 tile, a tile (row mode: and the e tile)
    __shared__ __attribute__((aligned(16))) float lds_b[P * STRIDE];          // theta2^T: B operand of dz theta2
    __shared__ __attribute__((aligned(16))) float rec_stage[(FLAGS || !NODE) ? 4 : kWaves * kRecStageFloats];   // staging of the record gather
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *tile_d = lds + wave * NT * TILE_F, *tile_a = tile_d + TILE_F;
    const int li = lane % LPR;
    const int jl = lane & 15, gl = lane >> 4;

    stage_matrix_lds<P>(lds_b, theta2, true);
    __syncthreads();

    f32x4 d2acc[CB][CB];
#pragma unroll
    for (int ib = 0; ib < CB; ++ib)
#pragma unroll
        for (int jb = 0; jb < CB; ++jb) d2acc[ib][jb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float4 cx4 = make_float4(0.f, 0.f, 0.f, 0.f), cp4 = cx4, cn4 = cx4;
    // FLAGS and row mode: sums and constants of column lane % P
    float fxj = 0.f, fpj = 0.f, fnj = 0.f, t1j = 0.f, qpj = 0.f, qnj = 0.f;
    if (FLAGS || !NODE) {
        t1j = theta1[lane % P];
        qpj = qvec[lane % P];
        qnj = qvec[P + lane % P];
    }

    const int n_tiles = (n_vrows + kWgRows - 1) / kWgRows;
    // ---- workgroup reductions, fixed order over the four waves, into this workgroup's compensated pair of
    // partial rows (see k_bwd_round); the accumulators start again at zero ----
    int n_flushed = 0;
    auto flush = [&](bool first) {
        __syncthreads();
#pragma unroll
        for (int ib = 0; ib < CB; ++ib) {
            float *slab = lds + wave * (16 * P);
#pragma unroll
            for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    slab[(4 * gl + rr) * P + 16 * jb + jl] = d2acc[ib][jb][rr];
                    d2acc[ib][jb][rr] = 0.f;
                }
            __syncthreads();
            for (int el = threadIdx.x; el < 16 * P; el += kThreads) {
                const float sum = (lds[el] + lds[16 * P + el]) + (lds[2 * 16 * P + el] + lds[3 * 16 * P + el]);
                const size_t at = (size_t)blockIdx.x * P * P + (size_t)ib * 16 * P + el;
                comp_add(d2_part + at, d2_part + (size_t)kBwdGrid * P * P + at, sum, first);
            }
            __syncthreads();
        }
        // the three column sums: lanes with equal li first, then the waves
#pragma unroll
        for (int m = LPR; m < 64; m <<= 1) {
            cx4.x += __shfl_xor(cx4.x, m); cx4.y += __shfl_xor(cx4.y, m); cx4.z += __shfl_xor(cx4.z, m); cx4.w += __shfl_xor(cx4.w, m);
            cp4.x += __shfl_xor(cp4.x, m); cp4.y += __shfl_xor(cp4.y, m); cp4.z += __shfl_xor(cp4.z, m); cp4.w += __shfl_xor(cp4.w, m);
            cn4.x += __shfl_xor(cn4.x, m); cn4.y += __shfl_xor(cn4.y, m); cn4.z += __shfl_xor(cn4.z, m); cn4.w += __shfl_xor(cn4.w, m);
        }
        if (FLAGS || !NODE) {
            if (lane < P) {
                lds[(wave * 3 + 0) * P + lane] = fxj;
                lds[(wave * 3 + 1) * P + lane] = fpj;
                lds[(wave * 3 + 2) * P + lane] = fnj;
            }
        } else if (lane < LPR) {
            st4(lds + (wave * 3 + 0) * P + 4 * lane, cx4);
            st4(lds + (wave * 3 + 1) * P + 4 * lane, cp4);
            st4(lds + (wave * 3 + 2) * P + 4 * lane, cn4);
        }
        cx4 = cp4 = cn4 = make_float4(0.f, 0.f, 0.f, 0.f);
        fxj = fpj = fnj = 0.f;
        __syncthreads();
        for (int el = threadIdx.x; el < 3 * P; el += kThreads) {
            const float sum = (lds[el] + lds[3 * P + el]) + (lds[2 * 3 * P + el] + lds[3 * 3 * P + el]);
            const size_t at = (size_t)blockIdx.x * 3 * P + el;
            comp_add(dc_part + at, dc_part + (size_t)kBwdGrid * 3 * P + at, sum, first);
        }
        __syncthreads();   // the tile area is free again
        ++n_flushed;
    };

    int it = 0;
    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x, ++it) {
        // (every wave of the workgroup makes the same number of iterations: the barriers inside are safe)
        if (it > 0 && it % kBwdFlushTiles == 0) flush(n_flushed == 0);
        const int r0 = t * kWgRows + wave * kTileRows;
        if (r0 >= n_vrows) continue;        // (node mode: S is a multiple of 16, tiles are whole)
        if constexpr (!NODE) {
            // ---- row mode: 16 consecutive rows (v, s) of the [N * S][p] matrices, any S ----
            float *tile_e = tile_a + TILE_F;
            const int r = r0 + jl;
            const bool valid = r < n_vrows;
            const int v = valid ? r / S : 0;
            const int s = valid ? r - v * S : 0;
            const int rb = valid ? rowptr[v] : 0, re = valid ? rowend[v] : 0;
            // the tile's rows of dz^2 (rows past the end are zero)
            for (int f = lane; f < kTileRows * LPR; f += 64) {
                const int row = f / LPR, c4 = f - row * LPR;
                const float4 d = r0 + row < n_vrows ? ld4(dz_in + (size_t)(r0 + row) * P + 4 * c4)
                                                    : make_float4(0.f, 0.f, 0.f, 0.f);
                st4(tile_d + row * STRIDE + 4 * c4, d);
            }
            __builtin_amdgcn_wave_barrier();
            {
                // e = dz^2 theta2, kept as a tile: each row meets its gathered sums below
                const Frag<P> afrag = load_a_frag_lds<P>(tile_d, lane);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                    acc = mfma_tile<P>(afrag, load_b_frag_lds<P>(lds_b, cb, lane), acc);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) tile_e[(4 * gl + rr) * STRIDE + 16 * cb + jl] = acc[rr];
                }
            }
            __builtin_amdgcn_wave_barrier();
            // the long rows of the tile: their four sums are ready, [hub][4][S][P]
            if (__builtin_amdgcn_ballot_w64(re - rb > kHubDegree) != 0ull) {
#pragma unroll 1
                for (int i = 0; i < kTileRows; ++i) {
                    if (__builtin_amdgcn_readlane(re, i) - __builtin_amdgcn_readlane(rb, i) <= kHubDegree) continue;
                    const int si = __builtin_amdgcn_readlane(s, i), vi = __builtin_amdgcn_readlane(v, i);
                    const float *hb = hub_sum4 + ((size_t)hub_index(ht, vi) * 4 * S + si) * P + (lane % P);
                    const float ev = tile_e[i * STRIDE + lane % P];
                    if (lane < P) tile_a[i * STRIDE + lane] = hb[0];
                    fxj = fmaf(ev, hb[(size_t)S * P], fxj);
                    fpj = fmaf(ev, hb[2 * (size_t)S * P], fpj);
                    if (NEG) fnj = fmaf(ev, hb[3 * (size_t)S * P], fnj);
                }
            }
            gather_tile_mu1_grad_rows<P, W, NEG>(tile_a, tile_e, ni, s, t1j, qpj, qnj, colidx, wagg, rb, re, kHubDegree,
                                                 lane, fxj, fpj, fnj);
            __builtin_amdgcn_wave_barrier();
            // dtheta2[i][j] += sum_r dz^2[r][i] a[r][j], as in node mode
            float ya[CB][4];
#pragma unroll
            for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) ya[jb][ks] = tile_a[(4 * gl + ks) * STRIDE + 16 * jb + jl];
#pragma unroll
            for (int ib = 0; ib < CB; ++ib) {
                float a2[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) a2[ks] = tile_d[(4 * gl + ks) * STRIDE + 16 * ib + jl];
#pragma unroll
                for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        d2acc[ib][jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[ks], ya[jb][ks], d2acc[ib][jb], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
        } else {
        const int v = r0 / S, s0 = r0 - v * S;
        const int b = rowptr[v], e = rowend[v];

        // this node's 16 rows of dz^2, lane (row c * RPI + lane / LPR, columns 4 * li ..)
        const NodeAcc<P> dz = load_node_block<P>(dz_in + (size_t)r0 * P, lane);
        store_node_block<P>(tile_d, dz, lane);

        NodeAcc4<P> g4;
        float cx16[FLAGS ? 16 : 1], cp16[FLAGS ? 16 : 1];
        if constexpr (FLAGS) {
            if (e - b > kHubDegree) {
                const int h = hub_index(ht, v);
                const float *hb = hub_sum4 + ((size_t)h * 4 * S + s0) * P + (lane % P);
#pragma unroll
                for (int st = 0; st < 16; ++st) {
                    if (lane < P) tile_a[st * STRIDE + lane] = hb[(size_t)st * P];
                    cx16[st] = hb[((size_t)S + st) * P];
                    cp16[st] = hb[(2 * (size_t)S + st) * P];
                }
            } else {
                gather_node_tile_flags_grad<P, W>(tile_a, cx16, cp16, ni, s0, t1j, qpj, colidx, b, e, lane,
                                                  ni.node(v)[ni.sn_off + 1], wagg);
            }
        } else if (e - b > kHubDegree) {
            const int h = hub_index(ht, v);
            const float *hb = hub_sum4 + ((size_t)h * 4 * S + s0) * P;
            g4.a = load_node_block_sm<P>(hb, lane);
            g4.cx = load_node_block_sm<P>(hb + (size_t)S * P, lane);
            g4.cp = load_node_block_sm<P>(hb + 2 * (size_t)S * P, lane);
            g4.cn = load_node_block_sm<P>(hb + 3 * (size_t)S * P, lane);
        } else {
            g4 = gather_node_block_mu1_grad<P, W, NEG>(ni, s0, theta1, qvec, colidx, wagg, b, e, lane,
                                                       rec_stage + (FLAGS ? 0 : wave * kRecStageFloats));
        }
        if constexpr (!FLAGS) store_node_block_sm<P>(tile_a, g4.a, lane);   // the four sums live in the state-major lane layout
        __builtin_amdgcn_wave_barrier();

        // e = dz^2 theta2 (row r, column j: sum_k dz^2[r][k] theta2[k][j])
        const Frag<P> afrag = load_a_frag_lds<P>(tile_d, lane);
        f32x4 acc[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            acc[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
            acc[cb] = mfma_tile<P>(afrag, load_b_frag_lds<P>(lds_b, cb, lane), acc[cb]);
        }
        // dtheta2[i][j] += sum_r dz^2[r][i] a[r][j]: 16x16 blocks, k runs over the 16 tile rows
        float ya[CB][4];
#pragma unroll
        for (int jb = 0; jb < CB; ++jb)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) ya[jb][ks] = tile_a[(4 * gl + ks) * STRIDE + 16 * jb + jl];
#pragma unroll
        for (int ib = 0; ib < CB; ++ib) {
            float a2[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) a2[ks] = tile_d[(4 * gl + ks) * STRIDE + 16 * ib + jl];
#pragma unroll
            for (int jb = 0; jb < CB; ++jb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    d2acc[ib][jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[ks], ya[jb][ks], d2acc[ib][jb], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();
        // e back into the layout of the gathered sums, through the dz tile
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) tile_d[(4 * gl + rr) * STRIDE + 16 * cb + jl] = acc[cb][rr];
        __builtin_amdgcn_wave_barrier();
        if constexpr (FLAGS) {
            if (lane < P) {
#pragma unroll
                for (int st = 0; st < 16; ++st) {
                    const float ev = tile_d[st * STRIDE + lane];
                    fxj = fmaf(ev, cx16[st], fxj);
                    fpj = fmaf(ev, cp16[st], fpj);
                }
            }
        } else
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const float4 e4 = ld4(tile_d + (NC * (lane / LPR) + c) * STRIDE + 4 * li);
            cx4.x = fmaf(e4.x, g4.cx.a[c].x, cx4.x); cx4.y = fmaf(e4.y, g4.cx.a[c].y, cx4.y);
            cx4.z = fmaf(e4.z, g4.cx.a[c].z, cx4.z); cx4.w = fmaf(e4.w, g4.cx.a[c].w, cx4.w);
            cp4.x = fmaf(e4.x, g4.cp.a[c].x, cp4.x); cp4.y = fmaf(e4.y, g4.cp.a[c].y, cp4.y);
            cp4.z = fmaf(e4.z, g4.cp.a[c].z, cp4.z); cp4.w = fmaf(e4.w, g4.cp.a[c].w, cp4.w);
            if (NEG) {
                cn4.x = fmaf(e4.x, g4.cn.a[c].x, cn4.x); cn4.y = fmaf(e4.y, g4.cn.a[c].y, cn4.y);
                cn4.z = fmaf(e4.z, g4.cn.a[c].z, cn4.z); cn4.w = fmaf(e4.w, g4.cn.a[c].w, cn4.w);
            }
        }
        __builtin_amdgcn_wave_barrier();
        }
    }

    flush(n_flushed == 0);
}

hipError_t launch_bwd_first(hipStream_t st, int p, int N, int S, const int32_t *rowptr, const int32_t *rowend,
                            const int32_t *colidx, const float *wagg, const float *dz_in, const NodeInfo &ni,
                            bool has_neg, const float *theta1, const float *theta2, const float *qvec, float *dc_part,
                            float *d2_part, const HubTable &ht, const float *hub_sum4) {
    const long n_vrows = (long)N * S;
#define S2V_LAUNCH_FIRST(PP, WW, NN)                                                                              \
    k_bwd_first<PP, WW, NN><<<kBwdGrid, kThreads, 0, st>>>((int)n_vrows, S, rowptr, rowend, colidx, wagg, dz_in, ni,  \
                                                           theta1, theta2, qvec, dc_part, d2_part, ht, hub_sum4)
#define S2V_LAUNCH_FIRST_N(PP, WW)                                                                                   \
    do {                                                                                                             \
        if (has_neg) S2V_LAUNCH_FIRST(PP, WW, true);                                                                 \
        else if (ni.flags16)                                                                                         \
            k_bwd_first<PP, WW, false, true><<<kBwdGrid, kThreads, 0, st>>>((int)n_vrows, S, rowptr, rowend, colidx, wagg, \
                                                                            dz_in, ni, theta1, theta2, qvec, dc_part, \
                                                                            d2_part, ht, hub_sum4);                   \
        else S2V_LAUNCH_FIRST(PP, WW, false);                                                                        \
    } while (0)
#define S2V_LAUNCH_FIRST_ROWS(PP, WW, NN)                                                                            \
    k_bwd_first<PP, WW, NN, false, false><<<kBwdGrid, kThreads, 0, st>>>((int)n_vrows, S, rowptr, rowend, colidx, wagg, \
                                                                         dz_in, ni, theta1, theta2, qvec, dc_part,      \
                                                                         d2_part, ht, hub_sum4)
#define S2V_LAUNCH_FIRST_W(PP)                                                                   \
    do {                                                                                         \
        if (S % 16 != 0) {                                                                       \
            if (wagg) { if (has_neg) S2V_LAUNCH_FIRST_ROWS(PP, true, true); else S2V_LAUNCH_FIRST_ROWS(PP, true, false); } \
            else { if (has_neg) S2V_LAUNCH_FIRST_ROWS(PP, false, true); else S2V_LAUNCH_FIRST_ROWS(PP, false, false); }    \
        } else if (wagg) S2V_LAUNCH_FIRST_N(PP, true);                                           \
        else S2V_LAUNCH_FIRST_N(PP, false);                                                      \
    } while (0)
    if (p == 32) S2V_LAUNCH_FIRST_W(32); else S2V_LAUNCH_FIRST_W(64);
#undef S2V_LAUNCH_FIRST_ROWS
#undef S2V_LAUNCH_FIRST_W
#undef S2V_LAUNCH_FIRST_N
#undef S2V_LAUNCH_FIRST
    return hipGetLastError();
}

// The four sums of the long rows for k_bwd_first: one wave per (segment, 16-state block),
// then the segments of a row added in order (k_hub_combine with rows of 4 * S * p floats).
template <int P, bool W, bool NEG>
__global__ __launch_bounds__(kThreads) void k_hub_partial_grad(int S, HubTable ht, const int32_t *__restrict__ rowend,
                                                               const int32_t *__restrict__ colidx,
                                                               const float *__restrict__ wagg, NodeInfo ni,
                                                               const float *__restrict__ theta1,
                                                               const float *__restrict__ qvec,
                                                               float *__restrict__ partial) {
    __shared__ __attribute__((aligned(16))) float rec_stage[kWaves * kRecStageFloats];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bpn = S / 16;
    const long items = (long)ht.n_segs * bpn;
    for (long item = (long)blockIdx.x * kWaves + wave; item < items; item += (long)gridDim.x * kWaves) {
        const int seg = (int)(item / bpn), s0 = (int)(item - (long)seg * bpn) * 16;
        const int b = ht.seg_begin[seg], e = min(ht.seg_end[seg], rowend[ht.seg_row[seg]]);
        const NodeAcc4<P> g4 = gather_node_block_mu1_grad<P, W, NEG>(ni, s0, theta1, qvec, colidx, wagg, b, e, lane,
                                                                     rec_stage + wave * kRecStageFloats);
        float *out = partial + ((size_t)seg * 4 * S + s0) * P;
        write_node_block_sm<P>(out, g4.a, lane);
        write_node_block_sm<P>(out + (size_t)S * P, g4.cx, lane);
        write_node_block_sm<P>(out + 2 * (size_t)S * P, g4.cp, lane);
        write_node_block_sm<P>(out + 3 * (size_t)S * P, g4.cn, lane);   // zeros when the graph has no negative weight
    }
}

// Row mode (S not a multiple of 16): one wave per (segment, state).
template <int P, bool W, bool NEG>
__global__ __launch_bounds__(kThreads) void k_hub_partial_grad_rows(int S, HubTable ht,
                                                                    const int32_t *__restrict__ rowend,
                                                                    const int32_t *__restrict__ colidx,
                                                                    const float *__restrict__ wagg, NodeInfo ni,
                                                                    const float *__restrict__ theta1,
                                                                    const float *__restrict__ qvec,
                                                                    float *__restrict__ partial) {
    constexpr int LPR = Geo<P>::LPR;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane % LPR;
    const float4 t1 = ld4(theta1 + 4 * li), qp = ld4(qvec + 4 * li), qn = ld4(qvec + P + 4 * li);
    const long items = (long)ht.n_segs * S;
    for (long item = (long)blockIdx.x * kWaves + wave; item < items; item += (long)gridDim.x * kWaves) {
        const int seg = (int)(item / S), s = (int)(item - (long)seg * S);
        const int b = ht.seg_begin[seg], e = min(ht.seg_end[seg], rowend[ht.seg_row[seg]]);
        const RowAcc4 g = gather_row_mu1_grad<P, W, NEG>(ni, s, t1, qp, qn, colidx, wagg, b, e, 0, false, lane);
        if (lane < LPR) {
            float *out = partial + ((size_t)seg * 4 * S + s) * P + 4 * lane;
            st4(out, g.a);
            st4(out + (size_t)S * P, g.cx);
            st4(out + 2 * (size_t)S * P, g.cp);
            st4(out + 3 * (size_t)S * P, g.cn);   // zeros when the graph has no negative weight
        }
    }
}

hipError_t launch_hub_sums_grad(hipStream_t st, int p, int S, const HubTable &ht, const int32_t *rowend,
                                const int32_t *colidx, const float *wagg, const NodeInfo &ni, bool has_neg,
                                const float *theta1, const float *qvec, float *partial4, float *hub_sum4) {
    if (ht.n_hubs == 0) return hipSuccess;
    // (every long row a single segment: its sums are the row's sums, written in place; see launch_hub_sums)
    const bool single = ht.n_segs == ht.n_hubs;
    if (single) partial4 = hub_sum4;
    const bool rows = S % 16 != 0;
    const long items = rows ? (long)ht.n_segs * S : (long)ht.n_segs * (S / 16);
    const int grid = (int)min((items + kWaves - 1) / kWaves, (long)65536);
#define S2V_LAUNCH_HG(PP, WW, NN)                                                                                          \
    do {                                                                                                                   \
        if (rows)                                                                                                          \
            k_hub_partial_grad_rows<PP, WW, NN><<<grid, kThreads, 0, st>>>(S, ht, rowend, colidx, wagg, ni, theta1, qvec,  \
                                                                          partial4);                                      \
        else                                                                                                               \
            k_hub_partial_grad<PP, WW, NN><<<grid, kThreads, 0, st>>>(S, ht, rowend, colidx, wagg, ni, theta1, qvec,       \
                                                                     partial4);                                           \
    } while (0)
#define S2V_LAUNCH_HG_N(PP, WW) \
    do { if (has_neg) S2V_LAUNCH_HG(PP, WW, true); else S2V_LAUNCH_HG(PP, WW, false); } while (0)
#define S2V_LAUNCH_HG_W(PP) \
    do { if (wagg) S2V_LAUNCH_HG_N(PP, true); else S2V_LAUNCH_HG_N(PP, false); } while (0)
    if (p == 32) S2V_LAUNCH_HG_W(32); else S2V_LAUNCH_HG_W(64);
#undef S2V_LAUNCH_HG_W
#undef S2V_LAUNCH_HG_N
#undef S2V_LAUNCH_HG
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || single) return err;
    return launch_hub_combine(st, 4 * S * p, ht, partial4, hub_sum4);
}

// ------------------------------------------------------------------------------------------
// The action node's own term of dz^T, which the MASK round leaves out:
//   dz^T[a_s][s] += da[s] (.) [mu^T[a_s][s] > 0] =: g_s.
// The round is linear in dz^T, so its effect is added here.  Only the rows u in N(a_s) see it:
//   G_u += g_s  (w_au g_s with a weighted sum)  =>  dz^{T-1}_u += (theta2^T g_s) (.) [mu^{T-1}_u > 0],  dtheta2 += g_s (sum_u mu^{T-1}_u)^T,
// plus the matching share of the sum x dz, sum s+- dz partials.  Grid = (kFixSplit, S): block
// (k, s) takes the entries of row a_s congruent to k modulo kFixSplit; thread = (slot, column).
// ------------------------------------------------------------------------------------------
template <int P>
__global__ __launch_bounds__(256) void k_bwd_action_fix(int S, const int32_t *__restrict__ rowptr,
                                                        const int32_t *__restrict__ rowend,
                                                        const int32_t *__restrict__ colidx,
                                                        const float *__restrict__ wagg /*NULL: unweighted sum*/,
                                                        const int32_t *__restrict__ action,
                                                        const unsigned long long *__restrict__ maskT,
                                                        const float *__restrict__ da,
                                                        const float *__restrict__ theta2,
                                                        const float *__restrict__ mu_prev, float *__restrict__ dz_out,
                                                        NodeInfo ni, float *__restrict__ dc_part,
                                                        float *__restrict__ d2_part) {
    constexpr int SLOTS = 256 / P;
    __shared__ float g[P], w[P];
    __shared__ float red[4][SLOTS][P];
    const int s = blockIdx.y, split = blockIdx.x;
    const int j = threadIdx.x % P, slot = threadIdx.x / P;
    const int a = action[s];
    if (threadIdx.x < P) {
        const unsigned long long word = maskT[(size_t)a * S + s];
        g[threadIdx.x] = ((word >> threadIdx.x) & 1ull) ? da[(size_t)s * P + threadIdx.x] : 0.f;
    }
    __syncthreads();
    if (threadIdx.x < P) {
        float acc = 0.f;
        for (int k = 0; k < P; ++k) acc += theta2[k * P + threadIdx.x] * g[k];
        w[threadIdx.x] = acc;
    }
    __syncthreads();
    float cx = 0.f, cp = 0.f, cn = 0.f, msum = 0.f;
    const int b = rowptr[a], e = rowend[a];
    for (int idx = b + split + slot * kFixSplit; idx < e; idx += SLOTS * kFixSplit) {
        const int u = colidx[idx];
        const size_t off = ((size_t)u * S + s) * P + j;
        const float mprev = mu_prev[off];
        const float wa = wagg ? wagg[idx] : 1.f;     // G_u += w_au g_s with a weighted sum
        const float d = mprev > 0.f ? wa * w[j] : 0.f;
        if (dz_out) dz_out[off] += d;
        const float3 q = ni.get(u, s);
        cx += q.x * d;
        cp += q.y * d;
        cn += q.z * d;
        msum += wa * mprev;
    }
    red[0][slot][j] = cx; red[1][slot][j] = cp; red[2][slot][j] = cn; red[3][slot][j] = msum;
    __syncthreads();
    const size_t row = (size_t)s * kFixSplit + split;
    if (threadIdx.x < P) {
        float t[4];
        for (int c = 0; c < 4; ++c) {
            float acc = 0.f;
            for (int k = 0; k < SLOTS; ++k) acc += red[c][k][threadIdx.x];
            t[c] = acc;
        }
        dc_part[row * 3 * P + threadIdx.x] = t[0];
        dc_part[row * 3 * P + P + threadIdx.x] = t[1];
        dc_part[row * 3 * P + 2 * P + threadIdx.x] = t[2];
        red[3][0][threadIdx.x] = t[3];
    }
    __syncthreads();
    for (int el = threadIdx.x; el < P * P; el += 256) {
        const int i = el / P, jj = el - i * P;
        d2_part[row * P * P + el] = g[i] * red[3][0][jj];
    }
}

hipError_t launch_bwd_action_fix(hipStream_t st, int p, int S, const int32_t *rowptr, const int32_t *rowend,
                                 const int32_t *colidx, const float *wagg,
                                 const int32_t *action, const unsigned long long *maskT, const BwdScratch &sc,
                                 const float *theta2, const float *mu_prev, float *dz_out, const NodeInfo &ni,
                                 float *dc_part, float *d2_part) {
    const dim3 grid(kFixSplit, S);
    if (p == 32)
        k_bwd_action_fix<32><<<grid, 256, 0, st>>>(S, rowptr, rowend, colidx, wagg, action, maskT, sc.da, theta2, mu_prev,
                                                   dz_out, ni, dc_part, d2_part);
    else
        k_bwd_action_fix<64><<<grid, 256, 0, st>>>(S, rowptr, rowend, colidx, wagg, action, maskT, sc.da, theta2, mu_prev,
                                                   dz_out, ni, dc_part, d2_part);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Final reductions.  k_colsum adds `rows` rows of width `width` in segments of rows_per_seg rows
// (double accumulator per segment, float out); called twice it gives a fixed two-level tree.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_colsum(int rows, int width, int rows_per_seg, const float *__restrict__ in,
                                                float *__restrict__ out) {
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= width) return;
    const int r0 = blockIdx.y * rows_per_seg, r1 = min(rows, r0 + rows_per_seg);
    double a0 = 0.0, a1 = 0.0;
    int r = r0;
    for (; r + 2 <= r1; r += 2) {
        a0 += (double)in[(size_t)r * width + col];
        a1 += (double)in[(size_t)(r + 1) * width + col];
    }
    if (r < r1) a0 += (double)in[(size_t)r * width + col];
    out[(size_t)blockIdx.y * width + col] = (float)(a0 + a1);
}

__global__ __launch_bounds__(128) void k_bwd_finish_vec(int p, const float *__restrict__ dvec,
                                                        const float *__restrict__ theta3,
                                                        const float *__restrict__ theta4, float *__restrict__ d1,
                                                        float *__restrict__ d3, float *__restrict__ d4) {
    const int j = threadIdx.x;
    const float *dqp = dvec + p, *dqn = dvec + 2 * p;
    if (j < p) {
        d1[j] = dvec[j];
        const float t4 = theta4[j];
        float up = 0.f, un = 0.f;
        for (int i = 0; i < p; ++i) {
            up += theta3[i * p + j] * dqp[i];
            un += theta3[i * p + j] * dqn[i];
        }
        d4[j] = (t4 > 0.f ? up : 0.f) - (t4 < 0.f ? un : 0.f);
    }
    for (int e = j; e < p * p; e += 128) {
        const int r = e / p, c = e - r * p;
        const float t4 = theta4[c];
        d3[e] = dqp[r] * fmaxf(t4, 0.f) + dqn[r] * fmaxf(-t4, 0.f);
    }
}

static hipError_t colsum_two_level(hipStream_t st, int rows, int width, const float *in, float *tmp, float *out) {
    constexpr int kSeg = 64;
    const int segs = (rows + kSeg - 1) / kSeg;
    const dim3 g1((width + 255) / 256, segs > 0 ? segs : 1);
    if (segs <= 1) {
        k_colsum<<<g1, 256, 0, st>>>(rows, width, kSeg, in, out);
        return hipGetLastError();
    }
    k_colsum<<<g1, 256, 0, st>>>(rows, width, kSeg, in, tmp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 g2((width + 255) / 256, 1);
    k_colsum<<<g2, 256, 0, st>>>(segs, width, segs, tmp, out);
    return hipGetLastError();
}

hipError_t launch_bwd_finish(hipStream_t st, int p, int dc_rows, int d2_rows, const BwdScratch &sc, const float *theta3,
                             const float *theta4, float *d1, float *d2, float *d3, float *d4) {
    hipError_t e = colsum_two_level(st, dc_rows, 3 * p, sc.dc_part, sc.red_tmp, sc.dvec);
    if (e != hipSuccess) return e;
    e = colsum_two_level(st, d2_rows, p * p, sc.d2_part, sc.red_tmp, d2);
    if (e != hipSuccess) return e;
    k_bwd_finish_vec<<<1, 128, 0, st>>>(p, sc.dvec, theta3, theta4, d1, d3, d4);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// theta <- theta - lr * grad over the seven tensors (4p^2 + 4p values).
// ------------------------------------------------------------------------------------------
struct SgdArgs {
    float *theta[7];
    const float *grad[7];
    int len[7];
};

__global__ __launch_bounds__(256) void k_sgd(SgdArgs a, float lr) {
    const int t = blockIdx.y;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < a.len[t]; i += gridDim.x * 256)
        a.theta[t][i] = a.theta[t][i] - lr * a.grad[t][i];
}

hipError_t launch_sgd(hipStream_t st, int p, float *const theta[7], const float *const grad[7], float lr) {
    SgdArgs a;
    const int len[7] = {p, p * p, p * p, p, 2 * p, p * p, p * p};
    for (int i = 0; i < 7; ++i) { a.theta[i] = theta[i]; a.grad[i] = grad[i]; a.len[i] = len[i]; }
    k_sgd<<<dim3((p * p + 255) / 256, 7), 256, 0, st>>>(a, lr);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Adam (the optimiser the paper trains with, Sec. 4.4), one step over the seven tensors:
//   m <- b1 m + (1-b1) g,  v <- b2 v + (1-b2) g^2,
//   theta <- theta - lr / (1 - b1^t) * m / (sqrt(v) / sqrt(1 - b2^t) + eps).
// ------------------------------------------------------------------------------------------
struct AdamArgs {
    float *theta[7];
    const float *grad[7];
    float *m[7];
    float *v[7];
    int len[7];
};

__global__ __launch_bounds__(256) void k_adam(AdamArgs a, float lr, float b1, float b2, float eps, float bias1,
                                              float bias2_sqrt) {
    const int t = blockIdx.y;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < a.len[t]; i += gridDim.x * 256) {
        const float g = a.grad[t][i];
        const float m = b1 * a.m[t][i] + (1.f - b1) * g;
        const float v = b2 * a.v[t][i] + (1.f - b2) * g * g;
        a.m[t][i] = m;
        a.v[t][i] = v;
        a.theta[t][i] = a.theta[t][i] - (lr / bias1) * (m / (sqrtf(v) / bias2_sqrt + eps));
    }
}

hipError_t launch_adam(hipStream_t st, int p, float *const theta[7], const float *const grad[7], float *const m[7],
                       float *const v[7], float lr, float b1, float b2, float eps, float bias1, float bias2_sqrt) {
    AdamArgs a;
    const int len[7] = {p, p * p, p * p, p, 2 * p, p * p, p * p};
    for (int i = 0; i < 7; ++i) { a.theta[i] = theta[i]; a.grad[i] = grad[i]; a.m[i] = m[i]; a.v[i] = v[i]; a.len[i] = len[i]; }
    k_adam<<<dim3((p * p + 255) / 256, 7), 256, 0, st>>>(a, lr, b1, b2, eps, bias1, bias2_sqrt);
    return hipGetLastError();
}

}  // namespace s2v
