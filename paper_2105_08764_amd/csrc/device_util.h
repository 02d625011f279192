// Device-side building blocks shared by the embedding kernels (forward and backward):
// the wave-level neighbour gather and the 16 x P by P x P product on the matrix cores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace s2v {

constexpr int kWaves = 4;         // waves per workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kTileRows = 16;     // rows of the (node, state) matrix one wave owns at a time
constexpr int kWgRows = kTileRows * kWaves;

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Geometry for embedding size P (32 or 64).  A row of P floats is covered by LPR lanes
// holding one float4 each, so one wave-wide load fetches NPL neighbour rows at once.
template <int P>
struct Geo {
    static constexpr int LPR = P / 4;
    static constexpr int NPL = 64 / LPR;
    static constexpr int KS = P / 4;        // k-steps of the 16x16x4 matrix instruction
    static constexpr int CB = P / 16;       // 16-wide column blocks of the output
    static constexpr int STRIDE = P + 4;    // LDS row stride in floats (keeps float4 alignment, spreads banks)
};

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// acc += v (W = false) or acc += w * v (W = true: the weighted neighbour sum)
template <bool W>
__device__ __forceinline__ float4 acc4(float4 a, float4 v, float w) {
    if (W) return make_float4(fmaf(w, v.x, a.x), fmaf(w, v.y, a.y), fmaf(w, v.z, a.z), fmaf(w, v.w, a.w));
    return add4(a, v);
}
__device__ __forceinline__ float readlane_f(float x, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

// The round-1 pre-activation of one (node, state, column) from the node's three scalars (mu^0 = 0 in
// Alg. 1, so z^1 = theta1 x + s+ q+ + s- q-).  Round 1 is recomputed wherever it is needed, forward (the
// neighbour rows of round 2, the stored round-1 rows) and backward (the relu decisions of the last reversed
// round): every such place calls this one function, whose order of operations is spelled out, so that all
// of them take the same decision on every relu and produce the same value bit for bit.
__device__ __forceinline__ float mu1_z(float x, float sp, float sn, float t1, float qp, float qn) {
    return __fmaf_rn(sn, qn, __fmaf_rn(sp, qp, __fmul_rn(x, t1)));
}
// The same when s- = 0 (graphs without a negative weight): mu1_z(x, sp, 0, t1, qp, qn) adds an exact zero.
__device__ __forceinline__ float mu1_z(float x, float sp, float t1, float qp) {
    return __fmaf_rn(sp, qp, __fmul_rn(x, t1));
}
__device__ __forceinline__ float4 mu1_row(float x, float sp, float sn, float4 t1, float4 qp, float4 qn) {
    return make_float4(fmaxf(mu1_z(x, sp, sn, t1.x, qp.x, qn.x), 0.f), fmaxf(mu1_z(x, sp, sn, t1.y, qp.y, qn.y), 0.f),
                       fmaxf(mu1_z(x, sp, sn, t1.z, qp.z, qn.z), 0.f), fmaxf(mu1_z(x, sp, sn, t1.w, qp.w, qn.w), 0.f));
}

// ---- row loaders: the float4 (columns 4*li .. 4*li+3) of neighbour u's row -------------------

// Row (u, s) of a [N][S][P] matrix in memory.
struct MemRow {
    const float *__restrict__ src;
    size_t row_stride;  // S * P
    size_t col_off;     // s * P + 4 * li
    __device__ __forceinline__ float4 operator()(int u) const { return ld4(src + (size_t)u * row_stride + col_off); }
};

// Row (u, s) of the round-1 embedding, recomputed instead of read: mu^0 = 0 makes
// mu^1_u = relu(theta1 x_u + s+_u q+ + s-_u q-) a function of three scalars per (node, state),
// read from the node's record.  A record of zeros gives a zero row.
struct Mu1Row {
    NodeInfo ni;
    int s;
    float4 t1, qp, qn;  // theta1, q+, q- at this lane's four columns
    __device__ __forceinline__ float4 operator()(int u) const {
        const float3 r = ni.get(u, s);
        return mu1_row(r.x, r.y, r.z, t1, qp, qn);
    }
};

// The same for S = 1, where a node's record is the 16 bytes {x, s+, s-, pad}: one load.
struct Mu1RowSingle {
    const float *__restrict__ base;
    float4 t1, qp, qn;
    __device__ __forceinline__ float4 operator()(int u) const {
        const float4 r = ld4(base + (size_t)u * 4);
        return mu1_row(r.x, r.y, r.z, t1, qp, qn);
    }
};

// Row (u, s) of the relu mask of an embedding, one 64-bit word per (node, state) with bit j set
// when entry j is positive, expanded to 0.0 / 1.0 floats: summing these rows counts, per column,
// the neighbours whose entry is positive (exact in float up to 2^24 neighbours).
struct BitsRow {
    const unsigned long long *__restrict__ mask;
    int S;
    int s;
    int shift;  // 4 * li
    __device__ __forceinline__ float4 operator()(int u) const {
        const unsigned nib = (unsigned)(mask[(size_t)u * S + s] >> shift);
        return make_float4((float)(nib & 1u), (float)((nib >> 1) & 1u), (float)((nib >> 2) & 1u),
                           (float)((nib >> 3) & 1u));
    }
};

// Sum over the stored entries [b, e) of one CSR row of the neighbours' P-float rows (row mode:
// any S).  All 64 lanes take part: lane = (group gq, lane-in-row li); one wave-wide load fetches
// NPL neighbour rows.  `cols` holds colidx[b + lane] for the first (up to) 64 entries, loaded by
// the caller ahead of time.  Returns the full row sum in every group.  W = true multiplies each
// neighbour's row by the weight of its entry (wagg is indexed like colidx).
template <int P, bool W = false, class Loader>
__device__ __forceinline__ float4 gather_row_sum(const Loader &row, const int *__restrict__ colidx,
                                                 const float *__restrict__ wagg, int b, int e, int cols, int lane) {
    constexpr int NPL = Geo<P>::NPL, LPR = Geo<P>::LPR;
    const int gq = lane / LPR;
    float4 total = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        if (base != b) cols = (lane < cnt) ? colidx[base + lane] : 0;
        float wv = 0.f;
        if (W) wv = (lane < cnt) ? wagg[base + lane] : 0.f;
        const int last = cnt - 1;
        // per-chunk accumulators folded into the running total: bounds the terms added into one float
        float4 a0 = make_float4(0.f, 0.f, 0.f, 0.f), a1 = a0, a2 = a0, a3 = a0;
        int s0 = 0;
        // Eight independent loads per lane while at least 4*NPL + 1 entries remain, else four.
        // Slots past the end re-read the last valid row (same cache line as a live lane, so no
        // extra memory traffic) and are dropped when accumulating.
        for (; cnt - s0 > 4 * NPL; s0 += 8 * NPL) {
            int sl[8];
            float4 v[8];
            float wk[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                sl[k] = s0 + gq + k * NPL;
                v[k] = row(__shfl(cols, min(sl[k], last)));
                wk[k] = W ? __shfl(wv, min(sl[k], last)) : 1.f;
            }
            if (sl[0] < cnt) a0 = acc4<W>(a0, v[0], wk[0]);
            if (sl[1] < cnt) a1 = acc4<W>(a1, v[1], wk[1]);
            if (sl[2] < cnt) a2 = acc4<W>(a2, v[2], wk[2]);
            if (sl[3] < cnt) a3 = acc4<W>(a3, v[3], wk[3]);
            if (sl[4] < cnt) a0 = acc4<W>(a0, v[4], wk[4]);
            if (sl[5] < cnt) a1 = acc4<W>(a1, v[5], wk[5]);
            if (sl[6] < cnt) a2 = acc4<W>(a2, v[6], wk[6]);
            if (sl[7] < cnt) a3 = acc4<W>(a3, v[7], wk[7]);
        }
        if (s0 < cnt) {
            int sl[4];
            float4 v[4];
            float wk[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                sl[k] = s0 + gq + k * NPL;
                v[k] = row(__shfl(cols, min(sl[k], last)));
                wk[k] = W ? __shfl(wv, min(sl[k], last)) : 1.f;
            }
            if (sl[0] < cnt) a0 = acc4<W>(a0, v[0], wk[0]);
            if (sl[1] < cnt) a1 = acc4<W>(a1, v[1], wk[1]);
            if (sl[2] < cnt) a2 = acc4<W>(a2, v[2], wk[2]);
            if (sl[3] < cnt) a3 = acc4<W>(a3, v[3], wk[3]);
        }
        total = add4(total, add4(add4(a0, a1), add4(a2, a3)));
    }
    float4 a0 = total;
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
        a0.x += __shfl_xor(a0.x, m);
        a0.y += __shfl_xor(a0.y, m);
        a0.z += __shfl_xor(a0.z, m);
        a0.w += __shfl_xor(a0.w, m);
    }
    return a0;
}

// Two short rows at once (each of at most 4 * NPL stored entries, possibly none): the loads of both rows are in
// flight together, so the pair costs one trip to memory instead of two.  Each row's terms are added exactly as
// gather_row_sum adds them for such a row: the same bits.  cols0 / cols1: colidx[b + lane] of the rows.
template <int P, bool W = false, class Loader>
__device__ __forceinline__ void gather_row_sum_pair(const Loader &row0, const Loader &row1,
                                                    const float *__restrict__ wagg, int b0, int e0, int cols0, int b1,
                                                    int e1, int cols1, int lane, float4 &out0, float4 &out1) {
    constexpr int NPL = Geo<P>::NPL, LPR = Geo<P>::LPR;
    const int gq = lane / LPR;
    const int cnt0 = e0 - b0, cnt1 = e1 - b1;
    float wv0 = 0.f, wv1 = 0.f;
    if (W) {
        wv0 = (lane < cnt0) ? wagg[b0 + lane] : 0.f;
        wv1 = (lane < cnt1) ? wagg[b1 + lane] : 0.f;
    }
    const int last0 = max(cnt0 - 1, 0), last1 = max(cnt1 - 1, 0);   // (an empty row re-reads a valid row: dropped below)
    int sl[4];
    float4 v0[4], v1[4];
    float wk0[4], wk1[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        sl[k] = gq + k * NPL;
        v0[k] = row0(__shfl(cols0, min(sl[k], last0)));
        v1[k] = row1(__shfl(cols1, min(sl[k], last1)));
        wk0[k] = W ? __shfl(wv0, min(sl[k], last0)) : 1.f;
        wk1[k] = W ? __shfl(wv1, min(sl[k], last1)) : 1.f;
    }
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 a[4], c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        a[k] = sl[k] < cnt0 ? acc4<W>(zero, v0[k], wk0[k]) : zero;
        c[k] = sl[k] < cnt1 ? acc4<W>(zero, v1[k], wk1[k]) : zero;
    }
    float4 t0 = cnt0 > 0 ? add4(zero, add4(add4(a[0], a[1]), add4(a[2], a[3]))) : zero;
    float4 t1 = cnt1 > 0 ? add4(zero, add4(add4(c[0], c[1]), add4(c[2], c[3]))) : zero;
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
        t0.x += __shfl_xor(t0.x, m); t0.y += __shfl_xor(t0.y, m); t0.z += __shfl_xor(t0.z, m); t0.w += __shfl_xor(t0.w, m);
        t1.x += __shfl_xor(t1.x, m); t1.y += __shfl_xor(t1.y, m); t1.z += __shfl_xor(t1.z, m); t1.w += __shfl_xor(t1.w, m);
    }
    out0 = t0;
    out1 = t1;
}

// The round-2 neighbour sum for S = 1 (records {x, s+, s-, pad}, see Mu1RowSingle), with the cheap
// case split off: for a neighbour with x = 0 and s- = 0 the recomputed row is
// relu(s+ q+) = s+ relu(q+) (s+ >= 0), i.e. linear in one scalar, so such neighbours only add
// s+ (times the edge weight when W) to a running scalar and the vector arithmetic runs for the
// others alone (a wave-uniform branch per wave-wide load).  On a partial solution that marks few
// nodes and with non-negative weights almost every neighbour is of the cheap kind.  Same
// arguments and result as gather_row_sum; rp = relu(q+) at this lane's columns.
template <int P, bool W>
__device__ __forceinline__ float4 gather_row_sum_mu1_single(const float *__restrict__ rec, float4 t1, float4 qp,
                                                            float4 qn, float4 rp, const int *__restrict__ colidx,
                                                            const float *__restrict__ wagg, int b, int e, int cols,
                                                            int lane) {
    constexpr int NPL = Geo<P>::NPL, LPR = Geo<P>::LPR;
    const int gq = lane / LPR;
    float4 total = make_float4(0.f, 0.f, 0.f, 0.f);
    float stotal = 0.f;
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        if (base != b) cols = (lane < cnt) ? colidx[base + lane] : 0;
        float wv = 0.f;
        if (W) wv = (lane < cnt) ? wagg[base + lane] : 0.f;
        const int last = cnt - 1;
        float4 a0 = make_float4(0.f, 0.f, 0.f, 0.f), a1 = a0;
        float s0acc = 0.f, s1acc = 0.f;
        for (int s0 = 0; s0 < cnt; s0 += 8 * NPL) {
            float4 r[8];
            float wk[8];
            int sl[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                sl[k] = s0 + gq + k * NPL;
                const int at = min(sl[k], last);   // past the end: a live lane's record again, dropped below
                r[k] = ld4(rec + (size_t)__shfl(cols, at) * 4);
                wk[k] = W ? __shfl(wv, at) : 1.f;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool live = sl[k] < cnt;
                const bool cheap = r[k].x == 0.f && r[k].z == 0.f;
                const float sadd = (live && cheap) ? wk[k] * r[k].y : 0.f;
                if (k & 1) s1acc += sadd; else s0acc += sadd;
                const bool full = live && !cheap;
                if (__ballot(full) != 0ull) {
                    const float4 m = mu1_row(r[k].x, r[k].y, r[k].z, t1, qp, qn);
                    const float wf = full ? wk[k] : 0.f;
                    if (k & 1) a1 = make_float4(fmaf(wf, m.x, a1.x), fmaf(wf, m.y, a1.y), fmaf(wf, m.z, a1.z), fmaf(wf, m.w, a1.w));
                    else a0 = make_float4(fmaf(wf, m.x, a0.x), fmaf(wf, m.y, a0.y), fmaf(wf, m.z, a0.z), fmaf(wf, m.w, a0.w));
                }
            }
        }
        total = add4(total, add4(a0, a1));
        stotal += s0acc + s1acc;
    }
    float4 a0 = make_float4(fmaf(stotal, rp.x, total.x), fmaf(stotal, rp.y, total.y), fmaf(stotal, rp.z, total.z),
                            fmaf(stotal, rp.w, total.w));
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
        a0.x += __shfl_xor(a0.x, m);
        a0.y += __shfl_xor(a0.y, m);
        a0.z += __shfl_xor(a0.z, m);
        a0.w += __shfl_xor(a0.w, m);
    }
    return a0;
}

// Round 2 for S = 1, a whole tile at once and one LANE per neighbour: the column indices of eight
// rows are fetched together, then the scalars of all their neighbours (up to 64 per row) with one
// load per row, so a wave has hundreds of them in flight instead of 32.  Cheap neighbours (see
// gather_row_sum_mu1_single) are summed by a wave reduction of one scalar; the few others are
// visited one by one, lane j forming column j of relu(x theta1 + s+ q+ + s- q-).
// MODE 1 (compact table): the first load reads the 4-byte table compact[u] (s+ of a cheap neighbour,
// NaN for any other) instead of the 16-byte record, and only the lanes that met a NaN fetch the record:
// the table is a quarter of the records' size, so more of it stays in the L2.
// MODE 2 (flag bits + per-row total; static graph without negative weights): even that table (4 N bytes)
// exceeds an L2 at a few million nodes, and a miss moves a whole cache line for four useful bytes: at
// 2 M nodes and 60 M entries the round fetched 5 GB that way.  Here the first load tests bit u of xbits
// (N / 8 bytes: always in the L2), only flagged neighbours (x_u != 0) fetch their record, and the sum of
// s+ over the unflagged ones is the row's precomputed total over all neighbours (fourth float of the
// row's own record) minus the s+ of the flagged ones.
// Rows with more than 64 entries continue in 64-entry chunks; rows longer than max_len are skipped
// (their sums are already in the tile).  rb / re: lane i (mod 16) holds begin / end of tile row i.
// The result of row i goes to tile[i * STRIDE + column].  lc = {theta1, q+, q-} in LDS ([3][P]).
// W (mode 2 only): the weighted neighbour sum; the row's total is then the weighted one, and a flagged
// neighbour's edge weight is read next to its column index.
template <int P, int MODE, bool W = false>
__device__ __forceinline__ void gather_tile_mu1_single(float *tile, const float *__restrict__ rec,
                                                       const float *__restrict__ compact,
                                                       const unsigned *__restrict__ xbits, const float *lc,
                                                       const int *__restrict__ colidx, int rb, int re, int max_len,
                                                       int lane, float total_mine = 0.f,
                                                       const float *__restrict__ wagg = nullptr) {
    static_assert(!W || MODE == 2, "only the flag-bit form has a weighted variant here");
    // total_mine (mode 2): lane i (mod 16) holds the total of s+ over all neighbours of tile row i
    constexpr int STRIDE = Geo<P>::STRIDE;
    const int j = lane % P;
    const float t1 = lc[j], qp = lc[P + j], qn = lc[2 * P + j];
    const float rp = fmaxf(qp, 0.f);
    // the scalars of neighbour u as {x, s+, s-}; a missing neighbour (u < 0) adds nothing.  In mode 2 an
    // unflagged neighbour comes back as all zeros (it is accounted for by the row's total).
    auto fetch = [&](int u, float &x, float &sp, float &sn) {
        x = 0.f; sp = 0.f; sn = 0.f;
        if (MODE == 1) {
            const float c = u >= 0 ? compact[u] : 0.f;
            if (c == c) { sp = c; return; }
            const float4 r = ld4(rec + (size_t)u * 4);
            x = r.x; sp = r.y; sn = r.z;
        } else if (MODE == 2) {
            const unsigned wd = u >= 0 ? xbits[u >> 5] : 0u;
            if ((wd >> (u & 31)) & 1u) {
                const float4 r = ld4(rec + (size_t)u * 4);
                x = r.x; sp = r.y; sn = r.z;
            }
        } else if (u >= 0) {
            const float4 r = ld4(rec + (size_t)u * 4);
            x = r.x; sp = r.y; sn = r.z;
        }
    };
    // Rows per pass: the loads of a pass (indices, then table entries, then the records that are needed) are
    // issued together, so a pass costs three trips to memory whatever its size.  The flag-bit form keeps two
    // registers less per row and takes the whole tile in one pass.
#ifndef S2V_R2_ROWS
#define S2V_R2_ROWS 16
#endif
    constexpr int RB = MODE == 2 ? S2V_R2_ROWS : 8;
#pragma unroll 1
    for (int half = 0; half < 16 / RB; ++half) {
        int cols[RB];
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            const int i = RB * half + k;
            // (i is wave-uniform: a lane read, not a shuffle through LDS)
            const int b = __builtin_amdgcn_readlane(rb, i), n = __builtin_amdgcn_readlane(re, i) - b;
            cols[k] = (n <= max_len && lane < n) ? colidx[b + lane] : -1;   // lane < n <= 64 entries of the first chunk
        }
        float rx[RB], rs[RB], rn[MODE == 2 ? 1 : RB];
        float rw[W ? RB : 1];   // edge weights of the flagged neighbours
        if constexpr (MODE == 1) {
            // all eight table loads first, then the record loads of the lanes that need one
            float c[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) c[k] = cols[k] >= 0 ? compact[cols[k]] : 0.f;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                rx[k] = 0.f; rs[k] = c[k]; rn[k] = 0.f;
                if (c[k] != c[k]) {
                    const float4 r = ld4(rec + (size_t)cols[k] * 4);
                    rx[k] = r.x; rs[k] = r.y; rn[k] = r.z;
                }
            }
        } else if constexpr (MODE == 2) {
            unsigned wd[RB];
#pragma unroll
            for (int k = 0; k < RB; ++k) wd[k] = cols[k] >= 0 ? xbits[cols[k] >> 5] : 0u;
#pragma unroll
            for (int k = 0; k < RB; ++k) {
                rx[k] = 0.f; rs[k] = 0.f;   // (no negative weights here: s- is zero and not kept)
                if (W) rw[W ? k : 0] = 0.f;
                if ((wd[k] >> (cols[k] & 31)) & 1u) {
                    const float2 r = *reinterpret_cast<const float2 *>(rec + (size_t)cols[k] * 4);
                    rx[k] = r.x; rs[k] = r.y;
                    if (W) rw[W ? k : 0] = wagg[__builtin_amdgcn_readlane(rb, RB * half + k) + lane];
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) fetch(cols[k], rx[k], rs[k], rn[k]);
        }
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            const int i = RB * half + k;
            const int b = __builtin_amdgcn_readlane(rb, i), e = __builtin_amdgcn_readlane(re, i);
            if (e - b > max_len) continue;                     // wave-uniform
            float ssum = 0.f, acc = 0.f;
            float flagged_sp = 0.f;                            // mode 2: s+ of the flagged neighbours (wave-uniform)
            float x = rx[k], sp = rs[k], sn = MODE == 2 ? 0.f : rn[MODE == 2 ? 0 : k];
            float wl = W ? rw[W ? k : 0] : 1.f;
            int base = b;
            while (true) {
                const bool cheap = x == 0.f && sn == 0.f;
                if (MODE != 2) ssum += cheap ? sp : 0.f;
                unsigned long long todo = __ballot(MODE == 2 ? x != 0.f : !cheap);
                while (todo != 0ull) {
                    const int l = __ffsll((long long)todo) - 1;
                    todo &= todo - 1ull;
                    const float xl = readlane_f(x, l), pl = readlane_f(sp, l), nl = readlane_f(sn, l);
                    const float m1 = fmaxf(mu1_z(xl, pl, nl, t1, qp, qn), 0.f);
                    if (W) {
                        const float wk = readlane_f(wl, l);
                        acc = fmaf(wk, m1, acc);
                        flagged_sp = fmaf(wk, pl, flagged_sp);
                    } else {
                        acc += m1;
                        if (MODE == 2) flagged_sp += pl;
                    }
                }
                base += 64;
                if (base >= e) break;                          // wave-uniform
                fetch((base + lane < e) ? colidx[base + lane] : -1, x, sp, sn);
                if (W) wl = (x != 0.f) ? wagg[base + lane] : 0.f;
            }
            if (MODE == 2) {
                ssum = readlane_f(total_mine, i) - flagged_sp;
            } else {
#pragma unroll
                for (int m = 1; m < 64; m <<= 1) ssum += __shfl_xor(ssum, m);
            }
            if (lane < P) tile[i * STRIDE + lane] = fmaf(ssum, rp, acc);
        }
    }
}

// Modes 0 and 1 of gather_tile_mu1_single for rows of several 64-entry chunks (the graphs of the inference loop,
// whose rows shrink from hundreds of entries): eight rows at a time as before, but chunk LEVEL by chunk level --
// the q-th chunks of all eight rows are fetched together (indices, then table entries, then the records that are
// needed), so eight rows of 200 entries cost four rounds of dependent loads instead of eight times four.  Every
// lane adds the same values in the same order as in gather_tile_mu1_single: the same bits.
template <int P, int MODE>
__device__ __forceinline__ void gather_tile_mu1_levels(float *tile, const float *__restrict__ rec,
                                                       const float *__restrict__ compact, const float *lc,
                                                       const int *__restrict__ colidx, int rb, int re, int max_len,
                                                       int lane) {
    static_assert(MODE == 0 || MODE == 1, "");
    constexpr int STRIDE = Geo<P>::STRIDE;
    const int j = lane % P;
    const float t1 = lc[j], qp = lc[P + j], qn = lc[2 * P + j];
    const float rp = fmaxf(qp, 0.f);
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        float ssum[8], acc[8];
        int nlev = 0;   // chunk levels of the longest row of this half that is gathered here (wave-uniform)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            ssum[k] = 0.f; acc[k] = 0.f;
            const int n = __builtin_amdgcn_readlane(re, 8 * half + k) - __builtin_amdgcn_readlane(rb, 8 * half + k);
            if (n <= max_len) nlev = max(nlev, (n + 63) >> 6);
        }
#pragma unroll 1
        for (int lev = 0; lev < nlev; ++lev) {
            int cols[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int b = __builtin_amdgcn_readlane(rb, 8 * half + k), n = __builtin_amdgcn_readlane(re, 8 * half + k) - b;
                const int i = 64 * lev + lane;
                cols[k] = (n <= max_len && i < n) ? colidx[b + i] : -1;
            }
            float rx[8], rs[8], rn[8];
            if constexpr (MODE == 1) {
                float c[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) c[k] = cols[k] >= 0 ? compact[cols[k]] : 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    rx[k] = 0.f; rs[k] = c[k]; rn[k] = 0.f;
                    if (c[k] != c[k]) {
                        const float4 r = ld4(rec + (size_t)cols[k] * 4);
                        rx[k] = r.x; rs[k] = r.y; rn[k] = r.z;
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    rx[k] = 0.f; rs[k] = 0.f; rn[k] = 0.f;
                    if (cols[k] >= 0) {
                        const float4 r = ld4(rec + (size_t)cols[k] * 4);
                        rx[k] = r.x; rs[k] = r.y; rn[k] = r.z;
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool cheap = rx[k] == 0.f && rn[k] == 0.f;
                ssum[k] += cheap ? rs[k] : 0.f;
                unsigned long long todo = __ballot(!cheap);
                while (todo != 0ull) {
                    const int l = __ffsll((long long)todo) - 1;
                    todo &= todo - 1ull;
                    const float xl = readlane_f(rx[k], l), pl = readlane_f(rs[k], l), nl = readlane_f(rn[k], l);
                    acc[k] += fmaxf(mu1_z(xl, pl, nl, t1, qp, qn), 0.f);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = 8 * half + k;
            if (__builtin_amdgcn_readlane(re, i) - __builtin_amdgcn_readlane(rb, i) > max_len) continue;   // wave-uniform
            float sv = ssum[k];
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) sv += __shfl_xor(sv, m);
            if (lane < P) tile[i * STRIDE + lane] = fmaf(sv, rp, acc[k]);
        }
    }
}

// The same for any S (row mode of round 2 with several states): tile row i is (node v_i, state s_i), and the
// record of neighbour u for that row is {x_u[s_i], s+_u, s-_u} of the general layout.  rb, re, s: lane i
// (mod 16) holds the range and the state of tile row i.  W: every neighbour's row times the weight of its entry.
template <int P, bool W>
__device__ __forceinline__ void gather_tile_mu1_rows(float *tile, const NodeInfo &ni, int s, const float *lc,
                                                     const int *__restrict__ colidx, const float *__restrict__ wagg,
                                                     int rb, int re, int max_len, int lane) {
    constexpr int STRIDE = Geo<P>::STRIDE;
    const int j = lane % P;
    const float t1 = lc[j], qp = lc[P + j], qn = lc[2 * P + j];
    const float rp = fmaxf(qp, 0.f);
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        float ssum[8], acc[8];
        int nlev = 0;   // chunk levels of the longest row of this half that is gathered here (wave-uniform)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            ssum[k] = 0.f; acc[k] = 0.f;
            const int n = __builtin_amdgcn_readlane(re, 8 * half + k) - __builtin_amdgcn_readlane(rb, 8 * half + k);
            if (n <= max_len) nlev = max(nlev, (n + 63) >> 6);
        }
#pragma unroll 1
        for (int lev = 0; lev < nlev; ++lev) {
            int cols[8];
            float wl[W ? 8 : 1];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int b = __builtin_amdgcn_readlane(rb, 8 * half + k), n = __builtin_amdgcn_readlane(re, 8 * half + k) - b;
                const int i = 64 * lev + lane;
                const bool ok = n <= max_len && i < n;
                cols[k] = ok ? colidx[b + i] : -1;
                if (W) wl[W ? k : 0] = ok ? wagg[b + i] : 0.f;
            }
            float rx[8], rs[8], rn[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int sk = __builtin_amdgcn_readlane(s, 8 * half + k);
                rx[k] = 0.f; rs[k] = 0.f; rn[k] = 0.f;
                if (cols[k] >= 0) {
                    const float3 r = ni.get(cols[k], sk);
                    rx[k] = r.x; rs[k] = r.y; rn[k] = r.z;
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool cheap = rx[k] == 0.f && rn[k] == 0.f;
                ssum[k] += cheap ? (W ? wl[W ? k : 0] * rs[k] : rs[k]) : 0.f;
                unsigned long long todo = __ballot(!cheap);
                while (todo != 0ull) {
                    const int l = __ffsll((long long)todo) - 1;
                    todo &= todo - 1ull;
                    const float xl = readlane_f(rx[k], l), pl = readlane_f(rs[k], l), nl = readlane_f(rn[k], l);
                    const float z = fmaxf(mu1_z(xl, pl, nl, t1, qp, qn), 0.f);
                    acc[k] = W ? fmaf(readlane_f(wl[W ? k : 0], l), z, acc[k]) : acc[k] + z;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = 8 * half + k;
            if (__builtin_amdgcn_readlane(re, i) - __builtin_amdgcn_readlane(rb, i) > max_len) continue;   // wave-uniform
            float sv = ssum[k];
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) sv += __shfl_xor(sv, m);
            if (lane < P) tile[i * STRIDE + lane] = fmaf(sv, rp, acc[k]);
        }
    }
}

// Node mode (S a multiple of 16): the 16 rows of a wave tile are 16 consecutive states
// s0 .. s0+15 of ONE node v, so every neighbour u contributes one contiguous block of 16 * P
// floats, mu[u][s0 .. s0+15][:].  A wave-wide float4 load covers RPI = 64 / LPR of those rows
// (1 KB, fully coalesced); NC = 16 / RPI loads cover the block.  Lane l, register c owns tile
// row c * RPI + l / LPR, columns 4 * (l % LPR) ..: no cross-lane reduction is needed, and the
// neighbour index is wave-uniform.
template <int P>
struct NodeAcc {
    float4 a[16 / Geo<P>::NPL];
};

#ifndef S2V_NODE_UNROLL
#define S2V_NODE_UNROLL 2
#endif

template <int P, bool W = false>
__device__ __forceinline__ NodeAcc<P> gather_node_block(const float *__restrict__ src, size_t node_stride /*S*P*/,
                                                        size_t blk_off /*s0*P*/, const int *__restrict__ colidx,
                                                        const float *__restrict__ wagg, int b, int e, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, U = S2V_NODE_UNROLL;
    // U accumulators per 64-entry chunk, folded into the running total after each chunk, so a
    // row of d entries adds at most about 64 / U + d / 64 terms into any one float.
    NodeAcc<P> total, acc[U];
#pragma unroll
    for (int c = 0; c < NC; ++c) total.a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *lane_src = src + blk_off + 4 * (size_t)lane;
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        const int cols = (lane < cnt) ? colidx[base + lane] : 0;
        float wv = 0.f;
        if (W) wv = (lane < cnt) ? wagg[base + lane] : 0.f;
#pragma unroll
        for (int k = 0; k < U; ++k)
#pragma unroll
            for (int c = 0; c < NC; ++c) acc[k].a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        int j = 0;
        for (; j + U <= cnt; j += U) {
            float4 v[U][NC];
            float wk[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const float *pk = lane_src + (size_t)__builtin_amdgcn_readlane(cols, j + k) * node_stride;
                wk[k] = W ? readlane_f(wv, j + k) : 1.f;
#pragma unroll
                for (int c = 0; c < NC; ++c) v[k][c] = ld4(pk + c * RPI * P);
            }
#pragma unroll
            for (int k = 0; k < U; ++k)
#pragma unroll
                for (int c = 0; c < NC; ++c) acc[k].a[c] = acc4<W>(acc[k].a[c], v[k][c], wk[k]);
        }
        for (; j < cnt; ++j) {
            const float *p0 = lane_src + (size_t)__builtin_amdgcn_readlane(cols, j) * node_stride;
            const float w0 = W ? readlane_f(wv, j) : 1.f;
            float4 v0[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) v0[c] = ld4(p0 + c * RPI * P);
#pragma unroll
            for (int c = 0; c < NC; ++c) acc[0].a[c] = acc4<W>(acc[0].a[c], v0[c], w0);
        }
#pragma unroll
        for (int k = 1; k < U; ++k)
#pragma unroll
            for (int c = 0; c < NC; ++c) acc[0].a[c] = add4(acc[0].a[c], acc[k].a[c]);
#pragma unroll
        for (int c = 0; c < NC; ++c) total.a[c] = add4(total.a[c], acc[0].a[c]);
    }
    return total;
}

// The gathers that recompute neighbour rows from the records use their own lane layout ("state-major"):
// lane l, register c owns tile row NC * (l / LPR) + c, so that a lane's NC states are consecutive and
// their x (or per-state s+-) come with ONE vector load per neighbour.
template <int NC>
__device__ __forceinline__ void ld_states(const float *p, float (&out)[NC]) {
    static_assert(NC == 4 || NC == 2 || NC == 1, "");
    if constexpr (NC == 4) {
        const float4 t = ld4(p);
        out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
    } else if constexpr (NC == 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        out[0] = t.x; out[1] = t.y;
    } else {
        out[0] = p[0];
    }
}
template <int P>
__device__ __forceinline__ void store_node_block_sm(float *tile, const NodeAcc<P> &acc, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
#pragma unroll
    for (int c = 0; c < NC; ++c) st4(tile + (NC * (lane / LPR) + c) * Geo<P>::STRIDE + 4 * (lane % LPR), acc.a[c]);
}
// state-major block from / to a plain [16][P] block in memory
template <int P>
__device__ __forceinline__ NodeAcc<P> load_node_block_sm(const float *__restrict__ blk, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
    NodeAcc<P> acc;
#pragma unroll
    for (int c = 0; c < NC; ++c) acc.a[c] = ld4(blk + (size_t)(NC * (lane / LPR) + c) * P + 4 * (lane % LPR));
    return acc;
}
template <int P>
__device__ __forceinline__ void write_node_block_sm(float *__restrict__ blk, const NodeAcc<P> &acc, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
#pragma unroll
    for (int c = 0; c < NC; ++c) st4(blk + (size_t)(NC * (lane / LPR) + c) * P + 4 * (lane % LPR), acc.a[c]);
}

// A batch of neighbour records for one 16-state block goes through wave-private LDS: the wave
// fetches the x of 16 neighbours with ONE float4 load (lane = (neighbour, group of four states)) and
// the per-node sums with one lane per neighbour, so a whole batch costs a single trip to memory;
// the lanes then read each neighbour's scalars back in their own (state-major) layout.
// Staged neighbour: x[16], then {s+, s-} (SHARED) or s+[16], s-[16] (per state).
template <bool SHARED>
struct RecStage {
    static constexpr int BATCH = SHARED ? 32 : 16;   // neighbours per batch
    static constexpr int NF = SHARED ? 20 : 52;      // floats per staged neighbour (multiple of 4)
};
constexpr int kRecStageFloats = 16 * 52;             // >= BATCH * NF of both forms

// cols: this lane's column index in the current 64-entry chunk; the batch is entries j0 .. j0 + m - 1.
template <bool SHARED>
__device__ __forceinline__ void stage_records(const NodeInfo &ni, int s0, int cols, int j0, int m, int lane,
                                              float *stage) {
    constexpr int BATCH = RecStage<SHARED>::BATCH, NF = RecStage<SHARED>::NF, NL = BATCH / 16;
    const int part = lane & 3;
    float4 x4[NL], p4[SHARED ? 1 : NL], n4[SHARED ? 1 : NL];
#pragma unroll
    for (int k = 0; k < NL; ++k) {
        const int n = 16 * k + (lane >> 2);
        const float *r = ni.node(__shfl(cols, j0 + min(n, m - 1)));   // past the end: a valid record, never consumed
        x4[k] = ld4(r + s0 + 4 * part);
        if (!SHARED) {
            p4[SHARED ? 0 : k] = ld4(r + ni.sp_off + s0 + 4 * part);
            n4[SHARED ? 0 : k] = ld4(r + ni.sn_off + s0 + 4 * part);
        }
    }
    float2 pn = make_float2(0.f, 0.f);
    if (SHARED) {
        const float *r = ni.node(__shfl(cols, j0 + min(lane & (BATCH - 1), m - 1)));
        pn = *reinterpret_cast<const float2 *>(r + ni.sp_off);          // s+ and s- are adjacent
    }
#pragma unroll
    for (int k = 0; k < NL; ++k) {
        float *dst = stage + (16 * k + (lane >> 2)) * NF + 4 * part;
        st4(dst, x4[k]);
        if (!SHARED) {
            st4(dst + 16, p4[SHARED ? 0 : k]);
            st4(dst + 32, n4[SHARED ? 0 : k]);
        }
    }
    if (SHARED && lane < BATCH) *reinterpret_cast<float2 *>(stage + lane * NF + 16) = pn;
}

// Neighbour n of the staged batch in this lane's layout: x, s+, s- of its NC consecutive states
// (s+ / s- in element 0 only when SHARED).
template <int NC, bool SHARED>
__device__ __forceinline__ void read_staged(const float *stage, int n, int q, float (&xs)[NC],
                                            float (&sp)[SHARED ? 1 : NC], float (&sn)[SHARED ? 1 : NC]) {
    const float *r = stage + n * RecStage<SHARED>::NF;
    ld_states<NC>(r + NC * q, xs);
    if constexpr (SHARED) {
        const float2 pn = *reinterpret_cast<const float2 *>(r + 16);
        sp[0] = pn.x;
        sn[0] = pn.y;
    } else {
        ld_states<NC>(r + 16 + NC * q, sp);
        ld_states<NC>(r + 32 + NC * q, sn);
    }
}

// Node mode with the round-1 rows recomputed from the neighbours' records (see Mu1Row): per
// neighbour the x of the 16 states and its edge sums, one pair per node (SHARED) or per state.
// `stage`: kRecStageFloats floats of wave-private LDS.
template <int P, bool W, bool SHARED>
__device__ __forceinline__ NodeAcc<P> gather_node_block_mu1_impl(const NodeInfo &ni, int s0,
                                                                 const float *__restrict__ theta1,
                                                                 const float *__restrict__ qvec,
                                                                 const int *__restrict__ colidx,
                                                                 const float *__restrict__ wagg, int b, int e,
                                                                 int lane, float *stage) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
    constexpr int BATCH = RecStage<SHARED>::BATCH;
    NodeAcc<P> total, acc;
#pragma unroll
    for (int c = 0; c < NC; ++c) total.a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int col = 4 * (lane % LPR);
    const float4 t1 = ld4(theta1 + col), qp = ld4(qvec + col), qn = ld4(qvec + P + col);
    const int q = lane / LPR;   // this lane owns states NC * q .. of the block (state-major layout)
    float ssum = 0.f;   // sum of (weight times) s+ over the neighbours whose rows are s+ relu(q+)
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        const int cols = (lane < cnt) ? colidx[base + lane] : 0;
        float wv = 0.f;
        if (W) wv = (lane < cnt) ? wagg[base + lane] : 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) acc.a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j0 = 0; j0 < cnt; j0 += BATCH) {
            const int m = min(BATCH, cnt - j0);
            stage_records<SHARED>(ni, s0, cols, j0, m, lane, stage);
            __builtin_amdgcn_wave_barrier();
            for (int n = 0; n < m; ++n) {
                float xs[NC], sp[SHARED ? 1 : NC], sn[SHARED ? 1 : NC];
                read_staged<NC, SHARED>(stage, n, q, xs, sp, sn);
                const float wk = W ? readlane_f(wv, j0 + n) : 1.f;
                if (SHARED) {
                    // x = 0 in all 16 states and s- = 0: the row is s+ relu(q+) in every state
                    bool any = false;
#pragma unroll
                    for (int c = 0; c < NC; ++c) any = any || xs[c] != 0.f;
                    if (sn[0] == 0.f && __ballot(any) == 0ull) {
                        ssum += wk * sp[0];
                        continue;
                    }
                }
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const float p_ = sp[SHARED ? 0 : c], n_ = sn[SHARED ? 0 : c], x_ = xs[c];
                    const float4 mm = mu1_row(x_, p_, n_, t1, qp, qn);
                    acc.a[c] = acc4<W>(acc.a[c], mm, wk);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) total.a[c] = add4(total.a[c], acc.a[c]);
    }
    if (SHARED) {
        const float4 rp = make_float4(fmaxf(qp.x, 0.f), fmaxf(qp.y, 0.f), fmaxf(qp.z, 0.f), fmaxf(qp.w, 0.f));
#pragma unroll
        for (int c = 0; c < NC; ++c)
            total.a[c] = make_float4(fmaf(ssum, rp.x, total.a[c].x), fmaf(ssum, rp.y, total.a[c].y),
                                     fmaf(ssum, rp.z, total.a[c].z), fmaf(ssum, rp.w, total.a[c].w));
    }
    return total;
}

template <int P, bool W = false>
__device__ __forceinline__ NodeAcc<P> gather_node_block_mu1(const NodeInfo &ni, int s0,
                                                            const float *__restrict__ theta1,
                                                            const float *__restrict__ qvec,
                                                            const int *__restrict__ colidx,
                                                            const float *__restrict__ wagg, int b, int e, int lane,
                                                            float *stage) {
    if (ni.ss == 0) return gather_node_block_mu1_impl<P, W, true>(ni, s0, theta1, qvec, colidx, wagg, b, e, lane, stage);
    return gather_node_block_mu1_impl<P, W, false>(ni, s0, theta1, qvec, colidx, wagg, b, e, lane, stage);
}

// Round 2 in node mode without reading the neighbours' records (static graph, no negative weight, plain
// neighbour sum; see NodeInfo::flags16).  For the 16 states s0 .. s0+15 of node v, row s of the tile is
//   sum_u mu^1_{u,s} = total_v relu(q+) + sum over the flagged (u, s) of [relu(x_{u,s} theta1 + s+_u q+) - s+_u relu(q+)],
// total_v = sum of s+ over all neighbours (computed once per graph): a neighbour outside the solution of
// state s has mu^1 = s+_u relu(q+).  One lane per neighbour fetches a 16-bit flag word; the records of the
// flagged neighbours only are touched (their s+, and x in the flagged states), and each flagged pair costs
// one p-wide vector operation (lane j = column j, one accumulator register per state).
// b .. e: a row of at most kHubDegree entries.  lc = {theta1, q+, q-} in LDS.  Writes tile[s * STRIDE + j].
template <int P, bool W = false>
__device__ __forceinline__ void gather_node_tile_flags(float *tile, const NodeInfo &ni, int s0, const float *lc,
                                                       const int *__restrict__ colidx, int b, int e, int lane,
                                                       float total, const float *__restrict__ wagg = nullptr,
                                                       int cols_first = 0, bool have_first = false) {
    constexpr int STRIDE = Geo<P>::STRIDE;
    const int j = lane % P;
    const float t1 = lc[j], qp = lc[P + j];
    const float rp = fmaxf(qp, 0.f);
    const int nb = ni.S >> 4, blk = s0 >> 4;
    float acc[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) acc[s] = 0.f;
    for (int base = b; base < e; base += 64) {
        // (have_first: the caller fetched colidx[b + lane] for the lanes below the row's length ahead of time)
        const int u = (base + lane < e) ? ((have_first && base == b) ? cols_first : colidx[base + lane]) : -1;
        const unsigned f = u >= 0 ? (unsigned)ni.flags16[(size_t)u * nb + blk] : 0u;
        if (__ballot(f != 0u) == 0ull) continue;                     // wave-uniform
        const float *r = ni.node(u >= 0 ? u : 0);
        const float sp = f != 0u ? r[ni.sp_off] : 0.f;
        float wl = 1.f;
        if (W) wl = f != 0u ? wagg[base + lane] : 0.f;
        float xs[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) xs[s] = ((f >> s) & 1u) ? r[s0 + s] : 0.f;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            unsigned long long todo = __ballot((f >> s) & 1u);
            while (todo != 0ull) {
                const int l = __ffsll((long long)todo) - 1;
                todo &= todo - 1ull;
                const float xl = readlane_f(xs[s], l), pl = readlane_f(sp, l);
                const float d = fmaxf(mu1_z(xl, pl, t1, qp), 0.f) - pl * rp;
                if (W) acc[s] = fmaf(readlane_f(wl, l), d, acc[s]);
                else acc[s] += d;
            }
        }
    }
    const float base_row = total * rp;
    if (lane < P) {
#pragma unroll
        for (int s = 0; s < 16; ++s) tile[s * STRIDE + lane] = base_row + acc[s];
    }
}

// The same for the sums of the last reversed round (see gather_node_block_mu1_grad for a, cx, cp; no
// negative weight, so cn = 0): per state s of the block and column j = lane,
//   a  = total relu(q+)   + sum over flagged (u, s) of [relu(z) - s+_u relu(q+)]
//   cx =                    sum over flagged (u, s) of x_{u,s} [z > 0]
//   cp = total [q+ > 0]   + sum over flagged (u, s) of s+_u ([z > 0] - [q+ > 0]),      z = x_{u,s} theta1 + s+_u q+
// (z comes from mu1_z as in gather_node_tile_flags, so forward and backward agree on every relu).
// a goes to tile_a[s * STRIDE + j]; cx and cp come back in registers (index = state).
template <int P, bool W = false>
__device__ __forceinline__ void gather_node_tile_flags_grad(float *tile_a, float (&cx)[16], float (&cp)[16],
                                                            const NodeInfo &ni, int s0, float t1, float qp,
                                                            const int *__restrict__ colidx, int b, int e, int lane,
                                                            float total, const float *__restrict__ wagg = nullptr) {
    constexpr int STRIDE = Geo<P>::STRIDE;
    const float rp = fmaxf(qp, 0.f);
    const float mq = qp > 0.f ? 1.f : 0.f;
    const int nb = ni.S >> 4, blk = s0 >> 4;
    float a[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) { a[s] = 0.f; cx[s] = 0.f; cp[s] = 0.f; }
    for (int base = b; base < e; base += 64) {
        const int u = (base + lane < e) ? colidx[base + lane] : -1;
        const unsigned f = u >= 0 ? (unsigned)ni.flags16[(size_t)u * nb + blk] : 0u;
        if (__ballot(f != 0u) == 0ull) continue;                     // wave-uniform
        const float *r = ni.node(u >= 0 ? u : 0);
        const float sp = f != 0u ? r[ni.sp_off] : 0.f;
        float wl = 1.f;
        if (W) wl = f != 0u ? wagg[base + lane] : 0.f;
        float xs[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) xs[s] = ((f >> s) & 1u) ? r[s0 + s] : 0.f;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            unsigned long long todo = __ballot((f >> s) & 1u);
            while (todo != 0ull) {
                const int l = __ffsll((long long)todo) - 1;
                todo &= todo - 1ull;
                const float xl = readlane_f(xs[s], l), pl = readlane_f(sp, l);
                const float z = mu1_z(xl, pl, t1, qp);
                const float m = z > 0.f ? 1.f : 0.f;
                const float wk = W ? readlane_f(wl, l) : 1.f;
                a[s] = fmaf(wk, fmaxf(z, 0.f) - pl * rp, a[s]);
                cx[s] = fmaf(wk * xl, m, cx[s]);
                cp[s] = fmaf(wk * pl, m - mq, cp[s]);
            }
        }
    }
    const float a0 = total * rp, c0 = total * mq;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        cp[s] += c0;
        if (lane < P) tile_a[s * STRIDE + lane] = a0 + a[s];
    }
}

// The neighbour sums that the LAST reversed round (t = 2) needs when it is taken from the scalars
// instead of gathering dz^2 (node mode).  With z_u = x_u theta1 + s+_u q+ + s-_u q- (the round-1
// pre-activation of neighbour u, recomputed as in gather_node_block_mu1) and m_u = [z_u > 0]:
//   a  = sum_u relu(z_u)    (the round-2 neighbour sum of mu^1: the second factor of dtheta2)
//   cx = sum_u x_u m_u,   cp = sum_u s+_u m_u,   cn = sum_u s-_u m_u
// each weighted by the edge weight when W.  NEG = false: no weight of the graph is negative, so
// s- = 0 everywhere and cn is not formed.  One running sum per quantity: callers pass at most
// kHubSegment entries (longer rows go through segments).
template <int P>
struct NodeAcc4 {
    NodeAcc<P> a, cx, cp, cn;
};

template <int P, bool W, bool SHARED, bool NEG>
__device__ __forceinline__ NodeAcc4<P> gather_node_block_mu1_grad_impl(const NodeInfo &ni, int s0,
                                                                       const float *__restrict__ theta1,
                                                                       const float *__restrict__ qvec,
                                                                       const int *__restrict__ colidx,
                                                                       const float *__restrict__ wagg, int b, int e,
                                                                       int lane, float *stage) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
    constexpr int BATCH = RecStage<SHARED>::BATCH;
    NodeAcc4<P> r;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        r.a.a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        r.cx.a[c] = r.a.a[c]; r.cp.a[c] = r.a.a[c]; r.cn.a[c] = r.a.a[c];
    }
    const int col = 4 * (lane % LPR);
    const float4 t1 = ld4(theta1 + col), qp = ld4(qvec + col), qn = ld4(qvec + P + col);
    const int q = lane / LPR;   // this lane owns states NC * q .. of the block (state-major layout)
    float ssum = 0.f;   // sum of (weight times) s+ over the neighbours with x = 0 in all states and s- = 0
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        const int cols = (lane < cnt) ? colidx[base + lane] : 0;
        float wv = 0.f;
        if (W) wv = (lane < cnt) ? wagg[base + lane] : 0.f;
        for (int j0 = 0; j0 < cnt; j0 += BATCH) {
            const int m = min(BATCH, cnt - j0);
            stage_records<SHARED>(ni, s0, cols, j0, m, lane, stage);
            __builtin_amdgcn_wave_barrier();
            for (int n = 0; n < m; ++n) {
                float xs[NC], sp[SHARED ? 1 : NC], sn[SHARED ? 1 : NC];
                read_staged<NC, SHARED>(stage, n, q, xs, sp, sn);
                const float w = W ? readlane_f(wv, j0 + n) : 1.f;
                if (SHARED) {
                    // x = 0 in all 16 states and s- = 0: z = s+ q+ in every state, so the neighbour adds
                    // s+ relu(q+) to a, s+ [q+ > 0] to cp and nothing to cx, cn
                    bool any = false;
#pragma unroll
                    for (int c = 0; c < NC; ++c) any = any || xs[c] != 0.f;
                    if (sn[0] == 0.f && __ballot(any) == 0ull) {
                        ssum += w * sp[0];
                        continue;
                    }
                }
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const float p_ = sp[SHARED ? 0 : c], n_ = NEG ? sn[SHARED ? 0 : c] : 0.f, x_ = xs[c];
                    // the forward pass's own function, so that the relu decisions agree
                    const float zx = mu1_z(x_, p_, n_, t1.x, qp.x, qn.x), zy = mu1_z(x_, p_, n_, t1.y, qp.y, qn.y);
                    const float zz = mu1_z(x_, p_, n_, t1.z, qp.z, qn.z), zw = mu1_z(x_, p_, n_, t1.w, qp.w, qn.w);
                    r.a.a[c].x = fmaf(w, fmaxf(zx, 0.f), r.a.a[c].x);
                    r.a.a[c].y = fmaf(w, fmaxf(zy, 0.f), r.a.a[c].y);
                    r.a.a[c].z = fmaf(w, fmaxf(zz, 0.f), r.a.a[c].z);
                    r.a.a[c].w = fmaf(w, fmaxf(zw, 0.f), r.a.a[c].w);
                    const float fx = zx > 0.f ? w : 0.f, fy = zy > 0.f ? w : 0.f;
                    const float fz = zz > 0.f ? w : 0.f, fw = zw > 0.f ? w : 0.f;
                    r.cx.a[c].x = fmaf(fx, x_, r.cx.a[c].x); r.cx.a[c].y = fmaf(fy, x_, r.cx.a[c].y);
                    r.cx.a[c].z = fmaf(fz, x_, r.cx.a[c].z); r.cx.a[c].w = fmaf(fw, x_, r.cx.a[c].w);
                    r.cp.a[c].x = fmaf(fx, p_, r.cp.a[c].x); r.cp.a[c].y = fmaf(fy, p_, r.cp.a[c].y);
                    r.cp.a[c].z = fmaf(fz, p_, r.cp.a[c].z); r.cp.a[c].w = fmaf(fw, p_, r.cp.a[c].w);
                    if (NEG) {
                        r.cn.a[c].x = fmaf(fx, n_, r.cn.a[c].x); r.cn.a[c].y = fmaf(fy, n_, r.cn.a[c].y);
                        r.cn.a[c].z = fmaf(fz, n_, r.cn.a[c].z); r.cn.a[c].w = fmaf(fw, n_, r.cn.a[c].w);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (SHARED) {
        const float4 ra = make_float4(ssum * fmaxf(qp.x, 0.f), ssum * fmaxf(qp.y, 0.f), ssum * fmaxf(qp.z, 0.f),
                                      ssum * fmaxf(qp.w, 0.f));
        const float4 rc = make_float4(qp.x > 0.f ? ssum : 0.f, qp.y > 0.f ? ssum : 0.f, qp.z > 0.f ? ssum : 0.f,
                                      qp.w > 0.f ? ssum : 0.f);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            r.a.a[c] = add4(r.a.a[c], ra);
            r.cp.a[c] = add4(r.cp.a[c], rc);
        }
    }
    return r;
}

template <int P, bool W, bool NEG>
__device__ __forceinline__ NodeAcc4<P> gather_node_block_mu1_grad(const NodeInfo &ni, int s0,
                                                                  const float *__restrict__ theta1,
                                                                  const float *__restrict__ qvec,
                                                                  const int *__restrict__ colidx,
                                                                  const float *__restrict__ wagg, int b, int e, int lane,
                                                                  float *stage) {
    if (ni.ss == 0)
        return gather_node_block_mu1_grad_impl<P, W, true, NEG>(ni, s0, theta1, qvec, colidx, wagg, b, e, lane, stage);
    return gather_node_block_mu1_grad_impl<P, W, false, NEG>(ni, s0, theta1, qvec, colidx, wagg, b, e, lane, stage);
}

// Row mode of the same (any S): the four sums of ONE row (v, s) over its stored entries [b, e), at this
// lane's four columns (4 * li ..).  A group of LPR lanes takes one neighbour at a time, four neighbours per
// group in flight; a wave-wide step whose neighbours all have x = 0 and s- = 0 only adds their s+ to a
// scalar (their row is s+ relu(q+), their mask [q+ > 0]).  The sums are returned complete in every group.
// cols: colidx[b + lane] of the first 64 entries when have_cols.  At most kHubSegment entries (the segments
// of the long rows are summed with this).
struct RowAcc4 {
    float4 a, cx, cp, cn;
};

template <int P, bool W, bool NEG>
__device__ __forceinline__ RowAcc4 gather_row_mu1_grad(const NodeInfo &ni, int s, float4 t1, float4 qp, float4 qn,
                                                       const int *__restrict__ colidx,
                                                       const float *__restrict__ wagg, int b, int e, int cols,
                                                       bool have_cols, int lane) {
    constexpr int NPL = Geo<P>::NPL, LPR = Geo<P>::LPR;
    const int gq = lane / LPR;
    RowAcc4 r;
    r.a = make_float4(0.f, 0.f, 0.f, 0.f);
    r.cx = r.a; r.cp = r.a; r.cn = r.a;
    float ssum = 0.f;
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        if (!(have_cols && base == b)) cols = (lane < cnt) ? colidx[base + lane] : 0;
        float wv = 0.f;
        if (W) wv = (lane < cnt) ? wagg[base + lane] : 0.f;
        const int last = cnt - 1;
        for (int s0 = 0; s0 < cnt; s0 += 4 * NPL) {
            float x_[4], p_[4], n_[4], wk[4];
            bool any = false;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                // slots past the end re-read the last neighbour with weight zero
                const int sl = s0 + gq + k * NPL;
                const int u = __shfl(cols, min(sl, last));
                if (ni.S == 1) {
                    const float4 rec = ld4(ni.base + (size_t)u * 4);
                    x_[k] = rec.x; p_[k] = rec.y; n_[k] = NEG ? rec.z : 0.f;
                } else {
                    x_[k] = ni.x(u, s); p_[k] = ni.sp(u, s); n_[k] = NEG ? ni.sn(u, s) : 0.f;
                }
                const float wl = W ? __shfl(wv, min(sl, last)) : 1.f;
                wk[k] = sl < cnt ? wl : 0.f;
                any = any || (sl < cnt && (x_[k] != 0.f || n_[k] != 0.f));
            }
            if (__ballot(any) == 0ull) {
#pragma unroll
                for (int k = 0; k < 4; ++k) ssum = fmaf(wk[k], p_[k], ssum);
                continue;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float w = wk[k];
                // the forward pass's own function, so that the relu decisions agree
                const float zx = mu1_z(x_[k], p_[k], n_[k], t1.x, qp.x, qn.x), zy = mu1_z(x_[k], p_[k], n_[k], t1.y, qp.y, qn.y);
                const float zz = mu1_z(x_[k], p_[k], n_[k], t1.z, qp.z, qn.z), zw = mu1_z(x_[k], p_[k], n_[k], t1.w, qp.w, qn.w);
                r.a.x = fmaf(w, fmaxf(zx, 0.f), r.a.x); r.a.y = fmaf(w, fmaxf(zy, 0.f), r.a.y);
                r.a.z = fmaf(w, fmaxf(zz, 0.f), r.a.z); r.a.w = fmaf(w, fmaxf(zw, 0.f), r.a.w);
                const float fx = zx > 0.f ? w : 0.f, fy = zy > 0.f ? w : 0.f;
                const float fz = zz > 0.f ? w : 0.f, fw = zw > 0.f ? w : 0.f;
                r.cx.x = fmaf(fx, x_[k], r.cx.x); r.cx.y = fmaf(fy, x_[k], r.cx.y);
                r.cx.z = fmaf(fz, x_[k], r.cx.z); r.cx.w = fmaf(fw, x_[k], r.cx.w);
                r.cp.x = fmaf(fx, p_[k], r.cp.x); r.cp.y = fmaf(fy, p_[k], r.cp.y);
                r.cp.z = fmaf(fz, p_[k], r.cp.z); r.cp.w = fmaf(fw, p_[k], r.cp.w);
                if (NEG) {
                    r.cn.x = fmaf(fx, n_[k], r.cn.x); r.cn.y = fmaf(fy, n_[k], r.cn.y);
                    r.cn.z = fmaf(fz, n_[k], r.cn.z); r.cn.w = fmaf(fw, n_[k], r.cn.w);
                }
            }
        }
    }
    // the neighbours that were summed as scalars: z = s+ q+ in every column
    r.a.x = fmaf(ssum, fmaxf(qp.x, 0.f), r.a.x); r.a.y = fmaf(ssum, fmaxf(qp.y, 0.f), r.a.y);
    r.a.z = fmaf(ssum, fmaxf(qp.z, 0.f), r.a.z); r.a.w = fmaf(ssum, fmaxf(qp.w, 0.f), r.a.w);
    r.cp.x += qp.x > 0.f ? ssum : 0.f; r.cp.y += qp.y > 0.f ? ssum : 0.f;
    r.cp.z += qp.z > 0.f ? ssum : 0.f; r.cp.w += qp.w > 0.f ? ssum : 0.f;
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
        r.a.x += __shfl_xor(r.a.x, m); r.a.y += __shfl_xor(r.a.y, m);
        r.a.z += __shfl_xor(r.a.z, m); r.a.w += __shfl_xor(r.a.w, m);
        r.cx.x += __shfl_xor(r.cx.x, m); r.cx.y += __shfl_xor(r.cx.y, m);
        r.cx.z += __shfl_xor(r.cx.z, m); r.cx.w += __shfl_xor(r.cx.w, m);
        r.cp.x += __shfl_xor(r.cp.x, m); r.cp.y += __shfl_xor(r.cp.y, m);
        r.cp.z += __shfl_xor(r.cp.z, m); r.cp.w += __shfl_xor(r.cp.w, m);
        if (NEG) {
            r.cn.x += __shfl_xor(r.cn.x, m); r.cn.y += __shfl_xor(r.cn.y, m);
            r.cn.z += __shfl_xor(r.cn.z, m); r.cn.w += __shfl_xor(r.cn.w, m);
        }
    }
    return r;
}

// The same sums for the 16 rows (v_i, s_i) of a row-mode tile at once, one LANE per stored entry: the column
// indices of eight rows are requested together, then the records of all their neighbours, so a tile costs a
// few trips to memory instead of two per row.  Neighbours with x = 0 and s- = 0 add their s+ to a scalar of
// their row; the others are visited one at a time with lane j forming column j = lane % P.  Row i's sum `a`
// goes to tile_a[i]; its cx, cp, cn meet row i of tile_e (e = dz^2 theta2) right away:
//   fx += e[i][j] cx_i[j],  fp += e[i][j] cp_i[j],  fn += e[i][j] cn_i[j].
// rb, re, s: lane i (mod 16) holds the range and the state of tile row i; rows longer than max_len are left
// to the caller.  t1, qp, qn: theta1, q+, q- at column j.
template <int P, bool W, bool NEG>
__device__ __forceinline__ void gather_tile_mu1_grad_rows(float *tile_a, const float *tile_e, const NodeInfo &ni,
                                                          int s, float t1, float qp, float qn,
                                                          const int *__restrict__ colidx,
                                                          const float *__restrict__ wagg, int rb, int re, int max_len,
                                                          int lane, float &fx, float &fp, float &fn) {
    constexpr int STRIDE = Geo<P>::STRIDE;
    const int j = lane % P;
    const float rp = fmaxf(qp, 0.f), mq = qp > 0.f ? 1.f : 0.f;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        float ssum[8], a[8], cx[8], cp[8], cn[NEG ? 8 : 1];
        int nlev = 0;   // chunk levels of the longest row of this half that is gathered here (wave-uniform)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            ssum[k] = 0.f; a[k] = 0.f; cx[k] = 0.f; cp[k] = 0.f; cn[NEG ? k : 0] = 0.f;
            const int n = __builtin_amdgcn_readlane(re, 8 * half + k) - __builtin_amdgcn_readlane(rb, 8 * half + k);
            if (n <= max_len) nlev = max(nlev, (n + 63) >> 6);
        }
#pragma unroll 1
        for (int lev = 0; lev < nlev; ++lev) {
            int cols[8];
            float wl[W ? 8 : 1];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int b = __builtin_amdgcn_readlane(rb, 8 * half + k), n = __builtin_amdgcn_readlane(re, 8 * half + k) - b;
                const int i = 64 * lev + lane;
                const bool ok = n <= max_len && i < n;
                cols[k] = ok ? colidx[b + i] : -1;
                if (W) wl[W ? k : 0] = ok ? wagg[b + i] : 0.f;
            }
            float rx[8], rs[8], rn[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int sk = __builtin_amdgcn_readlane(s, 8 * half + k);
                rx[k] = 0.f; rs[k] = 0.f; rn[k] = 0.f;
                if (cols[k] >= 0) {
                    if (ni.S == 1) {
                        const float4 r = ld4(ni.base + (size_t)cols[k] * 4);
                        rx[k] = r.x; rs[k] = r.y; rn[k] = NEG ? r.z : 0.f;
                    } else {
                        rx[k] = ni.x(cols[k], sk); rs[k] = ni.sp(cols[k], sk);
                        rn[k] = NEG ? ni.sn(cols[k], sk) : 0.f;
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool cheap = rx[k] == 0.f && rn[k] == 0.f;
                ssum[k] += cheap ? (W ? wl[W ? k : 0] * rs[k] : rs[k]) : 0.f;
                unsigned long long todo = __ballot(!cheap);
                while (todo != 0ull) {
                    const int l = __ffsll((long long)todo) - 1;
                    todo &= todo - 1ull;
                    const float xl = readlane_f(rx[k], l), pl = readlane_f(rs[k], l);
                    const float nl = NEG ? readlane_f(rn[k], l) : 0.f;
                    const float w = W ? readlane_f(wl[W ? k : 0], l) : 1.f;
                    // the forward pass's own function, so that the relu decisions agree
                    const float z = NEG ? mu1_z(xl, pl, nl, t1, qp, qn) : mu1_z(xl, pl, t1, qp);
                    const float m = z > 0.f ? w : 0.f;
                    a[k] = fmaf(w, fmaxf(z, 0.f), a[k]);
                    cx[k] = fmaf(m, xl, cx[k]);
                    cp[k] = fmaf(m, pl, cp[k]);
                    if (NEG) cn[k] = fmaf(m, nl, cn[k]);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = 8 * half + k;
            if (__builtin_amdgcn_readlane(re, i) - __builtin_amdgcn_readlane(rb, i) > max_len) continue;   // wave-uniform
            float sv = ssum[k];
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) sv += __shfl_xor(sv, m);
            const float ev = tile_e[i * STRIDE + j];
            if (lane < P) tile_a[i * STRIDE + lane] = fmaf(sv, rp, a[k]);
            fx = fmaf(ev, cx[k], fx);
            fp = fmaf(ev, fmaf(sv, mq, cp[k]), fp);
            if (NEG) fn = fmaf(ev, cn[NEG ? k : 0], fn);
        }
    }
}

// Row mode of the mask-word gather for a whole tile, one LANE per stored entry (as gather_tile_mu1_grad_rows):
// for each of the 16 rows (v_i, s_i), per column j = lane % P, the number of neighbours u whose relu-mask
// word (u, s_i) has bit j set (W: the sum of their edge weights), times scale_i[j] when the row is inside its
// state's graph (lane i (mod 16) holds in_graph for tile row i) and zero otherwise; written to tile[i][j].
// scale(s, j): the per-state factor.  Rows longer than max_len are left to the caller.
template <int P, bool W, class Scale>
__device__ __forceinline__ void gather_tile_bits_rows(float *tile, const unsigned long long *__restrict__ mask, int S,
                                                      int s, bool in_graph, const Scale &scale,
                                                      const int *__restrict__ colidx, const float *__restrict__ wagg,
                                                      int rb, int re, int max_len, int lane) {
    constexpr int STRIDE = Geo<P>::STRIDE;
    const int j = lane % P;
    const bool hi_half = j >= 32;
    const int sh = j & 31;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        float cnt[8];
        int nlev = 0;   // chunk levels of the longest row of this half that is gathered here (wave-uniform)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            cnt[k] = 0.f;
            const int n = __builtin_amdgcn_readlane(re, 8 * half + k) - __builtin_amdgcn_readlane(rb, 8 * half + k);
            if (n <= max_len) nlev = max(nlev, (n + 63) >> 6);
        }
#pragma unroll 1
        for (int lev = 0; lev < nlev; ++lev) {
            int cols[8];
            float wl[W ? 8 : 1];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int b = __builtin_amdgcn_readlane(rb, 8 * half + k), n = __builtin_amdgcn_readlane(re, 8 * half + k) - b;
                const int i = 64 * lev + lane;
                const bool ok = n <= max_len && i < n;
                cols[k] = ok ? colidx[b + i] : -1;
                if (W) wl[W ? k : 0] = ok ? wagg[b + i] : 0.f;
            }
            unsigned lo[8], hi[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int sk = __builtin_amdgcn_readlane(s, 8 * half + k);
                const unsigned long long wd = cols[k] >= 0 ? mask[(size_t)cols[k] * S + sk] : 0ull;
                lo[k] = (unsigned)wd;
                hi[k] = (unsigned)(wd >> 32);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                unsigned long long todo = __ballot((lo[k] | hi[k]) != 0u);
                while (todo != 0ull) {
                    const int l = __ffsll((long long)todo) - 1;
                    todo &= todo - 1ull;
                    const unsigned wlo = (unsigned)__builtin_amdgcn_readlane((int)lo[k], l);
                    const unsigned whi = (unsigned)__builtin_amdgcn_readlane((int)hi[k], l);
                    const unsigned bit = ((hi_half ? whi : wlo) >> sh) & 1u;
                    if (W) cnt[k] = fmaf((float)bit, readlane_f(wl[W ? k : 0], l), cnt[k]);
                    else cnt[k] += (float)bit;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = 8 * half + k;
            if (__builtin_amdgcn_readlane(re, i) - __builtin_amdgcn_readlane(rb, i) > max_len) continue;   // wave-uniform
            const bool ing = __builtin_amdgcn_readlane((int)in_graph, i) != 0;
            const int si = __builtin_amdgcn_readlane(s, i);
            if (lane < P) tile[i * STRIDE + lane] = ing ? cnt[k] * scale(si, j) : 0.f;
        }
    }
}

// Weighted form of gather_node_block_bits: per column, the sum of the weights of the neighbours whose
// entry is positive (per-chunk accumulators folded into a running total, as in the other gathers).
template <int P>
__device__ __forceinline__ NodeAcc<P> gather_node_block_bits_w(const unsigned long long *__restrict__ mask, int S,
                                                               int s0, const int *__restrict__ colidx,
                                                               const float *__restrict__ wagg, int b, int e, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
    NodeAcc<P> total, acc;
#pragma unroll
    for (int c = 0; c < NC; ++c) total.a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int shift = 4 * (lane % LPR);
    const int srow = s0 + lane / LPR;
    for (int base = b; base < e; base += 64) {
        const int n = min(64, e - base);
        const int cols = (lane < n) ? colidx[base + lane] : 0;
        const float wv = (lane < n) ? wagg[base + lane] : 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) acc.a[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < n; j += 4) {
            unsigned nib[4][NC];
            float wk[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int jj = min(j + k, n - 1);   // past the end: re-read the last word, weight 0 below
                const unsigned long long *w = mask + (size_t)__builtin_amdgcn_readlane(cols, jj) * S + srow;
                wk[k] = (j + k < n) ? readlane_f(wv, jj) : 0.f;
#pragma unroll
                for (int c = 0; c < NC; ++c) nib[k][c] = (unsigned)(w[c * RPI] >> shift);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const unsigned b4 = nib[k][c];
                    acc.a[c].x += (b4 & 1u) ? wk[k] : 0.f;
                    acc.a[c].y += (b4 & 2u) ? wk[k] : 0.f;
                    acc.a[c].z += (b4 & 4u) ? wk[k] : 0.f;
                    acc.a[c].w += (b4 & 8u) ? wk[k] : 0.f;
                }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) total.a[c] = add4(total.a[c], acc.a[c]);
    }
    return total;
}

// `stage` is wave-private LDS of at least kBitsStageBytes bytes.  The words of up to 32 neighbours
// are fetched at once (one wave-wide load brings the 16 consecutive state words of 4 neighbours),
// parked in `stage`, and each lane then counts its four columns for its NC states; counts are
// integers, so the order of the neighbours does not matter.
constexpr int kBitsStageBytes = 32 * 16 * 8;

template <int P>
__device__ __forceinline__ NodeAcc<P> gather_node_block_bits(const unsigned long long *__restrict__ mask, int S, int s0,
                                                             const int *__restrict__ colidx, int b, int e, int lane,
                                                             unsigned *stage, int cols0 = 0, bool have_cols0 = false,
                                                             const unsigned long long *words0 = nullptr) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
    int4 cnt[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) cnt[c] = make_int4(0, 0, 0, 0);
    const int shift = 4 * (lane % LPR);
    const int srow = lane / LPR;                 // this lane's state within a block of RPI states
    const int q = lane >> 4, st = lane & 15;     // load role: neighbour slot, state
    const int half = shift >> 5, sh = shift & 31;
    for (int base = b; base < e; base += 64) {
        const int n = min(64, e - base);
        // cols0: colidx[b + lane] of the first chunk, fetched by the caller ahead of time
        const int cols = (have_cols0 && base == b) ? cols0 : ((lane < n) ? colidx[base + lane] : 0);
        for (int j0 = 0; j0 < n; j0 += 32) {
            const int m = min(32, n - j0);       // neighbours in this batch
            unsigned long long wv[8];
            if (words0 && base == b && j0 == 0) {
                // words0: this first batch, fetched by the caller ahead of time in this very layout
#pragma unroll
                for (int k = 0; k < 8; ++k) wv[k] = words0[k];
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int jj = j0 + min(4 * k + q, m - 1);   // past the end: a valid word again, never counted
                    wv[k] = mask[(size_t)__shfl(cols, jj) * S + s0 + st];
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                stage[((4 * k + q) * 16 + st) * 2] = (unsigned)wv[k];
                stage[((4 * k + q) * 16 + st) * 2 + 1] = (unsigned)(wv[k] >> 32);
            }
            __builtin_amdgcn_wave_barrier();
            // four columns of one state packed as four byte counters (at most 32 per batch)
            unsigned packed[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) packed[c] = 0u;
            // (four neighbours per step, their LDS reads in flight together; the staging area holds 32 slots,
            //  and a slot past the last neighbour is read but not counted)
            for (int i = 0; i < m; i += 4) {
                unsigned w32[4][NC];
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < NC; ++c) w32[k][c] = stage[(((i + k) * 16) + c * RPI + srow) * 2 + half];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const unsigned live = i + k < m ? 0xFu : 0u;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const unsigned nib = (w32[k][c] >> sh) & live;
                        // bit t of the nibble -> bit 8 * t
                        packed[c] += __umul24(nib, 0x00204081u) & 0x01010101u;
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                cnt[c].x += (int)(packed[c] & 0xFFu);
                cnt[c].y += (int)((packed[c] >> 8) & 0xFFu);
                cnt[c].z += (int)((packed[c] >> 16) & 0xFFu);
                cnt[c].w += (int)(packed[c] >> 24);
            }
        }
    }
    NodeAcc<P> acc;
#pragma unroll
    for (int c = 0; c < NC; ++c)
        acc.a[c] = make_float4((float)cnt[c].x, (float)cnt[c].y, (float)cnt[c].z, (float)cnt[c].w);
    return acc;
}

// A segment of a long row for ONE state, round 2 (neighbour rows recomputed from the records): one LANE per
// neighbour, and the loads of the whole segment (at most 512 entries: eight per lane) issued together -- the column
// indices, then the records -- so the segment costs two trips to memory instead of two per 64 entries.  Neighbours
// with x = 0 and s- = 0 are summed as scalars (their row is s+ relu(q+)); the others are visited one at a time with
// lane j forming column j.  Returns column lane % P of the segment's sum.
template <int P, bool W>
__device__ __forceinline__ float gather_segment_mu1_lanes(const float *__restrict__ rec, float t1j, float qpj, float qnj,
                                                          const int *__restrict__ colidx, const float *__restrict__ wagg,
                                                          int b, int e, int lane) {
    constexpr int U = 8;
    const float rpj = fmaxf(qpj, 0.f);
    float ssum = 0.f, acc = 0.f;
    for (int base = b; base < e; base += 64 * U) {
        int c[U];
        float wv[W ? U : 1];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = base + 64 * u + lane;
            c[u] = i < e ? colidx[i] : -1;
            if (W) wv[W ? u : 0] = i < e ? wagg[i] : 0.f;
        }
        float4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = c[u] >= 0 ? ld4(rec + (size_t)c[u] * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool cheap = r[u].x == 0.f && r[u].z == 0.f;   // (a missing neighbour: all zeros, adds nothing)
            const float wl = W ? wv[W ? u : 0] : 1.f;
            ssum += cheap ? wl * r[u].y : 0.f;
            unsigned long long todo = __ballot(!cheap);
            while (todo != 0ull) {
                const int l = __ffsll((long long)todo) - 1;
                todo &= todo - 1ull;
                const float xl = readlane_f(r[u].x, l), pl = readlane_f(r[u].y, l), nl = readlane_f(r[u].z, l);
                const float m1 = fmaxf(mu1_z(xl, pl, nl, t1j, qpj, qnj), 0.f);
                if (W) acc = fmaf(readlane_f(wl, l), m1, acc);
                else acc += m1;
            }
        }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) ssum += __shfl_xor(ssum, m);
    return fmaf(ssum, rpj, acc);
}

// Index of node v among the long rows (v is known to be one): one load from the per-node table.
__device__ __forceinline__ int hub_index(const HubTable &ht, int v) { return ht.hub_of[v]; }

// A node-mode block read back from the hub sums instead of gathered.
template <int P>
__device__ __forceinline__ NodeAcc<P> load_node_block(const float *__restrict__ blk, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI;
    NodeAcc<P> acc;
#pragma unroll
    for (int c = 0; c < NC; ++c) acc.a[c] = ld4(blk + c * RPI * P + 4 * lane);
    return acc;
}

// Park a node-mode accumulator in the wave's LDS tile (row stride Geo<P>::STRIDE).
template <int P>
__device__ __forceinline__ void store_node_block(float *tile, const NodeAcc<P> &acc, int lane) {
    constexpr int RPI = Geo<P>::NPL, NC = 16 / RPI, LPR = Geo<P>::LPR;
#pragma unroll
    for (int c = 0; c < NC; ++c) st4(tile + (c * RPI + lane / LPR) * Geo<P>::STRIDE + 4 * (lane % LPR), acc.a[c]);
}

// The matrix-core product used everywhere:  D[i][j] = sum_k A[i][k] * B[j][k]  for a 16 x P
// tile A and a P x P matrix B, with v_mfma_f32_16x16x4_f32.  Operand layout of that
// instruction: lane l supplies A[l%16][k = l/16] and B[k = l/16][l%16]; it receives
// D[4*(l/16) + r][l%16] in result register r.  The k index is only summed over, so step ks
// lets lane group g = l/16 work on k = g*KS + ks: each lane then needs KS consecutive floats
// of "its" A row and of "its" B row, which are plain float4 loads.
template <int P>
struct Frag {
    float v[Geo<P>::KS];
};

// A-fragment of one wave's 16 x P tile held in LDS (row stride Geo<P>::STRIDE).
template <int P>
__device__ __forceinline__ Frag<P> load_a_frag_lds(const float *tile, int lane) {
    constexpr int KS = Geo<P>::KS;
    Frag<P> f;
    const float *row = tile + (lane & 15) * Geo<P>::STRIDE + (lane >> 4) * KS;
#pragma unroll
    for (int c = 0; c < KS / 4; ++c) {
        const float4 t = ld4(row + 4 * c);
        f.v[4 * c] = t.x; f.v[4 * c + 1] = t.y; f.v[4 * c + 2] = t.z; f.v[4 * c + 3] = t.w;
    }
    return f;
}

// B-fragments for column block cb of D = A * M^T, M row-major [P][P] (B[j][k] = M[j][k]).
template <int P>
__device__ __forceinline__ Frag<P> load_b_frag_rows(const float *__restrict__ m, int cb, int lane) {
    constexpr int KS = Geo<P>::KS;
    Frag<P> f;
    const float *row = m + (size_t)(16 * cb + (lane & 15)) * P + (lane >> 4) * KS;
#pragma unroll
    for (int c = 0; c < KS / 4; ++c) {
        const float4 t = ld4(row + 4 * c);
        f.v[4 * c] = t.x; f.v[4 * c + 1] = t.y; f.v[4 * c + 2] = t.z; f.v[4 * c + 3] = t.w;
    }
    return f;
}

// The P x P matrix M staged in LDS (row stride Geo<P>::STRIDE) by the whole workgroup; call
// __syncthreads() afterwards.  transpose = false keeps M[j][k]; true stores M[k][j] at [j][k], so
// that in both cases B-fragments are contiguous float4 reads of "row j".
template <int P>
__device__ __forceinline__ void stage_matrix_lds(float *dst, const float *__restrict__ m, bool transpose) {
    constexpr int STRIDE = Geo<P>::STRIDE;
    if (!transpose) {
        for (int f = threadIdx.x; f < P * P / 4; f += blockDim.x) {
            const int r = f / (P / 4), c4 = f % (P / 4);
            st4(dst + r * STRIDE + 4 * c4, ld4(m + r * P + 4 * c4));
        }
    } else {
        for (int f = threadIdx.x; f < P * P; f += blockDim.x) {
            const int k = f / P, j = f % P;
            dst[j * STRIDE + k] = m[f];
        }
    }
}

// B-fragment of column block cb from a matrix staged by stage_matrix_lds.
template <int P>
__device__ __forceinline__ Frag<P> load_b_frag_lds(const float *mat, int cb, int lane) {
    constexpr int KS = Geo<P>::KS;
    Frag<P> f;
    const float *row = mat + (16 * cb + (lane & 15)) * Geo<P>::STRIDE + (lane >> 4) * KS;
#pragma unroll
    for (int c = 0; c < KS / 4; ++c) {
        const float4 t = ld4(row + 4 * c);
        f.v[4 * c] = t.x; f.v[4 * c + 1] = t.y; f.v[4 * c + 2] = t.z; f.v[4 * c + 3] = t.w;
    }
    return f;
}

template <int P>
__device__ __forceinline__ f32x4 mfma_tile(const Frag<P> &a, const Frag<P> &b, f32x4 acc) {
#pragma unroll
    for (int ks = 0; ks < Geo<P>::KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[ks], b.v[ks], acc, 0, 0, 0);
    return acc;
}

}  // namespace s2v
