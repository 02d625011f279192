// Device-side building blocks shared by the embedding kernels (forward and backward):
// the wave-level neighbour gather and the 16 x P by P x P product on the matrix cores.
#pragma once
#include <hip/hip_runtime.h>

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

// Sum over the stored entries [b, e) of one CSR row of the P-float rows src[col * row_stride + col_off ..].
// All 64 lanes take part: lane = (group gq, lane-in-row li); col_off already includes 4 * li.
// `cols` holds colidx[b + lane] for the first (up to) 64 entries, loaded by the caller ahead of time.
// Returns the full row sum in every group (lanes with equal li hold equal values).
template <int P>
__device__ __forceinline__ float4 gather_row_sum(const float *__restrict__ src, size_t row_stride, size_t col_off,
                                                 const int *__restrict__ colidx, int b, int e, int cols, int lane) {
    constexpr int NPL = Geo<P>::NPL, LPR = Geo<P>::LPR;
    const int gq = lane / LPR;
    float4 a0 = make_float4(0.f, 0.f, 0.f, 0.f), a1 = a0, a2 = a0, a3 = a0;
    for (int base = b; base < e; base += 64) {
        const int cnt = min(64, e - base);
        if (base != b) cols = (lane < cnt) ? colidx[base + lane] : 0;
        const int last = cnt - 1;
        for (int s0 = 0; s0 < cnt; s0 += 4 * NPL) {
            // Four independent loads per lane; slots past the end re-read the last valid row
            // (same cache line as a live lane, so no extra traffic) and are dropped below.
            const int sl0 = s0 + gq, sl1 = sl0 + NPL, sl2 = sl1 + NPL, sl3 = sl2 + NPL;
            const int u0 = __shfl(cols, min(sl0, last));
            const int u1 = __shfl(cols, min(sl1, last));
            const int u2 = __shfl(cols, min(sl2, last));
            const int u3 = __shfl(cols, min(sl3, last));
            const float4 v0 = ld4(src + (size_t)u0 * row_stride + col_off);
            const float4 v1 = ld4(src + (size_t)u1 * row_stride + col_off);
            const float4 v2 = ld4(src + (size_t)u2 * row_stride + col_off);
            const float4 v3 = ld4(src + (size_t)u3 * row_stride + col_off);
            if (sl0 < cnt) a0 = add4(a0, v0);
            if (sl1 < cnt) a1 = add4(a1, v1);
            if (sl2 < cnt) a2 = add4(a2, v2);
            if (sl3 < cnt) a3 = add4(a3, v3);
        }
    }
    a0 = add4(add4(a0, a1), add4(a2, a3));
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
        a0.x += __shfl_xor(a0.x, m);
        a0.y += __shfl_xor(a0.y, m);
        a0.z += __shfl_xor(a0.z, m);
        a0.w += __shfl_xor(a0.w, m);
    }
    return a0;
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

// A-fragment straight from a row-major [rows][P] matrix in global memory; rows past n_rows read as zero.
template <int P>
__device__ __forceinline__ Frag<P> load_a_frag_global(const float *__restrict__ m, long row0, long n_rows, int lane) {
    constexpr int KS = Geo<P>::KS;
    Frag<P> f;
    const long r = row0 + (lane & 15);
    if (r < n_rows) {
        const float *row = m + (size_t)r * P + (lane >> 4) * KS;
#pragma unroll
        for (int c = 0; c < KS / 4; ++c) {
            const float4 t = ld4(row + 4 * c);
            f.v[4 * c] = t.x; f.v[4 * c + 1] = t.y; f.v[4 * c + 2] = t.z; f.v[4 * c + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < KS; ++c) f.v[c] = 0.f;
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

// B-fragments for column block cb of D = A * M, M row-major [P][P] (B[j][k] = M[k][j]).
template <int P>
__device__ __forceinline__ Frag<P> load_b_frag_cols(const float *__restrict__ m, int cb, int lane) {
    constexpr int KS = Geo<P>::KS;
    Frag<P> f;
    const float *col = m + (size_t)((lane >> 4) * KS) * P + 16 * cb + (lane & 15);
#pragma unroll
    for (int c = 0; c < KS; ++c) f.v[c] = col[(size_t)c * P];
    return f;
}

template <int P>
__device__ __forceinline__ f32x4 mfma_tile(const Frag<P> &a, const Frag<P> &b, f32x4 acc) {
#pragma unroll
    for (int ks = 0; ks < Geo<P>::KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[ks], b.v[ks], acc, 0, 0, 0);
    return acc;
}

}  // namespace s2v
