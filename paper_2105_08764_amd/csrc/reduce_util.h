// Reductions shared by stand-alone kernels and by kernels that fuse them: the second stage of the graph sum
// (Alg. 2 line 4) and the graph term of Eq. 2.  One body each, so that a fused launch gives the same bits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2v {

// Column `col` of the sum of the partial rows [rb, re) of a [rows][L] float matrix.  Called by all 1024 threads
// of a workgroup: thread = (row lane rl = tid / 16, column tid % 16 of a block of 16 columns); the row lanes
// take rows round-robin (double accumulators, four loads in flight each) and are added in lane order.
// The result is valid in the threads with rl == 0.  red: LDS, double [64][17].
__device__ __forceinline__ double gsum_stage2_cols(int L, int col, int rb, int re, const float *__restrict__ partial,
                                                   double (*red)[17]) {
    const int rl = threadIdx.x >> 4;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    int c = rb + rl;
    for (; c + 192 < re; c += 256) {
        const float v0 = partial[(size_t)c * L + col], v1 = partial[(size_t)(c + 64) * L + col];
        const float v2 = partial[(size_t)(c + 128) * L + col], v3 = partial[(size_t)(c + 192) * L + col];
        a0 += (double)v0; a1 += (double)v1; a2 += (double)v2; a3 += (double)v3;
    }
    for (; c < re; c += 64) a0 += (double)partial[(size_t)c * L + col];
    red[rl][threadIdx.x & 15] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    double acc = 0.0;
    if (rl == 0)
        for (int k = 0; k < 64; ++k) acc += red[k][threadIdx.x];
    __syncthreads();
    return acc;
}

// theta5[0:p] . relu(theta6 g) for the p-vector g (global or LDS), by the first 128 threads of a workgroup of
// at least 128 threads (all threads must call).  gs, red: LDS, 128 floats each.  Returned to every thread.
__device__ __forceinline__ float qa_value(int p, const float *__restrict__ theta5, const float *__restrict__ theta6,
                                          const float *g, float *gs, float *red) {
    const int i = threadIdx.x;
    if (i < p) gs[i] = g[i];
    __syncthreads();
    float term = 0.f;
    if (i < p) {
        // (double accumulation: p^2 operations per graph, and each of these p relu units carries 1/p of a
        //  state's whole gradient in training)
        double h = 0.0;
        for (int j = 0; j < p; ++j) h += (double)theta6[i * p + j] * (double)gs[j];
        term = theta5[i] * fmaxf((float)h, 0.f);
    }
    if (i < 128) red[i] = term;
    __syncthreads();
    for (int w = 64; w >= 1; w >>= 1) {
        if (i < w) red[i] += red[i + w];
        __syncthreads();
    }
    const float out = red[0];
    __syncthreads();
    return out;
}

}  // namespace s2v
