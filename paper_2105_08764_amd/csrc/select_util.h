// The selection rule shared by every kernel that picks nodes: candidates, the order-preserving key of a
// float32 score, and "better" = higher score, lower node index among equal scores (Alg. 3 line 7, Sec. 4.5.1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2v {

__device__ __forceinline__ bool is_candidate(const float *__restrict__ x, const uint8_t *__restrict__ cand, int v) {
    return cand ? (cand[v] != 0) : (x[v] == 0.f);
}

// Order-preserving map float -> uint32 (larger score = larger key); -0.0 is folded onto +0.0.
__device__ __forceinline__ uint32_t score_key(float q) {
    const uint32_t b = __float_as_uint(q + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_score(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// (val, idx) beats (val2, idx2) if the score is higher, or equal with a lower node index.
__device__ __forceinline__ void take_better(float &val, int &idx, float val2, int idx2) {
    if (val2 > val || (val2 == val && idx2 < idx)) { val = val2; idx = idx2; }
}

__device__ __forceinline__ bool beats(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

}  // namespace s2v
