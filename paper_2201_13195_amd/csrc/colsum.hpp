// Column sums of a row-major matrix, out[c] = sum_r A[r][c] (+ the old out[c]): the bias gradient
// db = dY^T 1 (Eq. 3).  One pass over A, bound by HBM.  Device body shared by the kernel of its own
// (plain.hip) and the launch it shares with dW = G^T X_proj (mfma.hip).
//
// A work-group owns LPR x 16 bytes of every row (LPR = 4: 32 bf16 or 16 fp32 columns): thread t
// (of the first 256) takes 16 bytes of rows t / LPR, t / LPR + 256 / LPR, ..., eight loads in
// flight, and keeps fp32 sums of its 8 (4) columns; the row groups of a column are then added
// through LDS in fixed order.  Column blocks that share a 128-byte line of A are numbered onto one
// XCD (work-groups are dealt round-robin to the 8 XCDs, each with its own L2), so HBM sees every
// line once.  Narrow matrices take one 16-byte piece per work-group, so that enough work-groups
// exist to pull the matrix in.  The result does not depend on the size of the work-group that runs
// the body (threads beyond the first 256 only take part in the barrier).
#pragma once
#include "common.hpp"

namespace rmm {

struct ColsumArgs {
    const void *A;  // n x d, 16-byte aligned, d a multiple of 16 bytes
    void *out;      // d
    int64_t n, d;
    int accumulate;
    int lpr;        // 16-byte pieces of a row per work-group: 4 or 1 (colsum_lpr)
};

// 16-byte pieces per row and work-group: four where that still gives 96 work-groups, else one
// (measured at 16384 x 1024 bf16: 15 us with one, 21 with two, 41 with four).
inline int colsum_lpr(int64_t d, int64_t elem_bytes) { return d * elem_bytes / 16 >= 384 ? 4 : 1; }
inline int64_t colsum_blocks(int64_t d, int64_t elem_bytes) {
    const int64_t vecs = d * elem_bytes / 16, lpr = colsum_lpr(d, elem_bytes);
    return (vecs + lpr - 1) / lpr;
}
inline bool colsum_wide_ok(const void *A, int64_t d, int64_t elem_bytes) {  // 16-byte loads apply
    return (d * elem_bytes) % 16 == 0 && (reinterpret_cast<uintptr_t>(A) & 15u) == 0;
}
constexpr int kColsumLdsFloats = 256 * 9;  // 256 row groups x (8 columns + 1), the larger of the two forms

// `lds` holds kColsumLdsFloats floats; block `blk` of `blocks`.
template <typename T>
__device__ __forceinline__ void colsum_body(const ColsumArgs &g, float *lds, int64_t blk, int64_t blocks) {
    constexpr int VEC = 16 / (int)sizeof(T), U = 8;
    const T *A = reinterpret_cast<const T *>(g.A);
    T *out = reinterpret_cast<T *>(g.out);
    const int tid = threadIdx.x, LPR = g.lpr, BC = VEC * LPR, RPP = 256 / LPR, PITCH = BC + 1;
    {
        const int64_t per = blocks / 8, rem = blocks % 8, x = blk % 8, r = blk / 8;
        blk = x * per + (x < rem ? x : rem) + r;
    }
    if (tid < 256) {
        const int cq = tid % LPR, rg = tid / LPR;
        const int64_t c = blk * BC + cq * VEC;
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
        if (c < g.d) {
            for (int64_t r0 = rg; r0 < g.n; r0 += (int64_t)RPP * U) {
                uint4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (r0 + u * RPP < g.n) v[u] = *reinterpret_cast<const uint4 *>(A + (r0 + u * RPP) * g.d + c);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (r0 + u * RPP >= g.n) break;
                    const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if constexpr (sizeof(T) == 2) {
                            acc[2 * q] += __uint_as_float(w[q] << 16);
                            acc[2 * q + 1] += __uint_as_float(w[q] & 0xFFFF0000u);
                        } else {
                            acc[q] += __uint_as_float(w[q]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) lds[rg * PITCH + cq * VEC + e] = acc[e];
    }
    __syncthreads();
    const int64_t col = blk * BC + tid;
    if (tid < BC && col < g.d) {
        float s = 0.0f;
        for (int r = 0; r < RPP; ++r) s += lds[r * PITCH + tid];
        if (g.accumulate) s += load_f32<T>(out + col);
        store_f32<T>(out + col, s);
    }
}

}  // namespace rmm
