// Plain LDS-tiled fp32-FMA kernels.
//
// These carry the fp32 data path of the layer (Algorithm 1 of the paper with
// every product accumulated in fp32 and the sketch generated with full-precision
// logf / sincospif), the bias-gradient column sum (Eq. 3), and the generator
// test hooks.  They are written for clarity: one 64x64 output tile per 256-thread
// work-group, 4x4 outputs per thread, operands staged through LDS 16 contraction
// steps at a time.  The bf16 hot path lives in the MFMA kernels.
#include "colsum.hpp"

namespace rmm {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T>
struct MemSrc {
    const T *p;
    int64_t s_outer, s_inner;  // element (r, c) of the logical operand at p[r*s_outer + c*s_inner]
    __device__ float at(int64_t r, int64_t c) const { return load_f32<T>(p + r * s_outer + c * s_inner); }
};

// Logical operand P^T: element (j, i) = P[i][j].
struct SketchSrc {
    int kind;
    SketchState st;
    __device__ float at(int64_t j, int64_t i) const { return sketch_entry_precise(kind, st, i, j); }
};

// The TM x TK tile of an operand (rows m0 .., contraction k0 .., k0 a multiple of TK) into LDS,
// zeros beyond the operand.
template <typename T>
__device__ __forceinline__ void fill_a_tile(const MemSrc<T> &A, float (&As)[TK][TM + 4], int64_t m0, int64_t k0, int64_t m,
                                            int64_t kk, int tid) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int e = tid + 256 * q, kl = e & 15, rl = e >> 4;
        As[kl][rl] = (m0 + rl < m && k0 + kl < kk) ? A.at(m0 + rl, k0 + kl) : 0.0f;
    }
}
// The same for P^T, with one Philox call serving all the entries it covers in the tile instead of
// one call per entry: a Gaussian call covers 8 consecutive tokens of a column (two calls per
// column and tile), a Rademacher call 128 (the tile's 16 tokens lie inside one call), and the
// SORS kind needs the tile's sign words once and one row number per column.  Values are those of
// sketch_entry_precise.
__device__ __forceinline__ void fill_a_tile(const SketchSrc &A, float (&As)[TK][TM + 4], int64_t m0, int64_t k0, int64_t m,
                                            int64_t kk, int tid) {
    static_assert(TK == 16 && TM == 64, "two 8-token groups per column, 64 columns");
    const SketchState &st = A.st;
    if (A.kind == 0) {
        if (tid < 2 * TM) {
            const int col = tid >> 1, grp = tid & 1;
            const int64_t j = m0 + col, t0 = k0 + 8 * grp;
            const Words4 r = philox4x32_10((uint32_t)(t0 >> 3), (uint32_t)j, st.off0, st.off1, st.key0, st.key1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float zc, zs;
                gauss_pair_precise(r.w[q], zc, zs);
                As[8 * grp + 2 * q][col] = (j < m && t0 + 2 * q < kk) ? zc : 0.0f;
                As[8 * grp + 2 * q + 1][col] = (j < m && t0 + 2 * q + 1 < kk) ? zs : 0.0f;
            }
        }
        return;
    }
    if (tid < TM) {
        const int col = tid;
        const int64_t j = m0 + col;
        const uint32_t t = (uint32_t)(k0 & 127), word = t >> 5, shift = t & 31;  // the 16 tokens share one word
        uint32_t bits, row = 0;
        if (A.kind == 1) {
            const Words4 r = philox4x32_10((uint32_t)(k0 >> 7), (uint32_t)j, st.off0, st.off1, st.key0, st.key1);
            bits = (word == 0 ? r.w[0] : word == 1 ? r.w[1] : word == 2 ? r.w[2] : r.w[3]) >> shift;
        } else {
            const Words4 rs = philox4x32_10((uint32_t)(k0 >> 7), kSorsSignColumn, st.off0, st.off1, st.key0, st.key1);
            const Words4 rr = philox4x32_10((uint32_t)(j >> 2), kSorsRowColumn, st.off0, st.off1, st.key0, st.key1);
            const uint32_t q = (uint32_t)(j & 3);
            bits = (word == 0 ? rs.w[0] : word == 1 ? rs.w[1] : word == 2 ? rs.w[2] : rs.w[3]) >> shift;
            row = (q == 0 ? rr.w[0] : q == 1 ? rr.w[1] : q == 2 ? rr.w[2] : rr.w[3]) & st.row_mask;
        }
#pragma unroll
        for (int i = 0; i < TK; ++i) {
            const uint32_t neg = ((bits >> i) ^ (uint32_t)__popc(row & (uint32_t)(k0 + i))) & 1u;
            As[i][col] = (j < m && k0 + i < kk) ? (neg ? -1.0f : 1.0f) : 0.0f;
        }
    }
}

// C[m x n] = alpha * A[m x kk] * B[kk x n] (+ bias).  A.at(row, kk), B.at(kk, col).
template <typename ASrc, typename BSrc, typename Tout, typename Tbias>
__global__ void __launch_bounds__(256) gemm_plain_kernel(ASrc A, BSrc B, Tout *__restrict__ C, int64_t ldc,
                                                         const Tbias *__restrict__ bias, int64_t m, int64_t n,
                                                         int64_t kk, float alpha, bool accumulate) {
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[TK][TN + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t m0 = (int64_t)blockIdx.y * TM, n0 = (int64_t)blockIdx.x * TN;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < kk; k0 += TK) {
        fill_a_tile(A, As, m0, k0, m, kk, tid);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q;  // 0..1023
            const int kl = e & 15, rl = e >> 4;
            Bs[kl][rl] = (n0 + rl < n && k0 + kl < kk) ? B.at(k0 + kl, n0 + rl) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kl = 0; kl < TK; ++kl) {
            float a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a[u] = As[kl][ty * 4 + u];
                b[u] = Bs[kl][tx * 4 + u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(a[u], b[v], acc[u][v]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t gm = m0 + ty * 4 + u;
        if (gm >= m) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t gn = n0 + tx * 4 + v;
            if (gn >= n) continue;
            float r = alpha * acc[u][v];
            if (bias != nullptr) r += load_f32<Tbias>(bias + gn);
            if (accumulate) r += load_f32<Tout>(C + gm * ldc + gn);
            store_f32<Tout>(C + gm * ldc + gn, r);
        }
    }
}

// Column sums with 16-byte loads (colsum.hpp) as a kernel of its own.
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(ColsumArgs g) {
    __shared__ float lds[kColsumLdsFloats];
    colsum_body<T>(g, lds, blockIdx.x, gridDim.x);
}

// The same for widths or addresses that rule out 16-byte loads: 64 columns per work-group, one
// element per load, 4 row lanes per column.
template <typename T>
__global__ void __launch_bounds__(256) colsum_narrow_kernel(const T *__restrict__ A, T *__restrict__ out, int64_t n,
                                                            int64_t d, bool accumulate) {
    __shared__ float part[4][64];
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 64 + cl;
    float s = 0.0f;
    if (c < d)
        for (int64_t r = rl; r < n; r += 4) s += load_f32<T>(A + r * d + c);
    part[rl][cl] = s;
    __syncthreads();
    if (rl == 0 && c < d) {
        float r = (part[0][cl] + part[1][cl]) + (part[2][cl] + part[3][cl]);
        if (accumulate) r += load_f32<T>(out + c);
        store_f32<T>(out + c, r);
    }
}

__global__ void debug_philox_kernel(SketchState st, uint32_t c0, uint32_t c1, int64_t ncalls,
                                    uint32_t *__restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ncalls) return;
    const Words4 r = philox4x32_10(c0 + (uint32_t)t, c1, st.off0, st.off1, st.key0, st.key1);
#pragma unroll
    for (int q = 0; q < 4; ++q) out[4 * t + q] = r.w[q];
}

__global__ void debug_sketch_tile_kernel(int kind, SketchState st, int64_t i0, int64_t j0, int64_t rows,
                                         int64_t cols, float *__restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows * cols) return;
    const int64_t r = e / cols, c = e % cols;
    out[e] = sketch_entry_precise(kind, st, i0 + r, j0 + c);
}

}  // namespace

template <typename Tin, typename Tout>
hipError_t launch_gemm_plain(const Tin *A, int64_t sam, int64_t sak, const Tin *B, int64_t sbk, int64_t sbn,
                             Tout *C, int64_t ldc, const Tin *bias, int64_t m, int64_t n, int64_t kk, float alpha,
                             hipStream_t stream, bool accumulate) {
    MemSrc<Tin> a{A, sam, sak}, b{B, sbk, sbn};
    dim3 grid((unsigned)((n + TN - 1) / TN), (unsigned)((m + TM - 1) / TM));
    gemm_plain_kernel<MemSrc<Tin>, MemSrc<Tin>, Tout, Tin><<<grid, 256, 0, stream>>>(a, b, C, ldc, bias, m, n, kk,
                                                                                      alpha, accumulate);
    return hipGetLastError();
}

template <typename Tin, typename Tout>
hipError_t launch_sketch_plain(const Tin *A, Tout *out, int64_t n, int64_t d, int64_t k, int kind, SketchState st,
                               float alpha, hipStream_t stream) {
    SketchSrc a{kind, st};
    MemSrc<Tin> b{A, d, 1};
    dim3 grid((unsigned)((d + TN - 1) / TN), (unsigned)((k + TM - 1) / TM));
    gemm_plain_kernel<SketchSrc, MemSrc<Tin>, Tout, Tin><<<grid, 256, 0, stream>>>(a, b, out, d, (const Tin *)nullptr,
                                                                                    k, d, n, alpha, false);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_colsum(const T *A, T *out, int64_t n, int64_t d, hipStream_t stream, bool accumulate) {
    if (colsum_wide_ok(A, d, sizeof(T))) {
        const ColsumArgs g{A, out, n, d, accumulate ? 1 : 0, colsum_lpr(d, sizeof(T))};
        colsum_kernel<T><<<(unsigned)colsum_blocks(d, sizeof(T)), 256, 0, stream>>>(g);
    } else
        colsum_narrow_kernel<T><<<(unsigned)((d + 63) / 64), 256, 0, stream>>>(A, out, n, d, accumulate);
    return hipGetLastError();
}

hipError_t launch_debug_philox(SketchState st, uint32_t c0, uint32_t c1, int64_t ncalls, uint32_t *out,
                               hipStream_t stream) {
    debug_philox_kernel<<<(unsigned)((ncalls + 255) / 256), 256, 0, stream>>>(st, c0, c1, ncalls, out);
    return hipGetLastError();
}

hipError_t launch_debug_sketch_tile(int kind, SketchState st, int64_t i0, int64_t j0, int64_t rows, int64_t cols,
                                    float *out, hipStream_t stream) {
    const int64_t total = rows * cols;
    debug_sketch_tile_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(kind, st, i0, j0, rows, cols, out);
    return hipGetLastError();
}

#define RMM_INSTANTIATE(Tin, Tout)                                                                              \
    template hipError_t launch_gemm_plain<Tin, Tout>(const Tin *, int64_t, int64_t, const Tin *, int64_t,       \
                                                     int64_t, Tout *, int64_t, const Tin *, int64_t, int64_t,   \
                                                     int64_t, float, hipStream_t, bool);                        \
    template hipError_t launch_sketch_plain<Tin, Tout>(const Tin *, Tout *, int64_t, int64_t, int64_t, int,     \
                                                       SketchState, float, hipStream_t);
RMM_INSTANTIATE(float, float)
RMM_INSTANTIATE(bf16_t, bf16_t)
#undef RMM_INSTANTIATE
template hipError_t launch_gemm_plain<bf16_t, float>(const bf16_t *, int64_t, int64_t, const bf16_t *, int64_t, int64_t,
                                                     float *, int64_t, const bf16_t *, int64_t, int64_t, int64_t,
                                                     float, hipStream_t, bool);
template hipError_t launch_colsum<float>(const float *, float *, int64_t, int64_t, hipStream_t, bool);
template hipError_t launch_colsum<bf16_t>(const bf16_t *, bf16_t *, int64_t, int64_t, hipStream_t, bool);

}  // namespace rmm
