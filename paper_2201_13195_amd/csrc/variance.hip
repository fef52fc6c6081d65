// Variance monitors (Section 2.3: Lemma 2.1, Lemma 2.2, Theorem 2.3): the reductions over
// X (n x d_in) and dY (n x d_out) that the closed forms need, and the closed forms themselves.
//
//   row_norms_kernel     one pass over X and dY: |X|_F^2, |dY|_F^2, sum_k |x_k|^2 |y_k|^2
//                        (one wave per token row, 16-byte loads, wave-level reduction)
//   sumsq_kernel         |A|_F^2 of an fp32 buffer (the fp32 path materialises X^T dY)
//   variance_finalize    fixed-order fp64 sums of the per-block partials, then D^2_SGD,
//                        D^2_RMM, alpha
// |X^T dY|_F^2 on the bf16 path comes from the MFMA kernel of mfma.hip (tile products are
// squared and summed in the epilogue, never stored).
#include "common.hpp"

namespace rmm {

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum of squares of one row, spread over the 64 lanes of a wave.
template <typename T>
__device__ __forceinline__ float row_sumsq(const T *row, int64_t d, int lane, bool vec) {
    float s = 0.0f;
    if (vec) {
        constexpr int PER = 16 / sizeof(T);  // elements per 16-byte load
        for (int64_t c = (int64_t)lane * PER; c < d; c += 64 * PER) {
            const uint4 q = *reinterpret_cast<const uint4 *>(row + c);
            if constexpr (sizeof(T) == 2) {
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float lo = __uint_as_float(w[i] << 16), hi = __uint_as_float(w[i] & 0xFFFF0000u);
                    s += lo * lo + hi * hi;
                }
            } else {
                const float f[4] = {__uint_as_float(q.x), __uint_as_float(q.y), __uint_as_float(q.z),
                                    __uint_as_float(q.w)};
#pragma unroll
                for (int i = 0; i < 4; ++i) s += f[i] * f[i];
            }
        }
    } else {
        for (int64_t c = lane; c < d; c += 64) {
            const float f = load_f32<T>(row + c);
            s += f * f;
        }
    }
    return wave_sum(s);
}

// part[3*b .. 3*b+2] = (sum |x_k|^2, sum |y_k|^2, sum |x_k|^2 |y_k|^2) over the rows of block b.
template <typename T>
__global__ void __launch_bounds__(256) row_norms_kernel(const T *__restrict__ X, const T *__restrict__ Y, int64_t n,
                                                        int64_t d_in, int64_t d_out, bool vec,
                                                        double *__restrict__ part) {
    __shared__ double red[4][3];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double ax = 0.0, ay = 0.0, ar = 0.0;
    for (int64_t r = (int64_t)blockIdx.x * 4 + wave; r < n; r += (int64_t)gridDim.x * 4) {
        const float sx = row_sumsq<T>(X + r * d_in, d_in, lane, vec);
        const float sy = row_sumsq<T>(Y + r * d_out, d_out, lane, vec);
        ax += sx, ay += sy, ar += (double)sx * (double)sy;
    }
    if (lane == 0) red[wave][0] = ax, red[wave][1] = ay, red[wave][2] = ar;
    __syncthreads();
    if (threadIdx.x < 3)
        part[3 * (int64_t)blockIdx.x + threadIdx.x] =
            (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

__global__ void __launch_bounds__(256) sumsq_kernel(const float *__restrict__ A, int64_t elems,
                                                    double *__restrict__ part) {
    __shared__ double red[4];
    double s = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < elems; e += (int64_t)gridDim.x * 256) {
        const double f = A[e];
        s += f * f;
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// One wave.  out[0..7] = |X|_F^2, |dY|_F^2, sum_k |x_k|^2 |y_k|^2, |X^T dY|_F^2,
// D^2_SGD (Lemma 2.1), D^2_RMM for sketch size k and the given kind (Lemma 2.2 with the sign of
// the |X^T dY|^2 term that the fourth moment of a Gaussian entry gives, minus 2 rows / k for
// Rademacher signs), alpha (Theorem 2.3), D^2_RMM as Lemma 2.2 prints it.
__global__ void __launch_bounds__(64) variance_finalize(const double *__restrict__ rows, int nb,
                                                        const double *__restrict__ xty, int nt, int64_t n,
                                                        int64_t k, int kind, double *__restrict__ out) {
    const int lane = threadIdx.x;
    double x2 = 0.0, y2 = 0.0, rw = 0.0, p2 = 0.0;
    for (int b = lane; b < nb; b += 64) x2 += rows[3 * b], y2 += rows[3 * b + 1], rw += rows[3 * b + 2];
    for (int t = lane; t < nt; t += 64) p2 += xty[t];
    x2 = wave_sum(x2), y2 = wave_sum(y2), rw = wave_sum(rw), p2 = wave_sum(p2);
    if (lane != 0) return;
    const double B = (double)n, kk = (double)k;
    out[0] = x2, out[1] = y2, out[2] = rw, out[3] = p2;
    out[4] = n > 1 ? B / (B - 1.0) * rw - p2 / (B - 1.0) : 0.0;
    out[5] = (x2 * y2 + p2 - (kind == 1 ? 2.0 * rw : 0.0)) / kk;
    out[6] = (x2 > 0.0 && y2 > 0.0) ? p2 / (x2 * y2) : 0.0;
    out[7] = (x2 * y2 - p2) / kk;
}

}  // namespace

int row_norm_blocks(int64_t n) {
    const int64_t b = (n + 3) / 4;
    return (int)(b < 2048 ? b : 2048);
}

int sumsq_blocks(int64_t elems) {
    const int64_t b = (elems + 255) / 256;
    return (int)(b < 1024 ? b : 1024);
}

template <typename T>
hipError_t launch_row_norms(const T *X, const T *Y, int64_t n, int64_t d_in, int64_t d_out, double *part,
                            hipStream_t stream) {
    constexpr int PER = 16 / sizeof(T);
    const bool vec = d_in % PER == 0 && d_out % PER == 0;
    row_norms_kernel<T><<<row_norm_blocks(n), 256, 0, stream>>>(X, Y, n, d_in, d_out, vec, part);
    return hipGetLastError();
}

hipError_t launch_sumsq(const float *A, int64_t elems, double *part, hipStream_t stream) {
    sumsq_kernel<<<sumsq_blocks(elems), 256, 0, stream>>>(A, elems, part);
    return hipGetLastError();
}

hipError_t launch_variance_finalize(const double *rows, int nb, const double *xty, int nt, int64_t n, int64_t k,
                                    int kind, double *out, hipStream_t stream) {
    variance_finalize<<<1, 64, 0, stream>>>(rows, nb, xty, nt, n, k, kind, out);
    return hipGetLastError();
}

template hipError_t launch_row_norms<float>(const float *, const float *, int64_t, int64_t, int64_t, double *,
                                            hipStream_t);
template hipError_t launch_row_norms<bf16_t>(const bf16_t *, const bf16_t *, int64_t, int64_t, int64_t, double *,
                                             hipStream_t);

}  // namespace rmm
