// Shared device helpers and the host-side launcher declarations of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "philox.hpp"

namespace rmm {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float((uint32_t)x << 16); }

// Round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ float load_f32(const T *p);
template <>
__device__ __forceinline__ float load_f32<float>(const float *p) { return *p; }
template <>
__device__ __forceinline__ float load_f32<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }

template <typename T>
__device__ __forceinline__ void store_f32(T *p, float v);
template <>
__device__ __forceinline__ void store_f32<float>(float *p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_f32<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// ---------------------------------------------------------------------------
// Host launchers (each returns the hipError_t of its launches).
// ---------------------------------------------------------------------------

// Plain LDS-tiled fp32-FMA kernels: the fp32 data path, and a slow bf16 one.
//   C[m x n] = alpha * A * B (+ bias[n] per row) (+ the old C if `accumulate`), A(m,kk) at
//   A[m*sam + kk*sak], B(kk,n) at B[kk*sbk + n*sbn], C row-major with leading dimension ldc.
template <typename Tin, typename Tout>
hipError_t launch_gemm_plain(const Tin *A, int64_t sam, int64_t sak, const Tin *B, int64_t sbk, int64_t sbn,
                             Tout *C, int64_t ldc, const Tin *bias, int64_t m, int64_t n, int64_t kk, float alpha,
                             hipStream_t stream, bool accumulate = false);
//   out[k x d] = alpha * P^T A with P the unscaled sketch (n x k) of `st`.
template <typename Tin, typename Tout>
hipError_t launch_sketch_plain(const Tin *A, Tout *out, int64_t n, int64_t d, int64_t k, int kind, SketchState st,
                               float alpha, hipStream_t stream);
//   out[d] = column sums of A[n x d] (+ the old out if `accumulate`).
template <typename T>
hipError_t launch_colsum(const T *A, T *out, int64_t n, int64_t d, hipStream_t stream, bool accumulate = false);

// bf16 MFMA path (mfma.hip).  Usable when mfma_shape_ok(); `ws` for the sketch
// must hold sketch_workspace_bf16() bytes (fp32 partial sums of the token slices).
// launch_sketch_bf16 records the optional event pair around its product kernel
// alone (the sum over token slices, when there is one, comes after `ev_end`).
bool mfma_shape_ok(int64_t n, int64_t d_in, int64_t d_out, int64_t k);
hipError_t launch_linear_nt_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, int64_t n,
                                 int64_t d_in, int64_t d_out, hipStream_t stream);
hipError_t launch_linear_nn_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, int64_t n, int64_t d_in,
                                 int64_t d_out, hipStream_t stream);
hipError_t launch_dw_bf16(const bf16_t *G, const bf16_t *X_proj, bf16_t *dW, int64_t k, int64_t d_in, int64_t d_out,
                          hipStream_t stream, bool accumulate = false);
// dW together with db = column sums of dY (n x d_out, 16-byte aligned, d_out a multiple of 8) in
// one launch; same results as launch_dw_bf16 followed by launch_colsum, bit for bit.
hipError_t launch_dw_colsum_bf16(const bf16_t *G, const bf16_t *X_proj, bf16_t *dW, int64_t k, int64_t d_in, int64_t d_out,
                                 const bf16_t *dY, bf16_t *dbias, int64_t n, hipStream_t stream, bool accumulate = false);
// `d_other` > 0 says that the sketch product belongs to a layer pass whose plain product has an
// n x d_other output (forward: d = d_in, d_other = d_out; backward: d = d_out, d_other = d_in): the
// token slicing is then the one the paired launch of that pass uses, so that the separate and the
// paired launches give the same bits.  0 = the product on its own (rmm_sketch).
size_t sketch_workspace_bf16(int64_t n, int64_t d, int64_t k, int64_t d_other = 0);
hipError_t launch_sketch_bf16(const bf16_t *A, bf16_t *out, int64_t n, int64_t d, int64_t k, int kind, SketchState st,
                              void *ws, hipStream_t stream, hipEvent_t ev_begin = nullptr,
                              hipEvent_t ev_end = nullptr, int64_t d_other = 0);

// One launch for the two products of a pass that do not depend on each other: Y = X W^T (+ bias)
// with the sketch product of X (forward), dX = dY W with the sketch product of dY (backward; G is
// k x d_out), followed by the sum over the sketch's token slices.  Results are bit-identical to
// the separate launches above (same kernels, same slices).  Only where *_pair_available() says so;
// the optional event pair brackets the paired kernel alone.
bool forward_pair_available(int64_t n, int64_t d_in, int64_t d_out, int64_t k);
hipError_t launch_forward_pair_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, bf16_t *X_proj,
                                    int64_t n, int64_t d_in, int64_t d_out, int64_t k, int kind, SketchState st, void *ws,
                                    hipStream_t stream, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
bool backward_pair_available(int64_t n, int64_t d_in, int64_t d_out, int64_t k);
// With `dbias` the launch also takes the column sums of dY (the bias gradient), on the compute units
// its last round leaves idle; backward_pair_takes_colsum() says where that beats the launch of dW.
hipError_t launch_backward_pair_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, bf16_t *G, int64_t n, int64_t d_in,
                                     int64_t d_out, int64_t k, int kind, SketchState st, void *ws, hipStream_t stream,
                                     hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr, bf16_t *dbias = nullptr,
                                     bool accumulate_dbias = false);
bool backward_pair_takes_colsum(int64_t n, int64_t d_in, int64_t d_out, int64_t k);

// SORS sketch kind, bf16 (sors.hip): signs, Walsh-Hadamard transform along the tokens and row
// selection in one kernel, no workspace.  Usable when sors_fast_ok(): d a multiple of 8 and at most
// 32768 tokens (the strip of one work-group has to fit in LDS); `st` made with the token count.
bool sors_fast_ok(int64_t n, int64_t d);
hipError_t launch_sors_bf16(const bf16_t *A, bf16_t *out, int64_t n, int64_t d, int64_t k, SketchState st,
                            hipStream_t stream);

// One launch for the plain product of a pass and the SORS sketch product of the same pass, where
// the plain product leaves compute units idle (mfma.hip decides, mfma_pair_sors.hip holds the
// kernels).  Same results as the separate launches, bit for bit.
bool sors_pair_available(int64_t n, int64_t d_sk, int64_t d_other, int64_t k);
hipError_t launch_forward_pair_sors_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, bf16_t *X_proj,
                                         int64_t n, int64_t d_in, int64_t d_out, int64_t k, SketchState st,
                                         hipStream_t stream, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
hipError_t launch_backward_pair_sors_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, bf16_t *G, int64_t n,
                                          int64_t d_in, int64_t d_out, int64_t k, SketchState st, hipStream_t stream,
                                          hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);

// Variance monitors (variance.hip, and the squared-norm epilogue of the MFMA kernel).
//   part[3*b..] = per-block (sum |x_k|^2, sum |y_k|^2, sum |x_k|^2 |y_k|^2); row_norm_blocks(n) blocks.
int row_norm_blocks(int64_t n);
template <typename T>
hipError_t launch_row_norms(const T *X, const T *Y, int64_t n, int64_t d_in, int64_t d_out, double *part,
                            hipStream_t stream);
//   part[b] = per-block sum of squares of an fp32 buffer; sumsq_blocks(elems) blocks.
int sumsq_blocks(int64_t elems);
hipError_t launch_sumsq(const float *A, int64_t elems, double *part, hipStream_t stream);
//   part[t] = sum of squares of tile t of X^T dY (d_in x d_out), bf16 MFMA path; xty_sumsq_tiles() tiles.
int xty_sumsq_tiles(int64_t n, int64_t d_in, int64_t d_out);
hipError_t launch_xty_sumsq_bf16(const bf16_t *X, const bf16_t *dY, double *part, int64_t n, int64_t d_in,
                                 int64_t d_out, hipStream_t stream);
hipError_t launch_variance_finalize(const double *rows, int nb, const double *xty, int nt, int64_t n, int64_t k,
                                    int kind, double *out, hipStream_t stream);

hipError_t launch_debug_philox(SketchState st, uint32_t c0, uint32_t c1, int64_t ncalls, uint32_t *out,
                               hipStream_t stream);
hipError_t launch_debug_sketch_tile(int kind, SketchState st, int64_t i0, int64_t j0, int64_t rows, int64_t cols,
                                    float *out, hipStream_t stream);

}  // namespace rmm
