// C ABI of the RMM linear layer: argument checks, workspace layout, dispatch.
// Semantics of every entry point are stated in include/rmm.h.
#include "../../include/rmm.h"

#include <math.h>

#include <mutex>

#include "common.hpp"

using namespace rmm;

namespace {

constexpr int64_t kMaxDim = (int64_t)1 << 31;
constexpr int64_t kMaxElems = (int64_t)1 << 40;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t elem_bytes(int dtype) { return dtype == RMM_DTYPE_BF16 ? 2 : 4; }

bool dims_ok(int64_t a, int64_t b) { return a >= 1 && b >= 1 && a < kMaxDim && b < kMaxDim && a * b < kMaxElems; }

bool desc_ok(const rmm_layer_desc_t *d) {
    if (d == nullptr) return false;
    if (d->dtype != RMM_DTYPE_F32 && d->dtype != RMM_DTYPE_BF16) return false;
    if (d->kind != RMM_SKETCH_GAUSSIAN && d->kind != RMM_SKETCH_RADEMACHER && d->kind != RMM_SKETCH_SORS) return false;
    return dims_ok(d->n, d->d_in) && dims_ok(d->n, d->d_out) && dims_ok(d->d_out, d->d_in) &&
           dims_ok(d->k, d->d_in) && dims_ok(d->k, d->d_out) && dims_ok(d->n, d->k);
}

// The plain kernels put the row tile index in gridDim.y.
bool grid_ok(int64_t rows) { return (rows + 63) / 64 <= 65535; }

bool use_mfma(const rmm_layer_desc_t *d) {
    return d->dtype == RMM_DTYPE_BF16 && mfma_shape_ok(d->n, d->d_in, d->d_out, d->k);
}

// Workspace layout.
//   sketch / forward: fp32 partial sums of the token slices of S^T A (MFMA path only).
//   backward: G = S^T dY (k x d_out, in the layer's dtype), then the partial sums.
size_t g_bytes(const rmm_layer_desc_t *d) { return round_up((size_t)d->k * d->d_out * elem_bytes(d->dtype), 256); }
// (the SORS kind has no token slices: its sketch products need no scratch)
bool sliced_sketch(const rmm_layer_desc_t *d) { return use_mfma(d) && d->kind != RMM_SKETCH_SORS; }
size_t ws_sketch(const rmm_layer_desc_t *d) {
    return sliced_sketch(d) ? round_up(sketch_workspace_bf16(d->n, d->d_in, d->k), 256) : 0;
}
size_t ws_forward(const rmm_layer_desc_t *d) {
    return sliced_sketch(d) ? round_up(sketch_workspace_bf16(d->n, d->d_in, d->k, d->d_out), 256) : 0;
}
size_t ws_backward(const rmm_layer_desc_t *d) {
    return g_bytes(d) + (sliced_sketch(d) ? round_up(sketch_workspace_bf16(d->n, d->d_out, d->k, d->d_in), 256) : 0);
}

// variance monitors: per-block partials (doubles), then, off the MFMA path, X^T dY in fp32.
int var_xty_partials(const rmm_layer_desc_t *d) {
    return use_mfma(d) ? xty_sumsq_tiles(d->n, d->d_in, d->d_out) : sumsq_blocks(d->d_in * d->d_out);
}
size_t var_partial_bytes(const rmm_layer_desc_t *d) {
    return round_up(((size_t)3 * row_norm_blocks(d->n) + (size_t)var_xty_partials(d)) * sizeof(double), 256);
}
size_t ws_variance(const rmm_layer_desc_t *d) {
    return var_partial_bytes(d) + (use_mfma(d) ? 0 : round_up((size_t)d->d_in * d->d_out * sizeof(float), 256));
}

int from_hip(hipError_t e) { return e == hipSuccess ? RMM_OK : RMM_ERR_LAUNCH; }

// Stages that exist only when the two independent products of a pass are launched one by one.
bool separate_stage(int stage) {
    return stage == RMM_STAGE_FWD_Y || stage == RMM_STAGE_FWD_XPROJ || stage == RMM_STAGE_FWD_XPROJ_PRODUCT ||
           stage == RMM_STAGE_BWD_DX || stage == RMM_STAGE_BWD_G || stage == RMM_STAGE_BWD_G_PRODUCT;
}

// Scratch of rmm_sketch_static: device memory that is part of the library's code object, so that
// entry point needs no workspace argument and no allocation.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and copies get the per-device address kept in
// g_static_scratch (every GPU holds its own copy of the array at its own address).
constexpr size_t kStaticScratchBytes = (size_t)RMM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_static_scratch[kMaxDevices];
std::mutex g_static_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up once per device).
int static_scratch_ptr(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RMM_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (g_static_scratch[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return RMM_ERR_LAUNCH;
        g_static_scratch[dev] = p;
    }
    *out = g_static_scratch[dev];
    return RMM_OK;
}

// Optional pair of caller-owned events bracketing one stage of a pass.
struct StageEvents {
    int stage = RMM_STAGE_NONE;
    hipEvent_t begin = nullptr, end = nullptr;
};

// Records the begin event on construction and the end event on destruction when
// `stage` is the one being timed.
class StageScope {
public:
    StageScope(const StageEvents &ev, int stage, hipStream_t stream)
        : ev_(ev), on_(ev.stage == stage && ev.begin != nullptr && ev.end != nullptr), stream_(stream) {
        if (on_) (void)hipEventRecord(ev_.begin, stream_);
    }
    ~StageScope() {
        if (on_) (void)hipEventRecord(ev_.end, stream_);
    }

private:
    const StageEvents &ev_;
    bool on_;
    hipStream_t stream_;
};

template <typename T>
int sketch_impl(int64_t n, int64_t d, int64_t k, int kind, SketchState st, const void *A, void *out, bool mfma,
                void *ws, hipStream_t stream, const StageEvents &ev = StageEvents(), int product_stage = RMM_STAGE_NONE,
                int64_t d_other = 0) {
    const bool timed = product_stage != RMM_STAGE_NONE && ev.stage == product_stage;
    if (kind == RMM_SKETCH_SORS && mfma && sors_fast_ok(n, d)) {  // fast transform; otherwise S is applied densely below
        StageScope scope(ev, product_stage, stream);
        return from_hip(launch_sors_bf16((const bf16_t *)A, (bf16_t *)out, n, d, k, st, stream));
    }
    if (mfma && kind != RMM_SKETCH_SORS)
        return from_hip(launch_sketch_bf16((const bf16_t *)A, (bf16_t *)out, n, d, k, kind, st, ws, stream,
                                           timed ? ev.begin : nullptr, timed ? ev.end : nullptr, d_other));
    StageScope scope(ev, product_stage, stream);  // the plain path is one kernel
    const float alpha = 1.0f / sqrtf((float)k);
    return from_hip(launch_sketch_plain<T, T>((const T *)A, (T *)out, n, d, k, kind, st, alpha, stream));
}

template <typename T>
int forward_impl(const rmm_layer_desc_t *d, SketchState st, const void *X, const void *W, const void *bias, void *Y,
                 void *X_proj, void *ws, hipStream_t stream, const StageEvents &ev) {
    const bool mfma = use_mfma(d);
    if (X_proj != nullptr && sliced_sketch(d) && !separate_stage(ev.stage) &&
        forward_pair_available(d->n, d->d_in, d->d_out, d->k)) {
        const bool timed = ev.stage == RMM_STAGE_FWD_PAIR;
        return from_hip(launch_forward_pair_bf16((const bf16_t *)X, (const bf16_t *)W, (const bf16_t *)bias, (bf16_t *)Y,
                                                 (bf16_t *)X_proj, d->n, d->d_in, d->d_out, d->k, d->kind, st, ws, stream,
                                                 timed ? ev.begin : nullptr, timed ? ev.end : nullptr));
    }
    if (X_proj != nullptr && mfma && d->kind == RMM_SKETCH_SORS && !separate_stage(ev.stage) &&
        sors_pair_available(d->n, d->d_in, d->d_out, d->k)) {
        const bool timed = ev.stage == RMM_STAGE_FWD_PAIR;
        return from_hip(launch_forward_pair_sors_bf16((const bf16_t *)X, (const bf16_t *)W, (const bf16_t *)bias, (bf16_t *)Y,
                                                      (bf16_t *)X_proj, d->n, d->d_in, d->d_out, d->k, st, stream,
                                                      timed ? ev.begin : nullptr, timed ? ev.end : nullptr));
    }
    {   // Y = X W^T (+ bias): A = X (n x d_in), B(kk, c) = W[c][kk].
        StageScope scope(ev, RMM_STAGE_FWD_Y, stream);
        hipError_t e =
            mfma ? launch_linear_nt_bf16((const bf16_t *)X, (const bf16_t *)W, (const bf16_t *)bias, (bf16_t *)Y,
                                         d->n, d->d_in, d->d_out, stream)
                 : launch_gemm_plain<T, T>((const T *)X, d->d_in, 1, (const T *)W, 1, d->d_in, (T *)Y, d->d_out,
                                           (const T *)bias, d->n, d->d_out, d->d_in, 1.0f, stream);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
    }
    if (X_proj == nullptr) return RMM_OK;  // no backward pass will follow: nothing to keep
    StageScope scope(ev, RMM_STAGE_FWD_XPROJ, stream);
    return sketch_impl<T>(d->n, d->d_in, d->k, d->kind, st, X, X_proj, mfma, ws, stream, ev,
                          RMM_STAGE_FWD_XPROJ_PRODUCT, d->d_out);
}

template <typename T>
int backward_impl(const rmm_layer_desc_t *d, SketchState st, const void *dY, const void *W, const void *X_proj,
                  void *dX, void *dW, void *dbias, void *ws, hipStream_t stream, const StageEvents &ev,
                  bool accumulate) {
    hipError_t e;
    const bool mfma = use_mfma(d);
    T *G = (T *)ws;  // G = S^T dY, k x d_out
    const bool paired_sors = mfma && d->kind == RMM_SKETCH_SORS && dX != nullptr && !separate_stage(ev.stage) &&
                             sors_pair_available(d->n, d->d_out, d->d_in, d->k);
    if (paired_sors) {
        const bool timed = ev.stage == RMM_STAGE_BWD_PAIR;
        e = launch_backward_pair_sors_bf16((const bf16_t *)dY, (const bf16_t *)W, (bf16_t *)dX, (bf16_t *)G, d->n, d->d_in,
                                           d->d_out, d->k, st, stream, timed ? ev.begin : nullptr, timed ? ev.end : nullptr);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
    }
    const bool paired = paired_sors || (sliced_sketch(d) && dX != nullptr && !separate_stage(ev.stage) &&
                                        backward_pair_available(d->n, d->d_in, d->d_out, d->k));
    const bool own_db_stage = ev.stage == RMM_STAGE_BWD_DW || ev.stage == RMM_STAGE_BWD_DBIAS;
    bool db_done = false;
    if (paired && !paired_sors) {
        const bool timed = ev.stage == RMM_STAGE_BWD_PAIR;
        db_done = dbias != nullptr && !own_db_stage && backward_pair_takes_colsum(d->n, d->d_in, d->d_out, d->k);
        e = launch_backward_pair_bf16((const bf16_t *)dY, (const bf16_t *)W, (bf16_t *)dX, (bf16_t *)G, d->n, d->d_in,
                                      d->d_out, d->k, d->kind, st, (char *)ws + g_bytes(d), stream,
                                      timed ? ev.begin : nullptr, timed ? ev.end : nullptr,
                                      db_done ? (bf16_t *)dbias : nullptr, accumulate);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
    }
    if (!paired && dX != nullptr) {  // dX = dY W: B(kk, c) = W[kk][c]
        StageScope scope(ev, RMM_STAGE_BWD_DX, stream);
        e = mfma ? launch_linear_nn_bf16((const bf16_t *)dY, (const bf16_t *)W, (bf16_t *)dX, d->n, d->d_in, d->d_out,
                                         stream)
                 : launch_gemm_plain<T, T>((const T *)dY, d->d_out, 1, (const T *)W, d->d_in, 1, (T *)dX, d->d_in,
                                           (const T *)nullptr, d->n, d->d_in, d->d_out, 1.0f, stream);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
    }
    if (!paired) {
        StageScope scope(ev, RMM_STAGE_BWD_G, stream);
        int rc = sketch_impl<T>(d->n, d->d_out, d->k, d->kind, st, dY, G, mfma, (char *)ws + g_bytes(d), stream, ev,
                                RMM_STAGE_BWD_G_PRODUCT, d->d_in);
        if (rc != RMM_OK) return rc;
    }
    if (mfma && dbias != nullptr && !db_done && !own_db_stage) {
        // dW and db in one launch (an event request for either stage keeps them apart)
        e = launch_dw_colsum_bf16((const bf16_t *)G, (const bf16_t *)X_proj, (bf16_t *)dW, d->k, d->d_in, d->d_out,
                                  (const bf16_t *)dY, (bf16_t *)dbias, d->n, stream, accumulate);
        return e == hipSuccess ? RMM_OK : RMM_ERR_LAUNCH;
    }
    {   // dW = G^T X_proj: A(r, kk) = G[kk][r], B(kk, c) = X_proj[kk][c]
        StageScope scope(ev, RMM_STAGE_BWD_DW, stream);
        e = mfma ? launch_dw_bf16((const bf16_t *)G, (const bf16_t *)X_proj, (bf16_t *)dW, d->k, d->d_in, d->d_out,
                                  stream, accumulate)
                 : launch_gemm_plain<T, T>(G, 1, d->d_out, (const T *)X_proj, d->d_in, 1, (T *)dW, d->d_in,
                                           (const T *)nullptr, d->d_out, d->d_in, d->k, 1.0f, stream, accumulate);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
    }
    if (dbias != nullptr && !db_done) {
        StageScope scope(ev, RMM_STAGE_BWD_DBIAS, stream);
        e = launch_colsum<T>((const T *)dY, (T *)dbias, d->n, d->d_out, stream, accumulate);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
    }
    return RMM_OK;
}

}  // namespace

extern "C" {

int rmm_version(void) { return 313; }

const char *rmm_status_string(int status) {
    switch (status) {
        case RMM_OK: return "ok";
        case RMM_ERR_INVALID_ARG: return "invalid argument";
        case RMM_ERR_UNSUPPORTED: return "size beyond the supported limits";
        case RMM_ERR_WORKSPACE: return "workspace missing or too small";
        case RMM_ERR_LAUNCH: return "HIP launch failed";
        case RMM_ERR_SCRATCH_LIMIT: return "shape needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

size_t rmm_workspace_bytes(const rmm_layer_desc_t *desc, int op) {
    if (desc == nullptr) return 0;
    rmm_layer_desc_t d = *desc;
    if (op == RMM_OP_SKETCH) d.d_out = d.d_in;
    if (!desc_ok(&d)) return 0;
    switch (op) {
        case RMM_OP_FORWARD: return ws_forward(&d);
        case RMM_OP_BACKWARD: return ws_backward(&d);
        case RMM_OP_SKETCH: return ws_sketch(&d);
        case RMM_OP_VARIANCE: return ws_variance(&d);
        default: return 0;
    }
}

int rmm_uses_paired_launch(const rmm_layer_desc_t *desc, int op) {
    if (!desc_ok(desc) || !use_mfma(desc)) return 0;
    if (desc->kind == RMM_SKETCH_SORS) {
        if (op == RMM_OP_FORWARD) return sors_pair_available(desc->n, desc->d_in, desc->d_out, desc->k) ? 1 : 0;
        if (op == RMM_OP_BACKWARD) return sors_pair_available(desc->n, desc->d_out, desc->d_in, desc->k) ? 1 : 0;
        return 0;
    }
    if (op == RMM_OP_FORWARD) return forward_pair_available(desc->n, desc->d_in, desc->d_out, desc->k) ? 1 : 0;
    if (op == RMM_OP_BACKWARD) return backward_pair_available(desc->n, desc->d_in, desc->d_out, desc->k) ? 1 : 0;
    return 0;
}

int rmm_sketch_profiled(int64_t n, int64_t d, int64_t k, int dtype, int kind, rmm_rng_state_t state, const void *A,
                        void *A_proj, void *ws, size_t ws_bytes, void *stream, void *ev_begin, void *ev_end) {
    rmm_layer_desc_t desc = {n, d, d, k, dtype, kind};
    if (!desc_ok(&desc) || A == nullptr || A_proj == nullptr) return RMM_ERR_INVALID_ARG;
    if (!aligned16(A) || !aligned16(A_proj) || !aligned16(ws)) return RMM_ERR_INVALID_ARG;
    if (!grid_ok(k)) return RMM_ERR_UNSUPPORTED;
    const size_t need = ws_sketch(&desc);
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return RMM_ERR_WORKSPACE;
    const SketchState st = make_state(state.seed, state.offset, n);
    hipStream_t s = (hipStream_t)stream;
    const bool mfma = use_mfma(&desc);
    StageEvents ev;
    ev.stage = RMM_STAGE_FWD_XPROJ_PRODUCT;
    ev.begin = (hipEvent_t)ev_begin;
    ev.end = (hipEvent_t)ev_end;
    return dtype == RMM_DTYPE_BF16
               ? sketch_impl<bf16_t>(n, d, k, kind, st, A, A_proj, mfma, ws, s, ev, RMM_STAGE_FWD_XPROJ_PRODUCT)
               : sketch_impl<float>(n, d, k, kind, st, A, A_proj, false, ws, s, ev, RMM_STAGE_FWD_XPROJ_PRODUCT);
}

int rmm_sketch(int64_t n, int64_t d, int64_t k, int dtype, int kind, rmm_rng_state_t state, const void *A,
               void *A_proj, void *ws, size_t ws_bytes, void *stream) {
    return rmm_sketch_profiled(n, d, k, dtype, kind, state, A, A_proj, ws, ws_bytes, stream, nullptr, nullptr);
}

int rmm_sketch_static(int64_t n, int64_t d, int64_t k, int dtype, int kind, rmm_rng_state_t state, const void *A,
                      void *A_proj, void *stream) {
    rmm_layer_desc_t desc = {n, d, d, k, dtype, kind};
    if (!desc_ok(&desc) || A == nullptr || A_proj == nullptr) return RMM_ERR_INVALID_ARG;
    if (!aligned16(A) || !aligned16(A_proj)) return RMM_ERR_INVALID_ARG;
    if (!grid_ok(k)) return RMM_ERR_UNSUPPORTED;
    const size_t need = ws_sketch(&desc);
    if (need > kStaticScratchBytes) return RMM_ERR_SCRATCH_LIMIT;
    void *ws = nullptr;
    if (need > 0) {  // the only HIP calls besides the launches: no allocation, no copy, no wait
        const int rc = static_scratch_ptr(&ws);
        if (rc != RMM_OK) return rc;
    }
    const SketchState st = make_state(state.seed, state.offset, n);
    hipStream_t s = (hipStream_t)stream;
    return dtype == RMM_DTYPE_BF16 ? sketch_impl<bf16_t>(n, d, k, kind, st, A, A_proj, use_mfma(&desc), ws, s)
                                   : sketch_impl<float>(n, d, k, kind, st, A, A_proj, false, ws, s);
}

int rmm_forward_profiled(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *X, const void *W,
                         const void *bias, void *Y, void *X_proj, void *ws, size_t ws_bytes, void *stream, int stage,
                         void *ev_begin, void *ev_end) {
    if (!desc_ok(desc) || X == nullptr || W == nullptr || Y == nullptr) return RMM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(W) || !aligned16(bias) || !aligned16(Y) || !aligned16(X_proj) || !aligned16(ws))
        return RMM_ERR_INVALID_ARG;
    if (!grid_ok(desc->n) || !grid_ok(desc->k)) return RMM_ERR_UNSUPPORTED;
    const size_t need = X_proj != nullptr ? ws_forward(desc) : 0;
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return RMM_ERR_WORKSPACE;
    const SketchState st = make_state(state.seed, state.offset, desc->n);
    hipStream_t s = (hipStream_t)stream;
    StageEvents ev;
    ev.stage = stage;
    ev.begin = (hipEvent_t)ev_begin;
    ev.end = (hipEvent_t)ev_end;
    return desc->dtype == RMM_DTYPE_BF16 ? forward_impl<bf16_t>(desc, st, X, W, bias, Y, X_proj, ws, s, ev)
                                         : forward_impl<float>(desc, st, X, W, bias, Y, X_proj, ws, s, ev);
}

int rmm_forward(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *X, const void *W, const void *bias,
                void *Y, void *X_proj, void *ws, size_t ws_bytes, void *stream) {
    return rmm_forward_profiled(desc, state, X, W, bias, Y, X_proj, ws, ws_bytes, stream, RMM_STAGE_NONE, nullptr,
                                nullptr);
}

static int backward_checked(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                            const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes,
                            void *stream, int stage, void *ev_begin, void *ev_end, bool accumulate) {
    if (!desc_ok(desc) || dY == nullptr || W == nullptr || X_proj == nullptr || dW == nullptr)
        return RMM_ERR_INVALID_ARG;
    if (!aligned16(dY) || !aligned16(W) || !aligned16(X_proj) || !aligned16(dX) || !aligned16(dW) || !aligned16(dbias) ||
        !aligned16(ws))
        return RMM_ERR_INVALID_ARG;
    if (!grid_ok(desc->n) || !grid_ok(desc->k) || !grid_ok(desc->d_out)) return RMM_ERR_UNSUPPORTED;
    const size_t need = ws_backward(desc);
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return RMM_ERR_WORKSPACE;
    const SketchState st = make_state(state.seed, state.offset, desc->n);
    hipStream_t s = (hipStream_t)stream;
    StageEvents ev;
    ev.stage = stage;
    ev.begin = (hipEvent_t)ev_begin;
    ev.end = (hipEvent_t)ev_end;
    return desc->dtype == RMM_DTYPE_BF16
               ? backward_impl<bf16_t>(desc, st, dY, W, X_proj, dX, dW, dbias, ws, s, ev, accumulate)
               : backward_impl<float>(desc, st, dY, W, X_proj, dX, dW, dbias, ws, s, ev, accumulate);
}

int rmm_backward_profiled(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                          const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes,
                          void *stream, int stage, void *ev_begin, void *ev_end) {
    return backward_checked(desc, state, dY, W, X_proj, dX, dW, dbias, ws, ws_bytes, stream, stage, ev_begin, ev_end,
                            false);
}

int rmm_backward(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                 const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes, void *stream) {
    return backward_checked(desc, state, dY, W, X_proj, dX, dW, dbias, ws, ws_bytes, stream, RMM_STAGE_NONE, nullptr,
                            nullptr, false);
}

int rmm_backward_accumulate(const rmm_layer_desc_t *desc, rmm_rng_state_t state, const void *dY, const void *W,
                            const void *X_proj, void *dX, void *dW, void *dbias, void *ws, size_t ws_bytes,
                            void *stream) {
    return backward_checked(desc, state, dY, W, X_proj, dX, dW, dbias, ws, ws_bytes, stream, RMM_STAGE_NONE, nullptr,
                            nullptr, true);
}

int rmm_variance_stats(const rmm_layer_desc_t *desc, const void *X, const void *dY, double *out, void *ws,
                       size_t ws_bytes, void *stream) {
    if (!desc_ok(desc) || X == nullptr || dY == nullptr || out == nullptr) return RMM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(dY) || !aligned16(ws) || ((uintptr_t)out & 7u) != 0) return RMM_ERR_INVALID_ARG;
    if (!use_mfma(desc) && !grid_ok(desc->d_in)) return RMM_ERR_UNSUPPORTED;  // plain X^T dY: d_in rows of tiles
    if (desc->kind == RMM_SKETCH_SORS) return RMM_ERR_UNSUPPORTED;  // Lemma 2.2 is about i.i.d. entries
    if (ws == nullptr || ws_bytes < ws_variance(desc)) return RMM_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int nb = row_norm_blocks(desc->n), nt = var_xty_partials(desc);
    double *rows = (double *)ws, *xty = rows + 3 * (size_t)nb;
    hipError_t e;
    if (desc->dtype == RMM_DTYPE_BF16) {
        e = launch_row_norms<bf16_t>((const bf16_t *)X, (const bf16_t *)dY, desc->n, desc->d_in, desc->d_out, rows, s);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
        if (use_mfma(desc)) {
            e = launch_xty_sumsq_bf16((const bf16_t *)X, (const bf16_t *)dY, xty, desc->n, desc->d_in, desc->d_out, s);
        } else {
            float *P = (float *)((char *)ws + var_partial_bytes(desc));  // P(i, j) = sum_t X[t][i] dY[t][j]
            e = launch_gemm_plain<bf16_t, float>((const bf16_t *)X, 1, desc->d_in, (const bf16_t *)dY, desc->d_out, 1, P,
                                                 desc->d_out, (const bf16_t *)nullptr, desc->d_in, desc->d_out,
                                                 desc->n, 1.0f, s);
            if (e == hipSuccess) e = launch_sumsq(P, desc->d_in * desc->d_out, xty, s);
        }
    } else {
        e = launch_row_norms<float>((const float *)X, (const float *)dY, desc->n, desc->d_in, desc->d_out, rows, s);
        if (e != hipSuccess) return RMM_ERR_LAUNCH;
        float *P = (float *)((char *)ws + var_partial_bytes(desc));
        e = launch_gemm_plain<float, float>((const float *)X, 1, desc->d_in, (const float *)dY, desc->d_out, 1, P,
                                            desc->d_out, (const float *)nullptr, desc->d_in, desc->d_out, desc->n,
                                            1.0f, s);
        if (e == hipSuccess) e = launch_sumsq(P, desc->d_in * desc->d_out, xty, s);
    }
    if (e != hipSuccess) return RMM_ERR_LAUNCH;
    return from_hip(launch_variance_finalize(rows, nb, xty, nt, desc->n, desc->k, desc->kind, out, s));
}

int rmm_debug_philox(rmm_rng_state_t state, uint32_t c0, uint32_t c1, int64_t ncalls, uint32_t *out, void *stream) {
    if (out == nullptr || ncalls < 1 || ncalls >= kMaxDim) return RMM_ERR_INVALID_ARG;
    return from_hip(
        launch_debug_philox(make_state(state.seed, state.offset), c0, c1, ncalls, out, (hipStream_t)stream));
}

int rmm_debug_sketch_tile(int kind, rmm_rng_state_t state, int64_t i0, int64_t j0, int64_t rows, int64_t cols,
                          float *P_out, void *stream) {
    if (P_out == nullptr || rows < 1 || cols < 1 || i0 < 0 || j0 < 0) return RMM_ERR_INVALID_ARG;
    if (kind != RMM_SKETCH_GAUSSIAN && kind != RMM_SKETCH_RADEMACHER) return RMM_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols) || rows * cols > kMaxDim || i0 + rows > kMaxDim || j0 + cols > kMaxDim)
        return RMM_ERR_UNSUPPORTED;  // one thread per entry, 2^23 work-groups at most
    return from_hip(launch_debug_sketch_tile(kind, make_state(state.seed, state.offset), i0, j0, rows, cols, P_out,
                                             (hipStream_t)stream));
}

}  // extern "C"
