// bf16 MFMA path of the RMM layer: which kernel of mfma_kernels.hpp serves which product at
// which shape, and the launches.
#include "mfma_pair.hpp"
#include "sors_kernels.hpp"

namespace rmm {

namespace {

// Prefetch depth (register sets of tiles in flight).  The kernels run whole groups of `depth`
// tiles, so a plain product takes the one of 4 and 3 that pads its contraction less; the
// 256 x 256 kernel and the sketch kernels need their registers for wide wave tiles and use 3.
int plain_depth(int64_t contraction, int bk) {
    const int64_t kt = (contraction + bk - 1) / bk;
    const int64_t pad4 = (kt + 3) / 4 * 4 - kt, pad3 = (kt + 2) / 3 * 3 - kt;
    return pad4 <= pad3 ? 4 : 3;
}

template <typename S, int AMODE, int BMODE, int OUT>
hipError_t launch(const GemmArgs &g, int splits, hipStream_t stream) {
    const int64_t tiles = ((g.M + S::BM - 1) / S::BM) * ((g.N + S::BN - 1) / S::BN);
    const dim3 grid((unsigned)tiles, 1, (unsigned)splits);
    if constexpr (AMODE >= A_GAUSS || std::is_same<S, ShapeLarge>::value) {
        gemm_mfma_kernel<S, AMODE, BMODE, OUT, 3><<<grid, S::THREADS, 0, stream>>>(g);
    } else {
        if (plain_depth(g.K < g.k_chunk ? g.K : g.k_chunk, S::BK) == 4)
            gemm_mfma_kernel<S, AMODE, BMODE, OUT, 4><<<grid, S::THREADS, 0, stream>>>(g);
        else
            gemm_mfma_kernel<S, AMODE, BMODE, OUT, 3><<<grid, S::THREADS, 0, stream>>>(g);
    }
    return hipGetLastError();
}

int64_t tiles_of(int64_t m, int64_t n, int64_t bm, int64_t bn) { return ((m + bm - 1) / bm) * ((n + bn - 1) / bn); }

// Tile shape of a plain product with an m x n output and contraction kk.
//   256 x 256 (8 waves, one work-group per compute unit) once there are at least 160 such tiles:
//     half the operand traffic per flop of the 128 x 128 tile, which needs more bytes per clock
//     from L2 than it delivers at full MFMA rate;
//   64 x 64 when there are fewer than 65 tiles of 128 x 128 (a quarter of the compute units);
//   128 x 128 x 64 with two wave groups splitting the contraction when there are at most 256
//     tiles and the contraction is 768 or longer (a compute unit then still holds 8 waves; at 768
//     it runs like the 4-wave tile on its own, and its 512 threads allow the paired launch);
//   128 x 128 x 32 with 4 waves otherwise (two work-groups per compute unit).
int gemm_cfg(int64_t m, int64_t n, int64_t kk) {
    if (tiles_of(m, n, ShapeLarge::BM, ShapeLarge::BN) >= 160) return GEMM_LARGE;
    const int64_t t128 = tiles_of(m, n, 128, 128);
    if (t128 < 65) return GEMM_TINY;
    if (t128 <= 256 && kk >= 768) return GEMM_SPLIT;
    return GEMM_MID;
}

template <int AMODE, int BMODE, int OUT>
hipError_t launch_gemm(int cfg, const GemmArgs &g, hipStream_t stream) {
    if (cfg == GEMM_LARGE) return launch<ShapeLarge, AMODE, BMODE, OUT>(g, 1, stream);
    if (cfg == GEMM_SPLIT) return launch<ShapeSplit, AMODE, BMODE, OUT>(g, 1, stream);
    if constexpr (OUT == OUT_BF16)
        if (cfg == GEMM_TINY) return launch<ShapeTiny, AMODE, BMODE, OUT>(g, 1, stream);
    return launch<ShapeMid, AMODE, BMODE, OUT>(g, 1, stream);
}

GemmArgs args_nt(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, int64_t n, int64_t d_in, int64_t d_out) {
    GemmArgs g{};
    g.A = X, g.lda = d_in, g.B = W, g.ldb = d_in, g.C = Y, g.ldc = d_out, g.bias = bias;
    g.M = n, g.N = d_out, g.K = d_in, g.alpha = 1.0f, g.k_chunk = (d_in + 127) / 128 * 128;
    return g;
}

GemmArgs args_nn(const bf16_t *dY, const bf16_t *W, bf16_t *dX, int64_t n, int64_t d_in, int64_t d_out) {
    GemmArgs g{};
    g.A = dY, g.lda = d_out, g.B = W, g.ldb = d_in, g.C = dX, g.ldc = d_in, g.bias = nullptr;
    g.M = n, g.N = d_in, g.K = d_out, g.alpha = 1.0f, g.k_chunk = (d_out + 127) / 128 * 128;
    return g;
}

// Which kernel serves a sketch product with k > 64 and how its token dimension is cut.
//   d >= 1024:               the work-group generates the 128 x 32 sketch tile into LDS and all
//                            eight waves read it, 512 columns per tile (an entry is generated once
//                            per 512 columns); 64-row tiles for k <= 512 (k = 410 pads to 448 rows
//                            instead of 512);
//   d a multiple of 384:     the same with 384-column tiles (d = 768);
//   other d below 1024:      128 x 256 tiles whose sketch fragments are generated in registers.
// Tokens are cut into `splits` slices of `k_chunk` tokens (a multiple of 128) so that about
// `target_wgs` work-groups exist (256 = one per compute unit; measured: more or fewer are slower
// when the product runs alone); with more than one slice the kernel writes fp32 partial results
// to workspace and reduce_partials_kernel sums them in slice order.
struct SketchPlan {
    int cfg, splits;
    int64_t k_chunk, tiles;
};

SketchPlan plan_sketch(int64_t n, int64_t d, int64_t k, int target_wgs = 256) {
    SketchPlan p;
    const bool rows64 = k <= 512;
    p.cfg = d >= 1024 ? (rows64 ? SK_WIDE64 : SK_WIDE) : d % 384 == 0 ? (rows64 ? SK_MID64 : SK_MID) : SK_NARROW;
    const int64_t bm = (p.cfg == SK_WIDE64 || p.cfg == SK_MID64) ? 64 : 128;
    const int64_t bn = p.cfg == SK_NARROW ? 256 : (p.cfg == SK_MID64 || p.cfg == SK_MID) ? 384 : 512;
    p.tiles = tiles_of(k, d, bm, bn);
    const int64_t blocks = (n + 127) / 128;
    int64_t s = target_wgs / p.tiles;
    if (s > blocks) s = blocks;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    p.k_chunk = (blocks + s - 1) / s * 128;
    p.splits = (int)((n + p.k_chunk - 1) / p.k_chunk);
    return p;
}

GemmArgs args_sketch(const bf16_t *A, int64_t n, int64_t d, int64_t k, SketchState st, const SketchPlan &p, bf16_t *out,
                     void *ws, bool always_partial = false) {
    GemmArgs g{};
    g.A = nullptr, g.lda = 0, g.B = A, g.ldb = d, g.bias = nullptr;
    g.M = k, g.N = d, g.K = n, g.st = st, g.ldc = d, g.k_chunk = p.k_chunk;
    if (p.splits == 1 && !always_partial) {
        g.C = out, g.alpha = 1.0f / sqrtf((float)k);
    } else {
        g.C = ws, g.alpha = 1.0f, g.split_stride = k * d;
    }
    return g;
}

template <int OUT>
hipError_t launch_sketch_cfg(int cfg, int kind, const GemmArgs &g, int splits, hipStream_t stream) {
    switch (cfg) {
        case SK_WIDE:
            return kind == 0 ? launch<ShapeSkWide, A_GAUSS_LDS, B_NCONTIG, OUT>(g, splits, stream)
                             : launch<ShapeSkWide, A_RADEM_LDS, B_NCONTIG, OUT>(g, splits, stream);
        case SK_WIDE64:
            return kind == 0 ? launch<ShapeSkWide64, A_GAUSS_LDS, B_NCONTIG, OUT>(g, splits, stream)
                             : launch<ShapeSkWide64, A_RADEM_LDS, B_NCONTIG, OUT>(g, splits, stream);
        case SK_MID64:
            return kind == 0 ? launch<ShapeSkMid64, A_GAUSS_LDS, B_NCONTIG, OUT>(g, splits, stream)
                             : launch<ShapeSkMid64, A_RADEM_LDS, B_NCONTIG, OUT>(g, splits, stream);
        case SK_MID:
            return kind == 0 ? launch<ShapeSkMid, A_GAUSS_LDS, B_NCONTIG, OUT>(g, splits, stream)
                             : launch<ShapeSkMid, A_RADEM_LDS, B_NCONTIG, OUT>(g, splits, stream);
        default:
            return kind == 0 ? launch<ShapeSkNarrow, A_GAUSS, B_NCONTIG, OUT>(g, splits, stream)
                             : launch<ShapeSkNarrow, A_RADEM, B_NCONTIG, OUT>(g, splits, stream);
    }
}

hipError_t launch_reduce(const void *ws, bf16_t *out, int64_t k, int64_t d, int splits, hipStream_t stream) {
    const int64_t elems = k * d;  // d % 8 == 0, so elems % 4 == 0
    reduce_partials_kernel<<<(unsigned)((elems / 4 + 255) / 256), 256, 0, stream>>>((const float *)ws, out, elems, splits,
                                                                                     elems, 1.0f / sqrtf((float)k));
    return hipGetLastError();
}

// The streaming kernel of small sketch sizes: token slices so that about one work-group per
// compute unit exists; 2 register sets of loads in flight.  Work-groups take 256 columns, or 128
// where that would leave slices of at most 2048 tokens (k <= 32) / 512 tokens (k <= 64): half as many,
// twice as long slices then halve the partial sums and the final cross-wave sum of a work-group
// (measured: 26.6 against 27.6 us at 16384 x 4096, k = 32; 11.7 against 15.3 us at 16384 x 1024),
// while on long slices the wider work-group is ahead (82.8 against 84.6 us at 65536 x 4096).
constexpr int64_t kSmallK = 64;
int smallk_slices_for(int64_t n, int64_t d, int64_t bn, int64_t *k_chunk) {
    const int64_t col_tiles = (d + bn - 1) / bn, blocks = (n + 127) / 128;
    int64_t s = 256 / col_tiles;
    if (s > blocks) s = blocks;
    if (s < 1) s = 1;
    *k_chunk = (blocks + s - 1) / s * 128;
    return (int)((n + *k_chunk - 1) / *k_chunk);
}
int64_t smallk_bn(int64_t n, int64_t d, int64_t k) {
    int64_t k_chunk;
    (void)smallk_slices_for(n, d, 256, &k_chunk);
    return k_chunk <= (k <= 32 ? 2048 : 512) ? 128 : 256;
}
int smallk_slices(int64_t n, int64_t d, int64_t k, int64_t *k_chunk) {
    return smallk_slices_for(n, d, smallk_bn(n, d, k), k_chunk);
}

template <int TM, int BN, int KIND>
hipError_t launch_smallk(const SmallkArgs &g, int slices, hipStream_t stream) {
    const dim3 grid((unsigned)((g.d + BN - 1) / BN), (unsigned)slices);
    if (slices == 1)
        sketch_smallk_kernel<TM, BN, KIND, 2, OUT_BF16><<<grid, 256, 0, stream>>>(g);
    else
        sketch_smallk_kernel<TM, BN, KIND, 2, OUT_F32_PARTIAL><<<grid, 256, 0, stream>>>(g);
    return hipGetLastError();
}

// Brackets a kernel with the caller's events (either may be null: nothing is recorded).
struct EventPair {
    hipEvent_t begin, end;
    hipStream_t stream;
    EventPair(hipEvent_t b, hipEvent_t e, hipStream_t s) : begin(b), end(e), stream(s) {
        if (begin != nullptr && end != nullptr) (void)hipEventRecord(begin, stream);
    }
    void done() {
        if (begin != nullptr && end != nullptr) (void)hipEventRecord(end, stream);
        begin = end = nullptr;
    }
    ~EventPair() { done(); }
};

// The paired launch exists for a plain product on 256 x 256 tiles, or on the 128 x 128 x 64 split
// tiles at prefetch depth 4 (both run with 512 threads, like the sketch kernels), next to a sketch
// product with an LDS-generated tile and at least two token slices.
// An unsliced sketch product (more than 128 tiles) joins too when it leaves at least 32 compute
// units idle: the plain product's tiles run there while its one long round lasts.  The paired
// kernel always writes fp32 partial results, so the single slice goes through the summing kernel
// like several would (same bits as the direct bf16 output: one rounding of the same fp32 value).
bool pair_ok(int cfg_a, int depth_a, const SketchPlan &p) {
    if (p.cfg == SK_NARROW) return false;
    if (p.splits < 2 && !(p.tiles > 128 && p.tiles <= 224)) return false;
    return cfg_a == GEMM_LARGE || (cfg_a == GEMM_SPLIT && depth_a == 4);
}

// Work-groups the sketch product of a pass should aim at when it is launched together with the
// pass's plain product (`blocks_a` tiles, flops_a flop): if the plain product leaves compute units
// idle in its last round and runs long enough for the whole sketch product (flops_sk, at about half
// the plain product's rate per compute unit) to finish on them, one work-group per idle compute
// unit (fewer, longer work-groups: less prologue, fewer partial sums); otherwise 256.
int paired_sketch_target(int64_t blocks_a, double flops_a, double flops_sk) {
    const int64_t idle = (256 - blocks_a % 256) % 256;
    if (idle >= 32 && 2.0 * flops_sk * (double)blocks_a <= (double)idle * flops_a) return (int)idle;
    return 256;
}

// Plan of the sketch product of X (forward) / dY (backward) inside a layer call.
SketchPlan plan_pass_sketch(int64_t n, int64_t d_sk, int64_t d_other, int64_t k) {
    // the plain product has an n x d_other output and contracts over d_sk
    const SketchPlan alone = plan_sketch(n, d_sk, k);
    const int cfg_a = gemm_cfg(n, d_other, d_sk);
    const int depth_a = cfg_a == GEMM_SPLIT ? plain_depth(d_sk, ShapeSplit::BK) : 3;
    if (!pair_ok(cfg_a, depth_a, alone)) return alone;
    const int64_t blocks_a = cfg_a == GEMM_LARGE ? tiles_of(n, d_other, ShapeLarge::BM, ShapeLarge::BN)
                                                 : tiles_of(n, d_other, ShapeSplit::BM, ShapeSplit::BN);
    const int target = paired_sketch_target(blocks_a, 2.0 * n * d_sk * d_other, 2.0 * n * k * d_sk);
    SketchPlan paired = plan_sketch(n, d_sk, k, target);
    if (target == 256) {
        // Short slices (at most 1024 tokens) pack better into the time the plain product's work-groups
        // take when there are a quarter more of them; long ones would only add a round.
        const SketchPlan finer = plan_sketch(n, d_sk, k, 320);
        if (finer.splits > paired.splits && finer.k_chunk <= 1024) paired = finer;
    }
    return paired.splits >= 2 || pair_ok(cfg_a, depth_a, paired) ? paired : alone;
}

}  // namespace

bool mfma_shape_ok(int64_t n, int64_t d_in, int64_t d_out, int64_t k) {
    // 16-byte chunks need widths that are multiples of 8; a buffer descriptor spans up to 256 rows
    // of an operand with 32-bit byte offsets, so a row has to stay below 2^22 elements.  The token
    // count and the sketch size are not limited here (operands of 2 GiB and more are fine).
    (void)n, (void)k;
    const int64_t lim = (int64_t)1 << 22;
    return d_in % 8 == 0 && d_out % 8 == 0 && d_in < lim && d_out < lim;
}

hipError_t launch_linear_nt_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, int64_t n,
                                 int64_t d_in, int64_t d_out, hipStream_t stream) {
    const GemmArgs g = args_nt(X, W, bias, Y, n, d_in, d_out);
    return launch_gemm<A_KCONTIG, B_KCONTIG, OUT_BF16>(gemm_cfg(g.M, g.N, g.K), g, stream);
}

hipError_t launch_linear_nn_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, int64_t n, int64_t d_in,
                                 int64_t d_out, hipStream_t stream) {
    const GemmArgs g = args_nn(dY, W, dX, n, d_in, d_out);
    return launch_gemm<A_KCONTIG, B_NCONTIG, OUT_BF16>(gemm_cfg(g.M, g.N, g.K), g, stream);
}

hipError_t launch_dw_bf16(const bf16_t *G, const bf16_t *X_proj, bf16_t *dW, int64_t k, int64_t d_in, int64_t d_out,
                          hipStream_t stream, bool accumulate) {
    GemmArgs g{};
    g.accumulate = accumulate ? 1 : 0;
    g.A = G, g.lda = d_out, g.B = X_proj, g.ldb = d_in, g.C = dW, g.ldc = d_in, g.bias = nullptr;
    g.M = d_out, g.N = d_in, g.K = k, g.alpha = 1.0f, g.k_chunk = (k + 127) / 128 * 128;
    return launch_gemm<A_MCONTIG, B_NCONTIG, OUT_BF16>(gemm_cfg(g.M, g.N, g.K), g, stream);
}

template <typename S>
static hipError_t launch_dw_colsum(const GemmArgs &g, const ColsumArgs &c, hipStream_t stream) {
    const int blocks_a = (int)tiles_of(g.M, g.N, S::BM, S::BN);
    const dim3 grid((unsigned)(blocks_a + colsum_blocks(c.d, 2)));
    if (plain_depth(g.K, S::BK) == 3)
        dw_colsum_kernel<S, 3><<<grid, S::THREADS, 0, stream>>>(g, c, blocks_a);
    else
        dw_colsum_kernel<S, 4><<<grid, S::THREADS, 0, stream>>>(g, c, blocks_a);
    return hipGetLastError();
}

hipError_t launch_dw_colsum_bf16(const bf16_t *G, const bf16_t *X_proj, bf16_t *dW, int64_t k, int64_t d_in, int64_t d_out,
                                 const bf16_t *dY, bf16_t *dbias, int64_t n, hipStream_t stream, bool accumulate) {
    GemmArgs g{};
    g.accumulate = accumulate ? 1 : 0;
    g.A = G, g.lda = d_out, g.B = X_proj, g.ldb = d_in, g.C = dW, g.ldc = d_in, g.bias = nullptr;
    g.M = d_out, g.N = d_in, g.K = k, g.alpha = 1.0f, g.k_chunk = (k + 127) / 128 * 128;
    const ColsumArgs c{dY, dbias, n, d_out, accumulate ? 1 : 0, colsum_lpr(d_out, 2)};
    switch (gemm_cfg(g.M, g.N, g.K)) {  // the tile dW runs with on its own
        case GEMM_LARGE: {  // 160 or more tiles of 256 x 256: dW fills the chip, the column sums follow as a launch of their own
            const hipError_t e = launch_dw_bf16(G, X_proj, dW, k, d_in, d_out, stream, accumulate);
            return e != hipSuccess ? e : launch_colsum<bf16_t>(dY, dbias, n, d_out, stream, accumulate);
        }
        case GEMM_SPLIT: return launch_dw_colsum<ShapeSplit>(g, c, stream);
        case GEMM_TINY: return launch_dw_colsum<ShapeTiny>(g, c, stream);
        default: return launch_dw_colsum<ShapeMid>(g, c, stream);
    }
}

// |X^T dY|_F^2 per tile for the variance monitors: the dW-type product (both operands stored
// [token][feature]) with the squared-norm epilogue; the tile menu of the other products without
// its 64 x 64 entry.
static int xty_cfg(int64_t m, int64_t n, int64_t kk) {
    const int cfg = gemm_cfg(m, n, kk);
    return cfg == GEMM_TINY ? (kk >= 1536 ? GEMM_SPLIT : GEMM_MID) : cfg;
}

int xty_sumsq_tiles(int64_t n, int64_t d_in, int64_t d_out) {
    const bool large = xty_cfg(d_in, d_out, n) == GEMM_LARGE;
    return (int)tiles_of(d_in, d_out, large ? ShapeLarge::BM : 128, large ? ShapeLarge::BN : 128);
}

hipError_t launch_xty_sumsq_bf16(const bf16_t *X, const bf16_t *dY, double *part, int64_t n, int64_t d_in,
                                 int64_t d_out, hipStream_t stream) {
    GemmArgs g{};
    g.A = X, g.lda = d_in, g.B = dY, g.ldb = d_out, g.C = part, g.ldc = d_out, g.bias = nullptr;
    g.M = d_in, g.N = d_out, g.K = n, g.alpha = 1.0f, g.k_chunk = (n + 127) / 128 * 128;
    return launch_gemm<A_MCONTIG, B_NCONTIG, OUT_SUMSQ>(xty_cfg(g.M, g.N, g.K), g, stream);
}

size_t sketch_workspace_bf16(int64_t n, int64_t d, int64_t k, int64_t d_other) {
    int64_t k_chunk;
    if (k <= kSmallK) {
        const int s = smallk_slices(n, d, k, &k_chunk);
        return s > 1 ? (size_t)s * (size_t)k * (size_t)d * sizeof(float) : 0;
    }
    if (d_other > 0) {  // inside a pass: a paired launch writes partial results even for a single slice
        const SketchPlan p = plan_pass_sketch(n, d, d_other, k);
        const int cfg_a = gemm_cfg(n, d_other, d);
        const bool paired = pair_ok(cfg_a, cfg_a == GEMM_SPLIT ? plain_depth(d, ShapeSplit::BK) : 3, p);
        return p.splits > 1 || paired ? (size_t)p.splits * (size_t)k * (size_t)d * sizeof(float) : 0;
    }
    const int s = plan_sketch(n, d, k).splits;
    return s > 1 ? (size_t)s * (size_t)k * (size_t)d * sizeof(float) : 0;
}

hipError_t launch_sketch_bf16(const bf16_t *A, bf16_t *out, int64_t n, int64_t d, int64_t k, int kind, SketchState st,
                              void *ws, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end, int64_t d_other) {
    EventPair pev(ev_begin, ev_end, stream);
    if (k <= kSmallK) {  // bound by one pass over A: streaming kernel
        SmallkArgs a{};
        a.A = A, a.n = n, a.d = d, a.k = k, a.st = st;
        const int slices = smallk_slices(n, d, k, &a.k_chunk);
        a.C = slices == 1 ? (void *)out : ws, a.alpha = 1.0f / sqrtf((float)k);
        const bool narrow = smallk_bn(n, d, k) == 128;
        hipError_t e;
        if (k <= 32)
            e = narrow ? (kind == 0 ? launch_smallk<1, 128, 0>(a, slices, stream) : launch_smallk<1, 128, 1>(a, slices, stream))
                       : (kind == 0 ? launch_smallk<1, 256, 0>(a, slices, stream) : launch_smallk<1, 256, 1>(a, slices, stream));
        else
            e = narrow ? (kind == 0 ? launch_smallk<2, 128, 0>(a, slices, stream) : launch_smallk<2, 128, 1>(a, slices, stream))
                       : (kind == 0 ? launch_smallk<2, 256, 0>(a, slices, stream) : launch_smallk<2, 256, 1>(a, slices, stream));
        pev.done();
        if (e != hipSuccess || slices == 1) return e;
        return launch_reduce(ws, out, k, d, slices, stream);
    }
    const SketchPlan p = d_other > 0 ? plan_pass_sketch(n, d, d_other, k) : plan_sketch(n, d, k);
    const GemmArgs g = args_sketch(A, n, d, k, st, p, out, ws);
    if (p.splits == 1) return launch_sketch_cfg<OUT_BF16>(p.cfg, kind, g, 1, stream);
    hipError_t e = launch_sketch_cfg<OUT_F32_PARTIAL>(p.cfg, kind, g, p.splits, stream);
    pev.done();
    if (e != hipSuccess) return e;
    return launch_reduce(ws, out, k, d, p.splits, stream);
}

bool forward_pair_available(int64_t n, int64_t d_in, int64_t d_out, int64_t k) {
    if (k <= kSmallK) return false;
    const int cfg = gemm_cfg(n, d_out, d_in);  // (the paired plan keeps >= 2 slices)
    return pair_ok(cfg, cfg == GEMM_SPLIT ? plain_depth(d_in, ShapeSplit::BK) : 3, plan_sketch(n, d_in, k));
}

hipError_t launch_forward_pair_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, bf16_t *X_proj,
                                    int64_t n, int64_t d_in, int64_t d_out, int64_t k, int kind, SketchState st, void *ws,
                                    hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
    const GemmArgs ga = args_nt(X, W, bias, Y, n, d_in, d_out);
    const SketchPlan p = plan_pass_sketch(n, d_in, d_out, k);
    const GemmArgs gb = args_sketch(X, n, d_in, k, st, p, X_proj, ws, true);
    EventPair pev(ev_begin, ev_end, stream);
    hipError_t e;
    if (gemm_cfg(ga.M, ga.N, ga.K) == GEMM_LARGE)
        e = launch_pair_nt(p.cfg, kind, ga, gb, (int)tiles_of(ga.M, ga.N, ShapeLarge::BM, ShapeLarge::BN), (int)p.tiles,
                           p.splits, stream);
    else
        e = launch_pair_nt_split(p.cfg, kind, ga, gb, (int)tiles_of(ga.M, ga.N, ShapeSplit::BM, ShapeSplit::BN), (int)p.tiles,
                                 p.splits, stream);
    pev.done();
    if (e != hipSuccess) return e;
    return launch_reduce(ws, X_proj, k, d_in, p.splits, stream);
}

bool backward_pair_available(int64_t n, int64_t d_in, int64_t d_out, int64_t k) {
    if (k <= kSmallK) return false;
    const int cfg = gemm_cfg(n, d_in, d_out);
    return pair_ok(cfg, cfg == GEMM_SPLIT ? plain_depth(d_out, ShapeSplit::BK) : 3, plan_sketch(n, d_out, k));
}

// Where the bias gradient goes in a backward pass that has the paired launch: into the launch of
// dW when that leaves at least 64 compute units idle (dW is short and mostly latency); otherwise
// into the paired launch when its last round leaves at least 16 idle (the sketch work-groups of
// that round run for long, and dY is being read there anyway); otherwise into the launch of dW.
bool backward_pair_takes_colsum(int64_t n, int64_t d_in, int64_t d_out, int64_t k) {
    if (!backward_pair_available(n, d_in, d_out, k)) return false;
    const int dw_cfg = gemm_cfg(d_out, d_in, k);
    const int64_t dw_tiles = dw_cfg == GEMM_LARGE ? tiles_of(d_out, d_in, ShapeLarge::BM, ShapeLarge::BN)
                             : dw_cfg == GEMM_TINY ? tiles_of(d_out, d_in, ShapeTiny::BM, ShapeTiny::BN)
                                                   : tiles_of(d_out, d_in, 128, 128);
    if ((256 - dw_tiles % 256) % 256 >= 64) return false;
    const int64_t blocks_a = gemm_cfg(n, d_in, d_out) == GEMM_LARGE ? tiles_of(n, d_in, ShapeLarge::BM, ShapeLarge::BN)
                                                                    : tiles_of(n, d_in, ShapeSplit::BM, ShapeSplit::BN);
    const SketchPlan p = plan_pass_sketch(n, d_out, d_in, k);
    const int64_t total = blocks_a + p.tiles * p.splits;
    return (256 - total % 256) % 256 >= 16;
}

hipError_t launch_backward_pair_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, bf16_t *G, int64_t n, int64_t d_in,
                                     int64_t d_out, int64_t k, int kind, SketchState st, void *ws, hipStream_t stream,
                                     hipEvent_t ev_begin, hipEvent_t ev_end, bf16_t *dbias, bool accumulate_dbias) {
    const GemmArgs ga = args_nn(dY, W, dX, n, d_in, d_out);
    const SketchPlan p = plan_pass_sketch(n, d_out, d_in, k);
    const GemmArgs gb = args_sketch(dY, n, d_out, k, st, p, G, ws, true);
    const ColsumArgs gc{dY, dbias, n, d_out, accumulate_dbias ? 1 : 0, colsum_lpr(d_out, 2)};
    const ColsumArgs *gcp = dbias != nullptr ? &gc : nullptr;
    EventPair pev(ev_begin, ev_end, stream);
    hipError_t e;
    if (gemm_cfg(ga.M, ga.N, ga.K) == GEMM_LARGE)
        e = launch_pair_nn_large(p.cfg, kind, ga, gb, (int)tiles_of(ga.M, ga.N, ShapeLarge::BM, ShapeLarge::BN), (int)p.tiles,
                                 p.splits, stream, gcp);
    else
        e = launch_pair_nn_split(p.cfg, kind, ga, gb, (int)tiles_of(ga.M, ga.N, ShapeSplit::BM, ShapeSplit::BN), (int)p.tiles,
                                 p.splits, stream, gcp);
    pev.done();
    if (e != hipSuccess) return e;
    return launch_reduce(ws, G, k, d_out, p.splits, stream);
}

// ---- SORS kind: the plain product of a pass together with the strips of its sketch product.
// Worth it when the plain product leaves at least 32 compute units idle in its last round (the
// sketch work-groups need a compute unit to themselves); the strip kernel's chunked form must
// apply (at least 4096 tokens after padding, at most 2048 sketch columns).
static int sors_chunks(int64_t n) {
    int l = 0;
    while (((int64_t)1 << l) < n) ++l;
    return l >= 12 ? 1 << (l - 11) : 0;
}

// 0: separate launches; 1: strips behind the plain tiles (they fill the compute units its last
// round leaves idle, at least 32 of them); 2: strips in front (the plain product runs three or more
// rounds and the strips, few and long, occupy at most a quarter of the chip beside its first rounds).
static int sors_pair_order(int64_t blocks_a, int64_t strip_groups) {
    if ((256 - blocks_a % 256) % 256 >= 32) return 1;
    if (blocks_a >= 256 && strip_groups <= 64) return 2;
    return 0;
}

bool sors_pair_available(int64_t n, int64_t d_sk, int64_t d_other, int64_t k) {
    if (!sors_fast_ok(n, d_sk) || sors_chunks(n) == 0 || k > 2048) return false;
    const int cfg = gemm_cfg(n, d_other, d_sk);
    if (!(cfg == GEMM_LARGE || (cfg == GEMM_SPLIT && plain_depth(d_sk, ShapeSplit::BK) == 4))) return false;
    const int64_t blocks_a = cfg == GEMM_LARGE ? tiles_of(n, d_other, ShapeLarge::BM, ShapeLarge::BN)
                                               : tiles_of(n, d_other, ShapeSplit::BM, ShapeSplit::BN);
    return sors_pair_order(blocks_a, (d_sk / 8 + 1) / 2) != 0;
}

static hipError_t launch_pass_sors(const GemmArgs &ga, bool row_indexed_b, const bf16_t *A, bf16_t *out, int64_t n, int64_t d_sk,
                                   int64_t k, SketchState st, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
    const int cfg = gemm_cfg(ga.M, ga.N, ga.K);
    const int blocks_a = (int)(cfg == GEMM_LARGE ? tiles_of(ga.M, ga.N, ShapeLarge::BM, ShapeLarge::BN)
                                                 : tiles_of(ga.M, ga.N, ShapeSplit::BM, ShapeSplit::BN));
    const SorsArgs gs{A, out, n, d_sk, k, st, 1.0f / sqrtf((float)k)};
    EventPair pev(ev_begin, ev_end, stream);
    return launch_pair_sors(cfg, row_indexed_b, ga, gs, blocks_a, sors_chunks(n), sors_pair_order(blocks_a, (d_sk / 8 + 1) / 2) == 2,
                            stream);
}

hipError_t launch_forward_pair_sors_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, bf16_t *X_proj,
                                         int64_t n, int64_t d_in, int64_t d_out, int64_t k, SketchState st,
                                         hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
    return launch_pass_sors(args_nt(X, W, bias, Y, n, d_in, d_out), false, X, X_proj, n, d_in, k, st, stream, ev_begin, ev_end);
}

hipError_t launch_backward_pair_sors_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, bf16_t *G, int64_t n,
                                          int64_t d_in, int64_t d_out, int64_t k, SketchState st, hipStream_t stream,
                                          hipEvent_t ev_begin, hipEvent_t ev_end) {
    return launch_pass_sors(args_nn(dY, W, dX, n, d_in, d_out), true, dY, G, n, d_out, k, st, stream, ev_begin, ev_end);
}

}  // namespace rmm
