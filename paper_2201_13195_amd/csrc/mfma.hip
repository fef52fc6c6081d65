// bf16 MFMA kernels of the RMM layer (gfx950).
//
// One tiled-GEMM kernel template covers the five products of Algorithm 1:
//
//   Y      = X W^T          A = X  (K-contiguous rows)      B = W      (K-contiguous rows)
//   dX     = dY W           A = dY (K-contiguous rows)      B = W      (N-contiguous rows)
//   X_proj = S^T X          A = P^T generated in registers  B = X      (N-contiguous rows)
//   G      = S^T dY         A = P^T generated in registers  B = dY     (N-contiguous rows)
//   dW     = G^T X_proj     A = G  (M-contiguous rows)      B = X_proj (N-contiguous rows)
//
// with C[M x N] = alpha * sum_kk A(m, kk) B(kk, n).  The contraction runs on
// v_mfma_f32_32x32x16_bf16 with fp32 accumulators.  Memory operands are staged
// through LDS in 16-byte chunks, double buffered.  An operand whose contraction
// index is its row index ("N-contiguous" / "M-contiguous") is read back from LDS
// with the transposing load ds_read_b64_tr_b16, which hands every lane four
// consecutive contraction elements of one column.  The sketch operand is never
// in memory: every lane makes the eight entries its MFMA operand register holds
// from one Philox-4x32-10 call (Gaussian: the call's 8 Box-Muller values are
// exactly 8 consecutive tokens of one sketch column; Rademacher: one byte of the
// call's 128 sign bits).  The 1/sqrt(k) of S = P/sqrt(k) is applied to the fp32
// accumulator, so P is exact in bf16 for Rademacher and rounded once for Gaussian.
#include "common.hpp"

#include <type_traits>

namespace rmm {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

enum { A_KCONTIG = 0, A_MCONTIG = 1, A_GAUSS = 2, A_RADEM = 3 };
enum { B_KCONTIG = 0, B_NCONTIG = 1 };
enum { OUT_BF16 = 0, OUT_F32_PARTIAL = 1 };

constexpr int KPAD = 8;   // elements of padding per row of a K-contiguous LDS tile (row stride 144 B at BK = 64)
constexpr int TPAD = 32;  // elements of padding per row of a transposed-read LDS tile (row stride = 64 mod 256 B)

struct GemmArgs {
    const bf16_t *A;
    int64_t lda;
    const bf16_t *B;
    int64_t ldb;
    void *C;
    int64_t ldc;
    const bf16_t *bias;
    int64_t M, N, K;
    int64_t a_bytes, b_bytes;  // byte sizes of the A and B operands in memory (each below 2^31)
    float alpha;
    SketchState st;
    int64_t k_chunk;       // contraction elements per blockIdx.z slice (multiple of 128)
    int64_t split_stride;  // fp32 elements between the partial results of two slices
#ifdef RMM_DEBUG_TRACE
    unsigned long long *trace;
#endif
};

// Eight unscaled Gaussian entries P[8*c0 .. 8*c0+7][j] as a bf16 MFMA operand.
__device__ __forceinline__ bf16x8_t gauss_operand(const SketchState &st, uint32_t c0, uint32_t j) {
    const Words4 r = philox4x32_10(c0, j, st.off0, st.off1, st.key0, st.key1);
    union {
        bf16x8_t v;
        bf16x2_t p[4];
    } out;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t w = r.w[q];
        const float u1 = (float)(2u * (w >> 16) + 1u) * (1.0f / 131072.0f);
        const float u2 = (float)(w & 0xFFFFu) * (1.0f / 65536.0f);                            // revolutions
        const float rad = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));  // -2 ln2 log2 u1
        f32x2_t z = {rad * __builtin_amdgcn_cosf(u2), rad * __builtin_amdgcn_sinf(u2)};
        out.p[q] = __builtin_convertvector(z, bf16x2_t);
    }
    return out.v;
}

// Eight Rademacher entries for tokens t0 .. t0+7 (t0 a multiple of 8) of column j,
// given the four words of the call that covers tokens 128*(t0/128) .. +127.
__device__ __forceinline__ bf16x8_t radem_operand(const Words4 &r, uint32_t t0) {
    const uint32_t t = t0 & 127u;
    const uint32_t word = (t >> 5) == 0 ? r.w[0] : (t >> 5) == 1 ? r.w[1] : (t >> 5) == 2 ? r.w[2] : r.w[3];
    const uint32_t bits = (word >> (t & 31u)) & 0xFFu;
    union {
        bf16x8_t v;
        uint32_t d[4];
    } out;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        out.d[q] = 0x3F803F80u | (((bits >> (2 * q)) & 1u) << 15) | (((bits >> (2 * q + 1)) & 1u) << 31);
    return out.v;
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int WAVES_K, int AMODE, int BMODE, int OUT>
struct Tile {
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N * WAVES_K;  // WAVES_K groups of waves split the contraction
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;            // 32x32 MFMA tiles per wave
    static constexpr bool A_IN_LDS = (AMODE == A_KCONTIG || AMODE == A_MCONTIG);
    static constexpr int A_STRIDE = AMODE == A_KCONTIG ? BK + KPAD : BM + TPAD;  // elements per LDS row
    static constexpr int A_ROWS = AMODE == A_KCONTIG ? BM : BK;
    static constexpr int B_STRIDE = BMODE == B_KCONTIG ? BK + KPAD : BN + TPAD;
    static constexpr int B_ROWS = BMODE == B_KCONTIG ? BN : BK;
    static constexpr int A_ELEMS = A_IN_LDS ? A_ROWS * A_STRIDE : 0;
    static constexpr int B_ELEMS = B_ROWS * B_STRIDE;
    static constexpr int STAGE_ELEMS = A_ELEMS + B_ELEMS;
    static constexpr int STAGES = 3;  // LDS stages: tile t is computed while tile t+2 is written
    static constexpr int LDS_BYTES = STAGES * STAGE_ELEMS * 2;
    static constexpr int A_CHUNKS = A_IN_LDS ? BM * BK / 8 / THREADS : 0;  // 16-byte chunks per thread and tile
    static constexpr int B_CHUNKS = BN * BK / 8 / THREADS;
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0 && BK % (16 * WAVES_K) == 0, "tile shape");
    static_assert((BM * BK / 8) % THREADS == 0 && (BN * BK / 8) % THREADS == 0, "chunks per thread");
};

// Operand fragment of the 32x32x16 MFMA from a K-contiguous LDS tile:
// lane l holds row (l % 32), contraction elements 8*(l / 32) .. +7.
__device__ __forceinline__ bf16x8_t frag_kcontig(const bf16_t *tile, int stride, int row0, int kk0, int lane) {
    const bf16_t *p = tile + (row0 + (lane & 31)) * stride + kk0 + ((lane >> 5) << 3);
    return *reinterpret_cast<const bf16x8_t *>(p);
}

// Same fragment from a tile stored [contraction row][column]: two transposing
// reads.  Within a block of 16 lanes, lane i points at row (i / 4), columns
// 4*(i % 4) .. +3 of a 4 x 16 patch; the load returns to lane L the four rows of
// column L.  Block b of the wave covers columns 16*(b % 2) .. +15 and
// contraction rows 8*(b / 2) .. +7 (in two patches of four rows).
__device__ __forceinline__ bf16x8_t frag_transposed(const bf16_t *tile, int stride, int col0, int kk0, int lane) {
    const int blk = lane >> 4, i = lane & 15;
    const bf16_t *p = tile + (kk0 + ((blk >> 1) << 3) + (i >> 2)) * stride + col0 + ((blk & 1) << 4) + ((i & 3) << 2);
    typedef __attribute__((address_space(3))) s16x4_t *lds_ptr_t;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * stride));
    union {
        s16x8_t s;
        bf16x8_t v;
    } out;
    out.s = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return out.v;
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int WAVES_K, int AMODE, int BMODE, int OUT, int D>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N * WAVES_K) gemm_mfma_kernel(GemmArgs g) {
    typedef Tile<BM, BN, BK, WAVES_M, WAVES_N, WAVES_K, AMODE, BMODE, OUT> T;
    __shared__ __attribute__((aligned(16))) bf16_t lds[T::STAGES * T::STAGE_ELEMS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Wave w works on the (wm, wn) part of the tile and, of every 16-deep contraction step s,
    // on those with s % WAVES_K == kg.
    const int kg = wave / (WAVES_M * WAVES_N), wmn = wave % (WAVES_M * WAVES_N);
    const int wm = wmn / WAVES_N, wn = wmn % WAVES_N;
    // Tile order.  Work-groups are dealt round-robin to the 8 XCDs (each with its own L2), so first
    // renumber them such that one XCD owns a contiguous run of positions; then walk the tile grid
    // in bands of GROUP_M tile rows, column by column, so that the work-groups resident on one XCD
    // at the same time form a compact block that shares A row blocks and B column blocks in L2.
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int64_t tiles = (int64_t)gridDim.x;
    int64_t tile = blockIdx.x;
    {
        const int64_t per = tiles / 8, rem = tiles % 8, x = tile % 8, r = tile / 8;
        tile = x * per + (x < rem ? x : rem) + r;   // XCD x owns `per` (+1 for the first `rem`) consecutive positions
    }
    constexpr int64_t GROUP_M = 8;
    const int64_t band = tile / (GROUP_M * tiles_n), in_band = tile % (GROUP_M * tiles_n);
    const int64_t band_rows = min(GROUP_M, tiles_m - band * GROUP_M);
    const int64_t m0 = (band * GROUP_M + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;
    const int64_t kk_begin = (int64_t)blockIdx.z * g.k_chunk;
    const int64_t kk_end = min(g.K, kk_begin + g.k_chunk);
    const int num_tiles = kk_end > kk_begin ? (int)((kk_end - kk_begin + BK - 1) / BK) : 0;

    f32x16_t acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // Global loads are buffer loads: an offset at or beyond the operand's byte size returns zeros
    // without touching memory, so tile edges and the tail of the contraction need no branches (a
    // chunk that must read as zero is simply given the offset 2^31).  Matrices are below 2^31 bytes.
    const __amdgpu_buffer_rsrc_t rsrc_a =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(g.A), (short)0, (int)g.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(g.B), (short)0, (int)g.b_bytes, 0x00020000);
    constexpr uint32_t OOB = 0x80000000u;

    // Per 16-byte chunk of a tile: byte offset in the operand for the first tile of this slice,
    // whether its row / column group exists at all, and its position along the contraction.
    uint32_t a_off[T::A_CHUNKS > 0 ? T::A_CHUNKS : 1], b_off[T::B_CHUNKS];
    bool a_ok[T::A_CHUNKS > 0 ? T::A_CHUNKS : 1], b_ok[T::B_CHUNKS];
    int a_kk[T::A_CHUNKS > 0 ? T::A_CHUNKS : 1], b_kk[T::B_CHUNKS];
    int a_lds[T::A_CHUNKS > 0 ? T::A_CHUNKS : 1], b_lds[T::B_CHUNKS];
    uint32_t a_step = 0, b_step = 0;  // bytes per tile along the contraction
    if constexpr (AMODE == A_KCONTIG) {  // A[m][kk], tile BM x BK
        a_step = BK * 2;
#pragma unroll
        for (int q = 0; q < T::A_CHUNKS; ++q) {
            const int c = tid + T::THREADS * q, row = c / (BK / 8), kc = c % (BK / 8);
            a_ok[q] = m0 + row < g.M;
            a_kk[q] = kc * 8;
            a_off[q] = (uint32_t)(((m0 + row) * g.lda + kk_begin + kc * 8) * 2);
            a_lds[q] = row * T::A_STRIDE + kc * 8;
        }
    } else if constexpr (AMODE == A_MCONTIG) {  // A stored [kk][m], tile BK x BM
        a_step = (uint32_t)(BK * g.lda * 2);
#pragma unroll
        for (int q = 0; q < T::A_CHUNKS; ++q) {
            const int c = tid + T::THREADS * q, row = c / (BM / 8), mc = c % (BM / 8);
            a_ok[q] = m0 + mc * 8 < g.M;
            a_kk[q] = row;
            a_off[q] = (uint32_t)(((kk_begin + row) * g.lda + m0 + mc * 8) * 2);
            a_lds[q] = row * T::A_STRIDE + mc * 8;
        }
    }
    if constexpr (BMODE == B_KCONTIG) {  // B stored [n][kk], tile BN x BK
        b_step = BK * 2;
#pragma unroll
        for (int q = 0; q < T::B_CHUNKS; ++q) {
            const int c = tid + T::THREADS * q, row = c / (BK / 8), kc = c % (BK / 8);
            b_ok[q] = n0 + row < g.N;
            b_kk[q] = kc * 8;
            b_off[q] = (uint32_t)(((n0 + row) * g.ldb + kk_begin + kc * 8) * 2);
            b_lds[q] = row * T::B_STRIDE + kc * 8;
        }
    } else {  // B stored [kk][n], tile BK x BN
        b_step = (uint32_t)(BK * g.ldb * 2);
#pragma unroll
        for (int q = 0; q < T::B_CHUNKS; ++q) {
            const int c = tid + T::THREADS * q, row = c / (BN / 8), nc = c % (BN / 8);
            b_ok[q] = n0 + nc * 8 < g.N;
            b_kk[q] = row;
            b_off[q] = (uint32_t)(((kk_begin + row) * g.ldb + n0 + nc * 8) * 2);
            b_lds[q] = row * T::B_STRIDE + nc * 8;
        }
    }
    const int kk_len = (int)(kk_end - kk_begin);  // contraction elements of this slice (may be <= 0)

    // D register sets hold the tiles in flight: tile t + D is requested while tile t is computed.
    u32x4_t ra[D][T::A_CHUNKS > 0 ? T::A_CHUNKS : 1], rb[D][T::B_CHUNKS];

    // Work-groups walk the contraction from different starting tiles (and wrap around): with a
    // power-of-two row pitch all rows of a tile fall on the same one or two L2 channels, and the
    // rotation spreads concurrently running work-groups over the channels.  The eight tiles of one
    // band column (same B column block, neighbouring A row blocks) share a starting tile so that
    // their common operand is fetched once into L2.
#ifndef RMM_STAGGER_DIV
#define RMM_STAGGER_DIV 8
#endif
    const int stagger = (num_tiles > 0 && RMM_STAGGER_DIV > 0) ? (int)((tile / RMM_STAGGER_DIV) % num_tiles) : 0;
    auto rotated = [&](int t) { return t + stagger - (t + stagger >= num_tiles ? num_tiles : 0); };

    auto issue = [&](int set, int t_seq) {  // request the t_seq-th tile of this slice into register set `set`
        const int t = t_seq < num_tiles ? rotated(t_seq) : t_seq;  // past the end: stays out of range, reads zeros
        const int kk_tile = t * BK;
        if constexpr (T::A_IN_LDS) {
#pragma unroll
            for (int q = 0; q < T::A_CHUNKS; ++q) {
                const bool ok = a_ok[q] && kk_tile + a_kk[q] < kk_len;
                ra[set][q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, ok ? a_off[q] + (uint32_t)t * a_step : OOB,
                                                                   0, 0);
            }
        }
#pragma unroll
        for (int q = 0; q < T::B_CHUNKS; ++q) {
            const bool ok = b_ok[q] && kk_tile + b_kk[q] < kk_len;
            rb[set][q] =
                __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, ok ? b_off[q] + (uint32_t)t * b_step : OOB, 0, 0);
        }
    };

    auto store_lds = [&](int set, int stage) {
        bf16_t *As = lds + stage * T::STAGE_ELEMS;
        bf16_t *Bs = As + T::A_ELEMS;
        if constexpr (T::A_IN_LDS) {
#pragma unroll
            for (int q = 0; q < T::A_CHUNKS; ++q) *reinterpret_cast<u32x4_t *>(As + a_lds[q]) = ra[set][q];
        }
#pragma unroll
        for (int q = 0; q < T::B_CHUNKS; ++q) *reinterpret_cast<u32x4_t *>(Bs + b_lds[q]) = rb[set][q];
    };

    // Operand fragments of one 16-deep contraction step.
    struct Frags {
        bf16x8_t a[T::TM], b[T::TN];
    };
    constexpr int KS = BK / 16 / WAVES_K;  // 16-deep contraction steps per tile and wave: kg, kg + WAVES_K, ...
    static_assert(KS >= 2, "the pipeline needs two contraction steps per tile and wave");

    // Fragments of step `ks` of the tile whose data sits in LDS stage `stage` and whose first
    // contraction index is kk0.  LDS reads (and the generator's ALU work) issued here run under
    // the MFMAs of the step before.
    Words4 rw[T::TM];  // Rademacher: the Philox words of the 128-token block the tile being fetched lies in
    auto load_frags = [&](Frags &f, int stage, int64_t kk0, int ks_local) {
        const int ks = ks_local * WAVES_K + kg;  // this wave's ks_local-th step of the tile
        const bf16_t *As = lds + stage * T::STAGE_ELEMS;
        const bf16_t *Bs = As + T::A_ELEMS;
#pragma unroll
        for (int a = 0; a < T::TM; ++a) {
            const int row0 = wm * T::WTM + a * 32;
            if constexpr (AMODE == A_KCONTIG) {
                f.a[a] = frag_kcontig(As, T::A_STRIDE, row0, ks * 16, lane);
            } else if constexpr (AMODE == A_MCONTIG) {
                f.a[a] = frag_transposed(As, T::A_STRIDE, row0, ks * 16, lane);
            } else {
                const uint32_t j = (uint32_t)(m0 + row0 + (lane & 31));
                const int64_t tok = kk0 + ks * 16 + ((lane >> 5) << 3);  // first of this lane's 8 tokens
                if constexpr (AMODE == A_GAUSS) {
                    f.a[a] = gauss_operand(g.st, (uint32_t)(tok >> 3), j);
                } else {
                    if (ks_local == 0)  // a tile (BK <= 128 tokens, aligned) never straddles two blocks
                        rw[a] = philox4x32_10((uint32_t)(kk0 >> 7), j, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
                    f.a[a] = radem_operand(rw[a], (uint32_t)tok);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < T::TN; ++b) {
            const int col0 = wn * T::WTN + b * 32;
            if constexpr (BMODE == B_KCONTIG)
                f.b[b] = frag_kcontig(Bs, T::B_STRIDE, col0, ks * 16, lane);
            else
                f.b[b] = frag_transposed(Bs, T::B_STRIDE, col0, ks * 16, lane);
        }
    };

    auto multiply = [&](const Frags &f) {
#pragma unroll
        for (int a = 0; a < T::TM; ++a)
#pragma unroll
            for (int b = 0; b < T::TN; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[b], f.a[a], acc[a][b], 0, 0, 0);
    };

    // Pipeline.  Global side: tiles t+3 .. t+D-1 are in flight in D register sets (tile u in set
    // u % D) while tile t is computed; the loop runs over whole groups of D tiles so that every
    // load's register set is fixed at compile time, and tiles past the end read as zeros.  LDS side:
    // three stages (tile u in stage u % 3).  During step t tile t+2 is written: its stage was last
    // read in step t-1, which every wave has left, and it is first read at the end of step t+1,
    // after the barrier that closes step t+1 ... so ONE barrier per step is enough, and the
    // fragments of the next 16-deep contraction step are always fetched before the MFMAs of the
    // current one are issued, also across the tile boundary.
    static_assert(D >= 3, "tile t+2 must have been requested before step t");
#ifdef RMM_DEBUG_TRACE
    unsigned long long *tr = g.trace ? g.trace + ((size_t)blockIdx.x + (size_t)gridDim.x * blockIdx.z) * 64 : nullptr;
    if (tr && tid == 0) tr[0] = clock64(), tr[62] = wall_clock64();
#endif
#pragma unroll
    for (int s = 0; s < D; ++s) issue(s, s);
    store_lds(0, 0);
    store_lds(1, 1);
    __syncthreads();
    Frags cur, nxt;
    load_frags(cur, 0, kk_begin + (int64_t)rotated(0) * BK, 0);
    const int groups = (num_tiles + D - 1) / D;
    int st_cur = 0;  // stage of tile t
#ifdef RMM_DEBUG_TRACE
    if (tr && tid == 0) tr[1] = clock64();
#endif
    for (int grp = 0; grp < groups; ++grp) {
#pragma unroll
        for (int s = 0; s < D; ++s) {
            const int t = grp * D + s;
            // A step past the end costs little when both operands are loaded (all zeros, no branch);
            // with a generated operand it would cost a full step of generator work, so leave
            // (only the last group can be short; the outer loop ends with it).
            if constexpr (!T::A_IN_LDS)
                if (t >= num_tiles) break;
            const int64_t kk_t = kk_begin + (int64_t)(t < num_tiles ? rotated(t) : 0) * BK;
            const int64_t kk_n = kk_begin + (int64_t)(t + 1 < num_tiles ? rotated(t + 1) : 0) * BK;
            const int st_next = st_cur == 2 ? 0 : st_cur + 1, st_write = st_next == 2 ? 0 : st_next + 1;
#ifndef RMM_DEBUG_NOLOAD
            issue(s, t + D);
#endif
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == KS - 1)
                    load_frags(nxt, st_next, kk_n, 0);
                else
                    load_frags(nxt, st_cur, kk_t, ks + 1);
                multiply(cur);  // tiles past the end are all zeros: no branch, the step stays one basic block
                cur = nxt;
                if (ks == 0) store_lds((s + 2) % D, st_write);
            }
            __builtin_amdgcn_iglp_opt(0);  // ask the scheduler to interleave LDS / global traffic with the MFMAs
            __syncthreads();
            st_cur = st_next;
#ifdef RMM_DEBUG_TRACE
            if (tr && tid == 0 && t + 2 < 60) tr[t + 2] = clock64();
#endif
        }
    }
#ifdef RMM_DEBUG_TRACE
    if (tr && tid == 0) tr[60] = clock64();
#endif

    // Epilogue.  The MFMA was issued with the operands swapped (B fragment first), so the
    // accumulators hold C^T tiles: register v of lane l is C(l % 32, 8*(v/4) + 4*(l/32) + v%4)
    // of its 32x32 tile, i.e. every lane owns four runs of four consecutive columns of one row.
    // Storing that directly would touch 32 rows with 16 bytes each per instruction; instead every
    // wave passes a strip of 32 rows x 128 bytes through a private piece of LDS and writes it out
    // with 16 bytes per lane, 8 lanes per row (full 128-byte lines).
    __syncthreads();  // all fragment reads of the main loop are done; LDS is free
    // Two wave groups that split the contraction each end up owning half of the 32x32 tiles of
    // their (identical) wave tile: a group parks the tiles the other one owns in LDS, 16 bytes per
    // lane and run with consecutive lanes consecutive, in rounds that fit the LDS, and adds what
    // the other group parked for it.  Both groups then write their halves.
    static_assert(WAVES_K <= 2, "the cross-group sum is written for two groups");
    constexpr int P = T::TM * T::TN;  // tiles per wave, numbered a * TN + b
    constexpr int OWN = P / WAVES_K;  // group kg owns tiles kg*OWN .. kg*OWN + OWN - 1
    if constexpr (WAVES_K == 2) {
        static_assert(P % 2 == 0, "an even number of tiles per wave");
        constexpr int CH_MAX = T::LDS_BYTES / (64 * T::THREADS);  // tiles per thread and round that fit
        static_assert(CH_MAX >= 1, "one tile per thread fits in LDS");
        constexpr int CH = OWN < CH_MAX ? OWN : CH_MAX;
        float4 *park = reinterpret_cast<float4 *>(lds);
        constexpr int GROUP_THREADS = T::THREADS / 2;
        const int partner = kg == 0 ? tid + GROUP_THREADS : tid - GROUP_THREADS;
        // `first` is a literal at every call, so all accumulator indices are static after unrolling.
        auto park_tiles = [&](auto first, int c0) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int p = decltype(first)::value + c0 + c;
                if (c0 + c < OWN) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        park[(c * 4 + q) * T::THREADS + tid] =
                            make_float4(acc[p / T::TN][p % T::TN][4 * q], acc[p / T::TN][p % T::TN][4 * q + 1],
                                        acc[p / T::TN][p % T::TN][4 * q + 2], acc[p / T::TN][p % T::TN][4 * q + 3]);
                }
            }
        };
        auto add_tiles = [&](auto first, int c0) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int p = decltype(first)::value + c0 + c;
                if (c0 + c < OWN) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 pv = park[(c * 4 + q) * T::THREADS + partner];
                        acc[p / T::TN][p % T::TN][4 * q] += pv.x, acc[p / T::TN][p % T::TN][4 * q + 1] += pv.y;
                        acc[p / T::TN][p % T::TN][4 * q + 2] += pv.z, acc[p / T::TN][p % T::TN][4 * q + 3] += pv.w;
                    }
                }
            }
        };
        using Zero = std::integral_constant<int, 0>;
        using Half = std::integral_constant<int, OWN>;
#pragma unroll
        for (int c0 = 0; c0 < OWN; c0 += CH) {
            if (kg == 0)
                park_tiles(Half(), c0);  // group 0 gives away the upper half
            else
                park_tiles(Zero(), c0);
            __syncthreads();
            if (kg == 0)
                add_tiles(Zero(), c0);
            else
                add_tiles(Half(), c0);
            __syncthreads();
        }
    }
    {
        constexpr int EB = OUT == OUT_BF16 ? 2 : 4;         // bytes per output element
        constexpr int CW = 128 / EB;                         // columns per strip: 64 (bf16) or 32 (fp32)
        constexpr int TPS = CW / 32;                         // 32-column MFMA tiles per strip
        constexpr int PITCH = 128 + 16;                      // bytes per strip row in LDS
        static_assert(T::THREADS / 64 * 32 * PITCH <= T::LDS_BYTES, "staging area fits in LDS");
        static_assert(WAVES_K == 1 || (OWN % TPS == 0 && T::TN % TPS == 0), "no strip straddles the two groups' tiles");
        char *stage = reinterpret_cast<char *>(lds) + wave * 32 * PITCH;
        const int r = lane & 31, h = lane >> 5;
#pragma unroll
        for (int a = 0; a < T::TM; ++a) {
            const int64_t row0 = m0 + wm * T::WTM + a * 32;
#pragma unroll
            for (int b0 = 0; b0 < T::TN; b0 += TPS) {
                if (WAVES_K > 1 && (a * T::TN + b0) / OWN != kg) continue;  // the other group's tiles
                const int64_t col0 = n0 + wn * T::WTN + b0 * 32;
#pragma unroll
                for (int bb = 0; bb < TPS; ++bb) {
                    if (b0 + bb >= T::TN) break;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float v[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) v[u] = acc[a][b0 + bb][4 * q + u];
                        const int c = bb * 32 + 8 * q + 4 * h;  // column inside the strip
                        if constexpr (OUT == OUT_BF16) {
#pragma unroll
                            for (int u = 0; u < 4; ++u) v[u] *= g.alpha;
                            if (g.bias != nullptr && col0 + c < g.N) {
                                const uint2 bv = *reinterpret_cast<const uint2 *>(g.bias + col0 + c);
                                v[0] += __uint_as_float(bv.x << 16);
                                v[1] += __uint_as_float(bv.x & 0xFFFF0000u);
                                v[2] += __uint_as_float(bv.y << 16);
                                v[3] += __uint_as_float(bv.y & 0xFFFF0000u);
                            }
                            union {
                                bf16x2_t hh[2];
                                uint2 u;
                            } o;
                            o.hh[0] = __builtin_convertvector((f32x2_t){v[0], v[1]}, bf16x2_t);  // nearest even
                            o.hh[1] = __builtin_convertvector((f32x2_t){v[2], v[3]}, bf16x2_t);
                            *reinterpret_cast<uint2 *>(stage + r * PITCH + c * 2) = o.u;
                        } else {
                            *reinterpret_cast<float4 *>(stage + r * PITCH + c * 4) = make_float4(v[0], v[1], v[2], v[3]);
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                // read back: lane l takes 16 bytes: chunk (l % 8) of row (l / 8) + 8*i
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int rr = (lane >> 3) + 8 * i, ch = lane & 7;
                    const uint4 d = *reinterpret_cast<const uint4 *>(stage + rr * PITCH + ch * 16);
                    const int64_t row = row0 + rr, col = col0 + ch * (16 / EB);
#ifdef RMM_DEBUG_NOEPI
                    if (g.alpha != 123.0f) continue;
#endif
                    if (row >= g.M || col >= g.N || ch * (16 / EB) >= (T::TN - b0) * 32) continue;
                    if constexpr (OUT == OUT_BF16)
                        *reinterpret_cast<uint4 *>(reinterpret_cast<bf16_t *>(g.C) + row * g.ldc + col) = d;
                    else
                        *reinterpret_cast<uint4 *>(reinterpret_cast<float *>(g.C) +
                                                   (int64_t)blockIdx.z * g.split_stride + row * g.ldc + col) = d;
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
#ifdef RMM_DEBUG_TRACE
    if (tr && tid == 0) tr[63] = clock64(), tr[61] = wall_clock64();
#endif
}

// out[r][c] (bf16) = alpha * sum_s part[s][r][c]; 8 columns per thread.
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float *__restrict__ part, bf16_t *__restrict__ out,
                                                              int64_t elems, int splits, int64_t split_stride,
                                                              float alpha) {
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= elems) return;
    float4 s = *reinterpret_cast<const float4 *>(part + e);
    for (int z = 1; z < splits; ++z) {
        const float4 p = *reinterpret_cast<const float4 *>(part + (int64_t)z * split_stride + e);
        s.x += p.x;
        s.y += p.y;
        s.z += p.z;
        s.w += p.w;
    }
    uint2 o;
    o.x = (uint32_t)f32_to_bf16(alpha * s.x) | ((uint32_t)f32_to_bf16(alpha * s.y) << 16);
    o.y = (uint32_t)f32_to_bf16(alpha * s.z) | ((uint32_t)f32_to_bf16(alpha * s.w) << 16);
    *reinterpret_cast<uint2 *>(out + e) = o;
}

// ---------------------------------------------------------------------------------------------
// Small sketch sizes (k <= 64): S^T A is bound by reading A once from HBM, so this kernel is a
// streaming pass.  A work-group owns 256 columns and one slice of tokens and walks the slice 64
// tokens at a time (global -> registers, D steps in flight -> LDS, two stages).  The four waves
// split the contraction: wave w takes tokens 16w .. 16w+15 of every step, for all 32*TM sketch
// columns and all 256 operand columns, so every sketch entry is generated exactly once per
// work-group and the generator's ALU work stays far below the memory time.  At the end the four
// partial accumulators are summed through LDS and written as fp32 partials of the slice (or,
// with a single slice, scaled and rounded to bf16).
struct SmallkArgs {
    const bf16_t *A;  // n x d
    void *C;          // bf16 k x d, or fp32 partials [slice][k][d]
    int64_t n, d, k;
    int64_t a_bytes;
    int64_t k_chunk;  // tokens per slice (multiple of 128)
    float alpha;
    SketchState st;
};

template <int TM, int KIND, int D, int OUT>
__global__ void __launch_bounds__(256) sketch_smallk_kernel(SmallkArgs g) {
    constexpr int BN = 256, BK = 64, STRIDE = BN + TPAD, STAGE_ELEMS = BK * STRIDE, CHUNKS = BN * BK / 8 / 256;
    constexpr int TN = BN / 32;
    __shared__ __attribute__((aligned(16))) bf16_t lds[2 * STAGE_ELEMS];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t n0 = (int64_t)blockIdx.x * BN;
    const int64_t kk_begin = (int64_t)blockIdx.y * g.k_chunk;
    const int kk_len = (int)(min(g.n, kk_begin + g.k_chunk) - kk_begin);  // >= 1: the host makes no empty slice
    const int num_tiles = (kk_len + BK - 1) / BK;

    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(g.A), (short)0, (int)g.a_bytes, 0x00020000);
    constexpr uint32_t OOB = 0x80000000u;
    uint32_t off[CHUNKS];
    int row_of[CHUNKS], lds_of[CHUNKS];
#pragma unroll
    for (int q = 0; q < CHUNKS; ++q) {
        const int c = tid + 256 * q, row = c / (BN / 8), nc = c % (BN / 8);
        row_of[q] = row, lds_of[q] = row * STRIDE + nc * 8;
        off[q] = n0 + nc * 8 < g.d ? (uint32_t)(((kk_begin + row) * g.d + n0 + nc * 8) * 2) : OOB;
    }
    const uint32_t step_bytes = (uint32_t)(BK * g.d * 2);

    u32x4_t rb[D][CHUNKS];
    auto issue = [&](int set, int t) {
#pragma unroll
        for (int q = 0; q < CHUNKS; ++q) {
            const bool ok = t * BK + row_of[q] < kk_len;  // also false for every t >= num_tiles
            rb[set][q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, ok ? off[q] + (uint32_t)t * step_bytes : OOB, 0, 0);
        }
    };
    auto store_lds = [&](int set, int stage) {
#pragma unroll
        for (int q = 0; q < CHUNKS; ++q)
            *reinterpret_cast<u32x4_t *>(lds + stage * STAGE_ELEMS + lds_of[q]) = rb[set][q];
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

#pragma unroll
    for (int s = 0; s < D; ++s) issue(s, s);
    store_lds(0, 0);
    __syncthreads();
    const int groups = (num_tiles + D - 1) / D;
    for (int grp = 0; grp < groups; ++grp) {
#pragma unroll
        for (int s = 0; s < D; ++s) {
            const int t = grp * D + s;
            issue(s, t + D);
            if (t < num_tiles) {
                const bf16_t *Bs = lds + (t & 1) * STAGE_ELEMS;
                const int tok = (int)kk_begin + t * BK + 16 * wave + ((lane >> 5) << 3);  // this lane's first token
                bf16x8_t af[TM], bfr[TN];
#pragma unroll
                for (int a = 0; a < TM; ++a) {
                    const uint32_t j = (uint32_t)(a * 32 + (lane & 31));
                    if constexpr (KIND == 0) {
                        af[a] = gauss_operand(g.st, (uint32_t)(tok >> 3), j);
                    } else {
                        const Words4 rw =
                            philox4x32_10((uint32_t)(tok >> 7), j, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
                        af[a] = radem_operand(rw, (uint32_t)tok);
                    }
                }
#pragma unroll
                for (int b = 0; b < TN; ++b) bfr[b] = frag_transposed(Bs, STRIDE, b * 32, 16 * wave, lane);
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b], af[a], acc[a][b], 0, 0, 0);
            }
            store_lds((s + 1) % D, (t + 1) & 1);
            __syncthreads();  // step t is consumed everywhere, step t+1 is visible
        }
    }

    // Sum the four waves' accumulators, 32 rows x 128 columns at a time: every wave puts its block
    // into its own LDS region, then all threads add the four regions and write full rows.
    // (Accumulator register v of lane l is C(l % 32, 8*(v/4) + 4*(l/32) + v%4) of a 32x32 tile.)
    constexpr int PITCH = 128 * 4 + 16;  // bytes per row of a region
    static_assert(4 * 32 * PITCH <= 2 * STAGE_ELEMS * 2, "reduction regions fit in LDS");
    char *region = reinterpret_cast<char *>(lds);
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int bb = 0; bb < 4; ++bb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16_t &t = acc[a][half * 4 + bb];
                    *reinterpret_cast<float4 *>(region + (wave * 32 + r) * PITCH + (bb * 32 + 8 * q + 4 * h) * 4) =
                        make_float4(t[4 * q], t[4 * q + 1], t[4 * q + 2], t[4 * q + 3]);
                }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int f = tid + 256 * i, row = f >> 5, c4 = f & 31;
                float4 s = *reinterpret_cast<const float4 *>(region + row * PITCH + c4 * 16);
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    const float4 p = *reinterpret_cast<const float4 *>(region + (w * 32 + row) * PITCH + c4 * 16);
                    s.x += p.x, s.y += p.y, s.z += p.z, s.w += p.w;
                }
                const int64_t grow = a * 32 + row, gcol = n0 + half * 128 + c4 * 4;
                if (grow < g.k && gcol < g.d) {  // d is a multiple of 4
                    if constexpr (OUT == OUT_BF16) {
                        union {
                            bf16x2_t hh[2];
                            uint2 u;
                        } o;
                        o.hh[0] = __builtin_convertvector((f32x2_t){g.alpha * s.x, g.alpha * s.y}, bf16x2_t);
                        o.hh[1] = __builtin_convertvector((f32x2_t){g.alpha * s.z, g.alpha * s.w}, bf16x2_t);
                        *reinterpret_cast<uint2 *>(reinterpret_cast<bf16_t *>(g.C) + grow * g.d + gcol) = o.u;
                    } else {
                        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(g.C) +
                                                    ((int64_t)blockIdx.y * g.k + grow) * g.d + gcol) = s;
                    }
                }
            }
            __syncthreads();
        }
}

// Prefetch depths (register sets of tiles in flight) to choose from.
#ifndef RMM_TUNE_D1
#define RMM_TUNE_D1 4
#endif
#ifndef RMM_TUNE_D2
#define RMM_TUNE_D2 3
#endif
#ifndef RMM_TUNE_SK_D
#define RMM_TUNE_SK_D 3
#endif

#ifdef RMM_DEBUG_TRACE
unsigned long long *g_trace = nullptr;
#endif
#ifndef RMM_TUNE_LARGE
#define RMM_TUNE_LARGE 256, 256, 32, 2, 4, 1
#endif
#ifndef RMM_TUNE_SPLIT_MIN_K
#define RMM_TUNE_SPLIT_MIN_K 1536
#endif
#ifndef RMM_TUNE_LARGE_MIN_TILES
#define RMM_TUNE_LARGE_MIN_TILES 160
#endif

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int WAVES_K, int AMODE, int BMODE, int OUT>
hipError_t launch(const GemmArgs &g_in, int splits, hipStream_t stream) {
    GemmArgs g = g_in;
#ifdef RMM_DEBUG_TRACE
    g.trace = (AMODE == RMM_DEBUG_TRACE_A && BMODE == RMM_DEBUG_TRACE_B) ? g_trace : nullptr;
#endif
    const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    dim3 grid((unsigned)tiles, 1, (unsigned)splits);
    // The kernel runs whole groups of D tiles; take the depth that wastes fewer.
    const int64_t kt = (min(g.K, g.k_chunk) + BK - 1) / BK;
    if constexpr (AMODE == A_GAUSS || AMODE == A_RADEM) {
        // The sketch kernels load one operand only and need their registers for wide wave tiles.
        gemm_mfma_kernel<BM, BN, BK, WAVES_M, WAVES_N, WAVES_K, AMODE, BMODE, OUT, RMM_TUNE_SK_D>
            <<<grid, 64 * WAVES_M * WAVES_N * WAVES_K, 0, stream>>>(g);
        return hipGetLastError();
    }
    const int64_t pad1 = (kt + RMM_TUNE_D1 - 1) / RMM_TUNE_D1 * RMM_TUNE_D1 - kt;
    const int64_t pad2 = (kt + RMM_TUNE_D2 - 1) / RMM_TUNE_D2 * RMM_TUNE_D2 - kt;
    if (pad1 <= pad2)
        gemm_mfma_kernel<BM, BN, BK, WAVES_M, WAVES_N, WAVES_K, AMODE, BMODE, OUT, RMM_TUNE_D1>
            <<<grid, 64 * WAVES_M * WAVES_N * WAVES_K, 0, stream>>>(g);
    else
        gemm_mfma_kernel<BM, BN, BK, WAVES_M, WAVES_N, WAVES_K, AMODE, BMODE, OUT, RMM_TUNE_D2>
            <<<grid, 64 * WAVES_M * WAVES_N * WAVES_K, 0, stream>>>(g);
    return hipGetLastError();
}

// Large outputs: 256x256 tiles (half the operand traffic per flop), one work-group per compute
// unit, prefetch depth 3.  Worth it once there is at least one such tile per compute unit.
template <int AMODE, int BMODE>
hipError_t launch_large(const GemmArgs &g_in, hipStream_t stream) {
    GemmArgs g = g_in;
#ifdef RMM_DEBUG_TRACE
    g.trace = nullptr;
#endif
    const int64_t tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    typedef Tile<RMM_TUNE_LARGE, AMODE, BMODE, OUT_BF16> T;
    gemm_mfma_kernel<RMM_TUNE_LARGE, AMODE, BMODE, OUT_BF16, 3><<<dim3((unsigned)tiles), T::THREADS, 0, stream>>>(g);
    return hipGetLastError();
}

bool large_tiles_pay(int64_t m, int64_t n) { return ((m + 255) / 256) * ((n + 255) / 256) >= RMM_TUNE_LARGE_MIN_TILES; }

// Few 128x128 tiles (at most one per compute unit) and a long contraction: two wave groups per
// tile split the contraction, so that a compute unit still holds eight waves.
bool split_waves_pay(int64_t m, int64_t n, int64_t kk) {
    return ((m + 127) / 128) * ((n + 127) / 128) <= 256 && kk >= RMM_TUNE_SPLIT_MIN_K;
}

}  // namespace

// Tile shapes: BM, BN, BK, waves along M, waves along N, wave groups along the contraction.
#ifndef RMM_TUNE_NT
#define RMM_TUNE_NT 128, 128, 32, 2, 2, 1
#endif
#ifndef RMM_TUNE_NN
#define RMM_TUNE_NN 128, 128, 32, 2, 2, 1
#endif
#ifndef RMM_TUNE_DW
#define RMM_TUNE_DW 128, 128, 32, 2, 2, 1
#endif
#ifndef RMM_TUNE_SPLIT
#define RMM_TUNE_SPLIT 128, 128, 64, 2, 2, 2
#endif
#ifndef RMM_TUNE_SK
#define RMM_TUNE_SK 128, 256, 64, 4, 1, 2
#endif
#ifndef RMM_TUNE_SK_BM
#define RMM_TUNE_SK_BM 128
#define RMM_TUNE_SK_BN 256
#endif
#ifndef RMM_TUNE_SK_WGS
#define RMM_TUNE_SK_WGS 256
#endif
// Streaming kernel for k <= 64: work-groups aimed at, prefetch depth for k <= 32 and for k <= 64.
#ifndef RMM_TUNE_SMALLK_WGS
#define RMM_TUNE_SMALLK_WGS 256
#endif
#ifndef RMM_TUNE_SMALLK_D1
#define RMM_TUNE_SMALLK_D1 4
#endif
#ifndef RMM_TUNE_SMALLK_D2
#define RMM_TUNE_SMALLK_D2 4
#endif

#ifdef RMM_DEBUG_TRACE
extern "C" void rmm_debug_set_trace(void *p) { g_trace = (unsigned long long *)p; }
#endif

bool mfma_shape_ok(int64_t n, int64_t d_in, int64_t d_out, int64_t k) {
    // 16-byte chunks need widths that are multiples of 8; buffer loads need operands below 2^31 bytes.
    const int64_t lim = ((int64_t)1 << 31) / 2;
    const int64_t rows = n > k ? n : k, cols = d_in > d_out ? d_in : d_out;
    return d_in % 8 == 0 && d_out % 8 == 0 && rows * cols < lim && d_in * d_out < lim;
}

hipError_t launch_linear_nt_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, int64_t n,
                                 int64_t d_in, int64_t d_out, hipStream_t stream) {
    GemmArgs g{};
    g.A = X, g.lda = d_in, g.B = W, g.ldb = d_in, g.C = Y, g.ldc = d_out, g.bias = bias;
    g.M = n, g.N = d_out, g.K = d_in, g.alpha = 1.0f, g.k_chunk = (d_in + 127) / 128 * 128;
    g.a_bytes = n * d_in * 2, g.b_bytes = d_out * d_in * 2;
    if (large_tiles_pay(g.M, g.N)) return launch_large<A_KCONTIG, B_KCONTIG>(g, stream);
    if (split_waves_pay(g.M, g.N, g.K)) return launch<RMM_TUNE_SPLIT, A_KCONTIG, B_KCONTIG, OUT_BF16>(g, 1, stream);
    return launch<RMM_TUNE_NT, A_KCONTIG, B_KCONTIG, OUT_BF16>(g, 1, stream);
}

hipError_t launch_linear_nn_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, int64_t n, int64_t d_in,
                                 int64_t d_out, hipStream_t stream) {
    GemmArgs g{};
    g.A = dY, g.lda = d_out, g.B = W, g.ldb = d_in, g.C = dX, g.ldc = d_in, g.bias = nullptr;
    g.M = n, g.N = d_in, g.K = d_out, g.alpha = 1.0f, g.k_chunk = (d_out + 127) / 128 * 128;
    g.a_bytes = n * d_out * 2, g.b_bytes = d_out * d_in * 2;
    if (large_tiles_pay(g.M, g.N)) return launch_large<A_KCONTIG, B_NCONTIG>(g, stream);
    if (split_waves_pay(g.M, g.N, g.K)) return launch<RMM_TUNE_SPLIT, A_KCONTIG, B_NCONTIG, OUT_BF16>(g, 1, stream);
    return launch<RMM_TUNE_NN, A_KCONTIG, B_NCONTIG, OUT_BF16>(g, 1, stream);
}

hipError_t launch_dw_bf16(const bf16_t *G, const bf16_t *X_proj, bf16_t *dW, int64_t k, int64_t d_in, int64_t d_out,
                          hipStream_t stream) {
    GemmArgs g{};
    g.A = G, g.lda = d_out, g.B = X_proj, g.ldb = d_in, g.C = dW, g.ldc = d_in, g.bias = nullptr;
    g.M = d_out, g.N = d_in, g.K = k, g.alpha = 1.0f, g.k_chunk = (k + 127) / 128 * 128;
    g.a_bytes = k * d_out * 2, g.b_bytes = k * d_in * 2;
    if (large_tiles_pay(g.M, g.N)) return launch_large<A_MCONTIG, B_NCONTIG>(g, stream);
    if (split_waves_pay(g.M, g.N, g.K)) return launch<RMM_TUNE_SPLIT, A_MCONTIG, B_NCONTIG, OUT_BF16>(g, 1, stream);
    return launch<RMM_TUNE_DW, A_MCONTIG, B_NCONTIG, OUT_BF16>(g, 1, stream);
}

// Token slices of the sketch product: at most one (tile, slice) pair per compute unit where
// the tile count allows, each slice a multiple of 128 tokens, none empty.
static int sketch_slices(int64_t n, int64_t d, int64_t k, int64_t *k_chunk) {
    const int64_t tiles = ((k + RMM_TUNE_SK_BM - 1) / RMM_TUNE_SK_BM) * ((d + RMM_TUNE_SK_BN - 1) / RMM_TUNE_SK_BN);
    const int64_t blocks = (n + 127) / 128;
    int64_t s = RMM_TUNE_SK_WGS / tiles;
    if (s > blocks) s = blocks;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    *k_chunk = (blocks + s - 1) / s * 128;
    return (int)((n + *k_chunk - 1) / *k_chunk);
}

// Same for the streaming kernel of small sketch sizes (256-column work-groups, one per compute unit).
constexpr int64_t kSmallK = 64;
static int smallk_slices(int64_t n, int64_t d, int64_t *k_chunk) {
    const int64_t col_tiles = (d + 255) / 256, blocks = (n + 127) / 128;
    int64_t s = RMM_TUNE_SMALLK_WGS / col_tiles;
    if (s > blocks) s = blocks;
    if (s < 1) s = 1;
    *k_chunk = (blocks + s - 1) / s * 128;
    return (int)((n + *k_chunk - 1) / *k_chunk);
}

size_t sketch_workspace_bf16(int64_t n, int64_t d, int64_t k) {
    int64_t k_chunk;
    const int s = k <= kSmallK ? smallk_slices(n, d, &k_chunk) : sketch_slices(n, d, k, &k_chunk);
    return s > 1 ? (size_t)s * (size_t)k * (size_t)d * sizeof(float) : 0;
}

template <int TM, int KIND>
static hipError_t launch_smallk(const SmallkArgs &g, int slices, hipStream_t stream) {
    constexpr int D = TM == 1 ? RMM_TUNE_SMALLK_D1 : RMM_TUNE_SMALLK_D2;
    dim3 grid((unsigned)((g.d + 255) / 256), (unsigned)slices);
    if (slices == 1)
        sketch_smallk_kernel<TM, KIND, D, OUT_BF16><<<grid, 256, 0, stream>>>(g);
    else
        sketch_smallk_kernel<TM, KIND, D, OUT_F32_PARTIAL><<<grid, 256, 0, stream>>>(g);
    return hipGetLastError();
}

namespace {
// Brackets the product kernel (not the sum over token slices) with the caller's events.
struct ProductEvents {
    hipEvent_t begin, end;
    hipStream_t stream;
    ProductEvents(hipEvent_t b, hipEvent_t e, hipStream_t s) : begin(b), end(e), stream(s) {
        if (begin != nullptr && end != nullptr) (void)hipEventRecord(begin, stream);
    }
    void done() {
        if (begin != nullptr && end != nullptr) (void)hipEventRecord(end, stream);
        begin = end = nullptr;
    }
    ~ProductEvents() { done(); }
};
}  // namespace

hipError_t launch_sketch_bf16(const bf16_t *A, bf16_t *out, int64_t n, int64_t d, int64_t k, int kind, SketchState st,
                              void *ws, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
    const float alpha = 1.0f / sqrtf((float)k);
    ProductEvents pev(ev_begin, ev_end, stream);
    if (k <= kSmallK) {  // bound by one pass over A: streaming kernel
        SmallkArgs a{};
        a.A = A, a.n = n, a.d = d, a.k = k, a.a_bytes = n * d * 2, a.st = st;
        const int slices = smallk_slices(n, d, &a.k_chunk);
        a.C = slices == 1 ? (void *)out : ws, a.alpha = alpha;
        hipError_t e = k <= 32 ? (kind == 0 ? launch_smallk<1, 0>(a, slices, stream) : launch_smallk<1, 1>(a, slices, stream))
                               : (kind == 0 ? launch_smallk<2, 0>(a, slices, stream) : launch_smallk<2, 1>(a, slices, stream));
        pev.done();
        if (e != hipSuccess || slices == 1) return e;
        const int64_t elems = k * d;
        reduce_partials_kernel<<<(unsigned)((elems / 4 + 255) / 256), 256, 0, stream>>>((const float *)ws, out, elems,
                                                                                         slices, k * d, alpha);
        return hipGetLastError();
    }
    GemmArgs g{};
    g.A = nullptr, g.lda = 0, g.B = A, g.ldb = d, g.bias = nullptr;
    g.M = k, g.N = d, g.K = n, g.st = st, g.ldc = d;
    g.a_bytes = 0, g.b_bytes = n * d * 2;
    const int splits = sketch_slices(n, d, k, &g.k_chunk);
    hipError_t e;
    if (splits == 1) {
        g.C = out, g.alpha = alpha;
        e = kind == 0 ? launch<RMM_TUNE_SK, A_GAUSS, B_NCONTIG, OUT_BF16>(g, 1, stream)
                      : launch<RMM_TUNE_SK, A_RADEM, B_NCONTIG, OUT_BF16>(g, 1, stream);
        return e;
    }
    g.C = ws, g.alpha = 1.0f, g.split_stride = k * d;
    e = kind == 0 ? launch<RMM_TUNE_SK, A_GAUSS, B_NCONTIG, OUT_F32_PARTIAL>(g, splits, stream)
                  : launch<RMM_TUNE_SK, A_RADEM, B_NCONTIG, OUT_F32_PARTIAL>(g, splits, stream);
    pev.done();
    if (e != hipSuccess) return e;
    const int64_t elems = k * d;  // d % 8 == 0, so elems % 4 == 0
    reduce_partials_kernel<<<(unsigned)((elems / 4 + 255) / 256), 256, 0, stream>>>((const float *)ws, out, elems,
                                                                                     splits, k * d, alpha);
    return hipGetLastError();
}

}  // namespace rmm
