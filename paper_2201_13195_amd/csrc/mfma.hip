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

namespace rmm {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

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
    float alpha;
    SketchState st;
    int64_t k_chunk;       // contraction elements per blockIdx.z slice (multiple of 128)
    int64_t split_stride;  // fp32 elements between the partial results of two slices
};

__device__ __forceinline__ uint4 ld16(const bf16_t *p, bool pred) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (pred) v = *reinterpret_cast<const uint4 *>(p);
    return v;
}

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

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int AMODE, int BMODE, int OUT>
struct Tile {
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
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
    static constexpr int LDS_BYTES = 2 * STAGE_ELEMS * 2;
    static constexpr int A_CHUNKS = A_IN_LDS ? BM * BK / 8 / THREADS : 0;  // 16-byte chunks per thread and tile
    static constexpr int B_CHUNKS = BN * BK / 8 / THREADS;
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0 && BK % 16 == 0, "tile shape");
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

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int AMODE, int BMODE, int OUT>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) gemm_mfma_kernel(GemmArgs g) {
    typedef Tile<BM, BN, BK, WAVES_M, WAVES_N, AMODE, BMODE, OUT> T;
    __shared__ __attribute__((aligned(16))) bf16_t lds[2 * T::STAGE_ELEMS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int64_t tiles_n = (g.N + BN - 1) / BN;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * BM, n0 = (int64_t)(blockIdx.x % tiles_n) * BN;
    const int64_t kk_begin = (int64_t)blockIdx.z * g.k_chunk;
    const int64_t kk_end = min(g.K, kk_begin + g.k_chunk);
    const int num_tiles = (int)((kk_end - kk_begin + BK - 1) / BK);

    f32x16_t acc[T::TM][T::TN];
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    uint4 ra[T::A_CHUNKS > 0 ? T::A_CHUNKS : 1], rb[T::B_CHUNKS];

    auto load_global = [&](int64_t kk0) {
        if constexpr (AMODE == A_KCONTIG) {  // A[m][kk], tile BM x BK
#pragma unroll
            for (int q = 0; q < T::A_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BK / 8), kc = c % (BK / 8);
                const int64_t gm = m0 + row, gk = kk0 + kc * 8;
                ra[q] = ld16(g.A + gm * g.lda + gk, gm < g.M && gk < kk_end);
            }
        } else if constexpr (AMODE == A_MCONTIG) {  // A stored [kk][m], tile BK x BM
#pragma unroll
            for (int q = 0; q < T::A_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BM / 8), mc = c % (BM / 8);
                const int64_t gk = kk0 + row, gm = m0 + mc * 8;
                ra[q] = ld16(g.A + gk * g.lda + gm, gk < kk_end && gm < g.M);
            }
        }
        if constexpr (BMODE == B_KCONTIG) {  // B stored [n][kk], tile BN x BK
#pragma unroll
            for (int q = 0; q < T::B_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BK / 8), kc = c % (BK / 8);
                const int64_t gn = n0 + row, gk = kk0 + kc * 8;
                rb[q] = ld16(g.B + gn * g.ldb + gk, gn < g.N && gk < kk_end);
            }
        } else {  // B stored [kk][n], tile BK x BN
#pragma unroll
            for (int q = 0; q < T::B_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BN / 8), nc = c % (BN / 8);
                const int64_t gk = kk0 + row, gn = n0 + nc * 8;
                rb[q] = ld16(g.B + gk * g.ldb + gn, gk < kk_end && gn < g.N);
            }
        }
    };

    auto store_lds = [&](int stage) {
        bf16_t *As = lds + stage * T::STAGE_ELEMS;
        bf16_t *Bs = As + T::A_ELEMS;
        if constexpr (AMODE == A_KCONTIG) {
#pragma unroll
            for (int q = 0; q < T::A_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BK / 8), kc = c % (BK / 8);
                *reinterpret_cast<uint4 *>(As + row * T::A_STRIDE + kc * 8) = ra[q];
            }
        } else if constexpr (AMODE == A_MCONTIG) {
#pragma unroll
            for (int q = 0; q < T::A_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BM / 8), mc = c % (BM / 8);
                *reinterpret_cast<uint4 *>(As + row * T::A_STRIDE + mc * 8) = ra[q];
            }
        }
        if constexpr (BMODE == B_KCONTIG) {
#pragma unroll
            for (int q = 0; q < T::B_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BK / 8), kc = c % (BK / 8);
                *reinterpret_cast<uint4 *>(Bs + row * T::B_STRIDE + kc * 8) = rb[q];
            }
        } else {
#pragma unroll
            for (int q = 0; q < T::B_CHUNKS; ++q) {
                const int c = tid + T::THREADS * q, row = c / (BN / 8), nc = c % (BN / 8);
                *reinterpret_cast<uint4 *>(Bs + row * T::B_STRIDE + nc * 8) = rb[q];
            }
        }
    };

    if (num_tiles > 0) {
        load_global(kk_begin);
        store_lds(0);
    }
    __syncthreads();

    for (int t = 0; t < num_tiles; ++t) {
        const int64_t kk0 = kk_begin + (int64_t)t * BK;
        const bool more = t + 1 < num_tiles;
        if (more) load_global(kk0 + BK);

        const bf16_t *As = lds + (t & 1) * T::STAGE_ELEMS;
        const bf16_t *Bs = As + T::A_ELEMS;

        Words4 rw[T::TM];
        if constexpr (AMODE == A_RADEM) {
#pragma unroll
            for (int a = 0; a < T::TM; ++a) {
                const uint32_t j = (uint32_t)(m0 + wm * T::WTM + a * 32 + (lane & 31));
                rw[a] = philox4x32_10((uint32_t)(kk0 >> 7), j, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
            }
        }

#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t af[T::TM], bfr[T::TN];
#pragma unroll
            for (int a = 0; a < T::TM; ++a) {
                const int row0 = wm * T::WTM + a * 32;
                if constexpr (AMODE == A_KCONTIG) {
                    af[a] = frag_kcontig(As, T::A_STRIDE, row0, ks * 16, lane);
                } else if constexpr (AMODE == A_MCONTIG) {
                    af[a] = frag_transposed(As, T::A_STRIDE, row0, ks * 16, lane);
                } else {
                    const uint32_t j = (uint32_t)(m0 + row0 + (lane & 31));
                    const int64_t tok = kk0 + ks * 16 + ((lane >> 5) << 3);  // first of this lane's 8 tokens
                    if constexpr (AMODE == A_GAUSS)
                        af[a] = gauss_operand(g.st, (uint32_t)(tok >> 3), j);
                    else
                        af[a] = radem_operand(rw[a], (uint32_t)tok);
                }
            }
#pragma unroll
            for (int b = 0; b < T::TN; ++b) {
                const int col0 = wn * T::WTN + b * 32;
                if constexpr (BMODE == B_KCONTIG)
                    bfr[b] = frag_kcontig(Bs, T::B_STRIDE, col0, ks * 16, lane);
                else
                    bfr[b] = frag_transposed(Bs, T::B_STRIDE, col0, ks * 16, lane);
            }
#pragma unroll
            for (int a = 0; a < T::TM; ++a)
#pragma unroll
                for (int b = 0; b < T::TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }

        if (more) store_lds((t + 1) & 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register v of lane l is C(8*(v/4) + 4*(l/32) + v%4, l%32) of its 32x32 tile.
#pragma unroll
    for (int a = 0; a < T::TM; ++a)
#pragma unroll
        for (int b = 0; b < T::TN; ++b) {
            const int64_t col = n0 + wn * T::WTN + b * 32 + (lane & 31);
            if (col >= g.N) continue;
            float bias = 0.0f;
            if constexpr (OUT == OUT_BF16)
                if (g.bias != nullptr) bias = bf16_to_f32(g.bias[col]);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm * T::WTM + a * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
                if (row >= g.M) continue;
                if constexpr (OUT == OUT_BF16) {
                    reinterpret_cast<bf16_t *>(g.C)[row * g.ldc + col] = f32_to_bf16(g.alpha * acc[a][b][v] + bias);
                } else {
                    reinterpret_cast<float *>(g.C)[(int64_t)blockIdx.z * g.split_stride + row * g.ldc + col] =
                        acc[a][b][v];
                }
            }
        }
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

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int AMODE, int BMODE, int OUT>
hipError_t launch(const GemmArgs &g, int splits, hipStream_t stream) {
    const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    dim3 grid((unsigned)tiles, 1, (unsigned)splits);
    gemm_mfma_kernel<BM, BN, BK, WAVES_M, WAVES_N, AMODE, BMODE, OUT><<<grid, 64 * WAVES_M * WAVES_N, 0, stream>>>(g);
    return hipGetLastError();
}

}  // namespace

bool mfma_shape_ok(int64_t n, int64_t d_in, int64_t d_out, int64_t k) {
    (void)n;
    (void)k;
    return d_in % 8 == 0 && d_out % 8 == 0;
}

hipError_t launch_linear_nt_bf16(const bf16_t *X, const bf16_t *W, const bf16_t *bias, bf16_t *Y, int64_t n,
                                 int64_t d_in, int64_t d_out, hipStream_t stream) {
    GemmArgs g{};
    g.A = X, g.lda = d_in, g.B = W, g.ldb = d_in, g.C = Y, g.ldc = d_out, g.bias = bias;
    g.M = n, g.N = d_out, g.K = d_in, g.alpha = 1.0f, g.k_chunk = (d_in + 127) / 128 * 128;
    return launch<128, 128, 64, 2, 2, A_KCONTIG, B_KCONTIG, OUT_BF16>(g, 1, stream);
}

hipError_t launch_linear_nn_bf16(const bf16_t *dY, const bf16_t *W, bf16_t *dX, int64_t n, int64_t d_in,
                                 int64_t d_out, hipStream_t stream) {
    GemmArgs g{};
    g.A = dY, g.lda = d_out, g.B = W, g.ldb = d_in, g.C = dX, g.ldc = d_in, g.bias = nullptr;
    g.M = n, g.N = d_in, g.K = d_out, g.alpha = 1.0f, g.k_chunk = (d_out + 127) / 128 * 128;
    return launch<128, 128, 64, 2, 2, A_KCONTIG, B_NCONTIG, OUT_BF16>(g, 1, stream);
}

hipError_t launch_dw_bf16(const bf16_t *G, const bf16_t *X_proj, bf16_t *dW, int64_t k, int64_t d_in, int64_t d_out,
                          hipStream_t stream) {
    GemmArgs g{};
    g.A = G, g.lda = d_out, g.B = X_proj, g.ldb = d_in, g.C = dW, g.ldc = d_in, g.bias = nullptr;
    g.M = d_out, g.N = d_in, g.K = k, g.alpha = 1.0f, g.k_chunk = (k + 127) / 128 * 128;
    return launch<128, 128, 64, 2, 2, A_MCONTIG, B_NCONTIG, OUT_BF16>(g, 1, stream);
}

int sketch_splits_bf16(int64_t n, int64_t d, int64_t k) {
    const int64_t tiles = ((k + 127) / 128) * ((d + 127) / 128);
    const int64_t chunks = (n + 127) / 128;  // slices are multiples of 128 tokens
    int64_t s = (2 * 256 + tiles - 1) / tiles;  // aim at two work-groups per compute unit
    if (s > chunks) s = chunks;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

size_t sketch_workspace_bf16(int64_t n, int64_t d, int64_t k) {
    const int s = sketch_splits_bf16(n, d, k);
    return s > 1 ? (size_t)s * (size_t)k * (size_t)d * sizeof(float) : 0;
}

hipError_t launch_sketch_bf16(const bf16_t *A, bf16_t *out, int64_t n, int64_t d, int64_t k, int kind, SketchState st,
                              void *ws, hipStream_t stream) {
    const int splits = sketch_splits_bf16(n, d, k);
    const float alpha = 1.0f / sqrtf((float)k);
    GemmArgs g{};
    g.A = nullptr, g.lda = 0, g.B = A, g.ldb = d, g.bias = nullptr;
    g.M = k, g.N = d, g.K = n, g.st = st, g.ldc = d;
    const int64_t chunks = (n + 127) / 128;
    g.k_chunk = (chunks + splits - 1) / splits * 128;
    hipError_t e;
    if (splits == 1) {
        g.C = out, g.alpha = alpha;
        e = kind == 0 ? launch<128, 128, 64, 2, 2, A_GAUSS, B_NCONTIG, OUT_BF16>(g, 1, stream)
                      : launch<128, 128, 64, 2, 2, A_RADEM, B_NCONTIG, OUT_BF16>(g, 1, stream);
        return e;
    }
    g.C = ws, g.alpha = 1.0f, g.split_stride = k * d;
    e = kind == 0 ? launch<128, 128, 64, 2, 2, A_GAUSS, B_NCONTIG, OUT_F32_PARTIAL>(g, splits, stream)
                  : launch<128, 128, 64, 2, 2, A_RADEM, B_NCONTIG, OUT_F32_PARTIAL>(g, splits, stream);
    if (e != hipSuccess) return e;
    const int64_t elems = k * d;  // d % 8 == 0, so elems % 4 == 0
    reduce_partials_kernel<<<(unsigned)((elems / 4 + 255) / 256), 256, 0, stream>>>((const float *)ws, out, elems,
                                                                                     splits, k * d, alpha);
    return hipGetLastError();
}

}  // namespace rmm
