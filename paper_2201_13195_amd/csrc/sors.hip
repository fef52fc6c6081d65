// The SORS sketch kind (subsampled orthonormal matrix with random signs; the paper names the
// family in Section 2.1 and points at its O(B N log B) cost in Section 3.5 and in the future-work
// paragraph, without a construction; the one used here is stated in include/rmm.h): the token signs,
// the Walsh-Hadamard transform along the token axis and the row selection in one pass over A.
//
//   A_proj[j][c] = (1 / sqrt(k)) * sum_i (-1)^popcount(i AND r_j) * sigma_i * A[i][c]
//
// A work-group owns C neighbouring columns of A and all tokens.  It reads its C x n strip once
// (one load of C bf16 per token row), keeps it as fp32 in LDS (one plane of n_pad tokens per
// column), runs the log2(n_pad) butterfly stages four at a time (a thread takes 16 tokens that
// differ in the four index bits of the pass into registers, does the four stages there and puts
// them back), and finally writes the k selected rows, scaled and rounded to bf16.  The first pass
// is fused with the load and the sign flip.  Bound: one read of A from HBM.
//
// LDS layout: plane c starts at c * PLANE; token t sits at t + t / 16 (one float of padding per 16
// tokens), which keeps the 16-token-stride accesses of the last pass and the 64-consecutive-token
// accesses of the other passes off each other's banks.
#include "sors_kernels.hpp"

namespace rmm {

namespace {

template <int L>
struct SorsShape {
    static constexpr int NP = 1 << L;                      // tokens the transform runs over
    static constexpr int C = L <= 12 ? 8 : (32768 >> L);   // columns per work-group: NP * C <= 32768 floats
    static constexpr int PLANE = NP + NP / 16;
    static constexpr int SIGN_WORDS = NP / 32;
    static_assert(L >= 13 && L <= 15, "8192 .. 32768 tokens");
};

// Butterfly stages over W index bits held in registers: v[i] and v[i + h] -> sum and difference.
template <int W, int C>
__device__ __forceinline__ void sors_butterflies(float (&v)[1 << W][C]) {
#pragma unroll
    for (int h = 1; h < (1 << W); h <<= 1)
#pragma unroll
        for (int i = 0; i < (1 << W); ++i)
            if ((i & h) == 0) {
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const float a = v[i][c], b = v[i + h][c];
                    v[i][c] = a + b;
                    v[i + h][c] = a - b;
                }
            }
}

// The stages of index bits SHIFT .. SHIFT + W - 1, on all planes, through registers.
template <int L, int SHIFT, int W>
__device__ __forceinline__ void sors_lds_pass(float *planes, int tid) {
    typedef SorsShape<L> S;
    constexpr int VEC = S::NP >> W;  // vectors of 2^W tokens per plane
    for (int item = tid; item < S::C * VEC; item += 256) {
        const int p = item / VEC, b = item % VEC;
        const int low = b & ((1 << SHIFT) - 1), high = b >> SHIFT;
        const int base = (high << (SHIFT + W)) | low;
        float *plane = planes + p * S::PLANE;
        float v[1 << W][1];
#pragma unroll
        for (int i = 0; i < (1 << W); ++i) v[i][0] = plane[sors_phys(base + (i << SHIFT))];
        sors_butterflies<W, 1>(v);
#pragma unroll
        for (int i = 0; i < (1 << W); ++i) plane[sors_phys(base + (i << SHIFT))] = v[i][0];
    }
}

template <int C>
struct SorsRow;  // C bf16 values of one row as one load / store
template <>
struct SorsRow<8> { typedef sors_u32x4_t type; };
template <>
struct SorsRow<4> { typedef sors_u32x2_t type; };
template <>
struct SorsRow<2> { typedef uint32_t type; };
template <>
struct SorsRow<1> { typedef uint16_t type; };

template <int L>
__global__ void __launch_bounds__(256) sors_kernel(SorsArgs g) {
    typedef SorsShape<L> S;
    constexpr int NP = S::NP, C = S::C;
    typedef typename SorsRow<C>::type row_t;
    __shared__ __attribute__((aligned(16))) float planes[C * S::PLANE];
    __shared__ uint32_t sign_words[S::SIGN_WORDS];
    const int tid = threadIdx.x;

    // Column groups that share 128-byte lines of A (8 groups of 8 columns) should meet in one L2:
    // work-groups are dealt round-robin to the 8 XCDs, so XCD x gets a contiguous run of groups.
    int64_t group = blockIdx.x;
    {
        const int64_t groups = gridDim.x, per = groups / 8, rem = groups % 8, x = group % 8, r = group / 8;
        group = x * per + (x < rem ? x : rem) + r;
    }
    const int64_t col0 = group * C;

    // sigma: the sign bits of tokens 128c .. 128c+127 are the four words of call c
    for (int c = tid; c < NP / 128; c += 256) {
        const Words4 w = philox4x32_10((uint32_t)c, kSorsSignColumn, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
#pragma unroll
        for (int q = 0; q < 4; ++q) sign_words[4 * c + q] = w.w[q];
    }
    __syncthreads();

    // First pass: the top four index bits.  A thread loads the 16 rows b, b + NP/16, ..., flips
    // signs, runs the four stages and parks the values in LDS.  Rows beyond n are zeros.
    constexpr int V = NP / 16;
    for (int b = tid; b < V; b += 256) {
        float v[16][C];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int t = b + i * V;
            union {
                row_t raw;
                bf16_t e[C];
            } in;
            if (t < g.n) {
                in.raw = *reinterpret_cast<const row_t *>(g.A + (int64_t)t * g.d + col0);
            } else {
#pragma unroll
                for (int c = 0; c < C; ++c) in.e[c] = 0;
            }
            const uint32_t flip = ((sign_words[t >> 5] >> (t & 31)) & 1u) << 31;
#pragma unroll
            for (int c = 0; c < C; ++c) v[i][c] = __uint_as_float(((uint32_t)in.e[c] << 16) ^ flip);
        }
        sors_butterflies<4, C>(v);
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int c = 0; c < C; ++c) planes[c * S::PLANE + sors_phys(b + i * V)] = v[i][c];
    }
    __syncthreads();

    // The other index bits, four at a time from the top; what is left below four goes last.
    constexpr int REST = L - 4;
    if constexpr (REST >= 4) {
        sors_lds_pass<L, REST - 4, 4>(planes, tid);
        __syncthreads();
    }
    if constexpr (REST >= 8) {
        sors_lds_pass<L, REST - 8, 4>(planes, tid);
        __syncthreads();
    }
    if constexpr (REST % 4 != 0) {
        sors_lds_pass<L, 0, REST % 4>(planes, tid);
        __syncthreads();
    }
    static_assert(REST < 12, "at most two full passes and one partial pass below the first");

    // Row selection: sketch columns 4q .. 4q+3 take their rows from the four words of call q.
    for (int64_t q = tid; q < (g.k + 3) / 4; q += 256) {
        const Words4 w = philox4x32_10((uint32_t)q, kSorsRowColumn, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = 4 * q + u;
            if (j >= g.k) break;
            const int at = sors_phys((int)(w.w[u] & g.st.row_mask));
            union {
                row_t raw;
                bf16_t e[C];
            } o;
#pragma unroll
            for (int c = 0; c < C; ++c) o.e[c] = f32_to_bf16(g.alpha * planes[c * S::PLANE + at]);
            *reinterpret_cast<row_t *>(g.out + j * g.d + col0) = o.raw;
        }
    }
}

template <int LC, bool ACC, int NPROB>
__global__ void __launch_bounds__(256 * NPROB) sors_strip_kernel(SorsArgs g, int chunks) {
    __shared__ float4 planes[NPROB * StripShape<LC>::REGION];
    __shared__ uint32_t sign_words[1024];  // up to 32768 tokens
    sors_strip_body<LC, ACC, NPROB>(g, chunks, planes, sign_words, blockIdx.x, gridDim.x);
}

template <int LC, bool ACC>
hipError_t launch_strip(const SorsArgs &g, int chunks, hipStream_t stream) {
    sors_strip_kernel<LC, ACC, 1><<<(unsigned)(g.d / 8), 256, 0, stream>>>(g, chunks);
    return hipGetLastError();
}

template <int L>
hipError_t launch_sors(const SorsArgs &g, hipStream_t stream) {
    sors_kernel<L><<<(unsigned)(g.d / SorsShape<L>::C), 256, 0, stream>>>(g);
    return hipGetLastError();
}

int log2_ceil(int64_t n) {
    int l = 0;
    while (((int64_t)1 << l) < n) ++l;
    return l;
}

}  // namespace

bool sors_fast_ok(int64_t n, int64_t d) { return d % 8 == 0 && n >= 1 && n <= 32768; }

hipError_t launch_sors_bf16(const bf16_t *A, bf16_t *out, int64_t n, int64_t d, int64_t k, SketchState st,
                            hipStream_t stream) {
    SorsArgs g{A, out, n, d, k, st, 1.0f / sqrtf((float)k)};
    // A kernel's transform length is at least 256; for fewer tokens the rows drawn below n_pad
    // are rows of the larger Walsh-Hadamard matrix restricted to its leading n_pad x n_pad block,
    // which is the n_pad-point matrix itself.
    const int l = log2_ceil(n) < 8 ? 8 : log2_ceil(n);
    if (l >= 12 && k <= kSorsAccMaxK) return launch_strip<11, true>(g, 1 << (l - 11), stream);  // chunks of 2048 tokens
    switch (l) {
        case 8: return launch_strip<8, false>(g, 1, stream);
        case 9: return launch_strip<9, false>(g, 1, stream);
        case 10: return launch_strip<10, false>(g, 1, stream);
        case 11: return launch_strip<11, false>(g, 1, stream);
        case 12: return launch_strip<12, false>(g, 1, stream);
        // more than 4096 tokens and more than 2048 sketch columns: whole strips in LDS, 4 / 2 / 1 columns wide
        case 13: return launch_sors<13>(g, stream);
        case 14: return launch_sors<14>(g, stream);
        case 15: return launch_sors<15>(g, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace rmm
