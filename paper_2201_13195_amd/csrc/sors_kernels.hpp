// Device code of the SORS sketch kind's strip kernel (see sors.hip for what it computes), kept in a
// header because it also runs inside the paired launches of a layer pass.
#pragma once
#include "common.hpp"

namespace rmm {

struct SorsArgs {
    const bf16_t *A;
    bf16_t *out;
    int64_t n, d, k;
    SketchState st;
    float alpha;
};

namespace {

typedef unsigned int sors_u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int sors_u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ int sors_phys(int t) { return t + (t >> 4); }

// ---------------------------------------------------------------------------------------------
// The kernel that serves the layer's shapes: strips of 8 columns (one 16-byte load per token row,
// the widest strip whose fp32 copy fits in LDS next to a second work-group's), tokens taken in
// chunks of CH = 2^LC.  The transform factors over the chunks,
//
//   out[j] = sum_chunks (-1)^popcount(hi(r_j) AND chunk) * T_chunk[lo(r_j)],
//   T_chunk = the CH-point transform of the chunk's signed tokens,
//
// so a work-group runs one CH-point transform per chunk in the same LDS buffer and adds the
// selected entries into per-thread accumulators (k <= 2048: 8 rows x 8 columns per thread), with
// the next chunk's rows already on their way from memory.  With a single chunk (CH >= n_pad) the
// selected rows are written directly and k is not limited.  Per chunk: the top LC - 8 index bits
// in registers while loading (2^(LC-8) rows per thread), then two LDS passes of four bits each,
// 16-byte LDS accesses throughout.  LDS layout: two halves (columns 0-3, 4-7) of float4 slots,
// token t at slot t + t / 16.
template <int LC>
struct StripShape {
    static constexpr int CH = 1 << LC, W0 = LC - 8, R0 = 1 << W0, SLOTS = CH + CH / 16;
    static constexpr int REGION = 2 * SLOTS + 4;  // float4 slots of one strip
    static_assert(LC >= 8 && LC <= 12, "chunks of 256 .. 4096 tokens");
};
constexpr int kSorsAccCalls = 2;                      // row-selection calls per thread with accumulators
constexpr int64_t kSorsAccMaxK = 256 * 4 * kSorsAccCalls;  // 2048

__device__ __forceinline__ void sors_butterflies4(float4 (&v)[16]) {
#pragma unroll
    for (int h = 1; h < 16; h <<= 1)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i & h) == 0) {
                const float4 a = v[i], b = v[i + h];
                v[i] = make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
                v[i + h] = make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w);
            }
}

// Index bits SHIFT .. SHIFT+3 of the chunk-local token index, both halves.
template <int LC, int SHIFT>
__device__ __forceinline__ void strip_lds_pass(float4 *planes, int tid) {
    typedef StripShape<LC> S;
    constexpr int VEC = S::CH / 16;
    for (int item = tid; item < 2 * VEC; item += 256) {
        const int h = item / VEC, b = item % VEC;
        const int low = b & ((1 << SHIFT) - 1), high = b >> SHIFT;
        const int base = (high << (SHIFT + 4)) | low;
        float4 *plane = planes + h * S::SLOTS;
        float4 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = plane[sors_phys(base + (i << SHIFT))];
        sors_butterflies4(v);
#pragma unroll
        for (int i = 0; i < 16; ++i) plane[sors_phys(base + (i << SHIFT))] = v[i];
    }
}

//
// NPROB = 2 puts two neighbouring strips into one work-group of 512 threads (thread 2r + p is
// thread r of strip p; separate LDS planes, offset by 64 bytes modulo 128 so that the interleaved
// lanes of the two strips stay on different banks): the form that shares a grid with the 512-thread
// work-groups of a plain product.  `block` of `blocks` numbers the work-group among those of the
// sketch product; LDS: NPROB * StripShape::REGION float4 slots and 1024 words.
template <int LC, bool ACC, int NPROB>
__device__ __forceinline__ void sors_strip_body(const SorsArgs &g, int chunks, float4 *planes_all, uint32_t *sign_words,
                                                int64_t block, int64_t blocks) {
    typedef StripShape<LC> S;
    constexpr int CH = S::CH, R0 = S::R0;
    const int prob = NPROB == 2 ? (int)(threadIdx.x & 1) : 0;
    const int tid = NPROB == 2 ? (int)(threadIdx.x >> 1) : (int)threadIdx.x;  // thread number inside the strip, 0 .. 255
    float4 *planes = planes_all + prob * S::REGION;

    // Strips that share 128-byte lines of A should meet in one L2: work-groups are dealt round-robin
    // to the 8 XCDs, so XCD x gets a contiguous run of strips.
    int64_t group = block;
    {
        const int64_t per = blocks / 8, rem = blocks % 8, x = group % 8, r = group / 8;
        group = x * per + (x < rem ? x : rem) + r;
    }
    const int64_t col0 = (group * NPROB + prob) * 8;
    const bool live = col0 < g.d;  // the last work-group's second strip may not exist

    for (int c = threadIdx.x; c < chunks * (CH / 128); c += 256 * NPROB) {
        const Words4 w = philox4x32_10((uint32_t)c, kSorsSignColumn, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
#pragma unroll
        for (int q = 0; q < 4; ++q) sign_words[4 * c + q] = w.w[q];
    }

    // Rows of this thread's sketch columns and their accumulators (ACC only).
    uint32_t rows[ACC ? kSorsAccCalls : 1][4];
    float4 acc[ACC ? kSorsAccCalls : 1][4][2];
    if constexpr (ACC) {
#pragma unroll
        for (int m = 0; m < kSorsAccCalls; ++m) {
            const Words4 w = philox4x32_10((uint32_t)(tid + 256 * m), kSorsRowColumn, g.st.off0, g.st.off1, g.st.key0,
                                           g.st.key1);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                rows[m][u] = w.w[u] & g.st.row_mask;
                acc[m][u][0] = acc[m][u][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }

    auto load_chunk = [&](int ch, sors_u32x4_t (&raw)[R0]) {
#pragma unroll
        for (int i = 0; i < R0; ++i) {
            const int64_t t = (int64_t)ch * CH + tid + i * 256;
            if (live && t < g.n)
                raw[i] = *reinterpret_cast<const sors_u32x4_t *>(g.A + t * g.d + col0);
            else
                raw[i] = (sors_u32x4_t){0u, 0u, 0u, 0u};
        }
    };

    sors_u32x4_t raw[R0], raw_next[R0];
    load_chunk(0, raw);
    __syncthreads();  // sign words
    for (int ch = 0; ch < chunks; ++ch) {
        // first pass: the chunk's top LC - 8 index bits, in registers, signs applied on the way
        {
            float4 v[R0][2];
#pragma unroll
            for (int i = 0; i < R0; ++i) {
                const int t = ch * CH + tid + i * 256;
                const uint32_t flip = ((sign_words[t >> 5] >> (t & 31)) & 1u) << 31;
                const sors_u32x4_t w = raw[i];  // eight bf16: element 2q in the low half of word q
                v[i][0] = make_float4(__uint_as_float((w.x << 16) ^ flip), __uint_as_float((w.x & 0xFFFF0000u) ^ flip),
                                      __uint_as_float((w.y << 16) ^ flip), __uint_as_float((w.y & 0xFFFF0000u) ^ flip));
                v[i][1] = make_float4(__uint_as_float((w.z << 16) ^ flip), __uint_as_float((w.z & 0xFFFF0000u) ^ flip),
                                      __uint_as_float((w.w << 16) ^ flip), __uint_as_float((w.w & 0xFFFF0000u) ^ flip));
            }
            if (ch + 1 < chunks) load_chunk(ch + 1, raw_next);  // arrives while this chunk is transformed
#pragma unroll
            for (int h = 1; h < R0; h <<= 1)
#pragma unroll
                for (int i = 0; i < R0; ++i)
                    if ((i & h) == 0) {
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const float4 a = v[i][e], b = v[i + h][e];
                            v[i][e] = make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
                            v[i + h][e] = make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w);
                        }
                    }
#pragma unroll
            for (int i = 0; i < R0; ++i) {
                const int at = sors_phys(tid + i * 256);
                planes[at] = v[i][0];
                planes[S::SLOTS + at] = v[i][1];
            }
        }
        __syncthreads();
        strip_lds_pass<LC, 4>(planes, tid);
        __syncthreads();
        strip_lds_pass<LC, 0>(planes, tid);
        __syncthreads();
        if constexpr (ACC) {
#pragma unroll
            for (int m = 0; m < kSorsAccCalls; ++m)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t r = rows[m][u];
                    const int at = sors_phys((int)(r & (CH - 1)));
                    const float sgn = (__popc((r >> LC) & (uint32_t)ch) & 1) ? -1.0f : 1.0f;
                    const float4 a = planes[at], b = planes[S::SLOTS + at];
                    acc[m][u][0].x += sgn * a.x, acc[m][u][0].y += sgn * a.y, acc[m][u][0].z += sgn * a.z, acc[m][u][0].w += sgn * a.w;
                    acc[m][u][1].x += sgn * b.x, acc[m][u][1].y += sgn * b.y, acc[m][u][1].z += sgn * b.z, acc[m][u][1].w += sgn * b.w;
                }
            __syncthreads();  // the next chunk overwrites the planes
#pragma unroll
            for (int i = 0; i < R0; ++i) raw[i] = raw_next[i];
        }
    }

    auto store_row = [&](int64_t j, const float4 &a, const float4 &b) {
        sors_u32x4_t o;
        o.x = (uint32_t)f32_to_bf16(g.alpha * a.x) | ((uint32_t)f32_to_bf16(g.alpha * a.y) << 16);
        o.y = (uint32_t)f32_to_bf16(g.alpha * a.z) | ((uint32_t)f32_to_bf16(g.alpha * a.w) << 16);
        o.z = (uint32_t)f32_to_bf16(g.alpha * b.x) | ((uint32_t)f32_to_bf16(g.alpha * b.y) << 16);
        o.w = (uint32_t)f32_to_bf16(g.alpha * b.z) | ((uint32_t)f32_to_bf16(g.alpha * b.w) << 16);
        if (live) *reinterpret_cast<sors_u32x4_t *>(g.out + j * g.d + col0) = o;
    };
    if constexpr (ACC) {
#pragma unroll
        for (int m = 0; m < kSorsAccCalls; ++m)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t j = 4 * (int64_t)(tid + 256 * m) + u;
                if (j < g.k) store_row(j, acc[m][u][0], acc[m][u][1]);
            }
    } else {
        for (int64_t q = tid; q < (g.k + 3) / 4; q += 256) {
            const Words4 w = philox4x32_10((uint32_t)q, kSorsRowColumn, g.st.off0, g.st.off1, g.st.key0, g.st.key1);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t j = 4 * q + u;
                if (j >= g.k) break;
                const int at = sors_phys((int)(w.w[u] & g.st.row_mask));
                store_row(j, planes[at], planes[S::SLOTS + at]);
            }
        }
    }
}

}  // namespace

}  // namespace rmm
