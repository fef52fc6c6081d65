// Device-side Philox-4x32-10 and the counter -> sketch-entry map.
//
// The sketch S of the RMM layer (paper: Section 2.1, Eq. 5; Algorithm 1 "generate /
// rematerialize S") is never stored: every kernel that needs a piece of it calls
// these functions.  The element map is the one documented in include/rmm.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rmm {

struct SketchState {
    uint32_t key0, key1;  // seed lo / hi
    uint32_t off0, off1;  // offset lo / hi  (counter words 2 and 3)
    uint32_t row_mask;    // SORS kind only: n_pad - 1, n_pad = the token count rounded up to a power of two
};

// `n` = the sketch's token count; it enters the SORS kind only (through n_pad).
__host__ __device__ inline SketchState make_state(uint64_t seed, uint64_t offset, int64_t n = 1) {
    SketchState s;
    s.key0 = (uint32_t)seed;
    s.key1 = (uint32_t)(seed >> 32);
    s.off0 = (uint32_t)offset;
    s.off1 = (uint32_t)(offset >> 32);
    uint32_t n_pad = 1;
    while ((int64_t)n_pad < n && n_pad < 0x80000000u) n_pad <<= 1;
    s.row_mask = n_pad - 1u;
    return s;
}

// Counter word 1 (the slot of the sketch column) of the calls behind the SORS kind's token signs
// and selected rows; no sketch has that many columns.
constexpr uint32_t kSorsSignColumn = 0xFFFFFFFFu, kSorsRowColumn = 0xFFFFFFFEu;

struct Words4 {
    uint32_t w[4];
};

// One Philox-4x32-10 block: ten rounds, key bumped by the Weyl constants before
// rounds 2..10.  The two 32x32->64 products per round map to v_mad_u64_u32 and each
// three-way xor to one v_bitop3_b32 (truth table 0x96 = a ^ b ^ c).
__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Words4 o;
    o.w[0] = c0;
    o.w[1] = c1;
    o.w[2] = c2;
    o.w[3] = c3;
    return o;
}

// Box-Muller pair of one 32-bit word, full-precision math (fp32 kernels).
// u1 = (hi16 + 1/2) / 2^16 in (0,1), u2 = lo16 / 2^16 in [0,1).
__device__ __forceinline__ void gauss_pair_precise(uint32_t w, float &z_cos, float &z_sin) {
    const float u1 = (float)(2u * (w >> 16) + 1u) * (1.0f / 131072.0f);
    const float u2x2 = (float)(w & 0xFFFFu) * (1.0f / 32768.0f);  // 2*u2, exact
    const float rad = sqrtf(-2.0f * logf(u1));
    float s, c;
    sincospif(u2x2, &s, &c);
    z_cos = rad * c;
    z_sin = rad * s;
}

// Unscaled sketch entry P[i][j] computed on its own (one Philox call per entry):
// the slow, obvious form used by the fp32 kernels and the debug export.
__device__ __forceinline__ float sketch_entry_precise(int kind, const SketchState &st, int64_t i, int64_t j) {
    if (kind == 0) {  // Gaussian
        const Words4 r = philox4x32_10((uint32_t)(i >> 3), (uint32_t)j, st.off0, st.off1, st.key0, st.key1);
        float zc, zs;
        gauss_pair_precise(r.w[(i & 7) >> 1], zc, zs);
        return (i & 1) ? zs : zc;
    }
    if (kind == 2) {  // SORS: sign of token i times entry (r_j, i) of the Walsh-Hadamard matrix
        const Words4 rs = philox4x32_10((uint32_t)(i >> 7), kSorsSignColumn, st.off0, st.off1, st.key0, st.key1);
        const Words4 rr = philox4x32_10((uint32_t)(j >> 2), kSorsRowColumn, st.off0, st.off1, st.key0, st.key1);
        const uint32_t t = (uint32_t)(i & 127);
        const uint32_t row = rr.w[j & 3] & st.row_mask;
        const uint32_t bit = ((rs.w[t >> 5] >> (t & 31)) ^ (uint32_t)__popc(row & (uint32_t)i)) & 1u;
        return bit ? -1.0f : 1.0f;
    }
    const Words4 r = philox4x32_10((uint32_t)(i >> 7), (uint32_t)j, st.off0, st.off1, st.key0, st.key1);
    const uint32_t t = (uint32_t)(i & 127);
    const uint32_t bit = (r.w[t >> 5] >> (t & 31)) & 1u;
    return bit ? -1.0f : 1.0f;
}

}  // namespace rmm
