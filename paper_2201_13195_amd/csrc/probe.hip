// Measurement probes: what this chip delivers to a kernel that does nothing but MFMAs, and to a
// kernel that does nothing but read memory.  bench.py reports the layer's kernels against these
// measured ceilings next to the published peaks (the shader clock under sustained MFMA load is
// well below the nominal one the published peak is quoted at).
#include "../../include/rmm.h"
#include "common.hpp"

namespace rmm {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// Four waves per work-group, each issuing 16 independent 32x32x16 bf16 MFMAs per iteration from
// operands that stay in registers.
__global__ void __launch_bounds__(256) probe_mfma_kernel(float *sink, int iters) {
    f32x16_t acc[16];
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.0f;
    // Operands with pseudo-random signs and mantissas (magnitudes in [0.5, 1)): constant operands
    // toggle few bits in the multipliers and draw less power than a real product does.
    bf16x8_t fa, fb;
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        h = h * 1664525u + 1013904223u;
        fa[i] = (__bf16)__uint_as_float(0x3F000000u | (h & 0x80000000u) | ((h >> 1) & 0x007F0000u));
        h = h * 1664525u + 1013904223u;
        fb[i] = (__bf16)__uint_as_float(0x3F000000u | (h & 0x80000000u) | ((h >> 1) & 0x007F0000u));
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 16; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[a], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[a][v];
    if (s == -1.0f) sink[threadIdx.x] = s;  // never true: keeps the loop alive
}

// Every work-group streams a contiguous share of the buffer with 16-byte loads, 8 in flight per
// thread, and folds what it read into one word so that the loads cannot be dropped.
__global__ void __launch_bounds__(256) probe_read_kernel(const u32x4_t *__restrict__ src, int64_t vecs, uint32_t *sink) {
    const int64_t per = (vecs + gridDim.x - 1) / gridDim.x;
    const int64_t begin = (int64_t)blockIdx.x * per, end = begin + per < vecs ? begin + per : vecs;
    uint32_t x = 0;
    int64_t i = begin + threadIdx.x;
    for (; i + 7 * 256 < end; i += 8 * 256) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < end; i += 256) {
        const u32x4_t v = __builtin_nontemporal_load(src + i);
        x ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (x == 0x9E3779B9u) sink[0] = x;  // practically never: keeps the loads alive
}

}  // namespace
}  // namespace rmm

extern "C" {

int rmm_probe_mfma(int work_groups, int iters, void *sink, void *stream) {
    if (work_groups < 1 || work_groups > (1 << 20) || iters < 1 || sink == nullptr) return RMM_ERR_INVALID_ARG;
    rmm::probe_mfma_kernel<<<work_groups, 256, 0, (hipStream_t)stream>>>((float *)sink, iters);
    return hipGetLastError() == hipSuccess ? RMM_OK : RMM_ERR_LAUNCH;
}

int rmm_probe_read(const void *src, size_t bytes, int work_groups, void *sink, void *stream) {
    if (src == nullptr || sink == nullptr || bytes < 16 || work_groups < 1 || work_groups > (1 << 20) ||
        (reinterpret_cast<uintptr_t>(src) & 15u) != 0)
        return RMM_ERR_INVALID_ARG;
    rmm::probe_read_kernel<<<work_groups, 256, 0, (hipStream_t)stream>>>((const rmm::u32x4_t *)src, (int64_t)(bytes / 16),
                                                                          (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? RMM_OK : RMM_ERR_LAUNCH;
}

}  // extern "C"
