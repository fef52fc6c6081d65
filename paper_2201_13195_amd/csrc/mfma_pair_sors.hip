// Paired-launch kernels for the SORS sketch kind: the tiles of a plain product (Y = X W^T or
// dX = dY W) and the strips of the sketch product of the same pass in one grid, for shapes whose
// plain product leaves compute units idle (see mfma_pair.hpp for the idea; the sketch half is the
// two-strip form of sors_strip_body).
#include "mfma_pair.hpp"
#include "sors_kernels.hpp"

namespace rmm {

namespace {

constexpr int kPairChunkLog = 11;  // chunks of 2048 tokens, as the strip kernel on its own

template <typename SA, int BMODE_A, int DA>
__global__ void __launch_bounds__(SA::THREADS) gemm_sors_pair_kernel(GemmArgs ga, SorsArgs gs, int blocks_a, int chunks,
                                                                     int sors_first) {
    typedef Tile<SA::BM, SA::BN, SA::BK, SA::WM, SA::WN, SA::WK, A_KCONTIG, BMODE_A, OUT_BF16> TA;
    typedef StripShape<kPairChunkLog> SS;
    static_assert(SA::THREADS == 512, "two strips of 256 threads");
    constexpr int BYTES_A = TA::STAGES * TA::STAGE_ELEMS * 2, PLANE_BYTES = 2 * SS::REGION * 16;
    constexpr int BYTES_S = PLANE_BYTES + 1024 * 4;
    __shared__ __attribute__((aligned(16))) unsigned char lds[BYTES_A > BYTES_S ? BYTES_A : BYTES_S];
    // The strips come last in the grid when they are to fill the compute units the plain product's
    // last round leaves idle, first when the plain product runs several full rounds and the (long)
    // strips should start with it rather than after it.
    const int strips = (int)gridDim.x - blocks_a;
    const int plain = sors_first ? (int)blockIdx.x - strips : (int)blockIdx.x;
    if (plain >= 0 && plain < blocks_a)
        gemm_tile<SA, A_KCONTIG, BMODE_A, OUT_BF16, DA>(ga, reinterpret_cast<bf16_t *>(lds), plain, blocks_a, 0);
    else
        sors_strip_body<kPairChunkLog, true, 2>(gs, chunks, reinterpret_cast<float4 *>(lds),
                                                reinterpret_cast<uint32_t *>(lds + PLANE_BYTES),
                                                sors_first ? (int64_t)blockIdx.x : (int64_t)blockIdx.x - blocks_a, strips);
}

template <typename SA, int BMODE_A, int DA>
hipError_t launch_impl(const GemmArgs &ga, const SorsArgs &gs, int blocks_a, int chunks, int sors_first, hipStream_t stream) {
    const unsigned strips2 = (unsigned)((gs.d / 8 + 1) / 2);
    gemm_sors_pair_kernel<SA, BMODE_A, DA><<<(unsigned)blocks_a + strips2, SA::THREADS, 0, stream>>>(ga, gs, blocks_a, chunks,
                                                                                                    sors_first);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pair_sors(int cfg_a, bool row_indexed_b, const GemmArgs &ga, const SorsArgs &gs, int blocks_a, int chunks,
                            bool sors_first, hipStream_t stream) {
    if (cfg_a == GEMM_LARGE)
        return row_indexed_b ? launch_impl<ShapeLarge, B_NCONTIG, 3>(ga, gs, blocks_a, chunks, sors_first ? 1 : 0, stream)
                             : launch_impl<ShapeLarge, B_KCONTIG, 3>(ga, gs, blocks_a, chunks, sors_first ? 1 : 0, stream);
    if (cfg_a == GEMM_SPLIT)
        return row_indexed_b ? launch_impl<ShapeSplit, B_NCONTIG, 4>(ga, gs, blocks_a, chunks, sors_first ? 1 : 0, stream)
                             : launch_impl<ShapeSplit, B_KCONTIG, 4>(ga, gs, blocks_a, chunks, sors_first ? 1 : 0, stream);
    return hipErrorInvalidValue;
}

}  // namespace rmm
