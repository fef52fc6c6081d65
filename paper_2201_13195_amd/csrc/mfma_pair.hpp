// Host-side interface between mfma.hip (kernel selection, single launches) and the translation
// units that hold the paired-launch kernels (mfma_pair_*.hip; separate files only to keep the
// build parallel).
#pragma once
#include "mfma_kernels.hpp"

namespace rmm {

// Tile shape a plain product runs with (Shape typedefs of mfma_kernels.hpp) and a sketch product's kernel.
enum { GEMM_LARGE = 0, GEMM_SPLIT = 1, GEMM_MID = 2, GEMM_TINY = 3 };
enum { SK_NARROW = 0, SK_WIDE = 1, SK_WIDE64 = 2, SK_MID64 = 3, SK_MID = 4 };

// One launch for a plain product (`ga`, `blocks_a` tiles) and a sketch product with an
// LDS-generated tile (`gb`, `tiles_b` tiles x `splits` token slices, fp32 partial results).
//   nt:       Y = X W^T, 256 x 256 tiles (GEMM_LARGE, prefetch depth 3)
//   nt_split: Y = X W^T, 128 x 128 x 64 tiles with two wave groups (GEMM_SPLIT, depth 4)
//   nn_large: dX = dY W, 256 x 256 tiles (GEMM_LARGE, depth 3)
//   nn_split: dX = dY W, 128 x 128 x 64 tiles with two wave groups (GEMM_SPLIT, depth 4)
// sk_cfg is one of SK_WIDE, SK_WIDE64, SK_MID64, SK_MID; anything else returns hipErrorInvalidValue.
// `gc`, if not null, adds the column blocks of a column-sum problem (colsum.hpp) behind the sketch work-groups.
// The sketch work-groups are put in front of the plain tiles when the sketch product is unsliced (few, long
// work-groups) or the plain product fills the chip at least once (256 tiles or more: measured 4 % faster at the
// RoBERTa-large shapes, 2-3 % slower where the plain product has 192 tiles and the sketch work-groups fill in behind).
hipError_t launch_pair_nt(int sk_cfg, int kind, const GemmArgs &ga, const GemmArgs &gb, int blocks_a, int tiles_b,
                          int splits, hipStream_t stream, const ColsumArgs *gc = nullptr);
hipError_t launch_pair_nt_split(int sk_cfg, int kind, const GemmArgs &ga, const GemmArgs &gb, int blocks_a, int tiles_b,
                                int splits, hipStream_t stream, const ColsumArgs *gc = nullptr);
hipError_t launch_pair_nn_large(int sk_cfg, int kind, const GemmArgs &ga, const GemmArgs &gb, int blocks_a, int tiles_b,
                                int splits, hipStream_t stream, const ColsumArgs *gc = nullptr);
hipError_t launch_pair_nn_split(int sk_cfg, int kind, const GemmArgs &ga, const GemmArgs &gb, int blocks_a, int tiles_b,
                                int splits, hipStream_t stream, const ColsumArgs *gc = nullptr);

// The same for the SORS sketch kind (mfma_pair_sors.hip): `gs` describes the sketch product, whose
// strips go two to a work-group; cfg_a is GEMM_LARGE (depth 3) or GEMM_SPLIT (depth 4), row_indexed_b
// says whether the plain product is dX = dY W (true) or Y = X W^T (false); `chunks` chunks of 2048 tokens;
// sors_first puts the strips' work-groups at the front of the grid instead of the back.
struct SorsArgs;
hipError_t launch_pair_sors(int cfg_a, bool row_indexed_b, const GemmArgs &ga, const SorsArgs &gs, int blocks_a, int chunks,
                            bool sors_first, hipStream_t stream);

// Shared body of launch_pair_nt, _nt_split, _nn_large and _nn_split.
template <typename SA, int BMODE_A, int DA>
hipError_t launch_pair_impl(int sk_cfg, int kind, const GemmArgs &ga, const GemmArgs &gb, int blocks_a, int tiles_b,
                            int splits, hipStream_t stream, const ColsumArgs *gc) {
    const int sketch_blocks = tiles_b * splits;
    const int sketch_first = splits == 1 || blocks_a >= 256 ? 1 : 0;
    const ColsumArgs c = gc != nullptr ? *gc : ColsumArgs{};
    const int col_blocks = gc != nullptr ? (int)colsum_blocks(c.d, 2) : 0;
    const dim3 grid((unsigned)(blocks_a + sketch_blocks + col_blocks));
    const int key = sk_cfg * 2 + (kind != 0 ? 1 : 0);
#define RMM_PAIR_CASE(CFG, SHAPE)                                                                                      \
    case CFG * 2:                                                                                                      \
        gemm_pair_kernel<SA, A_KCONTIG, BMODE_A, DA, SHAPE, A_GAUSS_LDS, 3>                                           \
            <<<grid, SA::THREADS, 0, stream>>>(ga, gb, blocks_a, tiles_b, sketch_blocks, col_blocks, sketch_first, c); \
        break;                                                                                                         \
    case CFG * 2 + 1:                                                                                                  \
        gemm_pair_kernel<SA, A_KCONTIG, BMODE_A, DA, SHAPE, A_RADEM_LDS, 3>                                           \
            <<<grid, SA::THREADS, 0, stream>>>(ga, gb, blocks_a, tiles_b, sketch_blocks, col_blocks, sketch_first, c); \
        break;
    switch (key) {
        RMM_PAIR_CASE(SK_WIDE, ShapeSkWide)
        RMM_PAIR_CASE(SK_WIDE64, ShapeSkWide64)
        RMM_PAIR_CASE(SK_MID64, ShapeSkMid64)
        RMM_PAIR_CASE(SK_MID, ShapeSkMid)
        default: return hipErrorInvalidValue;
    }
#undef RMM_PAIR_CASE
    return hipGetLastError();
}

}  // namespace rmm
