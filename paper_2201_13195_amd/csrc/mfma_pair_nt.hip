// Paired-launch kernels (see mfma_pair.hpp): launch_pair_nt.
#include "mfma_pair.hpp"

namespace rmm {

hipError_t launch_pair_nt(int sk_cfg, int kind, const GemmArgs &ga, const GemmArgs &gb, int blocks_a, int tiles_b,
                            int splits, hipStream_t stream, const ColsumArgs *gc) {
    return launch_pair_impl<ShapeLarge, B_KCONTIG, 3>(sk_cfg, kind, ga, gb, blocks_a, tiles_b, splits, stream, gc);
}

}  // namespace rmm
