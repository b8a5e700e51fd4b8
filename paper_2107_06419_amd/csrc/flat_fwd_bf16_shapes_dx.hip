// Tile shapes of the fused bf16 kernel for the head dimensions besides 64 and 128:
//   d = 32 : 4 wavefronts x 64 rows, 8 KiB per stage x 4 stages, two workgroups per CU
//   d = 96 : the d = 128 shape with rows padded to 256 bytes in LDS (8 wavefronts x 32 rows, 32 KiB x 3 stages)
//   d = 256: 4 wavefronts x 32 rows with 512 registers each (one wavefront per SIMD), tiles of 32 keys,
//            32 KiB per stage x 4 stages
#include "flat_fwd_bf16_kernel.hpp"

namespace flat {

FLAT_INSTANTIATE_BF16_SHAPE(32, 2, 4, 4)
FLAT_INSTANTIATE_BF16_SHAPE(32, 1, 4, 4)
FLAT_INSTANTIATE_BF16_SHAPE(96, 1, 8, 3)
FLAT_INSTANTIATE_BF16_SHAPE(96, 1, 4, 3)
FLAT_INSTANTIATE_BF16_SHAPE(256, 1, 4, 4)

hipError_t launch_fwd_bf16_sparse_dx(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                     float scale, hipStream_t stream) {
    if (d == 32) return launch_fwd_bf16_sparse_shape<32, 2, 4, 4>(Q, K, V, O, BH, prob, scale, stream);
    if (d == 96) return launch_fwd_bf16_sparse_shape<96, 1, 8, 3>(Q, K, V, O, BH, prob, scale, stream);
    return launch_fwd_bf16_sparse_shape<256, 1, 4, 4>(Q, K, V, O, BH, prob, scale, stream);
}

}  // namespace flat
