// The default tile shapes of the fused bf16 kernel (the kernel itself: flat_fwd_bf16_kernel.hpp):
//   d = 64 : 4 wavefronts x 64 rows, 16 KiB per stage x 4 stages, two workgroups per CU (128 of 160 KiB LDS)
//   d = 128: 8 wavefronts x 32 rows, 32 KiB per stage x 3 stages, one workgroup per CU (96 KiB)
#include "flat_fwd_bf16_kernel.hpp"

namespace flat {

FLAT_INSTANTIATE_BF16_SHAPE(64, 2, 4, 4)
FLAT_INSTANTIATE_BF16_SHAPE(128, 1, 8, 3)

hipError_t launch_fwd_bf16_sparse_dx(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                     float scale, hipStream_t stream);  // flat_fwd_bf16_shapes_dx.hip

// The block-sparse variant exists for the default shapes only: its row block (256 rows) is part of the ABI.
hipError_t launch_fwd_bf16_sparse(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                  float scale, hipStream_t stream) {
    if (d == 64) return launch_fwd_bf16_sparse_shape<64, 2, 4, 4>(Q, K, V, O, BH, prob, scale, stream);
    if (d != 128) return launch_fwd_bf16_sparse_dx(Q, K, V, O, BH, prob, d, scale, stream);
    return launch_fwd_bf16_sparse_shape<128, 1, 8, 3>(Q, K, V, O, BH, prob, scale, stream);
}

}  // namespace flat
