// Alternative tile shapes of the fused bf16 kernel, kept for the measured tile-shape sweep (table in flat_tiles.hip).
#include "flat_fwd_bf16_kernel.hpp"

namespace flat {

FLAT_INSTANTIATE_BF16_SHAPE(64, 1, 8, 4)
FLAT_INSTANTIATE_BF16_SHAPE(64, 1, 4, 4)
FLAT_INSTANTIATE_BF16_SHAPE(64, 2, 2, 4)
FLAT_INSTANTIATE_BF16_SHAPE(64, 1, 4, 3)

}  // namespace flat
