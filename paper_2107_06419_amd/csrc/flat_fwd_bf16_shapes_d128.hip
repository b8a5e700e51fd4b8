// Alternative tile shapes of the fused bf16 kernel, kept for the measured tile-shape sweep (table in flat_tiles.hip).
#include "flat_fwd_bf16_kernel.hpp"

namespace flat {

FLAT_INSTANTIATE_BF16_SHAPE(128, 1, 8, 4)
FLAT_INSTANTIATE_BF16_SHAPE(128, 1, 4, 3)
FLAT_INSTANTIATE_BF16_SHAPE(128, 2, 4, 3)

}  // namespace flat
