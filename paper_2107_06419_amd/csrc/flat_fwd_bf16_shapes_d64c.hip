// Tile shapes of the fused bf16 kernel with other key-tile lengths than the usual 64 (d = 64: 128 and 32 keys per
// tile), kept for the measured tile-shape sweep (table in flat_tiles.hip).
#include "flat_fwd_bf16_kernel.hpp"

namespace flat {

FLAT_INSTANTIATE_BF16_SHAPE_BC(64, 2, 8, 3, 128)
FLAT_INSTANTIATE_BF16_SHAPE_BC(64, 2, 8, 4, 128)
FLAT_INSTANTIATE_BF16_SHAPE_BC(64, 2, 4, 3, 128)
FLAT_INSTANTIATE_BF16_SHAPE_BC(64, 2, 4, 6, 32)

}  // namespace flat
