// Table of the tile shapes the fused bf16 kernel is built for, and the dispatch by index.  Index 0 of each head
// dimension is the shape flat_attn_fwd uses; the others exist so that the choice can be re-measured (the
// paper's map-space exploration, section 6.1, done by timing instead of a cost model; the trade-off being
// explored is the row granularity of section 5.3: fewer rows per workgroup re-fetch K and V more often and
// fill the matrix units less, more rows need more on-chip state).
#include "flat_launch.hpp"

namespace flat {

namespace {

using LaunchFn = hipError_t (*)(const void*, const void*, const void*, void*, int, const Bf16Problem&, float, int, hipStream_t);
using OccupancyFn = hipError_t (*)(int*);

struct Entry {
    TileShape shape;
    LaunchFn launch;
    OccupancyFn occupancy;
};

template <int D, int QB, int NW, int STAGES, int BCX = 0>
constexpr Entry entry() {
    constexpr int DP = D == 96 ? 128 : D, BC = BCX ? BCX : (D == 256 ? 32 : 64);  // as in Bf16Cfg: padded row length, keys per tile
    return Entry{TileShape{D, 32 * QB * NW, BC, NW, 32 * QB, STAGES, STAGES * 2 * BC * DP * 2},
                 &launch_fwd_bf16_shape<D, QB, NW, STAGES, BCX>, &fwd_bf16_shape_occupancy<D, QB, NW, STAGES, BCX>};
}

const Entry kD64[] = {entry<64, 2, 4, 4>(), entry<64, 2, 4, 3>(), entry<64, 2, 4, 6>(), entry<64, 2, 8, 4>(),
                      entry<64, 1, 8, 4>(), entry<64, 1, 4, 4>(), entry<64, 2, 2, 4>(), entry<64, 1, 4, 3>(),
                      // the key-tile axis: 128 keys per tile (512-row and 256-row workgroups), 32 keys per tile
                      entry<64, 2, 8, 3, 128>(), entry<64, 2, 8, 4, 128>(), entry<64, 2, 4, 3, 128>(), entry<64, 2, 4, 6, 32>()};
const Entry kD128[] = {entry<128, 1, 8, 3>(), entry<128, 1, 8, 4>(), entry<128, 1, 4, 3>(), entry<128, 2, 4, 3>()};
const Entry kD32[] = {entry<32, 2, 4, 4>(), entry<32, 1, 4, 4>()};
const Entry kD96[] = {entry<96, 1, 8, 3>(), entry<96, 1, 4, 3>()};
const Entry kD256[] = {entry<256, 1, 4, 4>()};

const Entry* table(int d) {
    switch (d) {
        case 32: return kD32;
        case 64: return kD64;
        case 96: return kD96;
        case 128: return kD128;
        case 256: return kD256;
        default: return nullptr;
    }
}

const Entry* find(int d, int index) {
    if (index < 0 || index >= tile_shape_count(d)) return nullptr;
    return &table(d)[index];
}

}  // namespace

int tile_shape_count(int d) {
    if (d == 64) return (int)(sizeof(kD64) / sizeof(kD64[0]));
    if (d == 128) return (int)(sizeof(kD128) / sizeof(kD128[0]));
    if (d == 32) return (int)(sizeof(kD32) / sizeof(kD32[0]));
    if (d == 96) return (int)(sizeof(kD96) / sizeof(kD96[0]));
    if (d == 256) return (int)(sizeof(kD256) / sizeof(kD256[0]));
    return 0;
}

bool tile_shape(int d, int index, TileShape* out) {
    const Entry* e = find(d, index);
    if (!e) return false;
    *out = e->shape;
    return true;
}

hipError_t tile_shape_occupancy(int d, int index, int* workgroups_per_cu) {
    const Entry* e = find(d, index);
    return e ? e->occupancy(workgroups_per_cu) : hipErrorInvalidValue;
}

hipError_t launch_fwd_bf16_tile(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                float scale, int causal, int index, hipStream_t stream) {
    const Entry* e = find(d, index);
    return e ? e->launch(Q, K, V, O, BH, prob, scale, causal, stream) : hipErrorInvalidValue;
}

// The shape flat_attn_fwd / flat_attn_fwd_cross run: index 0, except where a measured sweep (python -m
// paper_2107_06419_amd.tile_sweep --small: 1 to 512 heads of 128 to 8192 positions, both masks, several machines)
// shows the 128-row shape of the head dimension ahead:
//   * launches too small to give every compute unit a 256-row workgroup - at most 128 blocks of 256 query rows (causal:
//     256 at d = 32 / 64, 192 at d = 96 / 128): 1.3-1.5 times faster, simply because twice as many compute units work;
//   * d = 64 with the causal mask, up to 4096 positions and 1024 row blocks: ahead by up to 15 %, never behind;
//   * d = 32 (the vector side is the longer pole there and three workgroups per compute unit hide more of it): with
//     the causal mask up to 8192 positions (4-18 %), without it up to 4096 positions and 1024 row blocks (6 %).
// Beyond these ranges the 128-row shapes lose 1-15 %.  No other shape is ahead of index 0 by more than the
// run-to-run spread (the 512-row shape leads by 3 % for d = 64, causal, when B*H*ceil(N/512) is exactly 512, and
// trails by 2-15 % with more or fewer row blocks: no rule is built on that).
int default_tile_shape(int BH, int Nq, int d, int causal) {
    const long long blocks = (long long)BH * (((long long)Nq + 255) / 256);  // 256-row blocks in the launch
    switch (d) {
        case 32:
            if (causal) return (Nq > 128 && Nq <= 8192) ? 1 : 0;
            return (Nq > 512 && ((Nq <= 4096 && blocks <= 1024) || blocks <= 128)) ? 1 : 0;
        case 64:
            if (causal) return (Nq > 256 && blocks <= (Nq <= 4096 ? 1024 : 256)) ? 7 : 0;
            return (Nq > 256 && blocks <= 128) ? 7 : 0;
        case 96: return (Nq > 128 && blocks <= (causal ? 192 : 128)) ? 1 : 0;
        case 128: return (Nq > 128 && blocks <= (causal ? 192 : 128)) ? 2 : 0;
        default: return 0;
    }
}

hipError_t launch_fwd_bf16(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                           float scale, int causal, hipStream_t stream) {
    return launch_fwd_bf16_tile(Q, K, V, O, BH, prob, d, scale, causal, default_tile_shape(BH, prob.Nq, d, causal), stream);
}

}  // namespace flat
