// Host-side planning of a split-keys launch (no device code): how many workgroups share the keys of a row block,
// how many tiles each takes, and how large the workspace for their partial results is.
#include "flat_launch.hpp"

namespace flat {

namespace {
// the default tile shape of every head dimension: rows per workgroup, keys per tile, padded head dimension
struct Geometry { int rows, keys, dp; };
bool geometry(int d, Geometry* g) {
    switch (d) {
        case 32: *g = {256, 64, 32}; return true;
        case 64: *g = {256, 64, 64}; return true;
        case 96: *g = {256, 64, 128}; return true;
        case 128: *g = {256, 64, 128}; return true;
        case 256: *g = {128, 32, 256}; return true;
        default: return false;
    }
}
constexpr int kWorkgroupSlots = 512;   // 256 compute units x 2 resident workgroups of the d = 64 shape
constexpr int kMinTilesPerSplit = 8;   // below this the prologue and the merge outweigh the gain
}  // namespace

bool split_plan(int BH, int Nq, int Nk, int d, int n_splits_wanted, SplitPlan* out) {
    Geometry g;
    if (!geometry(d, &g) || BH <= 0 || Nq <= 0 || Nk <= 0) return false;
    SplitPlan p;
    p.rows_per_block = g.rows;
    p.keys_per_tile = g.keys;
    p.padded_d = g.dp;
    p.n_row_blocks = (int)(((long long)Nq + g.rows - 1) / g.rows);
    p.n_tiles = (int)(((long long)Nk + g.keys - 1) / g.keys);
    long long s = n_splits_wanted;
    if (s <= 0) {  // fill the chip about twice over, but keep every split long enough to pay for itself
        const long long blocks = (long long)BH * p.n_row_blocks;
        s = (2 * kWorkgroupSlots + blocks - 1) / blocks;
        const long long longest = (p.n_tiles + kMinTilesPerSplit - 1) / kMinTilesPerSplit;
        if (s > longest) s = longest;
    }
    if (s > p.n_tiles) s = p.n_tiles;
    if (s < 1) s = 1;
    p.tiles_per_split = (int)((p.n_tiles + s - 1) / s);
    p.n_splits = (p.n_tiles + p.tiles_per_split - 1) / p.tiles_per_split;  // no split is left without a tile
    const unsigned __int128 bytes = (unsigned __int128)BH * p.n_row_blocks * p.n_splits * g.rows * (g.dp + 2) * sizeof(float);
    if (bytes >= ((unsigned __int128)1 << 62) || (long long)BH * p.n_row_blocks * p.n_splits > 0x7fffffffLL) return false;
    if ((long long)BH * Nq > 0x7fffffffLL) return false;  // the merge launches one workgroup per (head, row)
    p.workspace_bytes = (size_t)bytes;
    *out = p;
    return true;
}

}  // namespace flat
