// Host-side planning of a split-keys launch (no device code): how many workgroups share the keys of a row block,
// how many tiles each takes, and how large the workspace for their partial results is.
#include "flat_launch.hpp"

namespace flat {

namespace {
// The tile shape a split-keys launch uses: rows per workgroup, keys per tile, padded head dimension, workgroups that
// fit a compute unit.  Every workgroup multiplies a full tile of `rows` rows whatever Nq is, so few query rows take a shape
// with fewer rows where flat_splitkv.hip builds one.
struct Geometry { int rows, keys, dp, per_cu; };
bool geometry(int d, int Nq, Geometry* g) {
    switch (d) {
        case 32:
            if (Nq <= 32) *g = {32, 64, 32, 6};
            else if (Nq <= 64) *g = {64, 64, 32, 4};
            else if (Nq <= 128) *g = {128, 64, 32, 2};
            else *g = {256, 64, 32, 2};
            return true;
        case 64:
            if (Nq <= 32) *g = {32, 64, 64, 3};
            else if (Nq <= 64) *g = {64, 64, 64, 2};
            else if (Nq <= 128) *g = {128, 64, 64, 2};
            else *g = {256, 64, 64, 2};
            return true;
        case 96:
            if (Nq <= 128) *g = {128, 64, 128, 1};
            else *g = {256, 64, 128, 1};
            return true;
        case 128:
            if (Nq <= 128) *g = {128, 64, 128, 1};
            else *g = {256, 64, 128, 1};
            return true;
        case 256: *g = {128, 32, 256, 1}; return true;
        default: return false;
    }
}
constexpr int kComputeUnits = 256;
constexpr int kMinTilesPerSplit = 8;   // below this the prologue and the merge outweigh the gain
}  // namespace

bool split_plan(int BH, int Nq, int Nk, int d, int n_splits_wanted, SplitPlan* out) {
    Geometry g;
    if (BH <= 0 || Nq <= 0 || Nk <= 0 || !geometry(d, Nq, &g)) return false;
    SplitPlan p;
    p.rows_per_block = g.rows;
    p.keys_per_tile = g.keys;
    p.padded_d = g.dp;
    p.n_row_blocks = (int)(((long long)Nq + g.rows - 1) / g.rows);
    p.n_tiles = (int)(((long long)Nk + g.keys - 1) / g.keys);
    long long s = n_splits_wanted;
    if (s <= 0) {  // one workgroup per slot of the chip (measured: more only adds partial results to write and merge), but
                   // keep every split long enough to pay for itself
        const long long blocks = (long long)BH * p.n_row_blocks;
        s = (kComputeUnits * g.per_cu + blocks - 1) / blocks;
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
