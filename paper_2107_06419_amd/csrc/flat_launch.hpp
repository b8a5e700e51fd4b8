// Host-side launchers of the attention kernels (one per translation unit); called by the C ABI
// in flat_api.hip after argument validation.  All tensors are device pointers, [B*H, N, d].
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace flat {

// Raise a kernel's dynamic-LDS limit once per device (bit = device ordinal) instead of on every launch.
inline hipError_t allow_dynamic_lds(const void* kern, int lds_bytes, std::atomic<uint64_t>* done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done->load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e == hipSuccess) done->fetch_or(bit, std::memory_order_release);
    return e;
}


// Sequence geometry of one fused bf16 launch.  Self-attention is Nq = Nk, causal_offset = 0, kv_lens = null.
struct Bf16Problem {
    int Nq;               // query rows per head (Q and O are [B*H, Nq, d])
    int Nk;               // key rows per head as laid out in memory (K and V are [B*H, Nk, d])
    int causal_offset;    // causal mask: query i sees keys 0 .. i + causal_offset (>= 0)
    int heads_per_batch;  // H, to find the batch entry of a head
    const int* kv_lens;   // device, one int per batch entry: keys that count (the rest is padding), or null
    // block-sparse launches only (else null / 0): CSR list of the 64-key tiles each 256-row block visits
    const int* tile_offsets;  // device, B*H*ceil(Nq/256) + 1 ints
    const int* tile_ids;      // device, n_tile_ids ints
    int n_tile_ids;
    // split-keys launches only (else 0 / null): the keys of a row block are divided over n_splits workgroups of
    // tiles_per_split tiles each, which leave their partial results in split_ws
    int n_splits;
    int tiles_per_split;
    float* split_ws;
};

hipError_t launch_fwd_bf16(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                           float scale, int causal, hipStream_t stream);

hipError_t launch_fwd_bf16_sparse(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                  float scale, hipStream_t stream);

// Split keys (flat_splitkv.hip): for few query rows over many keys, where one workgroup per row block leaves most
// of the chip idle.  The geometry is fixed per head dimension; split_plan fills in what a launch needs.
struct SplitPlan {
    int rows_per_block;    // query rows per workgroup of the shape used
    int keys_per_tile;
    int padded_d;          // accumulator columns stored per row
    int n_row_blocks;      // per head
    int n_tiles;           // key tiles per head
    int n_splits;          // after clamping to [1, n_tiles]
    int tiles_per_split;
    size_t workspace_bytes;
};
bool split_plan(int BH, int Nq, int Nk, int d, int n_splits_wanted, SplitPlan* out);  // n_splits_wanted <= 0: chosen here
hipError_t launch_fwd_bf16_split(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                 int rows_per_block, float scale, int causal, hipStream_t stream);
// The same launch with the partial results in a scratch array inside the library's device image (prob.split_ws is
// ignored): nothing is allocated.  The plan's workspace_bytes must not exceed kSplitStaticScratchBytes.
constexpr size_t kSplitStaticScratchBytes = (size_t)64 << 20;
hipError_t launch_fwd_bf16_split_static(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob,
                                        int d, int rows_per_block, float scale, int causal, hipStream_t stream);

// Tile shapes of the fused bf16 kernel (flat_tiles.hip).  Index 0 is the default of launch_fwd_bf16.
struct TileShape {
    int d;                   // head dimension the shape is built for
    int rows_per_workgroup;  // query rows per workgroup
    int keys_per_tile;       // keys per LDS stage
    int wavefronts;          // wavefronts per workgroup
    int rows_per_wavefront;
    int lds_stages;          // depth of the K/V ring
    int lds_bytes;           // dynamic LDS per workgroup
};
int tile_shape_count(int d);
int default_tile_shape(int BH, int Nq, int d, int causal);  // index launch_fwd_bf16 uses for this problem
bool tile_shape(int d, int index, TileShape* out);
hipError_t tile_shape_occupancy(int d, int index, int* workgroups_per_cu);
hipError_t launch_fwd_bf16_tile(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                float scale, int causal, int index, hipStream_t stream);
// One tile shape (D head dim, QB 32-row blocks per wavefront, NW wavefronts, STAGES ring depth): defined in
// flat_fwd_bf16_kernel.hpp, instantiated by the flat_fwd_bf16*.hip translation units.
template <int D, int QB, int NW, int STAGES, int BCX = 0>  // BCX: keys per tile, 0 = the head dimension's usual tile
hipError_t launch_fwd_bf16_shape(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, float scale,
                                 int causal, hipStream_t stream);
template <int D, int QB, int NW, int STAGES, int BCX = 0>
hipError_t fwd_bf16_shape_occupancy(int* workgroups_per_cu);

hipError_t launch_fwd_f32(const float* Q, const float* K, const float* V, float* O, int BH, int N, int d, float scale,
                          int causal, hipStream_t stream);

// GEMM -> row softmax -> GEMM through an fp32 [B*H, N, N] workspace.
hipError_t launch_unfused_bf16(const void* Q, const void* K, const void* V, void* O, int BH, int N, int d, float scale,
                               int causal, float* L, hipStream_t stream);

// MFMA-only throughput probe (flat_probe.hip): 512 workgroups x 4 wavefronts, each issuing `iters` rounds of
// four independent 32x32x16 bf16 MFMAs.  `sink` receives one float per thread.
hipError_t launch_mfma_probe(float* sink, int iters, int random_operands, hipStream_t stream);
double mfma_probe_flops(int iters);
size_t mfma_probe_sink_bytes();

// Instruction-mix probe (flat_probe.hip): 512 workgroups x 4 wavefronts loop over the fused d = 64 kernel's step
// (16 MFMAs + the softmax of two 32-row blocks) on synthetic data.  level 0 = registers only, 1 = + LDS operand reads,
// 2 = + one barrier per tile, 3 = + global -> LDS streaming of the tiles.  All operands are taken from `src`
// (mix_probe_src_bytes() of any finite bf16 data).  One trip of `iters` is 8 steps.
hipError_t launch_mix_probe(float* sink, const void* src, int level, int iters, hipStream_t stream);
double mix_probe_flops(int iters);
size_t mix_probe_sink_bytes();
size_t mix_probe_src_bytes();

}  // namespace flat
