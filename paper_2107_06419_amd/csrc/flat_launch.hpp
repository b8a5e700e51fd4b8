// Host-side launchers of the attention kernels (one per translation unit); called by the C ABI
// in flat_api.hip after argument validation.  All tensors are device pointers, [B*H, N, d].
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace flat {

hipError_t launch_fwd_bf16(const void* Q, const void* K, const void* V, void* O, int BH, int N, int d, float scale,
                           int causal, hipStream_t stream);

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

}  // namespace flat
