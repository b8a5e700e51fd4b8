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

}  // namespace flat
