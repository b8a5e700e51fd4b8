// MFMA-only throughput probe: what the matrix pipe of this GPU sustains on its own, with constant or with
// random operands.  It gives the attention numbers a measured ceiling next to the published peak: on
// MI355X the clock a kernel runs at depends on the power its operands draw, so a bf16 MFMA loop over
// random data sustains noticeably less than the same loop over constants.
#include "flat_common.hpp"
#include "flat_launch.hpp"

namespace flat {

constexpr int kProbeGrid = 512, kProbeBlock = 256;

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(kProbeBlock) void mfma_probe_kernel(float* __restrict__ sink, int iters, int random_operands) {
    bf16x8 av[4], bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = 1.0f, b = 0.0f;
            if (random_operands) {  // roughly uniform in [-2, 2): all mantissa and sign bits toggle
                a = (float)(int)(probe_hash(threadIdx.x * 64 + i * 8 + e) >> 8) * (1.0f / 4194304.0f) - 2.0f;
                b = (float)(int)(probe_hash(threadIdx.x * 64 + i * 8 + e + 7777) >> 8) * (1.0f / 4194304.0f) - 2.0f;
            }
            av[i][e] = (bf16)a;
            bv[i][e] = (bf16)b;
        }
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = mfma_bf16_32x32x16(av[i], bv[(i + u) & 3], acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[blockIdx.x * kProbeBlock + threadIdx.x] = s;
}

hipError_t launch_mfma_probe(float* sink, int iters, int random_operands, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeGrid), dim3(kProbeBlock), 0, stream, sink, iters, random_operands);
    return hipGetLastError();
}

double mfma_probe_flops(int iters) {
    const int rounded = (iters + 3) / 4 * 4;
    return (double)kProbeGrid * (kProbeBlock / 64) * rounded * 4.0 * 32768.0;
}

size_t mfma_probe_sink_bytes() { return (size_t)kProbeGrid * kProbeBlock * sizeof(float); }

}  // namespace flat
