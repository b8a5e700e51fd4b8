// Split-keys form of the fused bf16 kernel, for few query rows over many keys (a segment of new positions
// attending over a long cache).  The row granularity of the paper's section 5.3 trades on-chip memory against how
// well the compute array is filled; with a handful of row blocks the array stays empty whatever the tile size, so
// here the key loop of a row block is divided over several workgroups, each leaving (reference maximum, row sum,
// unnormalised output) in a workspace, and a second small kernel merges them.
#include "flat_fwd_bf16_kernel.hpp"

namespace flat {

// Second pass of a split-keys launch: one workgroup per (head, query row) merges the partial results of the splits.
// With m_s, l_s, O_s the reference maximum (log2 units), row sum and accumulators of split s:
//     M = max m_s over the splits that saw a key,   w_s = 2^(m_s - M),   O = sum_s w_s O_s / sum_s w_s l_s.
// The kernel is a chain of memory round trips, so it is written to have few of them: first thread t fetches (m, l) of
// splits t, t + 256, ... (all loads unconditional, hence in flight together), M and the sum of w_s l_s are reduced over
// the workgroup and the weights left in LDS; then thread t handles output columns 4 (t % quads) .. +3 of the splits
// t / quads, t / quads + lanes, ..., again with every load issued before its weight is looked at.  A split that saw
// no key has l = 0, hence weight 0, and its accumulators are left out.  Sums are taken in a fixed order, so
// the result is reproducible.
constexpr int kMergeThreads = 256;
constexpr int kMergeWeights = 2048;  // weights kept in LDS; splits beyond that have theirs recomputed from (m, l)

__device__ __forceinline__ float merge_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float merge_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ __launch_bounds__(kMergeThreads) void split_merge_kernel(const float* __restrict__ ws, bf16* __restrict__ O, int Nq,
                                                                    int n_row_blocks, int rows_per_block, int dp, int d,
                                                                    int n_splits) {
    __shared__ float red[4][kMergeThreads];
    __shared__ float wts[kMergeWeights];
    __shared__ float stat[2][kMergeThreads / 64];
    const int quads = d / 4;                        // 8 .. 64
    const int lanes = kMergeThreads / quads;        // split lanes (d = 96: 10, and the last 16 threads only meet the barriers)
    const int tid = threadIdx.x, quad = tid % quads, lane = tid / quads;
    const int first = lane < lanes ? lane : n_splits;  // first split of this thread in the second phase
    const int row = blockIdx.x % Nq, bh = blockIdx.x / Nq;
    const int rb = row / rows_per_block, r = row - rb * rows_per_block;
    const size_t stride = (size_t)rows_per_block * (dp + 2);
    const float* base = ws + (size_t)(bh * n_row_blocks + rb) * n_splits * stride;
    const size_t m_at = (size_t)rows_per_block * dp + r, l_at = m_at + rows_per_block;

    // phase 1: statistics.  The first split of a thread stays in registers (the usual case has no second one).
    float m0 = -INFINITY, l0 = 0.f;
    if (tid < n_splits) {
        m0 = base[tid * stride + m_at];
        l0 = base[tid * stride + l_at];
    }
    float M = l0 > 0.f ? m0 : -INFINITY;
    for (int s = tid + kMergeThreads; s < n_splits; s += kMergeThreads) {
        const float m = base[s * stride + m_at], l = base[s * stride + l_at];
        M = l > 0.f ? __builtin_fmaxf(M, m) : M;
    }
    M = merge_wave_max(M);
    if ((tid & 63) == 0) stat[0][tid >> 6] = M;
    __syncthreads();
    M = __builtin_fmaxf(__builtin_fmaxf(stat[0][0], stat[0][1]), __builtin_fmaxf(stat[0][2], stat[0][3]));

    auto weight = [&](float m, float l) { return l > 0.f ? __builtin_amdgcn_exp2f(m - M) : 0.f; };
    float L = 0.f;
    {
        const float w = weight(m0, l0);
        if (tid < n_splits) wts[tid] = w;
        L = w * l0;
    }
    for (int s = tid + kMergeThreads; s < n_splits; s += kMergeThreads) {
        const float l = base[s * stride + l_at];
        const float w = weight(base[s * stride + m_at], l);
        if (s < kMergeWeights) wts[s] = w;
        L += w * l;
    }
    L = merge_wave_sum(L);
    if ((tid & 63) == 0) stat[1][tid >> 6] = L;
    __syncthreads();
    L = (stat[1][0] + stat[1][1]) + (stat[1][2] + stat[1][3]);

    // phase 2: weighted sum of the accumulators
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int s = first; s < n_splits; s += lanes) {
        const float* part = base + s * stride;
        const floatx4 o = *(const floatx4*)(part + (size_t)r * dp + 4 * quad);
        const float w = s < kMergeWeights ? wts[s] : weight(part[m_at], part[l_at]);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = w > 0.f ? acc[e] + w * o[e] : acc[e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) red[e][tid] = acc[e];
    __syncthreads();
    if (lane != 0) return;
    for (int k = 1; k < lanes; ++k) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += red[e][k * quads + quad];
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    floatx2 out;
    out[0] = __builtin_bit_cast(float, pack_bf16(acc[0] * inv, acc[1] * inv));
    out[1] = __builtin_bit_cast(float, pack_bf16(acc[2] * inv, acc[3] * inv));
    *(floatx2*)(O + ((size_t)bh * Nq + row) * d + 4 * quad) = out;
}

// Split-keys launch of one tile shape: the partial pass, then the merge.  prob carries n_splits, tiles_per_split
// and the workspace (BH * ceil(Nq / BR) * n_splits * BR * (DP + 2) floats).
template <int D, int QB, int NW, int STAGES>
hipError_t launch_fwd_bf16_split_shape(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob,
                                       float scale, int causal, hipStream_t stream) {
    constexpr int BR = 32 * QB * NW;
    const hipError_t e = causal ? launch_cfg<D, QB, NW, STAGES, true, kSplit>(Q, K, V, O, BH, prob, scale, stream)
                                : launch_cfg<D, QB, NW, STAGES, false, kSplit>(Q, K, V, O, BH, prob, scale, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(split_merge_kernel, dim3((unsigned)BH * (unsigned)prob.Nq), dim3(kMergeThreads), 0, stream, prob.split_ws,
                       (bf16*)O, prob.Nq, (prob.Nq + BR - 1) / BR, BR, Bf16Cfg<D, STAGES, NW>::DP, D, prob.n_splits);
    return hipGetLastError();
}

// rows = rows per workgroup of the plan (split_plan): selects among the shapes built for a head dimension
hipError_t launch_fwd_bf16_split(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, int d,
                                 int rows, float scale, int causal, hipStream_t stream) {
    switch (d * 1000 + rows) {
        case 32032: return launch_fwd_bf16_split_shape<32, 1, 1, 3>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 32064: return launch_fwd_bf16_split_shape<32, 1, 2, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 32128: return launch_fwd_bf16_split_shape<32, 1, 4, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 32256: return launch_fwd_bf16_split_shape<32, 2, 4, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 64032: return launch_fwd_bf16_split_shape<64, 1, 1, 3>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 64064: return launch_fwd_bf16_split_shape<64, 1, 2, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 64128: return launch_fwd_bf16_split_shape<64, 1, 4, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 64256: return launch_fwd_bf16_split_shape<64, 2, 4, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 96128: return launch_fwd_bf16_split_shape<96, 1, 4, 3>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 96256: return launch_fwd_bf16_split_shape<96, 1, 8, 3>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 128128: return launch_fwd_bf16_split_shape<128, 1, 4, 3>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 128256: return launch_fwd_bf16_split_shape<128, 1, 8, 3>(Q, K, V, O, BH, prob, scale, causal, stream);
        case 256128: return launch_fwd_bf16_split_shape<256, 1, 4, 4>(Q, K, V, O, BH, prob, scale, causal, stream);
        default: return hipErrorInvalidValue;
    }
}

// ---- the same launch out of a scratch buffer that lives in the library's own device image ---------------------------------
// For callers that must not allocate.  The array below is a host-side handle only: its device address differs per
// GPU and is looked up once per device with hipGetSymbolAddress; kernels and launches only ever see that address.
static __device__ __align__(256) float scratch[kSplitStaticScratchBytes / sizeof(float)];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<float*> g_scratch_addr[kMaxDevices];  // device address of `scratch` on each GPU, null until first use there
}  // namespace

hipError_t launch_fwd_bf16_split_static(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob,
                                        int d, int rows, float scale, int causal, hipStream_t stream) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    float* addr = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!addr) {
        void* sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));  // with `dev` current: every GPU has its own copy
        if (e != hipSuccess) return e;
        if (!sym) return hipErrorInvalidSymbol;
        addr = static_cast<float*>(sym);
        g_scratch_addr[dev].store(addr, std::memory_order_release);
    }
    Bf16Problem p = prob;
    p.split_ws = addr;
    return launch_fwd_bf16_split(Q, K, V, O, BH, p, d, rows, scale, causal, stream);
}

}  // namespace flat
