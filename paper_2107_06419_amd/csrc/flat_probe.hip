// Throughput probes (measurement aids, no attention arithmetic is served from here).
//
// mfma_probe_kernel: an MFMA-only loop: what the matrix pipe of this GPU sustains on its own, with constant or
// with random operands.  On MI355X the clock a kernel runs at depends on the power its operands draw, so a bf16
// MFMA loop over random data sustains noticeably less than the same loop over constants.
//
// mix_probe_kernel<LEVEL>: the instruction mix of one step of the fused d = 64 kernel (16 MFMAs 32x32x16 and the
// 96 softmax vector instructions of two 32-row blocks against one 32-key block, scheduled by the same
// sched_group_barrier recipe), looped on synthetic data, with the kernel's data movement added rung by rung:
//   LEVEL 0  registers only: the ceiling this instruction mix can reach
//   LEVEL 1  + the K and V^T operand fragments read from LDS every step (4 ds_read_b128 + 8 ds_read_b64_tr_b16)
//   LEVEL 2  + one workgroup barrier per 64-key tile
//   LEVEL 3  + each 64-key K/V tile streamed global -> LDS (global_load_lds_dwordx4) from an L2-resident source
// LEVEL 3 has the structure of the fused kernel's main loop; the gaps between the rungs say what each part costs.
#include "flat_common.hpp"
#include "flat_launch.hpp"
#include "flat_fwd_bf16_kernel.hpp"

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


// ---- instruction-mix probe -------------------------------------------------------------------------------------
constexpr int kMixGrid = 512, kMixBlock = 256;      // two workgroups of four wavefronts per compute unit
constexpr int kMixSrcTiles = 64;                    // 64-key tiles in the global source (8 KiB per tile and tensor)
constexpr int kMixStepsPerIter = 8;                 // one loop trip = 4 tiles = 8 steps (the ring has 4 stages)
constexpr int kMixMfmaPerStep = 16;

template <int LEVEL>
__global__ __launch_bounds__(kMixBlock, 2) void mix_probe_kernel(float* __restrict__ sink, const char* __restrict__ src, int iters,
                                                                 float c) {
    using C = Bf16Cfg<64, 4, 4>;
    constexpr int QB = 2, DS = 4, DB = 2;
    __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    // All operands come from `src` (the caller's bf16 values), so that every level multiplies data of the same
    // distribution: the power an MFMA draws, and with it the clock, depends on its operands.
    constexpr int kSrcBytes = 2 * kMixSrcTiles * C::KBYTES;
    const uint4v* src16 = (const uint4v*)src;
    for (int i = tid; i < C::LDS_BYTES / 16; i += kMixBlock)
        ((uint4v*)smem)[i] = src16[(blockIdx.x * (C::LDS_BYTES / 16) + i) & (kSrcBytes / 16 - 1)];
    __syncthreads();
    auto src_frag = [&](int k) { return __builtin_bit_cast(bf16x8, src16[(tid * 32 + blockIdx.x * 7 + k) & (kSrcBytes / 16 - 1)]); };
    bf16x8 qf[QB][DS], kf[DS], vfA[2][DB], vfB[2][DB];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
        kf[ds] = src_frag(16 + ds);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) qf[qb][ds] = src_frag(qb * 4 + ds);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            vfA[t][db] = src_frag(20 + 2 * t + db);
            vfB[t][db] = src_frag(24 + 2 * t + db);
        }
    // the fused kernel's LDS addressing (operand reads and the wave-wide 1 KiB stores of the streaming loads)
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    int koff[DS], voff[DB][2];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) koff[ds] = (int)smem_base + l32 * C::ROWB + (((2 * ds + half) ^ C::swz(l32)) << 4);
    const int i16 = lane & 15, g16 = lane >> 4;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const int r = 8 * hi + 4 * (g16 >> 1) + (i16 >> 2);
            const int ch = 4 * db + 2 * (g16 & 1) + ((i16 >> 1) & 1);
            voff[db][hi] = (int)smem_base + r * C::ROWB + ((ch ^ C::swz(r)) << 4) + (i16 & 1) * 8;
        }
    uint32_t ld_off[C::LOADS];  // byte offset of this lane's 16 bytes inside a source tile
#pragma unroll
    for (int i = 0; i < C::LOADS; ++i) {
        const int row = (4 * i + wave) * C::ROWS_PER_LOAD + lane / C::CHUNKS;
        ld_off[i] = (uint32_t)row * C::ROWB + (((lane % C::CHUNKS) ^ C::swz(row)) << 4);
    }
    int src_tile = blockIdx.x & (kMixSrcTiles - 1);
    auto stream_tile = [&](int stage) __attribute__((always_inline)) {
        const char* ksrc = src + (size_t)src_tile * C::KBYTES;
        const char* vsrc = ksrc + (size_t)kMixSrcTiles * C::KBYTES;
        src_tile = (src_tile + 1) & (kMixSrcTiles - 1);
#pragma unroll
        for (int i = 0; i < C::LOADS; ++i) {
            const uint32_t dst = __builtin_amdgcn_readfirstlane(smem_base + stage * C::STAGE + (4 * i + wave) * 1024);
            dma16(ksrc, ld_off[i], dst);
            dma16(vsrc, ld_off[i], dst + C::KBYTES);
        }
    };

    floatx16 oacc[QB][DB], xA[QB], xB[QB];
    uint32_t pA[QB][8], pB[QB][8];
    float m[QB], lsum[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m[qb] = 0.125f * ((lane + qb) & 7);
        lsum[qb] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) xA[qb][r] = xB[qb][r] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            pA[qb][i] = 0x3f003e80u + (probe_hash(tid + i) & 63);
            pB[qb][i] = 0x3e803f00u + (probe_hash(tid + 99 + i) & 63);
        }
    }
#pragma unroll
    for (int ds = 0; ds < DS; ++ds)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) xA[qb] = mfma_bf16_32x32x16(kf[ds], qf[qb][ds], xA[qb]);
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};

    // One step, as in the fused kernel: matrix pipe Attend(previous block) and Logit(next block), vector ALU the
    // softmax of the current block; stage / kb are constants, so the LDS offsets fold into the instructions.
    auto step = [&](int stage, int next_stage, int kb, floatx16 (&xc)[QB], floatx16 (&xn)[QB], const uint32_t (&pp)[QB][8],
                    const bf16x8 (&vp)[2][DB], uint32_t (&pc)[QB][8], bf16x8 (&vc)[2][DB]) __attribute__((always_inline)) {
        typedef const bf16x8 __attribute__((address_space(3))) * lds_frag_ptr;
        if (LEVEL >= 1) {
            const int k_at = next_stage * C::STAGE + (kb ^ 1) * 32 * C::ROWB;
            const int v_at = stage * C::STAGE + C::KBYTES + kb * 32 * C::ROWB;
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                asm volatile("" : "+v"(koff[ds]));
                kf[ds] = *(lds_frag_ptr)(uintptr_t)(uint32_t)(koff[ds] + k_at);
            }
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                asm volatile("" : "+v"(voff[db][0]), "+v"(voff[db][1]));
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    vc[t][db] = concat(lds_read_tr16_at(voff[db][0] + v_at + t * 16 * C::ROWB),
                                       lds_read_tr16_at(voff[db][1] + v_at + t * 16 * C::ROWB));
            }
        } else {
            // registers only: tell the compiler the fragments may have changed, so that no product is hoisted
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) asm volatile("" : "+v"(kf[ds]));
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int db = 0; db < DB; ++db) asm volatile("" : "+v"(vc[t][db]));
        }
        __builtin_amdgcn_sched_barrier(0);
        float y[QB][16], bsum[QB];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    uint4v pw = {pp[qb][4 * t], pp[qb][4 * t + 1], pp[qb][4 * t + 2], pp[qb][4 * t + 3]};
                    oacc[qb][db] = mfma_bf16_32x32x16(vp[t][db], __builtin_bit_cast(bf16x8, pw), oacc[qb][db]);
                }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) xn[qb][r] = 0.f;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) xn[qb] = mfma_bf16_32x32x16(kf[ds], qf[qb][ds], xn[qb]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) y[qb][r] = __builtin_fmaf(xc[qb][r], c, -m[qb]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float l0 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 4) {
                float e[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) e[i] = __builtin_amdgcn_exp2f(y[qb][r + i]);
                const uint32_t pk0 = pack_bf16(e[0], e[1]), pk1 = pack_bf16(e[2], e[3]);
                pc[qb][r >> 1] = pk0;
                pc[qb][(r >> 1) + 1] = pk1;
                l0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk0), ones, l0, false);
                l0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk1), ones, l0, false);
            }
            bsum[qb] = l0;
        }
#pragma unroll
        for (int g = 0; g < kMixMfmaPerStep; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // the fused kernel's test for a logit far above the reference maximum, with a stand-in for its rare path
        bool jump = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) jump |= !(bsum[qb] <= kSumJump);
        if (__builtin_amdgcn_ballot_w64(jump) != 0) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float a = y[qb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) a = __builtin_fmaxf(a, y[qb][r]);
                a = halves_max(a);
                m[qb] += __builtin_fmaxf(a, 0.f);
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    pc[qb][r] = pack_bf16(__builtin_amdgcn_exp2f(y[qb][2 * r] - a), __builtin_amdgcn_exp2f(y[qb][2 * r + 1] - a));
                bsum[qb] = 1.0f;
            }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) lsum[qb] += bsum[qb];
    };

    if (LEVEL >= 3) {
#pragma unroll
        for (int t = 0; t < 3; ++t) stream_tile(t);
        wait_vm<0>();
        __syncthreads();
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int sj = 0; sj < 4; ++sj) {  // tile in ring stage sj, consumed as two 32-key blocks
            const int sn = (sj + 1) & 3, sd = (sj + 3) & 3;
            if (LEVEL >= 1)
                step(sj, sj, 0, xA, xB, pB, vfB, pA, vfA);
            else
                step(sj, sj, 0, xA, xB, pB, vfA, pA, vfA);
            if (LEVEL >= 3) wait_vm<(4 - 3) * 2 * C::LOADS>();
            if (LEVEL >= 2) __syncthreads();
            if (LEVEL >= 3) stream_tile(sd);
            if (LEVEL >= 1)
                step(sj, sn, 1, xB, xA, pA, vfA, pB, vfB);
            else
                step(sj, sn, 1, xB, xA, pA, vfA, pB, vfA);
        }
    }
    if (LEVEL >= 3) wait_vm<0>();
    float s = 0.f;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        s += lsum[qb];
#pragma unroll
        for (int r = 0; r < 16; ++r) s += xA[qb][r] + oacc[qb][0][r] + oacc[qb][1][r];
    }
    sink[blockIdx.x * kMixBlock + tid] = s;
}

hipError_t launch_mix_probe(float* sink, const void* src, int level, int iters, hipStream_t stream) {
    const float c = 0.125f * kLog2e;
    const char* s8 = static_cast<const char*>(src);
    switch (level) {
        case 0: hipLaunchKernelGGL(mix_probe_kernel<0>, dim3(kMixGrid), dim3(kMixBlock), 0, stream, sink, s8, iters, c); break;
        case 1: hipLaunchKernelGGL(mix_probe_kernel<1>, dim3(kMixGrid), dim3(kMixBlock), 0, stream, sink, s8, iters, c); break;
        case 2: hipLaunchKernelGGL(mix_probe_kernel<2>, dim3(kMixGrid), dim3(kMixBlock), 0, stream, sink, s8, iters, c); break;
        default: hipLaunchKernelGGL(mix_probe_kernel<3>, dim3(kMixGrid), dim3(kMixBlock), 0, stream, sink, s8, iters, c); break;
    }
    return hipGetLastError();
}

double mix_probe_flops(int iters) {
    return (double)kMixGrid * (kMixBlock / 64) * iters * kMixStepsPerIter * kMixMfmaPerStep * 32768.0;
}

size_t mix_probe_sink_bytes() { return (size_t)kMixGrid * kMixBlock * sizeof(float); }

size_t mix_probe_src_bytes() { return (size_t)2 * kMixSrcTiles * Bf16Cfg<64, 4, 4>::KBYTES; }

}  // namespace flat
