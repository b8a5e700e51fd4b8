// Fused attention forward for gfx950 in fp32 throughout (fp32 MFMA 32x32x2, fp32 probabilities).
// Same dataflow as the bf16 kernel (paper sections 4-5: one pass over blocks of query rows with
// Logit, softmax and Attend interleaved), sized for small problems: 4 wavefronts x 32 query rows
// per workgroup, 32 keys per tile, one LDS stage fed from a register prefetch of the next tile.
#include "flat_common.hpp"
#include "flat_launch.hpp"

namespace flat {

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void fwd_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                      const float* __restrict__ V, float* __restrict__ O, int N,
                                                      int n_qtiles, int n_blocks, int blocks_per_xcd, float c) {
    constexpr int BR = 128, BC = 32, KS = D / 2, DB = D / 32, KLD = D + 1;  // KLD: odd row pitch, conflict-free column reads
    __shared__ float Ks[BC * KLD];
    __shared__ __attribute__((aligned(16))) float Vs[BC * D];

    const int logical = xcd_logical_block(blockIdx.x, blocks_per_xcd);
    if (logical >= n_blocks) return;
    const int bh = logical / n_qtiles;
    int qt = logical - bh * n_qtiles;
    if (CAUSAL) qt = n_qtiles - 1 - qt;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const size_t head = (size_t)bh * N * D;
    const float* Qh = Q + head;
    const float* Kh = K + head;
    const float* Vh = V + head;
    float* Oh = O + head;
    const int q0w = qt * BR + wave * 32;
    const int qrow = q0w + l32;

    float qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = qrow < N ? Qh[(size_t)qrow * D + 2 * ks + half] : 0.f;

    floatx16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m = -INFINITY, lsum = 0.f;

    int kv_len = N;
    if (CAUSAL) kv_len = min(N, qt * BR + BR);
    const int n_tiles = (kv_len + BC - 1) / BC;

    // K/V tiles are fetched one tile ahead into registers and written to LDS once the previous tile's readers
    // are done, so the global-memory latency overlaps the MFMAs of the tile before.
    constexpr int LD = BC * D / 4 / 256;  // float4 loads per thread, tile and tensor
    floatx4 kreg[LD], vreg[LD];
    auto fetch_tile = [&](int jbase) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int ch = tid + 256 * i;
            const int row = ch / (D / 4), col = (ch % (D / 4)) * 4;
            kreg[i] = floatx4{0, 0, 0, 0};
            vreg[i] = floatx4{0, 0, 0, 0};
            if (jbase + row < N) {
                kreg[i] = *(const floatx4*)(Kh + (size_t)(jbase + row) * D + col);
                vreg[i] = *(const floatx4*)(Vh + (size_t)(jbase + row) * D + col);
            }
        }
    };
    if (n_tiles > 0) fetch_tile(0);

    for (int j = 0; j < n_tiles; ++j) {
        const int jbase = j * BC;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int ch = tid + 256 * i;
            const int row = ch / (D / 4), col = (ch % (D / 4)) * 4;
            Ks[row * KLD + col] = kreg[i][0];
            Ks[row * KLD + col + 1] = kreg[i][1];
            Ks[row * KLD + col + 2] = kreg[i][2];
            Ks[row * KLD + col + 3] = kreg[i][3];
            *(floatx4*)(Vs + row * D + col) = vreg[i];
        }
        __syncthreads();
        if (j + 1 < n_tiles) fetch_tile(jbase + BC);
        if (CAUSAL && jbase > q0w + 31) continue;  // every key of this tile is masked for this wavefront

        // Logit: S^T[key, query]
        floatx16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s = mfma_f32_32x32x2(Ks[l32 * KLD + 2 * ks + half], qf[ks], s);

        const bool masked = (jbase + BC > N) || (CAUSAL && jbase + BC - 1 > q0w);
        uint32_t okmask = 0xffffu;
        if (masked) {
            okmask = 0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = jbase + acc_row(r, half);
                const bool ok = key < N && (!CAUSAL || key <= qrow);
                okmask |= ok ? (1u << r) : 0u;
                s[r] = ok ? s[r] : -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(mx, s[r]);
        mx = halves_max(mx);
        const float m_new = __builtin_fmaxf(m, mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        lsum *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        m = m_new;
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float x = __builtin_fmaf(s[r], c, -m_new);
            if (masked) x = (okmask >> r) & 1u ? x : -INFINITY;
            p[r] = __builtin_amdgcn_exp2f(x);
            lsum += p[r];
        }
        // Attend: O^T[dcol, query] += V^T[dcol, key] P^T[key, query]; step r contracts the two keys
        // acc_row(r, 0) and acc_row(r, 1) held by the two wave halves.
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key_local = acc_row(r, half);
#pragma unroll
            for (int db = 0; db < DB; ++db) oacc[db] = mfma_f32_32x32x2(Vs[key_local * D + 32 * db + l32], p[r], oacc[db]);
        }
    }

    const float inv = 1.0f / halves_sum(lsum);
    if (qrow < N) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                floatx4 w = {oacc[db][4 * rq] * inv, oacc[db][4 * rq + 1] * inv, oacc[db][4 * rq + 2] * inv,
                             oacc[db][4 * rq + 3] * inv};
                *(floatx4*)(Oh + (size_t)qrow * D + 32 * db + 8 * rq + 4 * half) = w;
            }
    }
}

template <int D, bool CAUSAL>
static hipError_t launch_cfg(const float* Q, const float* K, const float* V, float* O, int BH, int N, float scale,
                             hipStream_t stream) {
    const int n_qtiles = (N + 127) / 128;
    const int n_blocks = BH * n_qtiles;
    const int blocks_per_xcd = (n_blocks + 7) / 8;
    hipLaunchKernelGGL((fwd_f32_kernel<D, CAUSAL>), dim3(blocks_per_xcd * 8), dim3(256), 0, stream, Q, K, V, O, N,
                       n_qtiles, n_blocks, blocks_per_xcd, scale * kLog2e);
    return hipGetLastError();
}

hipError_t launch_fwd_f32(const float* Q, const float* K, const float* V, float* O, int BH, int N, int d, float scale,
                          int causal, hipStream_t stream) {
    if (d == 64)
        return causal ? launch_cfg<64, true>(Q, K, V, O, BH, N, scale, stream)
                      : launch_cfg<64, false>(Q, K, V, O, BH, N, scale, stream);
    return causal ? launch_cfg<128, true>(Q, K, V, O, BH, N, scale, stream)
                  : launch_cfg<128, false>(Q, K, V, O, BH, N, scale, stream);
}

}  // namespace flat
