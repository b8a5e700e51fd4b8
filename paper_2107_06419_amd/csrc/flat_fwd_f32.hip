// Fused attention forward for gfx950 in fp32 throughout (fp32 MFMA 32x32x2, fp32 probabilities).
// Same dataflow as the bf16 kernel (paper sections 4-5: one pass over blocks of query rows with
// Logit, softmax and Attend interleaved), sized for small problems: 4 wavefronts x 32 query rows
// per workgroup, 32 keys per tile, one LDS stage fed from a register prefetch of the next tile; small problems
// take a second form that splits the keys over the wavefronts of a workgroup (fwd_f32_splitkeys_kernel).
#include "flat_common.hpp"
#include "flat_launch.hpp"

namespace flat {

// One 32-key tile for one wavefront (32 query rows): Logit, exact online softmax, Attend.  Ks holds the tile's
// keys with row pitch D + 1, Vs its values with row pitch D.
template <int D, bool CAUSAL>
__device__ __forceinline__ void f32_tile(const float* Ks, const float* Vs, int jbase, int N, int q0w, int qrow, float c,
                                         const float (&qf)[D / 2], floatx16 (&oacc)[D / 32], float& m, float& lsum, int l32,
                                         int half) {
    constexpr int BC = 32, KS = D / 2, DB = D / 32, KLD = D + 1;
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

        f32_tile<D, CAUSAL>(Ks, Vs, jbase, N, q0w, qrow, c, qf, oacc, m, lsum, l32, half);
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

// Small problems: with 128 rows per workgroup a short sequence leaves most of the chip idle (B*H*N/32 wavefronts
// in all).  This form gives a workgroup only 32 query rows and lets its four wavefronts split the KEYS: wavefront
// w takes the 32-key tiles w, w+4, ... through an LDS region of its own (no workgroup barrier in the loop), and
// the four partial results (running max, sum, unnormalised output) are merged through LDS at the end with the
// same rescaling as a step of the online softmax.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void fwd_f32_splitkeys_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                                const float* __restrict__ V, float* __restrict__ O, int N,
                                                                int n_qtiles, int n_blocks, int blocks_per_xcd, float c) {
    constexpr int BC = 32, KS = D / 2, DB = D / 32, KLD = D + 1, WAVE_LDS = BC * KLD + BC * D;  // floats per wavefront
    extern __shared__ __attribute__((aligned(16))) float lds[];

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
    const int q0w = qt * 32;  // all four wavefronts work on the same 32 rows
    const int qrow = q0w + l32;
    float* Ks = lds + wave * WAVE_LDS;
    float* Vs = Ks + BC * KLD;  // BC * KLD * 4 bytes is a multiple of 16

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
    if (CAUSAL) kv_len = min(N, q0w + 32);
    const int n_tiles = (kv_len + BC - 1) / BC;
    constexpr int LD = BC * D / 4 / 64;  // float4 loads per lane, tile and tensor
    for (int j = wave; j < n_tiles; j += 4) {
        const int jbase = j * BC;
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int ch = lane + 64 * i;
            const int row = ch / (D / 4), col = (ch % (D / 4)) * 4;
            floatx4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
            if (jbase + row < N) {
                kv = *(const floatx4*)(Kh + (size_t)(jbase + row) * D + col);
                vv = *(const floatx4*)(Vh + (size_t)(jbase + row) * D + col);
            }
            Ks[row * KLD + col] = kv[0];
            Ks[row * KLD + col + 1] = kv[1];
            Ks[row * KLD + col + 2] = kv[2];
            Ks[row * KLD + col + 3] = kv[3];
            *(floatx4*)(Vs + row * D + col) = vv;
        }
        // The region is private to this wavefront, but lanes read what other lanes wrote: order the wavefront's
        // LDS stores before its reads, and the reads before the next tile's stores.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        f32_tile<D, CAUSAL>(Ks, Vs, jbase, N, q0w, qrow, c, qf, oacc, m, lsum, l32, half);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // merge: wavefronts 1..3 publish (m, l, O) in their own regions (layout [value][lane], conflict-free)
    lsum = halves_sum(lsum);
    if (wave != 0) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) Ks[(db * 16 + r) * 64 + lane] = oacc[db][r];
        Ks[DB * 16 * 64 + lane] = m;
        Ks[(DB * 16 + 1) * 64 + lane] = lsum;
    }
    __syncthreads();
    if (wave != 0) return;
    float mw[4], lw[4], M = m;
    mw[0] = m;
    lw[0] = lsum;
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        const float* part = lds + w * WAVE_LDS;
        mw[w] = part[DB * 16 * 64 + lane];
        lw[w] = part[(DB * 16 + 1) * 64 + lane];
        M = __builtin_fmaxf(M, mw[w]);
    }
    float L = 0.f, sc[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        sc[w] = __builtin_amdgcn_exp2f(mw[w] - M);  // a wavefront that saw no key has m = -inf: weight 0
        L += lw[w] * sc[w];
    }
    const float inv = 1.0f / L;  // wavefront 0 always sees key 0, so L > 0
    if (qrow < N) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                floatx4 w4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * rq + e;
                    float acc = oacc[db][r] * sc[0];
#pragma unroll
                    for (int w = 1; w < 4; ++w) acc += (lds + w * WAVE_LDS)[(db * 16 + r) * 64 + lane] * sc[w];
                    w4[e] = acc * inv;
                }
                *(floatx4*)(Oh + (size_t)qrow * D + 32 * db + 8 * rq + 4 * half) = w4;
            }
    }
}

template <int D, bool CAUSAL>
static hipError_t launch_cfg(const float* Q, const float* K, const float* V, float* O, int BH, int N, float scale,
                             hipStream_t stream) {
    // 128 rows per workgroup fill the chip (256 compute units, a few workgroups each) only from about 1024 row
    // blocks on; below that, 32 rows per workgroup with the keys split over its wavefronts.
    const int n_qtiles_big = (N + 127) / 128;
    if ((long long)BH * n_qtiles_big < 1024 && N > 128) {
        const int n_qtiles = (N + 31) / 32;
        const int n_blocks = BH * n_qtiles;
        const int blocks_per_xcd = (n_blocks + 7) / 8;
        constexpr int lds = 4 * (32 * (D + 1) + 32 * D) * (int)sizeof(float);
        auto kern = fwd_f32_splitkeys_kernel<D, CAUSAL>;
        static std::atomic<uint64_t> attr_done{0};
        hipError_t e = allow_dynamic_lds((const void*)kern, lds, &attr_done);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(blocks_per_xcd * 8), dim3(256), lds, stream, Q, K, V, O, N, n_qtiles, n_blocks,
                           blocks_per_xcd, scale * kLog2e);
        return hipGetLastError();
    }
    const int n_qtiles = n_qtiles_big;
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
