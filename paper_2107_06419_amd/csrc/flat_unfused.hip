// Operator-by-operator attention for gfx950: the baseline dataflow of the paper's Fig.
// "flat_dataflow"(a).  Three kernels with the N x N intermediate in device memory:
//   1. logits_kernel   L = Q K^T * scale        -> fp32 [BH, N, N]        (Logit, section 2 step 2)
//   2. softmax_kernel  each row of L replaced by its softmax (in place)  (step 3)
//   3. attend_kernel   O = A V, A read back from memory                   (Attend, step 4)
// This is what the fused kernel is measured against: same MFMA instructions, but the intermediate
// crosses HBM four times (write, read, write, read), which is the traffic section 3 analyses.
#include "flat_common.hpp"
#include "flat_launch.hpp"

namespace flat {

// ---------------------------------------------------------------------------------------------
// 1. L[bh, i, j] = scale * sum_k Q[bh,i,k] K[bh,j,k].  Workgroup = 128 x 128 tile of L; wave w owns
//    rows 32w..32w+31 and all 128 columns.  Operands go straight from global memory into MFMA
//    fragments (the contraction is only d long).
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void logits_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                     float* __restrict__ L, int N, float scale) {
    constexpr int DS = D / 16;
    const int bh = blockIdx.z;
    const int row0 = blockIdx.y * 128, col0 = blockIdx.x * 128;
    if (CAUSAL && col0 > row0 + 127) return;  // wholly above the diagonal: the softmax kernel writes zeros there
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const size_t head = (size_t)bh * N * D;
    const bf16* Qh = Q + head;
    const bf16* Kh = K + head;
    float* Lh = L + (size_t)bh * N * N;

    const int qrow = row0 + 32 * wave + l32;
    bf16x8 qf[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
        uint4v z = {0, 0, 0, 0};
        if (qrow < N) z = *(const uint4v*)(Qh + (size_t)qrow * D + ds * 16 + half * 8);
        qf[ds] = __builtin_bit_cast(bf16x8, z);
    }
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int key = col0 + 32 * cb + l32;
        floatx16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            uint4v z = {0, 0, 0, 0};
            if (key < N) z = *(const uint4v*)(Kh + (size_t)key * D + ds * 16 + half * 8);
            s = mfma_bf16_32x32x16(qf[ds], __builtin_bit_cast(bf16x8, z), s);  // rows = queries, columns = keys
        }
        if (key < N) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + 32 * wave + acc_row(r, half);
                if (row < N) Lh[(size_t)row * N + key] = s[r] * scale;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 2. One workgroup per row; the row is replaced by exp(x - max) / sum.  Keys beyond the causal limit are
//    written as exact zeros.  Two forms:
//    - softmax_row_regs: rows of up to THREADS * 4 * CH logits (N a multiple of 4, at most 65536) are held in
//      registers, CH float4 per thread, so memory sees one read and one write of the row;
//    - softmax_row_stream: any N; a running (max, sum) pass and a second pass that reads the row again.
__device__ __forceinline__ void online_combine(float& m, float& s, float m2, float s2) {
    const float mn = __builtin_fmaxf(m, m2);
    const float a = (m == -INFINITY) ? 0.f : __expf(m - mn);
    const float b = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
    s = s * a + s2 * b;
    m = mn;
}

template <bool IS_MAX, int WAVES>
__device__ __forceinline__ float block_reduce(float v, float* slots) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float o = __shfl_xor(v, off);
        v = IS_MAX ? __builtin_fmaxf(v, o) : v + o;
    }
    if ((threadIdx.x & 63) == 0) slots[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = slots[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) r = IS_MAX ? __builtin_fmaxf(r, slots[w]) : r + slots[w];
    return r;
}

template <bool CAUSAL, int CH, int THREADS>
__global__ __launch_bounds__(THREADS) void softmax_row_regs(float* __restrict__ L, int N) {
    constexpr int WAVES = THREADS / 64;
    __shared__ float smax[WAVES], ssum[WAVES];
    const size_t rowid = blockIdx.x;  // bh * N + i
    const int i = (int)(rowid % (size_t)N);
    float* row = L + rowid * (size_t)N;
    const int nk = CAUSAL ? i + 1 : N;
    const int tid = threadIdx.x;

    floatx4 x[CH];
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int j = (c * THREADS + tid) * 4;
        x[c] = floatx4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (j < nk) x[c] = *(const floatx4*)(row + j);  // j < nk <= N and N % 4 == 0, so j + 3 < N
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (CAUSAL && j + e >= nk) x[c][e] = -INFINITY;
            m = __builtin_fmaxf(m, x[c][e]);
        }
    }
    m = block_reduce<true, WAVES>(m, smax);  // key 0 is always valid, so m is finite
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[c][e] = __expf(x[c][e] - m);  // masked and out-of-row slots: exp(-inf) = 0
            s += x[c][e];
        }
    s = block_reduce<false, WAVES>(s, ssum);
    const float inv = 1.0f / s;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int j = (c * THREADS + tid) * 4;
        if (j < N) *(floatx4*)(row + j) = floatx4{x[c][0] * inv, x[c][1] * inv, x[c][2] * inv, x[c][3] * inv};
    }
}

template <bool CAUSAL>
__global__ __launch_bounds__(256) void softmax_row_stream(float* __restrict__ L, int N) {
    const size_t rowid = blockIdx.x;  // bh * N + i
    const int i = (int)(rowid % (size_t)N);
    float* row = L + rowid * (size_t)N;
    const int nk = CAUSAL ? i + 1 : N;
    const int tid = threadIdx.x;

    float m = -INFINITY, s = 0.f;
    for (int j = tid; j < nk; j += 256) {
        const float x = row[j];
        if (x > m) {
            s = s * __expf(m - x) + 1.f;
            m = x;
        } else {
            s += __expf(x - m);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(m, off), s2 = __shfl_xor(s, off);
        online_combine(m, s, m2, s2);
    }
    __shared__ float sm[4], ss[4];
    if ((tid & 63) == 0) {
        sm[tid >> 6] = m;
        ss[tid >> 6] = s;
    }
    __syncthreads();
    m = sm[0];
    s = ss[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) online_combine(m, s, sm[w], ss[w]);
    const float inv = 1.0f / s;
    for (int j = tid; j < N; j += 256) row[j] = (j < nk) ? __expf(row[j] - m) * inv : 0.f;
}

template <bool CAUSAL>
static void launch_softmax(float* L, int BH, int N, hipStream_t stream) {
    const dim3 grid((unsigned)((size_t)BH * N));
    const bool vec = (N & 3) == 0;
    if (vec && N <= 1024)
        hipLaunchKernelGGL((softmax_row_regs<CAUSAL, 1, 256>), grid, dim3(256), 0, stream, L, N);
    else if (vec && N <= 4096)
        hipLaunchKernelGGL((softmax_row_regs<CAUSAL, 4, 256>), grid, dim3(256), 0, stream, L, N);
    else if (vec && N <= 16384)
        hipLaunchKernelGGL((softmax_row_regs<CAUSAL, 16, 256>), grid, dim3(256), 0, stream, L, N);
    else if (vec && N <= 65536)
        hipLaunchKernelGGL((softmax_row_regs<CAUSAL, 16, 1024>), grid, dim3(1024), 0, stream, L, N);
    else
        hipLaunchKernelGGL((softmax_row_stream<CAUSAL>), grid, dim3(256), 0, stream, L, N);
}

// ---------------------------------------------------------------------------------------------
// 3. O[bh, i, :] = sum_j A[bh,i,j] V[bh,j,:].  Workgroup = 128 query rows, wave w owns rows
//    32w..32w+31.  A is read as fp32 from global memory directly in MFMA A-operand order (8
//    consecutive keys per lane) and rounded to bf16; V tiles (64 keys) go through LDS and are read
//    transposed with ds_read_b64_tr_b16.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attend_kernel(const float* __restrict__ A, const bf16* __restrict__ V,
                                                     bf16* __restrict__ O, int N) {
    constexpr int DB = D / 32, BC = 64, VSTRIDE = D * 2 + 64, CHUNKS = D * 2 / 16, LOADS = BC * CHUNKS / 256;
    __shared__ __attribute__((aligned(16))) char Vs[BC * VSTRIDE];
    const int bh = blockIdx.y;
    const int row0 = blockIdx.x * 128;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const float* Ah = A + (size_t)bh * N * N;
    const char* Vh = (const char*)(V + (size_t)bh * N * D);
    bf16* Oh = O + (size_t)bh * N * D;
    const int arow = row0 + 32 * wave + l32;  // the query row whose probabilities this lane loads
    const bool vec_ok = (N & 3) == 0;

    floatx16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;

    int kv_len = N;
    if (CAUSAL) kv_len = min(N, row0 + 128);
    const int n_tiles = (kv_len + BC - 1) / BC;
    const int i16 = lane & 15, g16 = lane >> 4;
    const int v_lane_off = (8 * (g16 >> 1) + (i16 >> 2)) * VSTRIDE + (16 * (g16 & 1) + 4 * (i16 & 3)) * 2;

    for (int j = 0; j < n_tiles; ++j) {
        const int jbase = j * BC;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int ch = tid + 256 * i;
            const int r = ch / CHUNKS, col = ch % CHUNKS;
            uint4v z = {0, 0, 0, 0};
            if (jbase + r < N) z = *(const uint4v*)(Vh + (size_t)(jbase + r) * (D * 2) + col * 16);
            *(uint4v*)(Vs + r * VSTRIDE + col * 16) = z;
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 4; ++t) {  // 16 keys per MFMA
            const int k0 = jbase + 16 * t + 8 * half;
            float a[8];
            if (arow < N && vec_ok && k0 + 8 <= N) {
                const floatx4 a0 = *(const floatx4*)(Ah + (size_t)arow * N + k0);
                const floatx4 a1 = *(const floatx4*)(Ah + (size_t)arow * N + k0 + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    a[e] = a0[e];
                    a[4 + e] = a1[e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = (arow < N && k0 + e < N) ? Ah[(size_t)arow * N + k0 + e] : 0.f;
            }
            uint4v pw = {pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(a[4], a[5]), pack_bf16(a[6], a[7])};
            const bf16x8 af = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const char* vp = Vs + (16 * t) * VSTRIDE + v_lane_off + db * 64;
                const bf16x8 vf = concat(lds_read_tr16(vp), lds_read_tr16(vp + 4 * VSTRIDE));
                oacc[db] = mfma_bf16_32x32x16(af, vf, oacc[db]);  // rows = queries, columns = head dim
            }
        }
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + 32 * wave + acc_row(r, half);
            if (row < N) Oh[(size_t)row * D + 32 * db + l32] = (bf16)oacc[db][r];
        }
}

template <int D, bool CAUSAL>
static hipError_t launch_cfg(const void* Q, const void* K, const void* V, void* O, int BH, int N, float scale, float* L,
                             hipStream_t stream) {
    const int nt = (N + 127) / 128;
    hipLaunchKernelGGL((logits_kernel<D, CAUSAL>), dim3(nt, nt, BH), dim3(256), 0, stream, (const bf16*)Q, (const bf16*)K, L,
                       N, scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    launch_softmax<CAUSAL>(L, BH, N, stream);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attend_kernel<D, CAUSAL>), dim3(nt, BH), dim3(256), 0, stream, (const float*)L, (const bf16*)V,
                       (bf16*)O, N);
    return hipGetLastError();
}

hipError_t launch_unfused_bf16(const void* Q, const void* K, const void* V, void* O, int BH, int N, int d, float scale,
                               int causal, float* L, hipStream_t stream) {
    if (d == 64)
        return causal ? launch_cfg<64, true>(Q, K, V, O, BH, N, scale, L, stream)
                      : launch_cfg<64, false>(Q, K, V, O, BH, N, scale, L, stream);
    return causal ? launch_cfg<128, true>(Q, K, V, O, BH, N, scale, L, stream)
                  : launch_cfg<128, false>(Q, K, V, O, BH, N, scale, L, stream);
}

}  // namespace flat
