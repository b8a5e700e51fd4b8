// Fused attention forward for gfx950, bf16 in / fp32 accumulate / bf16 out.
//
// Dataflow (paper sections 4-5: fused Logit-softmax-Attend with a shared outer loop over batch,
// head and blocks of query rows, the two inner loops interleaved):
//   one workgroup = one (batch, head, block of BR query rows); its 4 wavefronts own QW = BR/4 rows
//   each.  The key/value sequence is streamed in tiles of BC = 64 keys through LDS (two stages, the
//   paper's double-buffered operand tiles).  Per tile a wavefront computes
//       S^T = K_tile Q^T           (Logit, MFMA 32x32x16 bf16; the transposed product is chosen so
//                                   that a lane owns ONE query column: row max / row sum are then
//                                   in-lane reductions plus one exchange between wave halves)
//       P   = exp2(c S - m)        (row softmax numerator with running max m, fp32, then bf16 RNE)
//       O^T += V_tile^T P^T        (Attend; the accumulator layout of S^T is already the B-operand
//                                   layout of this product, so P never leaves registers;
//                                   V^T operands come from ds_read_b64_tr_b16 on row-major V)
// and only Q, K, V are read and O written: the N x N intermediate never exists off-chip.
// Unlike the paper's row-granularity tile, which keeps a whole R x N logit slab on chip, the row
// max and sum are carried as running values, so on-chip state is independent of N.
#include "flat_common.hpp"
#include "flat_launch.hpp"

namespace flat {

// LDS tile layout.  Rows are stored unpadded (ROWB = 2 D bytes) because tiles arrive by
// global_load_lds_dwordx4, which writes the 64 lanes of a wavefront to 1024 contiguous LDS bytes
// (lane l at base + 16 l).  Bank conflicts are avoided instead by an XOR swizzle of the 16-byte
// chunk index within a row: chunk c of row r lives in slot c ^ swz(r).  The LDS serves 256 bytes
// per clock: a ds_read_b128 touches 16 rows at one chunk index per clock, a ds_read_b64_tr_b16
// touches 4 rows x 64 bytes; swz() is chosen so that both patterns hit every bank once.
template <int D>
struct Bf16Cfg {
    static constexpr int BC = 64;                     // keys per tile
    static constexpr int ROWB = D * 2;                // bytes per row
    static constexpr int CHUNKS = ROWB / 16;          // 16-byte chunks per row
    static constexpr int KBYTES = BC * ROWB;
    static constexpr int VBYTES = BC * ROWB;
    static constexpr int STAGE = KBYTES + VBYTES;
    static constexpr int ROWS_PER_LOAD = 1024 / ROWB; // rows covered by one wave-wide 16-byte-per-lane load
    static constexpr int LOADS = BC / ROWS_PER_LOAD / 4;  // such loads per wavefront per tensor per tile
    static constexpr int LDS_BYTES = 2 * STAGE;
    __device__ static __forceinline__ int swz(int r) {
        if (D == 64) return (((r >> 1) & 1) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1);  // 128-byte rows: 2 rows per 256 B
        return ((r & 3) << 2) | ((r >> 2) & 3);                                              // 256-byte rows
    }
};

template <int D, int QB, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void fwd_bf16_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                          const bf16* __restrict__ V, bf16* __restrict__ O, int N,
                                                          int n_qtiles, int n_blocks, int blocks_per_xcd, float c) {
    using C = Bf16Cfg<D>;
    constexpr int QW = 32 * QB, BR = 4 * QW, BC = C::BC, DS = D / 16, DB = D / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int logical = xcd_logical_block(blockIdx.x, blocks_per_xcd);
    if (logical >= n_blocks) return;
    const int bh = logical / n_qtiles;
    int qt = logical - bh * n_qtiles;
    if (CAUSAL) qt = n_qtiles - 1 - qt;  // longest rows first

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const size_t head = (size_t)bh * N * D;
    const bf16* Qh = Q + head;
    const char* Kh = (const char*)(K + head);
    const char* Vh = (const char*)(V + head);
    bf16* Oh = O + head;
    const int q0w = qt * BR + wave * QW;

    // Q^T fragments (B operand of S^T = K Q^T): column = query, 8 consecutive head-dim elements
    bf16x8 qf[QB][DS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = q0w + 32 * qb + l32;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            uint4v z = {0, 0, 0, 0};
            if (row < N) z = *(const uint4v*)(Qh + (size_t)row * D + ds * 16 + half * 8);
            qf[qb][ds] = __builtin_bit_cast(bf16x8, z);
        }
    }

    floatx16 oacc[QB][DB];
    float m[QB], lsum[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m[qb] = -INFINITY;
        lsum[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
    }

    int kv_len = N;
    if (CAUSAL) kv_len = min(N, qt * BR + BR);
    const int n_tiles = (kv_len + BC - 1) / BC;

    // global -> LDS copy of one K tile and one V tile, no registers in between.  Wave w issues load
    // i for the 1024-byte LDS block (4 i + w); lane l fills slot (l % CHUNKS) of row (l / CHUNKS) of
    // that block, so it fetches the chunk whose swizzled position that is.  Keys beyond N are clamped
    // to the last key: their logits are masked and their (finite) values meet a zero probability.
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    const int ld_row = lane / C::CHUNKS;
    auto issue_tile_loads = [&](int tile, int stage) {
        char* Kb = smem + stage * C::STAGE;
        char* Vb = Kb + C::KBYTES;
#pragma unroll
        for (int i = 0; i < C::LOADS; ++i) {
            const int blk = 4 * i + wave;
            const int row = blk * C::ROWS_PER_LOAD + ld_row;
            const int chunk = (lane % C::CHUNKS) ^ C::swz(row);
            const int key = min(tile * BC + row, N - 1);
            const size_t off = (size_t)key * C::ROWB + chunk * 16;
            __builtin_amdgcn_global_load_lds((gptr_t)(Kh + off), (lptr_t)(Kb + blk * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(Vh + off), (lptr_t)(Vb + blk * 1024), 16, 0, 0);
        }
    };
    auto wait_tile_loads = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    // per-lane LDS byte offsets of the MFMA operand reads (row part + swizzled chunk), one per
    // compile-time chunk index
    int koff[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) koff[ds] = l32 * C::ROWB + (((2 * ds + half) ^ C::swz(l32)) << 4);
    const int i16 = lane & 15, g16 = lane >> 4;
    int voff[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const int r = 8 * hi + 4 * (g16 >> 1) + (i16 >> 2);             // row within a 16-key step
            const int ch = 4 * db + 2 * (g16 & 1) + ((i16 >> 1) & 1);      // 16-byte chunk holding this lane's 4 columns
            voff[db][hi] = r * C::ROWB + ((ch ^ C::swz(r)) << 4) + (i16 & 1) * 8;
        }
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};

    // One tile = 64 keys, processed as two blocks of 32 keys so that only a 32 x QW logit block and its
    // probabilities are live at a time.
    auto compute_tile = [&](int stage, int jbase, bool masked) {
        const char* Kb = smem + stage * C::STAGE;
        const char* Vb = Kb + C::KBYTES;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            // ---- Logit: S^T[key, query] for keys jbase + 32 kb .. + 31
            floatx16 s[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[qb][r] = 0.f;
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                const bf16x8 kf = *(const bf16x8*)(Kb + kb * 32 * C::ROWB + koff[ds]);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) s[qb] = mfma_bf16_32x32x16(kf, qf[qb][ds], s[qb]);
            }
            // ---- row softmax with running max / sum; a lane owns query (l32) of each 32-row block
            uint32_t p[QB][8];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                uint32_t okmask = 0xffffffffu;
                if (masked) {
                    const int qidx = q0w + 32 * qb + l32;
                    okmask = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = jbase + 32 * kb + acc_row(r, half);
                        const bool ok = key < N && (!CAUSAL || key <= qidx);
                        okmask |= ok ? (1u << r) : 0u;
                        s[qb][r] = ok ? s[qb][r] : -INFINITY;
                    }
                }
                float mx = s[qb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(mx, s[qb][r]);
                mx = halves_max(mx);
                // mx * c is NaN only if c == 0 and the block is fully masked; fmaxf then keeps m
                const float m_new = __builtin_fmaxf(m[qb], mx * c);
                if (__builtin_amdgcn_ballot_w64(m_new != m[qb]) != 0) {
                    const float alpha = __builtin_amdgcn_exp2f(m[qb] - m_new);
                    lsum[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
                    m[qb] = m_new;
                }
                float ls = lsum[qb];
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float x0 = __builtin_fmaf(s[qb][r], c, -m_new);
                    float x1 = __builtin_fmaf(s[qb][r + 1], c, -m_new);
                    if (masked) {
                        x0 = (okmask >> r) & 1u ? x0 : -INFINITY;
                        x1 = (okmask >> (r + 1)) & 1u ? x1 : -INFINITY;
                    }
                    const float p0 = __builtin_amdgcn_exp2f(x0);
                    const float p1 = __builtin_amdgcn_exp2f(x1);
                    const uint32_t pk = pack_bf16(p0, p1);
                    p[qb][r >> 1] = pk;
                    // row sum of the ROUNDED probabilities, so that sum and the Attend operand agree
                    ls = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, ls, false);
                }
                lsum[qb] = ls;
            }
            // ---- Attend: O^T[dcol, query] += V^T[dcol, key] P^T[key, query]
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const char* vrow = Vb + (kb * 32 + t * 16) * C::ROWB;  // swz() only looks at row bits below 16
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x4 lo = lds_read_tr16(vrow + voff[db][0]);
                    const bf16x4 hi = lds_read_tr16(vrow + voff[db][1]);
                    const bf16x8 vf = concat(lo, hi);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        uint4v pw = {p[qb][4 * t], p[qb][4 * t + 1], p[qb][4 * t + 2], p[qb][4 * t + 3]};
                        oacc[qb][db] = mfma_bf16_32x32x16(vf, __builtin_bit_cast(bf16x8, pw), oacc[qb][db]);
                    }
                }
            }
        }
    };

    issue_tile_loads(0, 0);
    wait_tile_loads();
    __syncthreads();
#pragma unroll 1
    for (int j = 0; j < n_tiles; ++j) {
        const bool more = j + 1 < n_tiles;
        if (more) issue_tile_loads(j + 1, (j + 1) & 1);  // that stage was last read before the previous barrier
        const int jbase = j * BC;
        const bool active = !CAUSAL || jbase <= q0w + QW - 1;
        if (active) {
            const bool masked = (jbase + BC > N) || (CAUSAL && jbase + BC - 1 > q0w);
            if (masked)
                compute_tile(j & 1, jbase, true);
            else
                compute_tile(j & 1, jbase, false);
        }
        wait_tile_loads();
        __syncthreads();
    }

    // ---- epilogue: O = O_acc / l, rounded to bf16; a lane holds 4 consecutive head-dim elements per register quad
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float inv = 1.0f / halves_sum(lsum[qb]);
        const int row = q0w + 32 * qb + l32;
        if (row < N) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int dcol = 32 * db + 8 * rq + 4 * half;
                    floatx2 w;
                    w[0] = __builtin_bit_cast(float, pack_bf16(oacc[qb][db][4 * rq] * inv, oacc[qb][db][4 * rq + 1] * inv));
                    w[1] = __builtin_bit_cast(float, pack_bf16(oacc[qb][db][4 * rq + 2] * inv, oacc[qb][db][4 * rq + 3] * inv));
                    *(floatx2*)(Oh + (size_t)row * D + dcol) = w;
                }
        }
    }
}

template <int D, int QB, bool CAUSAL>
static hipError_t launch_cfg(const void* Q, const void* K, const void* V, void* O, int BH, int N, float scale,
                             hipStream_t stream) {
    constexpr int BR = 128 * QB;
    const int n_qtiles = (N + BR - 1) / BR;
    const long long n_blocks_ll = (long long)BH * n_qtiles;
    const int n_blocks = (int)n_blocks_ll;
    const int blocks_per_xcd = (n_blocks + 7) / 8;
    auto kern = fwd_bf16_kernel<D, QB, CAUSAL>;
    constexpr int lds = Bf16Cfg<D>::LDS_BYTES;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(blocks_per_xcd * 8), dim3(256), lds, stream, (const bf16*)Q, (const bf16*)K,
                       (const bf16*)V, (bf16*)O, N, n_qtiles, n_blocks, blocks_per_xcd, scale * kLog2e);
    return hipGetLastError();
}

hipError_t launch_fwd_bf16(const void* Q, const void* K, const void* V, void* O, int BH, int N, int d, float scale,
                           int causal, hipStream_t stream) {
    if (d == 64) {
        return causal ? launch_cfg<64, 2, true>(Q, K, V, O, BH, N, scale, stream)
                      : launch_cfg<64, 2, false>(Q, K, V, O, BH, N, scale, stream);
    }
    return causal ? launch_cfg<128, 1, true>(Q, K, V, O, BH, N, scale, stream)
                  : launch_cfg<128, 1, false>(Q, K, V, O, BH, N, scale, stream);
}

}  // namespace flat
