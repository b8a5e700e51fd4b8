// Fused attention forward for gfx950, bf16 in / fp32 accumulate / bf16 out.
//
// Dataflow (paper sections 4-5: fused Logit-softmax-Attend with a shared outer loop over batch,
// head and blocks of query rows, the two inner loops interleaved):
//   one workgroup = one (batch, head, block of BR query rows); its NW wavefronts own QW = BR/NW
//   rows each.  The key/value sequence is streamed in tiles of 64 keys through a ring of LDS stages
//   (the paper's double-buffered operand tiles, deepened to hide HBM/L2 latency).  Each tile is
//   consumed as two blocks of 32 keys; per block a wavefront computes
//       S^T = K_blk Q^T            (Logit, MFMA 32x32x16 bf16; the transposed product is chosen so
//                                   that a lane owns ONE query column: row max / row sum are then
//                                   in-lane reductions plus one exchange between wave halves)
//       P   = exp2(c S - m)        (row softmax numerator against a reference max m, fp32 -> bf16 RNE)
//       O^T += V_blk^T P^T         (Attend; the accumulator layout of S^T is already the B-operand
//                                   layout of this product, so P never leaves registers;
//                                   V^T operands come from ds_read_b64_tr_b16 on row-major V)
// and only Q, K, V are read and O written: the N x N intermediate never exists off-chip.
// Unlike the paper's row-granularity tile, which keeps a whole R x N logit slab on chip, the row
// max and sum are carried as running values, so on-chip state is independent of N.
//
// Reference max and optimistic exponentiation.  softmax is invariant to the constant subtracted per
// row, so m need not be the exact running maximum.  It starts as the (scaled) logit of key 0, which
// every query sees, so the row sum is at least 1 relative to it and can never underflow.  The steady
// state exponentiates against the current m WITHOUT computing the block maximum; a logit far above m
// shows up as a jump of the fp32 row sum (more than kSumJump per lane and block, i.e. some
// probability above 2^10), and only then the block takes the exact path: row maximum, raise m,
// rescale O and l, recompute the block's probabilities.  Probabilities therefore stay below 2^14
// relative to m, far inside bf16/fp32 range, and for typical data the exact path runs in the first
// blocks only.
#pragma once
#include "flat_common.hpp"
#include "flat_launch.hpp"

namespace flat {

constexpr float kSumJump = 16384.0f;  // per lane and 32-key block: 16 probabilities

// Checking build (-DFLAT_SYNC_EVERY_PHASE): nothing is left in flight across a phase of the ring.  Every
// streaming load is awaited in full and fenced by a barrier on both sides, and every LDS operand read is awaited
// before the step goes on.  The release build overlaps these phases and counts on its vmcnt arithmetic and on
// one barrier per tile; the two builds must produce bit-identical results, which a GPU test checks.
#ifdef FLAT_SYNC_EVERY_PHASE
constexpr bool kSyncEveryPhase = true;
#else
constexpr bool kSyncEveryPhase = false;
#endif

// Head dimensions.  D is the head dimension of the tensors in memory (32, 64, 96, 128 or 256); the tiles in LDS
// and the matrix products use DP = D rounded up to a power of two (96 -> 128: the missing columns of Q are zero,
// so whatever the padded K columns hold drops out of the logits, and the padded output columns are not stored).
// A tile holds BC keys: 64 (two 32-key blocks), or 32 at d = 256, where 64 keys of K and V would take 64 KiB; a tile
// shape may ask for another multiple of 32 (BCX: 32, 64 or 128) so that this axis of the map space can be measured too.
//
// LDS tile layout.  Rows are stored unpadded (ROWB = 2 DP bytes) because tiles arrive by
// global_load_lds_dwordx4, which writes the 64 lanes of a wavefront to 1024 contiguous LDS bytes
// (lane l at base + 16 l).  Bank conflicts are avoided instead by an XOR swizzle of the 16-byte
// chunk index within a row: chunk c of row r lives in slot c ^ swz(r).  The LDS serves 256 bytes
// per clock: a ds_read_b128 touches 16 rows at one chunk index per clock, a ds_read_b64_tr_b16
// touches 4 rows x 64 bytes; swz() is chosen so that both patterns hit every bank once.
template <int D, int STAGES, int NW, int BCX = 0>
struct Bf16Cfg {
    static_assert(D == 32 || D == 64 || D == 96 || D == 128 || D == 256, "head dimension not built");
    static constexpr int DP = D == 96 ? 128 : D;      // head dimension of the tiles and products
    static constexpr int BC = BCX ? BCX : (D == 256 ? 32 : 64);  // keys per tile
    static constexpr int ROWB = DP * 2;               // bytes per row in LDS
    static constexpr int GROWB = D * 2;               // bytes per row in global memory
    static constexpr int CHUNKS = ROWB / 16;          // 16-byte chunks per LDS row
    static constexpr int GCHUNKS = GROWB / 16;        // ... of which this many exist in memory
    static constexpr int KBYTES = BC * ROWB;
    static constexpr int VBYTES = BC * ROWB;
    static constexpr int STAGE = KBYTES + VBYTES;
    static constexpr int ROWS_PER_LOAD = 1024 / ROWB; // rows covered by one wave-wide 16-byte-per-lane load
    static constexpr int LOADS = BC / ROWS_PER_LOAD / NW; // such loads per wavefront per tensor per tile
    static_assert(LOADS >= 1 && LOADS * ROWS_PER_LOAD * NW == BC, "the wavefronts must share a tile's rows evenly");
    static constexpr int LDS_BYTES = STAGES * STAGE;
    __device__ static __forceinline__ int swz(int r) {
        if (ROWB == 64) return (r >> 2) & 3;                                                    // 4 rows per 256 B
        if (ROWB == 128) return (((r >> 1) & 1) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1);  // 2 rows per 256 B
        return ((r & 3) << 2) | ((r >> 2) & 3);                                                 // rows of 256 B or more
    }
};

// One wave-wide global -> LDS copy, 16 bytes per lane: lane l's bytes land at lds_base + 16 l.
// Issued as inline asm so that the compiler does not serialise later LDS reads of OTHER stages
// behind it; completion is awaited explicitly with wait_vm<n>() before the stage is published by
// a barrier.  lds_base must be wave-uniform.  The statement overwrites m0, which the compiler reserves and does
// not accept on a clobber list; the kernels here contain nothing else that lives in m0 (no indirect register
// indexing, no LDS-direct or message instructions), and a host-side test checks the generated assembly for that.
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(gbase) : "memory");
}
// s_waitcnt vmcnt(CNT) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4, lgkmcnt 11:8).  Emitted through the builtin so that the compiler's own wait bookkeeping
// sees it.
template <int CNT>
__device__ __forceinline__ void wait_vm() {
    static_assert(CNT >= 0 && CNT < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((CNT & 15) | ((CNT >> 4) << 14) | (7 << 4) | (15 << 8));
}

constexpr int kMaxSparseTiles = 2048;  // block-sparse: listed tiles per row block that fit the LDS copy of the list (8 KiB)

// Template parameters: D head dimension (32, 64, 96, 128, 256), QB 32-row blocks per wavefront, NW wavefronts per workgroup, STAGES
// depth of the K/V ring, CAUSAL mask, MODE: kDense, kSparse = block-sparse variant (the workgroup visits only the 64-key tiles
// listed for its row block, ids ascending, staged in LDS behind the ring; everything else as in the dense kernel).
// Two wavefronts per SIMD (256 registers each), except 64 rows per wavefront at d = 128 and every shape at d = 256,
// whose accumulators alone need more: those run one wavefront per SIMD with the full 512 registers.

// kSplit = the keys of one row block are divided over prob.n_splits workgroups, each of which leaves its
// unnormalised result (reference maximum, row sum, accumulators) in a workspace for split_merge_kernel.
constexpr int kDense = 0, kSparse = 1, kSplit = 2;

template <int D, int QB, int NW, int STAGES, bool CAUSAL, int MODE = kDense, int BCX = 0>
__global__ __launch_bounds__(64 * NW, ((D == 128 && QB == 2) || D == 256) ? 1 : 2) void fwd_bf16_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                          const bf16* __restrict__ V, bf16* __restrict__ O,
                                                          const Bf16Problem prob, int n_qtiles, int n_blocks,
                                                          int blocks_per_xcd, float c) {
    using C = Bf16Cfg<D, STAGES, NW, BCX>;
    constexpr bool SPARSE = MODE == kSparse, SPLIT = MODE == kSplit;
    constexpr int DP = C::DP, QW = 32 * QB, BR = NW * QW, BC = C::BC, DS = DP / 16, DB = DP / 32;
    constexpr int KB = BC / 32;    // 32-key blocks per tile
    constexpr int KB64 = 64 / BC;  // tiles per 64 keys (the unit of a block-sparse list)
    static_assert(KB == 1 || KB == 2 || KB == 4, "a tile is one, two or four 32-key blocks");
    static_assert(KB != 1 || STAGES % 2 == 0, "with one block per tile the unrolled loop needs an even ring");
    static_assert(!SPARSE || KB64 >= 1, "block-sparse lists name 64-key tiles");
    constexpr int LOADS_PER_TILE = 2 * C::LOADS;  // DMA instructions per wavefront per tile (K and V)
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Which (head, row block) this workgroup takes.  Workgroup ids are dealt round-robin to the 8 XCDs, so XCD x
    // sees the ids x, x+8, ...: position t = id / 8 of its own sequence.
    // Without a mask all blocks cost the same: XCD x takes the contiguous range [x, x+1) * blocks_per_xcd of
    // (head, row block) pairs, so that the workgroups sharing one head's K/V share one L2.
    // With the causal mask row block q costs ~ q+1 tiles, and the order decides the load balance.  All blocks are
    // ranked heaviest first across ALL heads (rank g = rows-from-the-end * heads + head) and dealt to the XCDs
    // like cards (XCD x gets ranks x, x+8, ...): every XCD gets the same mix, its late, dynamically placed
    // workgroups are the light ones, and with a head count that is a multiple of 8 it still sees only its own
    // heads.  When two workgroups fit a compute unit the hardware places positions t and t+32 of an XCD's
    // sequence on the same unit in the first round; the second half of every 64 positions is therefore taken in
    // reverse, which pairs the k-th heaviest of the 64 with the k-th lightest.
    static_assert(!(CAUSAL && SPARSE), "the block-sparse variant has no causal form");
    int bh, qt;
    if (!CAUSAL) {
        const int logical = xcd_logical_block(blockIdx.x, blocks_per_xcd);
        if (logical >= n_blocks) return;
        bh = logical / n_qtiles;
        qt = logical - bh * n_qtiles;
    } else {
        constexpr int kByLds = (160 * 1024) / C::LDS_BYTES, kByRegs = 8 / NW;  // two wavefronts per SIMD
        constexpr bool kTwoPerUnit = (kByLds < kByRegs ? kByLds : kByRegs) == 2;
        const int x = blockIdx.x & 7, t = blockIdx.x >> 3;
        int r = t;
        if (kTwoPerUnit && (t | 63) < blocks_per_xcd && (t & 32)) r = (t & ~31) + 31 - (t & 31);
        const int g = 8 * r + x;
        if (g >= n_blocks) return;
        const int heads = n_blocks / n_qtiles;
        const int from_end = g / heads;
        bh = g - from_end * heads;
        qt = n_qtiles - 1 - from_end;
    }

    int split = 0;
    if (SPLIT) {  // the launch counts (row block, split) pairs per head; the splits of a row block are neighbours
        split = qt % prob.n_splits;
        qt /= prob.n_splits;
    }
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    // Nq query rows per head; N = number of keys of this head that count (the padded tail of a shorter batch
    // entry is masked like the tail of a ragged tile); causal: query i sees keys 0 .. i + off.
    const int Nq = prob.Nq, off = prob.causal_offset;
    int N = prob.Nk;
    if (prob.kv_lens) N = max(1, min(prob.Nk, prob.kv_lens[bh / prob.heads_per_batch]));
    const size_t head_q = (size_t)bh * Nq * D, head_k = (size_t)bh * prob.Nk * D;
    const bf16* Qh = Q + head_q;
    const char* Kh = (const char*)(K + head_k);
    const char* Vh = (const char*)(V + head_k);
    bf16* Oh = O + head_q;
    const int q0w = qt * BR + wave * QW;

    // Q^T fragments (B operand of S^T = K Q^T): column = query, 8 consecutive head-dim elements
    bf16x8 qf[QB][DS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = q0w + 32 * qb + l32;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            uint4v z = {0, 0, 0, 0};  // rows past the end and the padded head-dim columns are zero
            if (row < Nq && ds * 16 + half * 8 < D) z = *(const uint4v*)(Qh + (size_t)row * D + ds * 16 + half * 8);
            qf[qb][ds] = __builtin_bit_cast(bf16x8, z);
        }
    }

    // Block-sparse: copy this row block's tile list into LDS (ids forced into range; a wrong list can give a
    // wrong result but no stray access).
    int* const sp_ids = (int*)(smem + C::LDS_BYTES);
    int sp_count = 0;
    if (SPARSE) {
        const int n_ktiles = (N + 63) / 64;  // list entries name 64-key tiles
        const int row_block = bh * ((Nq + 255) / 256) + (qt * BR) / 256;  // lists are per 256 query rows; BR divides 256
        const int lo = max(0, min(prob.n_tile_ids, prob.tile_offsets[row_block]));
        const int hi = max(lo, min(prob.n_tile_ids, prob.tile_offsets[row_block + 1]));
        sp_count = min(hi - lo, kMaxSparseTiles);
        for (int i = tid; i < sp_count; i += 64 * NW) sp_ids[i] = max(0, min(n_ktiles - 1, prob.tile_ids[lo + i]));
        __syncthreads();
    }
    // Split keys: this workgroup takes tiles [t0, t0 + tiles_per_split) of those its row block sees.
    int kv_len = N;
    if (CAUSAL) kv_len = min(N, qt * BR + BR + off);
    const int t0 = SPLIT ? split * prob.tiles_per_split : 0;
    // j-th tile this workgroup visits (a listed 64-key tile is KB64 consecutive tiles)
    auto tile_of = [&](int j) __attribute__((always_inline)) {
        if (SPLIT) return t0 + j;
        if (!SPARSE) return j;
        return KB64 == 1 ? sp_ids[j] : sp_ids[j / KB64] * KB64 + j % KB64;
    };

    float m[QB];  // reference max of each row, set in the prologue below

    floatx16 oacc[QB][DB];
    float lsum[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        lsum[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
    }

    const int n_tiles_seen = (kv_len + BC - 1) / BC;  // tiles the row block sees
    const int n_tiles = SPARSE ? sp_count * KB64                                              // tiles this workgroup visits
                        : SPLIT ? max(0, min(n_tiles_seen - t0, prob.tiles_per_split)) : n_tiles_seen;

    // ---- global -> LDS streaming.  Wave w issues load i of a tile for the 1024-byte LDS block
    // (NW i + w); lane l fills slot (l % CHUNKS) of row (l / CHUNKS) of that block, so it fetches
    // the chunk whose swizzled position that is (for a padded head dimension, a chunk that does not
    // exist in memory is replaced by one of the same row that does: its content never matters).
    // Keys beyond N are clamped to the last key: their logits are masked and their (finite) values
    // meet a zero probability.
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    int ld_row[C::LOADS], ld_chunk_off[C::LOADS];
#pragma unroll
    for (int i = 0; i < C::LOADS; ++i) {
        ld_row[i] = (NW * i + wave) * C::ROWS_PER_LOAD + lane / C::CHUNKS;
        const int chunk = (lane % C::CHUNKS) ^ C::swz(ld_row[i]);
        ld_chunk_off[i] = (chunk < C::GCHUNKS ? chunk : chunk - (C::CHUNKS - C::GCHUNKS)) * 16;
    }
    auto issue_tile_loads = [&](int j, int stage) __attribute__((always_inline)) {  // j-th visited tile, stage = j % STAGES
        const uint32_t stage_base = smem_base + (uint32_t)stage * C::STAGE;
        const int tile = tile_of(j);
#pragma unroll
        for (int i = 0; i < C::LOADS; ++i) {
            const int key = min(tile * BC + ld_row[i], N - 1);
            const uint32_t voff = (uint32_t)key * C::GROWB + ld_chunk_off[i];
            const uint32_t lds_k = __builtin_amdgcn_readfirstlane(stage_base + (NW * i + wave) * 1024);
            dma16(Kh, voff, lds_k);
            dma16(Vh, voff, lds_k + C::KBYTES);
        }
    };

    // per-lane LDS byte addresses of the MFMA operand reads (ring base + row part + swizzled chunk), one per
    // compile-time chunk index
    int koff[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) koff[ds] = (int)smem_base + l32 * C::ROWB + (((2 * ds + half) ^ C::swz(l32)) << 4);
    const int i16 = lane & 15, g16 = lane >> 4;
    int voff[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const int r = 8 * hi + 4 * (g16 >> 1) + (i16 >> 2);         // row within a 16-key step
            const int ch = 4 * db + 2 * (g16 & 1) + ((i16 >> 1) & 1);  // 16-byte chunk holding this lane's 4 columns
            voff[db][hi] = (int)smem_base + r * C::ROWB + ((ch ^ C::swz(r)) << 4) + (i16 & 1) * 8;
        }
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};

    // ---- block = 32 keys.  Pieces of the per-block work; the main loop below software-pipelines them so
    // that the matrix pipe works on PV of block b-1 and on S of block b+1 while the vector ALU does the
    // softmax of block b.
    // (stage, kb) locate a block: ring stage of its tile and which half of the tile.  In the unrolled main loop
    // both are compile-time constants and fold into the immediate offsets of the LDS reads.
    auto read_k = [&](int stage, int kb, bf16x8 (&kf)[DS]) __attribute__((always_inline)) {  // K fragments (A operand of S^T = K Q^T) of one block
        typedef const bf16x8 __attribute__((address_space(3))) * lds_frag_ptr;
        const int block_off = stage * C::STAGE + kb * 32 * C::ROWB;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            // Declaring the lane offset "modified" keeps (offset + constant) from being hoisted out of the loop
            // into one register per stage; inside the loop the constant folds into the DS offset field.
            asm volatile("" : "+v"(koff[ds]));
            kf[ds] = *(lds_frag_ptr)(uintptr_t)(uint32_t)(koff[ds] + block_off);
        }
    };
    auto read_v = [&](int stage, int kb, bf16x8 (&vf)[2][DB]) __attribute__((always_inline)) {  // V^T fragments (A operand of O^T += V^T P^T)
        const int block_off = stage * C::STAGE + C::KBYTES + kb * 32 * C::ROWB;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            asm volatile("" : "+v"(voff[db][0]), "+v"(voff[db][1]));
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int off = block_off + t * 16 * C::ROWB;  // swz() only looks at row bits below 16
                vf[t][db] = concat(lds_read_tr16_at(voff[db][0] + off), lds_read_tr16_at(voff[db][1] + off));
            }
        }
    };
    auto logits = [&](const bf16x8 (&kf)[DS], floatx16 (&x)[QB]) __attribute__((always_inline)) {  // S^T = K Q^T
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) x[qb][r] = 0.f;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) x[qb] = mfma_bf16_32x32x16(kf[ds], qf[qb][ds], x[qb]);
    };
    auto attend = [&](const bf16x8 (&vf)[2][DB], const uint32_t (&p)[QB][8]) __attribute__((always_inline)) {  // O^T += V^T P^T
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    uint4v pw = {p[qb][4 * t], p[qb][4 * t + 1], p[qb][4 * t + 2], p[qb][4 * t + 3]};
                    oacc[qb][db] = mfma_bf16_32x32x16(vf[t][db], __builtin_bit_cast(bf16x8, pw), oacc[qb][db]);
                }
    };
    // x <- c S - m (masked keys -> -inf)
    auto shift = [&](int blk, bool masked, floatx16 (&x)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float mref = m[qb];
#pragma unroll
            for (int r = 0; r < 16; ++r) x[qb][r] = __builtin_fmaf(x[qb][r], c, -mref);
            if (masked) {
                const int qidx = q0w + 32 * qb + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = blk * 32 + acc_row(r, half);
                    const bool ok = key < N && (!CAUSAL || key <= qidx + off);
                    x[qb][r] = ok ? x[qb][r] : -INFINITY;  // exp2 -> probability exactly 0
                }
            }
        }
    };
    auto row_max = [&](const floatx16 (&x)[QB], float (&mx)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float a = x[qb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) a = __builtin_fmaxf(a, x[qb][r]);
            mx[qb] = halves_max(a);
        }
    };
    // p <- bf16(exp2(x)); bsum <- this block's sum of the ROUNDED probabilities (so that the row sum and the
    // Attend operand agree).  One accumulator chain per query block: its links are spread through the step
    // anyway, and a second chain costs more in merging than it gains.
    auto softmax_b = [&](floatx16 (&x)[QB], uint32_t (&p)[QB][8], float (&bsum)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float l0 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 4) {
                float e[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) e[i] = __builtin_amdgcn_exp2f(x[qb][r + i]);
                const uint32_t pk0 = pack_bf16(e[0], e[1]), pk1 = pack_bf16(e[2], e[3]);
                p[qb][r >> 1] = pk0;
                p[qb][(r >> 1) + 1] = pk1;
                l0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk0), ones, l0, false);
                l0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk1), ones, l0, false);
            }
            bsum[qb] = l0;
        }
    };
    // Rare path: raise the reference max of every row whose block maximum lies above it, rescale O and l,
    // and shift the block's exponents accordingly.
    auto rescale = [&](floatx16 (&x)[QB], const float (&mx)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float delta = __builtin_fmaxf(mx[qb], 0.f);
            const float alpha = __builtin_amdgcn_exp2f(-delta);
            m[qb] += delta;
            lsum[qb] *= alpha;
#pragma unroll
            for (int r = 0; r < 16; ++r) x[qb][r] -= delta;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
        }
    };
    // ---- prologue: fill STAGES-1 stages.  The full wait at its end also retires the Q loads above, so that no
    // wait on them is left inside the loops (it would drain the prefetch ring every iteration).  The streaming
    // loads go out before the first-key loads below are waited for, so that a workgroup's start is one memory round
    // trip, not two in a row (short sequences consist of little else).
#pragma unroll
    for (int t = 0; t < STAGES - 1; ++t)
        if (t < n_tiles) issue_tile_loads(t, t);
    // reference max of each row = c * (q . k_first), k_first = the first key the row block sees (key 0 unless
    // block-sparse or split), from the Q fragments already in registers
    {
        float k0[DS][8];
        const int first_key = SPLIT ? min(t0 * BC, N - 1) : (SPARSE && sp_count > 0) ? sp_ids[0] * 64 : 0;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            uint4v kv = {0, 0, 0, 0};
            if (ds * 16 + half * 8 < D) kv = *(const uint4v*)(Kh + (size_t)first_key * C::GROWB + ds * 32 + half * 16);
            const bf16x8 kb8 = __builtin_bit_cast(bf16x8, kv);
#pragma unroll
            for (int e = 0; e < 8; ++e) k0[ds][e] = (float)kb8[e];
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float dot = 0.f;
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = __builtin_fmaf((float)qf[qb][ds][e], k0[ds][e], dot);
            m[qb] = halves_sum(dot) * c;
        }
    }
    wait_vm<0>();
    __syncthreads();

    // With d = 128 two sets of V fragments do not fit the register file next to the accumulators: then one
    // set is used, refilled in the middle of each step right after the MFMAs that consumed it were issued.
    constexpr bool kTwoVSets = (DP <= 64);
    // d = 256 (one wavefront per SIMD, accumulators in the upper half of its 512 registers): the other half has to
    // hold everything the vector ALU touches, so K fragments are kept 8 at a time and V fragments one 16-key half
    // at a time, and the Attend of a block follows its softmax in the same step instead of being owed to the next.
    constexpr bool kWide = (DP == 256);
    constexpr int KFN = kWide ? DS / 2 : DS;
    // Pipeline state: xA/xB hold the logits of the current / next block, pA/pB and vfA/vfB the
    // probabilities and V fragments of the block whose Attend is still owed.
    floatx16 xA[QB], xB[QB];
    uint32_t pA[QB][8], pB[QB][8];
    bf16x8 vfA[2][DB], vfB[2][DB];  // vfB stays unused with one set; the wide form uses vfA[0] only
    bf16x8 kf[DS];                  // the wide form uses the first KFN
    float mx[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int i = 0; i < 8; ++i) pB[qb][i] = 0u;  // the Attend owed before block 0 adds nothing
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int db = 0; db < DB; ++db) vfA[t][db] = vfB[t][db] = __builtin_bit_cast(bf16x8, (uint4v){0, 0, 0, 0});
    // wide form: K fragments ds = h KFN .. of one block, and the V fragments of one 16-key half t
    auto read_k_half = [&](int stage, int kb, int h) __attribute__((always_inline)) {
        typedef const bf16x8 __attribute__((address_space(3))) * lds_frag_ptr;
        const int block_off = stage * C::STAGE + kb * 32 * C::ROWB;
#pragma unroll
        for (int i = 0; i < KFN; ++i) {
            asm volatile("" : "+v"(koff[h * KFN + i]));
            kf[i] = *(lds_frag_ptr)(uintptr_t)(uint32_t)(koff[h * KFN + i] + block_off);
        }
    };
    auto read_v_half = [&](int stage, int kb, int t) __attribute__((always_inline)) {
        const int off = stage * C::STAGE + C::KBYTES + kb * 32 * C::ROWB + t * 16 * C::ROWB;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            asm volatile("" : "+v"(voff[db][0]), "+v"(voff[db][1]));
            vfA[0][db] = concat(lds_read_tr16_at(voff[db][0] + off), lds_read_tr16_at(voff[db][1] + off));
        }
    };
    auto logits_half = [&](int h, floatx16 (&x)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < KFN; ++i)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) x[qb] = mfma_bf16_32x32x16(kf[i], qf[qb][h * KFN + i], x[qb]);
    };
    auto attend_half = [&](int t, const uint32_t (&p)[QB][8]) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                uint4v pw = {p[qb][4 * t], p[qb][4 * t + 1], p[qb][4 * t + 2], p[qb][4 * t + 3]};
                oacc[qb][db] = mfma_bf16_32x32x16(vfA[0][db], __builtin_bit_cast(bf16x8, pw), oacc[qb][db]);
            }
    };
    if (kWide) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) xA[qb][r] = 0.f;
        read_k_half(0, 0, 0);
        logits_half(0, xA);
        __builtin_amdgcn_sched_barrier(0);
        read_k_half(0, 0, 1);
        logits_half(1, xA);
    } else {
        read_k(0, 0, kf);
        logits(kf, xA);
    }

    // One step = one block b:   matrix pipe: Attend(b-1) and S(b+1);   vector ALU: softmax(b).
    // Stage bookkeeping (tile j = blocks 2j, 2j+1; reads of step b touch K of block b+1 and V of block b):
    //   after step 2j   : wait for tile j+1, barrier  (also: every wave is past step 2j-1, the last reader of tile j-1)
    //   before step 2j+1: start streaming tile j+STAGES-1 into the stage that held tile j-1
    auto step = [&](int blk, int stage, int next_stage, bool masked, floatx16 (&xc)[QB], floatx16 (&xn)[QB], const uint32_t (&pp)[QB][8],
                    const bf16x8 (&vp)[2][DB], uint32_t (&pc)[QB][8], bf16x8 (&vc)[2][DB]) __attribute__((always_inline)) {
        if (kWide) {
            // Wide head: S(b+1) in two halves with the softmax of block b spread under them, then Attend(b) in its
            // two key halves; every batch of LDS reads has eight MFMAs (256 matrix-pipe cycles) ahead of its use.
            constexpr auto kLgkm0 = (63 & 15) | ((63 >> 4) << 14) | (7 << 4) | (0 << 8);
            float bs[QB];
            read_k_half(next_stage, 0, 0);
            read_v_half(stage, 0, 0);
            if (kSyncEveryPhase) __builtin_amdgcn_s_waitcnt(kLgkm0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) xn[qb][r] = 0.f;
            logits_half(0, xn);
            shift(blk, masked, xc);
#pragma unroll
            for (int g = 0; g < QB * KFN; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (QB * 16) / (QB * KFN), 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            read_k_half(next_stage, 0, 1);
            if (kSyncEveryPhase) __builtin_amdgcn_s_waitcnt(kLgkm0);
            __builtin_amdgcn_sched_barrier(0);
            logits_half(1, xn);
            softmax_b(xc, pc, bs);
#pragma unroll
            for (int g = 0; g < QB * KFN; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (QB * 32) / (QB * KFN), 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            bool jumped = false;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) jumped |= !(bs[qb] <= kSumJump);
            if (__builtin_amdgcn_ballot_w64(jumped) != 0) {  // exact path, before this block's Attend
                row_max(xc, mx);
                rescale(xc, mx);
                softmax_b(xc, pc, bs);
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) lsum[qb] += bs[qb];
            attend_half(0, pc);
            __builtin_amdgcn_sched_barrier(0);
            read_v_half(stage, 0, 1);
            if (kSyncEveryPhase) __builtin_amdgcn_s_waitcnt(kLgkm0);
            __builtin_amdgcn_sched_barrier(0);
            attend_half(1, pc);
            return;
        }
        read_k(next_stage, (blk + 1) & (KB - 1), kf);
        if (kTwoVSets) read_v(stage, blk & (KB - 1), vc);
        if (kSyncEveryPhase) __builtin_amdgcn_s_waitcnt((63 & 15) | ((63 >> 4) << 14) | (7 << 4) | (0 << 8));  // lgkmcnt(0) only
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads at the top: they have a whole step to land
        float bsum[QB];
        constexpr int kMfmaPerStep = 2 * QB * DB + QB * DS, kValuPerMfma = (QB * 48) / kMfmaPerStep;
        if (kTwoVSets) {
            // one scheduling region: spread the MFMAs evenly through the softmax instructions
            attend(vp, pp);
            logits(kf, xn);
            shift(blk, masked, xc);
            softmax_b(xc, pc, bsum);
#pragma unroll
            for (int g = 0; g < kMfmaPerStep; ++g) {  // vector work first: measured about 1 % faster than MFMA first
                __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);  // one MFMA's share of the vector work
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);             // one MFMA
            }
        } else {
            // two regions; the single V fragment set (vp and vc are the same registers) is refilled between them
            attend(vp, pp);
            shift(blk, masked, xc);
#pragma unroll
            for (int g = 0; g < 2 * QB * DB; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (QB * 16) / (2 * QB * DB), 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            read_v(stage, blk & (KB - 1), vc);
            if (kSyncEveryPhase) __builtin_amdgcn_s_waitcnt((63 & 15) | ((63 >> 4) << 14) | (7 << 4) | (0 << 8));
            __builtin_amdgcn_sched_barrier(0);
            logits(kf, xn);
            softmax_b(xc, pc, bsum);
#pragma unroll
            for (int g = 0; g < QB * DS; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (QB * 32) / (QB * DS), 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        bool jump = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) jump |= !(bsum[qb] <= kSumJump);
        if (__builtin_amdgcn_ballot_w64(jump) != 0) {  // exact path: xc still holds c S - m of this block
            row_max(xc, mx);
            rescale(xc, mx);
            softmax_b(xc, pc, bsum);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            lsum[qb] += bsum[qb];
        }
    };
    // Ring bookkeeping around the steps of one tile.  sync_before_last_step: wait for tile j+1 (of the tiles in
    // flight only STAGES-3 may still be outstanding), barrier (every wavefront is then also past its last read of
    // tile j-1), and start streaming tile j+STAGES-1 into the stage that held tile j-1.
    auto sync_and_stream = [&](int j, int sj) __attribute__((always_inline)) {
        if (kSyncEveryPhase || j + STAGES - 2 >= n_tiles)
            wait_vm<0>();
        else
            wait_vm<(STAGES - 3) * LOADS_PER_TILE>();
        __syncthreads();
        if (j + STAGES - 1 < n_tiles) issue_tile_loads(j + STAGES - 1, sj == 0 ? STAGES - 1 : sj - 1);
        if (kSyncEveryPhase) {  // every wavefront runs this the same number of times, so the barrier is safe here
            wait_vm<0>();
            __syncthreads();
        }
    };
    // Two or four blocks per tile: the last step already reads K of the next tile, so the synchronisation sits
    // before it.  One block per tile: it sits before the tile's only step, and consecutive tiles alternate the
    // roles of the two logit / probability register sets (`odd`).
    auto tile_steps = [&](int j, int sj, bool masked, bool odd) __attribute__((always_inline)) {  // sj = j % STAGES
        const int sn = sj + 1 == STAGES ? 0 : sj + 1;       // stage of tile j+1
        // first 32-key block of the tile, as a key position / 32 (only the masked form of a step looks at it)
        const int kb0 = KB * (((SPARSE && masked) || SPLIT) ? tile_of(j) : j);
        if (KB >= 2) {
#pragma unroll
            for (int i = 0; i < KB; i += 2) {
                if (kTwoVSets)
                    step(kb0 + i, sj, sj, masked, xA, xB, pB, vfB, pA, vfA);
                else
                    step(kb0 + i, sj, sj, masked, xA, xB, pB, vfA, pA, vfA);
                const bool last = i + 2 == KB;
                if (last) sync_and_stream(j, sj);
                if (kTwoVSets)
                    step(kb0 + i + 1, sj, last ? sn : sj, masked, xB, xA, pA, vfA, pB, vfB);
                else
                    step(kb0 + i + 1, sj, last ? sn : sj, masked, xB, xA, pA, vfA, pB, vfA);
            }
        } else {
            sync_and_stream(j, sj);
            if (!odd) {
                if (kTwoVSets)
                    step(kb0, sj, sn, masked, xA, xB, pB, vfB, pA, vfA);
                else
                    step(kb0, sj, sn, masked, xA, xB, pB, vfA, pA, vfA);
            } else {
                if (kTwoVSets)
                    step(kb0, sj, sn, masked, xB, xA, pA, vfA, pB, vfB);
                else
                    step(kb0, sj, sn, masked, xB, xA, pA, vfA, pB, vfA);
            }
        }
    };

    // Per wavefront the tiles fall into three consecutive ranges: fully visible, partly masked
    // (sequence tail or causal diagonal), and not visible at all (the wavefront then only keeps
    // streaming and synchronising for the others).
    const int n_vis_blocks = (N + 31) / 32;
    // (block-sparse: the list is ascending, so only its last 64 keys can hold the ragged end of the sequence)
    // (split keys: the same ranges, counted from the first tile of the split and cut to its length)
    const int n_unm_all = (CAUSAL ? min((q0w + off + 1) / 32, N / 32) : N / 32) / KB;
    const int n_act_all = ((CAUSAL ? min(n_vis_blocks, (q0w + QW - 1 + off) / 32 + 1) : n_vis_blocks) + KB - 1) / KB;
    const int n_unm_tiles = SPARSE ? max(n_tiles - KB64, 0) : max(0, min(n_unm_all - t0, n_tiles));
    const int n_act_tiles = SPARSE ? n_tiles : max(0, min(n_act_all - t0, n_tiles));
    int j = 0;
    // main loop: STAGES fully visible tiles per trip, so that every ring stage index is a constant
#pragma unroll 1
    for (; j + STAGES <= n_unm_tiles; j += STAGES) {
#pragma unroll
        for (int sj = 0; sj < STAGES; ++sj) tile_steps(j + sj, sj, false, (sj & 1) != 0);
    }
    // remaining visible tiles and the partly masked ones (masking a fully visible tile changes nothing)
    int sj = 0;  // j is a multiple of STAGES here (even, where that matters)
    bool owed_in_a = false;  // one block per tile only: the last step left its probabilities in pA, not pB
    if (KB >= 2) {
#pragma unroll 1
        for (; j < n_act_tiles; ++j) {
            tile_steps(j, sj, true, false);
            sj = sj + 1 == STAGES ? 0 : sj + 1;
        }
    } else {
#pragma unroll 1
        for (; j < n_act_tiles; j += 2) {
            tile_steps(j, sj, true, false);
            sj = sj + 1 == STAGES ? 0 : sj + 1;
            if (j + 1 < n_act_tiles) {
                tile_steps(j + 1, sj, true, true);
                sj = sj + 1 == STAGES ? 0 : sj + 1;
            } else {
                owed_in_a = true;
            }
        }
        if (j > n_act_tiles) j = n_act_tiles;
    }
    // the Attend still owed for the last block
    if (kWide) {
        // nothing is owed: every step ran its own Attend
    } else if (owed_in_a) {
        attend(vfA, pA);
    } else {
        attend(kTwoVSets ? vfB : vfA, pB);
    }
#pragma unroll 1
    for (; j < n_tiles; ++j) {
        sync_and_stream(j, sj);
        sj = sj + 1 == STAGES ? 0 : sj + 1;
    }

    // ---- split keys: leave the unnormalised partial result in the workspace.  Per (head, row block, split):
    // BR rows x DP accumulators, then BR reference maxima, then BR row sums, all fp32.
    if (SPLIT) {
        const int n_row_blocks = n_qtiles / prob.n_splits;  // per head
        float* part = prob.split_ws + ((size_t)(bh * n_row_blocks + qt) * prob.n_splits + split) * (size_t)(BR * (DP + 2));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float total = halves_sum(lsum[qb]);
            const int r_wg = wave * QW + 32 * qb + l32;  // row within the row block
            if (qt * BR + r_wg >= Nq) continue;          // rows past the end are never merged
            if (half == 0) {
                part[BR * DP + r_wg] = m[qb];
                part[BR * DP + BR + r_wg] = total;
            }
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    floatx4 w4 = {oacc[qb][db][4 * rq], oacc[qb][db][4 * rq + 1], oacc[qb][db][4 * rq + 2], oacc[qb][db][4 * rq + 3]};
                    *(floatx4*)(part + (size_t)r_wg * DP + 32 * db + 8 * rq + 4 * half) = w4;
                }
        }
        return;
    }
    // ---- epilogue: O = O_acc / l, rounded to bf16; a lane holds 4 consecutive head-dim elements per register quad
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float total = halves_sum(lsum[qb]);
        const float inv = (SPARSE && n_tiles == 0) ? 0.f : 1.0f / total;  // a row block with an empty list yields zeros
        const int row = q0w + 32 * qb + l32;
        if (row < Nq) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int dcol = 32 * db + 8 * rq + 4 * half;
                    if (32 * db + 8 * rq >= D) continue;  // padded head-dim columns
                    floatx2 w;
                    w[0] = __builtin_bit_cast(float, pack_bf16(oacc[qb][db][4 * rq] * inv, oacc[qb][db][4 * rq + 1] * inv));
                    w[1] = __builtin_bit_cast(float, pack_bf16(oacc[qb][db][4 * rq + 2] * inv, oacc[qb][db][4 * rq + 3] * inv));
                    *(floatx2*)(Oh + (size_t)row * D + dcol) = w;
                }
        }
    }
}

template <int D, int QB, int NW, int STAGES, bool CAUSAL, int MODE = kDense, int BCX = 0>
inline hipError_t launch_cfg(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, float scale,
                             hipStream_t stream) {
    constexpr int BR = 32 * QB * NW;
    // split keys: the kernel sees (row block, split) pairs where the other modes see row blocks
    const int n_qtiles = (prob.Nq + BR - 1) / BR * (MODE == kSplit ? prob.n_splits : 1);
    const int n_blocks = BH * n_qtiles;
    const int blocks_per_xcd = (n_blocks + 7) / 8;
    auto kern = fwd_bf16_kernel<D, QB, NW, STAGES, CAUSAL, MODE, BCX>;
    constexpr int lds = Bf16Cfg<D, STAGES, NW, BCX>::LDS_BYTES + (MODE == kSparse ? kMaxSparseTiles * (int)sizeof(int) : 0);
    static std::atomic<uint64_t> attr_done{0};  // one flag per kernel instantiation
    hipError_t e = allow_dynamic_lds((const void*)kern, lds, &attr_done);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(blocks_per_xcd * 8), dim3(64 * NW), lds, stream, (const bf16*)Q, (const bf16*)K,
                       (const bf16*)V, (bf16*)O, prob, n_qtiles, n_blocks, blocks_per_xcd, scale * kLog2e);
    return hipGetLastError();
}

// The two mask variants of one tile shape behind one call; defined here, instantiated explicitly by the
// translation units that own the shapes (declared in flat_launch.hpp).
template <int D, int QB, int NW, int STAGES, int BCX>
hipError_t launch_fwd_bf16_shape(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob, float scale,
                                 int causal, hipStream_t stream) {
    return causal ? launch_cfg<D, QB, NW, STAGES, true, kDense, BCX>(Q, K, V, O, BH, prob, scale, stream)
                  : launch_cfg<D, QB, NW, STAGES, false, kDense, BCX>(Q, K, V, O, BH, prob, scale, stream);
}

// Workgroups of this shape that fit one compute unit at a time (registers and LDS), as the runtime reports it.
template <int D, int QB, int NW, int STAGES, int BCX>
hipError_t fwd_bf16_shape_occupancy(int* workgroups_per_cu) {
    auto kern = fwd_bf16_kernel<D, QB, NW, STAGES, false, kDense, BCX>;
    constexpr int lds = Bf16Cfg<D, STAGES, NW, BCX>::LDS_BYTES;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(workgroups_per_cu, kern, 64 * NW, lds);
}

// Block-sparse launch of one tile shape (its row block is the shape's rows per workgroup).
template <int D, int QB, int NW, int STAGES>
hipError_t launch_fwd_bf16_sparse_shape(const void* Q, const void* K, const void* V, void* O, int BH, const Bf16Problem& prob,
                                        float scale, hipStream_t stream) {
    return launch_cfg<D, QB, NW, STAGES, false, kSparse>(Q, K, V, O, BH, prob, scale, stream);
}

#define FLAT_INSTANTIATE_BF16_SHAPE_BC(D, QB, NW, STAGES, BCX)                                                               \
    template hipError_t launch_fwd_bf16_shape<D, QB, NW, STAGES, BCX>(const void*, const void*, const void*, void*, int,    \
                                                                      const Bf16Problem&, float, int, hipStream_t);        \
    template hipError_t fwd_bf16_shape_occupancy<D, QB, NW, STAGES, BCX>(int*);
#define FLAT_INSTANTIATE_BF16_SHAPE(D, QB, NW, STAGES) FLAT_INSTANTIATE_BF16_SHAPE_BC(D, QB, NW, STAGES, 0)

}  // namespace flat
