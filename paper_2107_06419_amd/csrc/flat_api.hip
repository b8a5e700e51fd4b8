// C ABI of the attention library (see include/flat_attn.h for the contract).
// Every argument check below runs before the first HIP call, so a host without a GPU can
// exercise the error paths.
#include "../../include/flat_attn.h"

#include <math.h>
#include <stdint.h>

#include "flat_launch.hpp"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

// Head dimensions: the fused bf16 kernel is built for five, the fp32 variant and the unfused baseline for two.
bool fused_bf16_head_dim(int d) { return d == 32 || d == 64 || d == 96 || d == 128 || d == 256; }
bool basic_head_dim(int d) { return d == 64 || d == 128; }

// Shape / pointer checks shared by all entry points.  `elem` = bytes per tensor element; `all_dims`: the entry
// point takes every head dimension of the fused bf16 kernel.
int check_common(const void* Q, const void* K, const void* V, const void* O, int B, int H, int N, int d, float scale,
                 int mask_kind, size_t elem, bool all_dims = false) {
    if (!Q || !K || !V || !O) return FLAT_ERR_NULL;
    if (B <= 0 || H <= 0 || N <= 0) return FLAT_ERR_SHAPE;
    if (!(all_dims ? fused_bf16_head_dim(d) : basic_head_dim(d))) return FLAT_ERR_UNSUPPORTED;
    if (mask_kind != FLAT_MASK_NONE && mask_kind != FLAT_MASK_CAUSAL) return FLAT_ERR_UNSUPPORTED;
    if (!(scale >= 0.0f) || isinf(scale)) return FLAT_ERR_UNSUPPORTED;  // also rejects NaN
    // B*H must fit the grid; B*H*N*d*elem and B*H*N*N*4 must fit 63 bits
    const long long BH = (long long)B * H;
    if (BH > 0x7fffffffLL / (((long long)N + 127) / 128)) return FLAT_ERR_SHAPE;
    const unsigned __int128 tensor = (unsigned __int128)BH * (unsigned)N * (unsigned)d * elem;
    const unsigned __int128 square = (unsigned __int128)BH * (unsigned)N * (unsigned)N * 4u;
    const unsigned __int128 lim = (unsigned __int128)1 << 62;
    if (tensor >= lim || square >= lim) return FLAT_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return FLAT_ERR_ALIGN;
    const size_t bytes = (size_t)tensor;
    if (overlaps(O, bytes, Q, bytes) || overlaps(O, bytes, K, bytes) || overlaps(O, bytes, V, bytes)) return FLAT_ERR_ALIAS;
    return FLAT_OK;
}

// The checks of check_common with separate lengths for the query side (Q, O) and the key side (K, V); on success
// *qbytes / *kbytes are the sizes of one query-side / key-side tensor.
int check_cross(const void* Q, const void* K, const void* V, const void* O, int B, int H, int Nq, int Nk, int d, float scale,
                int mask_kind, const int* kv_lens, size_t* qbytes_out, size_t* kbytes_out) {
    if (!Q || !K || !V || !O) return FLAT_ERR_NULL;
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0) return FLAT_ERR_SHAPE;
    if (!fused_bf16_head_dim(d)) return FLAT_ERR_UNSUPPORTED;
    if (mask_kind != FLAT_MASK_NONE && mask_kind != FLAT_MASK_CAUSAL) return FLAT_ERR_UNSUPPORTED;
    if (!(scale >= 0.0f) || isinf(scale)) return FLAT_ERR_UNSUPPORTED;
    if (mask_kind == FLAT_MASK_CAUSAL && Nk < Nq) return FLAT_ERR_UNSUPPORTED;  // some query would see no key
    const long long BH = (long long)B * H;
    if (BH > 0x7fffffffLL / (((long long)Nq + 127) / 128)) return FLAT_ERR_SHAPE;
    const unsigned long long per_head_q = (unsigned long long)Nq * (unsigned)d * 2u, per_head_k = (unsigned long long)Nk * (unsigned)d * 2u;
    if (per_head_q > 0xffffffffULL || per_head_k > 0xffffffffULL) return FLAT_ERR_SHAPE;  // 32-bit byte offsets within a head
    const unsigned __int128 qbytes128 = (unsigned __int128)BH * per_head_q, kbytes128 = (unsigned __int128)BH * per_head_k;
    const unsigned __int128 lim = (unsigned __int128)1 << 62;
    if (qbytes128 >= lim || kbytes128 >= lim) return FLAT_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return FLAT_ERR_ALIGN;
    if (kv_lens && (reinterpret_cast<uintptr_t>(kv_lens) & 3u)) return FLAT_ERR_ALIGN;
    const size_t qbytes = (size_t)qbytes128, kbytes = (size_t)kbytes128;
    if (overlaps(O, qbytes, Q, qbytes) || overlaps(O, qbytes, K, kbytes) || overlaps(O, qbytes, V, kbytes)) return FLAT_ERR_ALIAS;
    if (kv_lens && overlaps(O, qbytes, kv_lens, (size_t)B * sizeof(int))) return FLAT_ERR_ALIAS;
    *qbytes_out = qbytes;
    *kbytes_out = kbytes;
    return FLAT_OK;
}

}  // namespace

extern "C" {

int flat_attn_fwd(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                  int mask_kind, void* stream) {
    const int rc = check_common(Q, K, V, O, B, H, N, d, scale, mask_kind, 2, true);
    if (rc != FLAT_OK) return rc;
    if ((unsigned long long)N * (unsigned)d * 2u > 0xffffffffULL) return FLAT_ERR_SHAPE;  // the kernel addresses one head with 32-bit byte offsets
    const flat::Bf16Problem prob{N, N, 0, H, nullptr, nullptr, nullptr, 0};
    const hipError_t e = flat::launch_fwd_bf16(Q, K, V, O, B * H, prob, d, scale, mask_kind == FLAT_MASK_CAUSAL,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

int flat_attn_fwd_cross(const void* Q, const void* K, const void* V, void* O, int B, int H, int Nq, int Nk, int d, float scale,
                        int mask_kind, const int* kv_lens, void* stream) {
    size_t qbytes = 0, kbytes = 0;
    const int rc = check_cross(Q, K, V, O, B, H, Nq, Nk, d, scale, mask_kind, kv_lens, &qbytes, &kbytes);
    if (rc != FLAT_OK) return rc;
    const flat::Bf16Problem prob{Nq, Nk, mask_kind == FLAT_MASK_CAUSAL ? Nk - Nq : 0, H, kv_lens, nullptr, nullptr, 0};
    const hipError_t e = flat::launch_fwd_bf16(Q, K, V, O, B * H, prob, d, scale, mask_kind == FLAT_MASK_CAUSAL,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

int flat_attn_fwd_splitkv_splits(int B, int H, int Nq, int Nk, int d, int n_splits) {
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || (long long)B * H > 0x7fffffffLL) return FLAT_ERR_SHAPE;
    if (!fused_bf16_head_dim(d)) return FLAT_ERR_UNSUPPORTED;
    flat::SplitPlan plan;
    if (!flat::split_plan(B * H, Nq, Nk, d, n_splits, &plan)) return FLAT_ERR_SHAPE;
    return plan.n_splits;
}

size_t flat_attn_fwd_splitkv_workspace_bytes(int B, int H, int Nq, int Nk, int d, int n_splits) {
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || (long long)B * H > 0x7fffffffLL || !fused_bf16_head_dim(d)) return 0;
    flat::SplitPlan plan;
    return flat::split_plan(B * H, Nq, Nk, d, n_splits, &plan) ? plan.workspace_bytes : 0;
}

int flat_attn_fwd_splitkv(const void* Q, const void* K, const void* V, void* O, int B, int H, int Nq, int Nk, int d, float scale,
                          int mask_kind, const int* kv_lens, int n_splits, void* workspace, size_t workspace_bytes, void* stream) {
    size_t qbytes = 0, kbytes = 0;
    const int rc = check_cross(Q, K, V, O, B, H, Nq, Nk, d, scale, mask_kind, kv_lens, &qbytes, &kbytes);
    if (rc != FLAT_OK) return rc;
    if (!workspace) return FLAT_ERR_NULL;
    if (!aligned16(workspace)) return FLAT_ERR_ALIGN;
    flat::SplitPlan plan;
    if (!flat::split_plan(B * H, Nq, Nk, d, n_splits, &plan)) return FLAT_ERR_SHAPE;
    if (workspace_bytes < plan.workspace_bytes) return FLAT_ERR_WORKSPACE;
    if (overlaps(workspace, plan.workspace_bytes, Q, qbytes) || overlaps(workspace, plan.workspace_bytes, K, kbytes) ||
        overlaps(workspace, plan.workspace_bytes, V, kbytes) || overlaps(workspace, plan.workspace_bytes, O, qbytes))
        return FLAT_ERR_ALIAS;
    if (kv_lens && overlaps(workspace, plan.workspace_bytes, kv_lens, (size_t)B * sizeof(int))) return FLAT_ERR_ALIAS;
    flat::Bf16Problem prob{Nq, Nk, mask_kind == FLAT_MASK_CAUSAL ? Nk - Nq : 0, H, kv_lens, nullptr, nullptr, 0};
    prob.n_splits = plan.n_splits;
    prob.tiles_per_split = plan.tiles_per_split;
    prob.split_ws = static_cast<float*>(workspace);
    const hipError_t e = flat::launch_fwd_bf16_split(Q, K, V, O, B * H, prob, d, plan.rows_per_block, scale,
                                                     mask_kind == FLAT_MASK_CAUSAL, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

int flat_attn_fwd_splitkv_static(const void* Q, const void* K, const void* V, void* O, int B, int H, int Nq, int Nk, int d,
                                 float scale, int mask_kind, const int* kv_lens, int n_splits, void* stream) {
    size_t qbytes = 0, kbytes = 0;
    const int rc = check_cross(Q, K, V, O, B, H, Nq, Nk, d, scale, mask_kind, kv_lens, &qbytes, &kbytes);
    if (rc != FLAT_OK) return rc;
    flat::SplitPlan plan;
    if (!flat::split_plan(B * H, Nq, Nk, d, n_splits, &plan)) return FLAT_ERR_SHAPE;
    if (plan.workspace_bytes > flat::kSplitStaticScratchBytes) {
        if (n_splits > 0) return FLAT_ERR_WORKSPACE;  // the caller's choice does not fit the built-in scratch buffer
        // the library's choice: as many splits as the buffer holds
        const size_t per_split = plan.workspace_bytes / (size_t)plan.n_splits;
        const size_t fit = flat::kSplitStaticScratchBytes / per_split;
        if (fit < 1 || !flat::split_plan(B * H, Nq, Nk, d, (int)fit, &plan) || plan.workspace_bytes > flat::kSplitStaticScratchBytes)
            return FLAT_ERR_WORKSPACE;
    }
    flat::Bf16Problem prob{Nq, Nk, mask_kind == FLAT_MASK_CAUSAL ? Nk - Nq : 0, H, kv_lens, nullptr, nullptr, 0};
    prob.n_splits = plan.n_splits;
    prob.tiles_per_split = plan.tiles_per_split;
    const hipError_t e = flat::launch_fwd_bf16_split_static(Q, K, V, O, B * H, prob, d, plan.rows_per_block, scale,
                                                            mask_kind == FLAT_MASK_CAUSAL, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

int flat_attn_fwd_f32(const float* Q, const float* K, const float* V, float* O, int B, int H, int N, int d, float scale,
                      int mask_kind, void* stream) {
    const int rc = check_common(Q, K, V, O, B, H, N, d, scale, mask_kind, 4);
    if (rc != FLAT_OK) return rc;
    const hipError_t e = flat::launch_fwd_f32(Q, K, V, O, B * H, N, d, scale, mask_kind == FLAT_MASK_CAUSAL,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

size_t flat_attn_unfused_workspace_bytes(int B, int H, int N, int d, int dtype) {
    if (B <= 0 || H <= 0 || N <= 0 || (d != 64 && d != 128) || dtype != FLAT_DTYPE_BF16) return 0;
    const unsigned __int128 square = (unsigned __int128)B * (unsigned)H * (unsigned)N * (unsigned)N * 4u;
    if (square >= ((unsigned __int128)1 << 62)) return 0;
    return (size_t)square;
}

int flat_attn_unfused(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                      int mask_kind, void* workspace, size_t workspace_bytes, int dtype, void* stream) {
    if (dtype != FLAT_DTYPE_BF16) return FLAT_ERR_UNSUPPORTED;
    const int rc = check_common(Q, K, V, O, B, H, N, d, scale, mask_kind, 2);
    if (rc != FLAT_OK) return rc;
    if (!workspace) return FLAT_ERR_NULL;
    if (!aligned16(workspace)) return FLAT_ERR_ALIGN;
    if ((long long)B * H > 65535) return FLAT_ERR_SHAPE;                       // grid z/y limit of the GEMM launches
    if ((unsigned long long)B * H * N > 0x7fffffffULL) return FLAT_ERR_SHAPE;  // one workgroup per row in the softmax
    const size_t need = flat_attn_unfused_workspace_bytes(B, H, N, d, dtype);
    if (need == 0) return FLAT_ERR_SHAPE;
    if (workspace_bytes < need) return FLAT_ERR_WORKSPACE;
    const size_t tbytes = (size_t)B * H * N * d * 2;
    if (overlaps(workspace, need, Q, tbytes) || overlaps(workspace, need, K, tbytes) || overlaps(workspace, need, V, tbytes) ||
        overlaps(workspace, need, O, tbytes))
        return FLAT_ERR_ALIAS;
    const hipError_t e = flat::launch_unfused_bf16(Q, K, V, O, B * H, N, d, scale, mask_kind == FLAT_MASK_CAUSAL,
                                                   static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

int flat_attn_fwd_blocksparse(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                              const int* tile_offsets, const int* tile_ids, int n_tile_ids, void* stream) {
    const int rc = check_common(Q, K, V, O, B, H, N, d, scale, FLAT_MASK_NONE, 2, true);
    if (rc != FLAT_OK) return rc;
    if (!tile_offsets || !tile_ids) return FLAT_ERR_NULL;
    if (N > FLAT_SPARSE_BLOCK_KEYS * 2048) return FLAT_ERR_SHAPE;  // a row block's list must fit its LDS copy
    if (n_tile_ids < 0) return FLAT_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(tile_offsets) & 3u) || (reinterpret_cast<uintptr_t>(tile_ids) & 3u)) return FLAT_ERR_ALIGN;
    const size_t tbytes = (size_t)B * H * N * d * 2;
    const size_t n_row_blocks = (size_t)B * H * ((N + FLAT_SPARSE_BLOCK_ROWS - 1) / FLAT_SPARSE_BLOCK_ROWS);
    if (overlaps(O, tbytes, tile_offsets, (n_row_blocks + 1) * sizeof(int)) ||
        (n_tile_ids > 0 && overlaps(O, tbytes, tile_ids, (size_t)n_tile_ids * sizeof(int))))
        return FLAT_ERR_ALIAS;
    const flat::Bf16Problem prob{N, N, 0, H, nullptr, tile_offsets, tile_ids, n_tile_ids};
    const hipError_t e = flat::launch_fwd_bf16_sparse(Q, K, V, O, B * H, prob, d, scale, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

int flat_attn_tile_shape_count(int d) { return flat::tile_shape_count(d); }

int flat_attn_tile_shape_get(int d, int index, flat_tile_shape* out) {
    if (!out) return FLAT_ERR_NULL;
    if (!fused_bf16_head_dim(d)) return FLAT_ERR_UNSUPPORTED;
    flat::TileShape t;
    if (!flat::tile_shape(d, index, &t)) return FLAT_ERR_SHAPE;
    out->d = t.d;
    out->rows_per_workgroup = t.rows_per_workgroup;
    out->keys_per_tile = t.keys_per_tile;
    out->wavefronts = t.wavefronts;
    out->rows_per_wavefront = t.rows_per_wavefront;
    out->lds_stages = t.lds_stages;
    out->lds_bytes = t.lds_bytes;
    return FLAT_OK;
}

int flat_attn_tile_shape_occupancy(int d, int index) {
    if (!fused_bf16_head_dim(d)) return FLAT_ERR_UNSUPPORTED;
    if (index < 0 || index >= flat::tile_shape_count(d)) return FLAT_ERR_SHAPE;
    int n = 0;
    return flat::tile_shape_occupancy(d, index, &n) == hipSuccess ? n : FLAT_ERR_HIP;
}

int flat_attn_tile_shape_default(int B, int H, int Nq, int d, int mask_kind) {
    if (B <= 0 || H <= 0 || Nq <= 0 || (long long)B * H > 0x7fffffffLL) return FLAT_ERR_SHAPE;
    if (!fused_bf16_head_dim(d)) return FLAT_ERR_UNSUPPORTED;
    if (mask_kind != FLAT_MASK_NONE && mask_kind != FLAT_MASK_CAUSAL) return FLAT_ERR_UNSUPPORTED;
    return flat::default_tile_shape(B * H, Nq, d, mask_kind == FLAT_MASK_CAUSAL);
}

int flat_attn_fwd_tile(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                       int mask_kind, int tile_shape, void* stream) {
    const int rc = check_common(Q, K, V, O, B, H, N, d, scale, mask_kind, 2, true);
    if (rc != FLAT_OK) return rc;
    if ((unsigned long long)N * (unsigned)d * 2u > 0xffffffffULL) return FLAT_ERR_SHAPE;
    if (tile_shape < 0 || tile_shape >= flat::tile_shape_count(d)) return FLAT_ERR_SHAPE;
    const flat::Bf16Problem prob{N, N, 0, H, nullptr, nullptr, nullptr, 0};
    const hipError_t e = flat::launch_fwd_bf16_tile(Q, K, V, O, B * H, prob, d, scale, mask_kind == FLAT_MASK_CAUSAL, tile_shape,
                                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

const char* flat_attn_status_string(int status) {
    switch (status) {
        case FLAT_OK: return "FLAT_OK";
        case FLAT_ERR_NULL: return "FLAT_ERR_NULL: a required pointer is NULL";
        case FLAT_ERR_SHAPE: return "FLAT_ERR_SHAPE: B, H or N not positive, or the problem is too large to index";
        case FLAT_ERR_UNSUPPORTED:
            return "FLAT_ERR_UNSUPPORTED: d must be 32, 64, 96, 128 or 256 (64 or 128 for the fp32 and unfused paths), mask_kind 0 or 1, "
                   "scale finite and >= 0, Nk >= Nq with the causal mask";
        case FLAT_ERR_ALIGN: return "FLAT_ERR_ALIGN: pointers must be 16-byte aligned";
        case FLAT_ERR_WORKSPACE:
            return "FLAT_ERR_WORKSPACE: a workspace is smaller than the matching *_workspace_bytes() call says, or the request needs "
                   "more than the built-in scratch buffer of flat_attn_fwd_splitkv_static holds";
        case FLAT_ERR_HIP: return "FLAT_ERR_HIP: the HIP runtime refused a launch";
        case FLAT_ERR_ALIAS: return "FLAT_ERR_ALIAS: an output, workspace or sink overlaps another buffer";
        default: return "unknown flat_status";
    }
}

int flat_attn_version(void) { return 300; }

}  // extern "C"
