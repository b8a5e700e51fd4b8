/*
 * flat_attn.h -- C ABI of the fused-attention library for AMD MI355X (gfx950).
 *
 * The library computes, for every (batch, head) of [B,H,N,d] tensors,
 *
 *     L = Q K^T * scale        (Logit operator,  paper section 2, step 2)
 *     A = softmax_row(L)       (row normalisation along the key dimension, step 3 / section 5.2)
 *     O = A V                  (Attend operator, step 4)
 *
 * in two ways:
 *   - flat_attn_fwd / flat_attn_fwd_f32: the fused, query-row-tiled dataflow of the paper's
 *     sections 4-5 (shared outer loop over batch, head and row blocks; Logit, softmax and
 *     Attend interleaved per block) -- the N x N intermediate never leaves the chip;
 *   - flat_attn_unfused: the operator-by-operator baseline of Fig. "flat_dataflow"(a), with L
 *     materialised in device memory (GEMM -> row softmax in place -> GEMM).
 *
 * Conventions common to all entry points
 *   - Q, K, V, O are DEVICE pointers to contiguous [B,H,N,d] arrays, d fastest; element type
 *     bf16 (flat_attn_fwd, flat_attn_unfused) or float (flat_attn_fwd_f32).  All four must
 *     be 16-byte aligned.  Q, K, V are only read.  O must not overlap Q, K or V.
 *   - Self-attention: queries and keys both number N.  Any N >= 1 is accepted.
 *   - Head dimension d: 32, 64, 96, 128 or 256 for the fused bf16 entry points (flat_attn_fwd, _fwd_cross,
 *     _fwd_blocksparse, _fwd_tile): the head sizes of the model families in the paper's workload list (section 6,
 *     "Workloads").  64 or 128 for flat_attn_fwd_f32 and flat_attn_unfused.  Anything else: FLAT_ERR_UNSUPPORTED.
 *   - scale multiplies the logits before softmax; it must be finite and >= 0.
 *   - mask_kind: FLAT_MASK_NONE, or FLAT_MASK_CAUSAL (key j contributes to query i iff j <= i;
 *     a masked key has probability exactly 0).
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return without synchronising.
 *   - The caller owns every buffer.  The library allocates and frees nothing and keeps no
 *     state between calls; calls from different threads are independent.
 *   - Return value: FLAT_OK, or a negative flat_status.  Argument checks run before any
 *     HIP call, so they can be exercised on a machine without a GPU.  FLAT_ERR_HIP reports a
 *     failed launch; no partial work is rolled back.
 *   - Results of the fused kernels are bitwise reproducible from run to run (fixed reduction
 *     order, no atomics).
 */
#ifndef FLAT_ATTN_H
#define FLAT_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FLAT_OK = 0,
    FLAT_ERR_NULL = -1,        /* a required pointer is NULL */
    FLAT_ERR_SHAPE = -2,       /* B, H or N is not positive, or B*H*N*N / B*H*N*d overflows */
    FLAT_ERR_UNSUPPORTED = -3, /* head dimension not built, unknown mask_kind or dtype, scale negative or not finite, causal with Nk < Nq */
    FLAT_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned */
    FLAT_ERR_WORKSPACE = -5,   /* a workspace is smaller than the matching *_workspace_bytes() call says */
    FLAT_ERR_HIP = -6,         /* the HIP runtime refused a launch */
    FLAT_ERR_ALIAS = -7        /* O overlaps Q, K or V */
} flat_status;

typedef enum { FLAT_MASK_NONE = 0, FLAT_MASK_CAUSAL = 1 } flat_mask_kind;

typedef enum { FLAT_DTYPE_BF16 = 0 } flat_dtype;

/*
 * Fused attention forward, bf16 in / bf16 out, fp32 accumulation (sections 4-5: fused
 * Logit-softmax-Attend at row granularity).  Probabilities are rounded to bf16 before the
 * second contraction; row maxima and row sums are kept in fp32.
 *   Q, K, V: device, const bf16 [B,H,N,d].   O: device, bf16 [B,H,N,d], fully overwritten.
 *   One head of one tensor (N*d*2 bytes) must stay below 4 GiB, else FLAT_ERR_SHAPE.
 */
int flat_attn_fwd(const void* Q, const void* K, const void* V, void* O,
                  int B, int H, int N, int d, float scale, int mask_kind, void* stream);

/*
 * The same kernel for queries and keys of different number, and for batches whose entries have different
 * key counts.  The paper's workload list (section 6, "Workloads") has TransformerXL and T5 in it, models that
 * attend over cached earlier segments or over another sequence, i.e. over more or other keys than queries; the
 * dataflow of section 5 tiles the query rows and streams the keys, so only the loop bounds change.
 *   Q: device, const bf16 [B,H,Nq,d].  K, V: device, const bf16 [B,H,Nk,d].  O: device, bf16 [B,H,Nq,d].
 *   mask_kind FLAT_MASK_CAUSAL: the queries are the LAST Nq positions of the key sequence, i.e. key j
 *     contributes to query i iff j <= i + (Nk - Nq); needs Nk >= Nq (else FLAT_ERR_UNSUPPORTED).
 *   kv_lens: NULL, or device pointer to B ints (4-byte aligned, only read): batch entry b uses its first
 *     kv_lens[b] keys, the rest of its Nk rows is padding with probability exactly 0.  Values are clamped to
 *     [1, Nk] on the device; with the causal mask the alignment above still refers to Nk.
 *   Nq = Nk, kv_lens = NULL gives exactly flat_attn_fwd.  One head of Q or K (N*d*2 bytes) must stay below 4 GiB.
 */
int flat_attn_fwd_cross(const void* Q, const void* K, const void* V, void* O,
                        int B, int H, int Nq, int Nk, int d, float scale, int mask_kind,
                        const int* kv_lens, void* stream);

/*
 * flat_attn_fwd_cross for FEW query rows over MANY keys (a segment of new positions attending over a long cache:
 * the TransformerXL case of the paper's workload list, section 6 "Workloads").  Section 5.3 weighs the row
 * granularity by how well it fills the compute array; with only a handful of row blocks no tile size fills it,
 * so here the key loop of every row block is divided over n_splits workgroups that leave partial results
 * (reference maximum, row sum, unnormalised output, all fp32) in `workspace`, and a second kernel merges them.
 * Same arguments, masks, key counts and tolerance as flat_attn_fwd_cross, plus
 *   n_splits: parts the key sequence is divided into, clamped to [1, number of key tiles]; <= 0 lets the library
 *     choose (one workgroup per compute-unit slot, at least 8 key tiles per split).
 *     flat_attn_fwd_splitkv_splits returns the number actually used (or a negative flat_status).
 *   workspace: device, 16-byte aligned, at least flat_attn_fwd_splitkv_workspace_bytes() bytes (same B, H, Nq,
 *     Nk, d, n_splits; 0 means the arguments are invalid), overwritten; it must not overlap any other buffer
 *     (FLAT_ERR_ALIAS).  FLAT_ERR_WORKSPACE if too small.
 * The result differs from flat_attn_fwd_cross in the last bits (different summation order), and is itself
 * bitwise reproducible for a given n_splits.  Two launches (partial pass, merge) are enqueued on `stream`.
 */
int flat_attn_fwd_splitkv_splits(int B, int H, int Nq, int Nk, int d, int n_splits);
size_t flat_attn_fwd_splitkv_workspace_bytes(int B, int H, int Nq, int Nk, int d, int n_splits);
int flat_attn_fwd_splitkv(const void* Q, const void* K, const void* V, void* O,
                          int B, int H, int Nq, int Nk, int d, float scale, int mask_kind,
                          const int* kv_lens, int n_splits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * flat_attn_fwd_splitkv for callers that cannot allocate device memory or hand over a workspace: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  The partial results go to a scratch
 * buffer of FLAT_SPLITKV_STATIC_BYTES that is part of the library's device image (every GPU the library runs on
 * holds its own copy until the process ends); the call allocates and frees nothing.
 *   Arguments and results as flat_attn_fwd_splitkv without workspace / workspace_bytes.
 *   n_splits > 0 whose partial results need more than FLAT_SPLITKV_STATIC_BYTES: FLAT_ERR_WORKSPACE (use fewer
 *     splits, or flat_attn_fwd_splitkv with a workspace of your own).  n_splits <= 0: the library's choice, reduced
 *     to what the buffer holds; FLAT_ERR_WORKSPACE if not even one split fits (B*H*ceil(Nq/rows per block) too large).
 *   With the same n_splits in effect the output is bit-identical to flat_attn_fwd_splitkv.
 *   All calls on one GPU share the one buffer: calls that may overlap in time on the same GPU (different streams,
 *   different threads) race and must be serialised by the caller.  Nothing in the buffer needs clearing between calls:
 *   every launch overwrites all it later reads.
 */
#define FLAT_SPLITKV_STATIC_BYTES (64u << 20)
int flat_attn_fwd_splitkv_static(const void* Q, const void* K, const void* V, void* O,
                                 int B, int H, int Nq, int Nk, int d, float scale, int mask_kind,
                                 const int* kv_lens, int n_splits, void* stream);

/*
 * Block-sparse variant.  The paper asks (section 8.2, compatibility with sparse-attention accelerators) whether
 * the Logit/Attend pair stays worth fusing when the N x N matrix is pruned, and prunes it randomly at 50 %.  On
 * this hardware pruning pays only at about the granularity the kernel works at, so the pattern is given in blocks of
 * FLAT_SPARSE_BLOCK_ROWS query rows x FLAT_SPARSE_BLOCK_KEYS keys: query i sees key j iff tile j / 64 is listed
 * for row block i / 256 of its (batch, head).  Unlisted tiles are neither loaded nor computed.
 *   Q, K, V, O: as flat_attn_fwd (self-attention, N <= 131072).  No causal form.
 *   tile_offsets: device, B*H*ceil(N/256) + 1 ints, only read: row block r = (b*H + h)*ceil(N/256) + i/256 owns
 *     tile_ids[tile_offsets[r] .. tile_offsets[r+1]).
 *   tile_ids: device, n_tile_ids ints in [0, ceil(N/64)), ascending and distinct within a row block.
 *   The lists live on the device and are not validated by the host: out-of-range offsets and ids are clamped
 *     (never a stray access), duplicate or unsorted ids give a wrong result.  A row block with an empty list
 *     produces zeros.  Listing every tile for every row block reproduces flat_attn_fwd bit for bit.
 */
#define FLAT_SPARSE_BLOCK_ROWS 256
#define FLAT_SPARSE_BLOCK_KEYS 64
int flat_attn_fwd_blocksparse(const void* Q, const void* K, const void* V, void* O,
                              int B, int H, int N, int d, float scale,
                              const int* tile_offsets, const int* tile_ids, int n_tile_ids, void* stream);

/*
 * Same dataflow in fp32 throughout (fp32 matrix instructions, fp32 probabilities).
 *   Q, K, V: device, const float [B,H,N,d].  O: device, float [B,H,N,d].
 */
int flat_attn_fwd_f32(const float* Q, const float* K, const float* V, float* O,
                      int B, int H, int N, int d, float scale, int mask_kind, void* stream);

/*
 * Unfused baseline (Fig. "flat_dataflow"(a); the off-chip traffic this path pays is the
 * O(B H N^2) intermediate of section 3.3).  Three launches on `stream`:
 *   1. L = Q K^T * scale written as fp32 [B,H,N,N] into `workspace`;
 *   2. each row of L replaced in place by its softmax (masked keys become 0);
 *   3. O = A V reading the fp32 probabilities back (rounded to bf16 as they are loaded).
 * workspace: device, 16-byte aligned, at least flat_attn_unfused_workspace_bytes() bytes;
 *   contents on return are the probabilities A.  dtype: FLAT_DTYPE_BF16.
 */
size_t flat_attn_unfused_workspace_bytes(int B, int H, int N, int d, int dtype);

int flat_attn_unfused(const void* Q, const void* K, const void* V, void* O,
                      int B, int H, int N, int d, float scale, int mask_kind,
                      void* workspace, size_t workspace_bytes, int dtype, void* stream);

/*
 * Tile shapes of the fused bf16 kernel.  The paper picks its tile sizes by a map-space exploration over a
 * cost model (section 6.1) and discusses what the row granularity trades (section 5.3: fewer query rows per
 * tile re-fetch the keys more often and fill the compute array less; more rows need more on-chip memory).
 * Here the exploration is done by measurement: the library is built with several shapes per head dimension,
 * flat_attn_fwd uses index 0, except where the 128-row shape (d = 64: index 7, d = 128: index 2, d = 32 and 96:
 * index 1) measures ahead: launches of few row blocks (at most 128 blocks of 256 query rows; 256 with the causal
 * mask at d = 32 and 64, 192 at d = 96 and 128: 1.3-1.5 times faster), d = 64 with the causal mask up to 4096
 * positions and 1024 row blocks, and d = 32 for short sequences.  flat_attn_fwd_tile runs any shape so that the
 * choice can be re-timed.
 *   flat_attn_tile_shape_count(d): number of shapes for head dimension d (0 if d is not one of 32, 64, 96, 128, 256).
 *   flat_attn_tile_shape_get: fills *out (HOST pointer) for 0 <= index < count; FLAT_ERR_SHAPE otherwise.
 *   flat_attn_tile_shape_occupancy: workgroups of that shape resident per compute unit on the current
 *     device (registers and LDS permitting), or a negative flat_status; the only one of the three that
 *     needs a GPU.
 *   flat_attn_tile_shape_default: the index flat_attn_fwd (N = Nq) and flat_attn_fwd_cross (Nq query rows) take for a
 *     problem, or a negative flat_status; host arithmetic only.
 *   flat_attn_fwd_tile: flat_attn_fwd with the shape chosen by the caller; same arguments, checks and
 *     result tolerance (different shapes sum in different orders, so results differ in the last bits).
 */
typedef struct {
    int d;                  /* head dimension the shape is built for */
    int rows_per_workgroup; /* query rows per workgroup (the paper's R of R-Gran) */
    int keys_per_tile;      /* keys staged in LDS per ring stage */
    int wavefronts;         /* wavefronts per workgroup */
    int rows_per_wavefront; /* query rows owned by one wavefront */
    int lds_stages;         /* depth of the K/V ring in LDS */
    int lds_bytes;          /* LDS bytes per workgroup */
} flat_tile_shape;

int flat_attn_tile_shape_count(int d);
int flat_attn_tile_shape_get(int d, int index, flat_tile_shape* out);
int flat_attn_tile_shape_occupancy(int d, int index);
int flat_attn_tile_shape_default(int B, int H, int Nq, int d, int mask_kind);
int flat_attn_fwd_tile(const void* Q, const void* K, const void* V, void* O,
                       int B, int H, int N, int d, float scale, int mask_kind, int tile_shape, void* stream);

/* Human-readable name of a flat_status value (static storage, never NULL). */
const char* flat_attn_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int flat_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLAT_ATTN_H */
