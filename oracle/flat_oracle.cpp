// CPU oracle for multi-head attention:  L = Q K^T * scale,  A = softmax_row(L),  O = A V.
//
// THIS IS TEST INFRASTRUCTURE, not part of the product.  Only the test-suite,
// the smoke check and the benchmark's cpu_baseline leg may call it.  It shares
// no code with the GPU library and knows nothing about tiles, LDS or MFMA.
//
// What it follows (paper section 2, "Computation operators"):
//   step 2  Logit:   a d-long dot product of every query vector with every key
//                    vector of the same (batch, head) -> [B,H,N,N]
//   step 3  Softmax: per query row, a reduction over the N scores of that row
//                    and a rescale of each score by the reduced value; the
//                    reduction runs along the key dimension (section 5.2)
//   step 4  Attend:  a weighted sum of the value vectors with those weights
//                    -> [B,H,N,d]
// The fused dataflow of the paper does not change what is computed (abstract:
// functionality is unaltered), so the oracle is the plain definition with the
// whole logit row materialised, in double precision, one operator after the
// other -- exactly the operator-by-operator baseline of Fig. "flat_dataflow"(a).
//
// Readings where the paper is silent:
//   * softmax(x)_j = exp(x_j - max x) / sum_j exp(x_j - max x)
//   * the logit is multiplied by `scale` before softmax
//   * mask_kind 1 (causal): key j contributes to query i iff j <= i; a masked
//     key has probability exactly 0 and is skipped
//
// Parity pins (tests/test_oracle_pins.py): brute force without max-subtraction
// on tiny shapes, closed forms (zero keys -> column mean of V; dominant key;
// constant V; causal row 0; N = 1; softmax([0, ln 2]) = [1/3, 2/3]), and
// invariants (rows sum to 1; key/value permutation; per-row logit shift;
// power-of-two rescaling; linearity in V; head independence), plus an
// independent float64 array-library evaluation.  No function here is unpinned.
//
// Layout: all tensors contiguous, [B,H,N,d] with d fastest.  Inputs are the
// already-rounded bf16/fp32 values widened exactly to double.

#include <atomic>
#include <cmath>
#include <cstdint>
#include <thread>
#include <vector>

namespace {

// step 2: logits of one query row against all visible keys of one head
void logit_row(const double* q_row, const double* K_head, int64_t n_keys, int d, double scale, double* L_row) {
    for (int64_t j = 0; j < n_keys; ++j) {
        const double* k_row = K_head + j * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += q_row[c] * k_row[c];
        L_row[j] = dot * scale;
    }
}

// step 3: softmax over the first n_keys entries of a row
void softmax_row(const double* L_row, int64_t n_keys, double* A_row) {
    double m = L_row[0];
    for (int64_t j = 1; j < n_keys; ++j) m = L_row[j] > m ? L_row[j] : m;
    double Z = 0.0;
    for (int64_t j = 0; j < n_keys; ++j) {
        A_row[j] = std::exp(L_row[j] - m);
        Z += A_row[j];
    }
    for (int64_t j = 0; j < n_keys; ++j) A_row[j] /= Z;
}

// step 4: weighted sum of value rows
void attend_row(const double* A_row, const double* V_head, int64_t n_keys, int d, double* O_row) {
    for (int c = 0; c < d; ++c) O_row[c] = 0.0;
    for (int64_t j = 0; j < n_keys; ++j) {
        const double a = A_row[j];
        const double* v_row = V_head + j * d;
        for (int c = 0; c < d; ++c) O_row[c] += a * v_row[c];
    }
}

inline int64_t visible_keys(int64_t i, int64_t N, int mask_kind) { return mask_kind == 1 ? i + 1 : N; }

}  // namespace

extern "C" {

// Number of hardware threads the host reports (what `threads <= 0` resolves to).
int flat_oracle_hw_threads(void) {
    unsigned n = std::thread::hardware_concurrency();
    return n == 0 ? 1 : (int)n;
}

// Logits and probabilities of ONE head for a set of query rows (for the pins).
//   Q, K: [N,d] doubles of that head.  rows: n_rows query indices.
//   L_out, A_out: [n_rows, N]; entries of masked keys are written as 0 in A_out and
//   as -infinity in L_out.  Either output may be null.
int flat_oracle_logits_softmax(const double* Q, const double* K, int64_t N, int d, double scale, int mask_kind,
                               const int64_t* rows, int64_t n_rows, double* L_out, double* A_out) {
    if (!Q || !K || !rows || N <= 0 || d <= 0 || n_rows < 0) return -1;
    if (mask_kind != 0 && mask_kind != 1) return -3;
    std::vector<double> L(N), A(N);
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t i = rows[r];
        if (i < 0 || i >= N) return -2;
        const int64_t nk = visible_keys(i, N, mask_kind);
        logit_row(Q + i * d, K, nk, d, scale, L.data());
        softmax_row(L.data(), nk, A.data());
        for (int64_t j = 0; j < N; ++j) {
            if (L_out) L_out[r * N + j] = j < nk ? L[j] : -INFINITY;
            if (A_out) A_out[r * N + j] = j < nk ? A[j] : 0.0;
        }
    }
    return 0;
}

// Attention output for a set of query rows of every (batch, head).
//   Q, K, V: [B,H,N,d] doubles.  rows: n_rows query indices in [0,N) used for every
//   head, or null for all rows (then n_rows is ignored and taken as N).
//   O: [B,H,n_rows,d] doubles.
//   threads: worker threads; <= 0 means all hardware threads.  Work is split over
//   (batch, head, block of rows); each row is computed independently, so the result
//   does not depend on the thread count.
// Returns 0, or a negative code for bad arguments.
int flat_oracle_attention(const double* Q, const double* K, const double* V, double* O, int B, int H, int64_t N, int d,
                          double scale, int mask_kind, const int64_t* rows, int64_t n_rows, int threads) {
    if (!Q || !K || !V || !O || B <= 0 || H <= 0 || N <= 0 || d <= 0) return -1;
    if (mask_kind != 0 && mask_kind != 1) return -3;
    if (!rows) n_rows = N;
    if (n_rows < 0) return -1;
    if (rows)
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= N) return -2;
    if (threads <= 0) threads = flat_oracle_hw_threads();

    const int64_t block = 16;  // rows per work item
    const int64_t blocks_per_head = (n_rows + block - 1) / block;
    const int64_t n_items = (int64_t)B * H * blocks_per_head;
    std::atomic<int64_t> next(0);

    auto worker = [&]() {
        std::vector<double> L(N), A(N);
        for (;;) {
            const int64_t item = next.fetch_add(1);
            if (item >= n_items) break;
            const int64_t bh = item / blocks_per_head;
            const int64_t r0 = (item % blocks_per_head) * block;
            const int64_t r1 = r0 + block < n_rows ? r0 + block : n_rows;
            const double* Qh = Q + bh * N * d;
            const double* Kh = K + bh * N * d;
            const double* Vh = V + bh * N * d;
            for (int64_t r = r0; r < r1; ++r) {
                const int64_t i = rows ? rows[r] : r;
                const int64_t nk = visible_keys(i, N, mask_kind);
                logit_row(Qh + i * d, Kh, nk, d, scale, L.data());
                softmax_row(L.data(), nk, A.data());
                attend_row(A.data(), Vh, nk, d, O + (bh * n_rows + r) * d);
            }
        }
    };

    if (threads == 1) {
        worker();
    } else {
        std::vector<std::thread> pool;
        for (int t = 0; t < threads; ++t) pool.emplace_back(worker);
        for (auto& th : pool) th.join();
    }
    return 0;
}

// Attention with Nq queries and Nk keys per head, for a set of query rows of every (batch, head).
// The operators are those above; only the set of keys a query sees changes.  Readings (the paper does not
// treat these cases; its workload list merely contains models that need them):
//   * Q: [B,H,Nq,d], K, V: [B,H,Nk,d] doubles, O: [B,H,n_rows,d].
//   * kv_lens (may be null): B counts; batch entry b uses its first kv_lens[b] keys (1 <= kv_lens[b] <= Nk), the
//     remaining rows of K and V are padding with probability exactly 0.
//   * mask_kind 1 (causal): the queries are the last Nq positions of the key sequence, so key j contributes to
//     query i iff j <= i + (Nk - Nq); needs Nk >= Nq.  With kv_lens the alignment still refers to Nk.
//   In every case the visible keys of a row are a prefix 0 .. n-1 of the key sequence, n >= 1.
// Pins (tests/test_oracle_cross_pins.py): equals flat_oracle_attention when Nq = Nk and kv_lens is null; the last Nq
// rows of causal self-attention over Nk positions; attention over K, V truncated to kv_lens[b]; brute force
// over explicit visibility tests on tiny shapes.
int flat_oracle_attention_cross(const double* Q, const double* K, const double* V, double* O, int B, int H, int64_t Nq,
                                int64_t Nk, int d, double scale, int mask_kind, const int64_t* kv_lens, const int64_t* rows,
                                int64_t n_rows, int threads) {
    if (!Q || !K || !V || !O || B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return -1;
    if (mask_kind != 0 && mask_kind != 1) return -3;
    if (mask_kind == 1 && Nk < Nq) return -3;
    if (kv_lens)
        for (int b = 0; b < B; ++b)
            if (kv_lens[b] < 1 || kv_lens[b] > Nk) return -2;
    if (!rows) n_rows = Nq;
    if (n_rows < 0) return -1;
    if (rows)
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= Nq) return -2;
    if (threads <= 0) threads = flat_oracle_hw_threads();

    const int64_t n_items = (int64_t)B * H;
    std::atomic<int64_t> next(0);
    auto worker = [&]() {
        std::vector<double> L(Nk), A(Nk);
        for (;;) {
            const int64_t bh = next.fetch_add(1);
            if (bh >= n_items) break;
            const int64_t len = kv_lens ? kv_lens[bh / H] : Nk;
            const double* Qh = Q + bh * Nq * d;
            const double* Kh = K + bh * Nk * d;
            const double* Vh = V + bh * Nk * d;
            for (int64_t r = 0; r < n_rows; ++r) {
                const int64_t i = rows ? rows[r] : r;
                int64_t n = len;
                if (mask_kind == 1) {
                    const int64_t last = i + (Nk - Nq);  // last key position this query may see
                    n = last + 1 < len ? last + 1 : len;
                }
                logit_row(Qh + i * d, Kh, n, d, scale, L.data());
                softmax_row(L.data(), n, A.data());
                attend_row(A.data(), Vh, n, d, O + (bh * n_rows + r) * d);
            }
        }
    };
    if (threads == 1) {
        worker();
    } else {
        std::vector<std::thread> pool;
        for (int t = 0; t < threads; ++t) pool.emplace_back(worker);
        for (auto& th : pool) th.join();
    }
    return 0;
}

// Block-sparse attention: query i of a head sees key j iff tile j / block_keys is listed for the row block
// i / block_rows of that head.  The operators are those above, applied to the visible keys only: they are
// gathered (in ascending order) into contiguous K and V rows first.  Reading: the paper prunes the N x N matrix
// randomly (section 8.2) without saying at what granularity; here the pattern is an input, at block granularity.
//   tile_offsets: B*H*ceil(N/block_rows) + 1 counts (CSR); row block r = bh*ceil(N/block_rows) + i/block_rows owns
//   tile_ids[tile_offsets[r] .. tile_offsets[r+1]), ids in [0, ceil(N/block_keys)), ascending and distinct.
//   A row block with an empty list gives a zero row.  rows / n_rows / threads as in flat_oracle_attention.
// Pins (tests/test_oracle_sparse_pins.py): every tile listed = flat_oracle_attention; the listed keys gathered by
// the test = flat_oracle_attention_cross over them; a prefix of tiles = truncated K, V; brute force over an explicit
// per-pair visibility test.
int flat_oracle_attention_blocksparse(const double* Q, const double* K, const double* V, double* O, int B, int H, int64_t N,
                                      int d, double scale, int64_t block_rows, int64_t block_keys,
                                      const int64_t* tile_offsets, const int64_t* tile_ids, const int64_t* rows,
                                      int64_t n_rows, int threads) {
    if (!Q || !K || !V || !O || !tile_offsets || !tile_ids || B <= 0 || H <= 0 || N <= 0 || d <= 0) return -1;
    if (block_rows <= 0 || block_keys <= 0) return -1;
    const int64_t n_rb = (N + block_rows - 1) / block_rows, n_kt = (N + block_keys - 1) / block_keys;
    const int64_t n_lists = (int64_t)B * H * n_rb;
    if (tile_offsets[0] != 0) return -2;
    for (int64_t r = 0; r < n_lists; ++r) {
        if (tile_offsets[r + 1] < tile_offsets[r]) return -2;
        for (int64_t e = tile_offsets[r]; e < tile_offsets[r + 1]; ++e) {
            if (tile_ids[e] < 0 || tile_ids[e] >= n_kt) return -2;
            if (e > tile_offsets[r] && tile_ids[e] <= tile_ids[e - 1]) return -2;
        }
    }
    if (!rows) n_rows = N;
    if (n_rows < 0) return -1;
    if (rows)
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= N) return -2;
    if (threads <= 0) threads = flat_oracle_hw_threads();

    const int64_t n_items = (int64_t)B * H;
    std::atomic<int64_t> next(0);
    auto worker = [&]() {
        std::vector<double> L(N), A(N), Kg((size_t)N * d), Vg((size_t)N * d);
        for (;;) {
            const int64_t bh = next.fetch_add(1);
            if (bh >= n_items) break;
            const double* Qh = Q + bh * N * d;
            const double* Kh = K + bh * N * d;
            const double* Vh = V + bh * N * d;
            int64_t gathered_for = -1, n = 0;  // row block whose keys Kg, Vg hold
            for (int64_t r = 0; r < n_rows; ++r) {
                const int64_t i = rows ? rows[r] : r;
                const int64_t rb = bh * n_rb + i / block_rows;
                if (rb != gathered_for) {
                    n = 0;
                    for (int64_t e = tile_offsets[rb]; e < tile_offsets[rb + 1]; ++e) {
                        const int64_t j0 = tile_ids[e] * block_keys;
                        const int64_t j1 = j0 + block_keys < N ? j0 + block_keys : N;
                        for (int64_t j = j0; j < j1; ++j, ++n)
                            for (int c = 0; c < d; ++c) {
                                Kg[n * d + c] = Kh[j * d + c];
                                Vg[n * d + c] = Vh[j * d + c];
                            }
                    }
                    gathered_for = rb;
                }
                double* O_row = O + (bh * n_rows + r) * d;
                if (n == 0) {
                    for (int c = 0; c < d; ++c) O_row[c] = 0.0;
                    continue;
                }
                logit_row(Qh + i * d, Kg.data(), n, d, scale, L.data());
                softmax_row(L.data(), n, A.data());
                attend_row(A.data(), Vg.data(), n, d, O_row);
            }
        }
    };
    if (threads == 1) {
        worker();
    } else {
        std::vector<std::thread> pool;
        for (int t = 0; t < threads; ++t) pool.emplace_back(worker);
        for (auto& th : pool) th.join();
    }
    return 0;
}

}  // extern "C"
