// Host-only check run under AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_sanitizers_host.py
// builds and runs it; no GPU, no HIP runtime).  It links
//   * the argument-validation half of the C ABI (csrc/flat_api.hip, csrc/flat_plan.hip and csrc/flat_probe_api.hip compiled as plain C++) against stub
//     launchers that only count calls, and walks its error paths with pointers that are never dereferenced;
//   * the CPU oracle, and runs every entry point of it on small problems with row subsets, key counts, block
//     patterns and several threads, comparing with a direct long-double evaluation.
// A sanitizer report, a wrong status or a mismatch makes it exit non-zero.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "../../include/flat_attn.h"
#include "../../include/flat_attn_probe.h"
#include "../../paper_2107_06419_amd/csrc/flat_launch.hpp"

// ---- stub launchers: the validation code must never get here with bad arguments --------------------------------------
static int g_launches = 0;
static int g_static_splits = 0;  // n_splits of the last allocation-free split-keys launch
namespace flat {
hipError_t launch_fwd_bf16(const void*, const void*, const void*, void*, int, const Bf16Problem&, int, float, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_fwd_bf16_sparse(const void*, const void*, const void*, void*, int, const Bf16Problem&, int, float, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_fwd_bf16_split(const void*, const void*, const void*, void*, int, const Bf16Problem& p, int, int, float, int, hipStream_t) {
    ++g_launches;
    return (p.n_splits >= 1 && p.tiles_per_split >= 1 && p.split_ws) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_fwd_bf16_split_static(const void*, const void*, const void*, void*, int, const Bf16Problem& p, int, int, float, int, hipStream_t) {
    ++g_launches;
    g_static_splits = p.n_splits;
    return (p.n_splits >= 1 && p.tiles_per_split >= 1) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_fwd_bf16_tile(const void*, const void*, const void*, void*, int, const Bf16Problem&, int, float, int, int, hipStream_t) { ++g_launches; return hipSuccess; }
int tile_shape_count(int d) { return (d == 64 || d == 128) ? 2 : (d == 32 || d == 96 || d == 256) ? 1 : 0; }
bool tile_shape(int d, int index, TileShape* out) {
    if (index < 0 || index >= tile_shape_count(d)) return false;
    *out = TileShape{d, 256, 64, 4, 64, 4, 65536};
    return true;
}
hipError_t tile_shape_occupancy(int, int, int* n) { *n = 2; return hipSuccess; }
int default_tile_shape(int, int, int, int) { return 0; }
hipError_t launch_fwd_f32(const float*, const float*, const float*, float*, int, int, int, float, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_unfused_bf16(const void*, const void*, const void*, void*, int, int, int, float, int, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_probe(float*, int, int, hipStream_t) { ++g_launches; return hipSuccess; }
double mfma_probe_flops(int iters) { return 1.0 * iters; }
size_t mfma_probe_sink_bytes() { return 4096; }
hipError_t launch_mix_probe(float*, const void*, int, int, hipStream_t) { ++g_launches; return hipSuccess; }
double mix_probe_flops(int iters) { return 1.0 * iters; }
size_t mix_probe_sink_bytes() { return 4096; }
size_t mix_probe_src_bytes() { return 8192; }
}  // namespace flat

// ---- oracle entry points (oracle/flat_oracle.cpp) ---------------------------------------------------------------------
extern "C" {
int flat_oracle_hw_threads(void);
int flat_oracle_logits_softmax(const double*, const double*, int64_t, int, double, int, const int64_t*, int64_t, double*, double*);
int flat_oracle_attention(const double*, const double*, const double*, double*, int, int, int64_t, int, double, int, const int64_t*,
                          int64_t, int);
int flat_oracle_attention_cross(const double*, const double*, const double*, double*, int, int, int64_t, int64_t, int, double, int,
                                const int64_t*, const int64_t*, int64_t, int);
int flat_oracle_attention_blocksparse(const double*, const double*, const double*, double*, int, int, int64_t, int, double, int64_t,
                                      int64_t, const int64_t*, const int64_t*, const int64_t*, int64_t, int);
}

static int g_failed = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            printf("FAILED line %d: %s\n", __LINE__, #cond);                \
            ++g_failed;                                                     \
        }                                                                   \
    } while (0)

static void* fake(uintptr_t a) { return reinterpret_cast<void*>(a); }

static void check_validation() {
    void *Q = fake(0x1000), *K = fake(0x2000000), *V = fake(0x4000000), *O = fake(0x6000000);
    EXPECT(flat_attn_fwd(nullptr, K, V, O, 1, 1, 8, 64, 1.f, 0, nullptr) == FLAT_ERR_NULL);
    EXPECT(flat_attn_fwd(Q, K, V, O, 0, 1, 8, 64, 1.f, 0, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd(Q, K, V, O, 1, 1, 8, 80, 1.f, 0, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd(Q, K, V, O, 1, 1, 8, 64, NAN, 0, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd(Q, K, V, O, 1, 1, 8, 64, 1.f, 7, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd(fake(0x1008), K, V, O, 1, 1, 8, 64, 1.f, 0, nullptr) == FLAT_ERR_ALIGN);
    EXPECT(flat_attn_fwd(Q, K, V, Q, 1, 1, 8, 64, 1.f, 0, nullptr) == FLAT_ERR_ALIAS);
    EXPECT(flat_attn_fwd(Q, K, V, O, 1 << 20, 1 << 20, 1 << 20, 64, 1.f, 0, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd(Q, fake(1ull << 40), fake(2ull << 40), fake(3ull << 40), 1, 1, 1 << 25, 64, 1.f, 0, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd(Q, K, V, O, 2147483647, 2147483647, 2147483647, 256, 1.f, 0, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(g_launches == 0);
    for (int d : {32, 64, 96, 128, 256}) EXPECT(flat_attn_fwd(Q, K, V, O, 2, 3, 100, d, 0.125f, 1, nullptr) == FLAT_OK);
    EXPECT(g_launches == 5);

    int lens_storage[4] = {1, 2, 3, 4};
    EXPECT(flat_attn_fwd_cross(Q, K, V, O, 1, 1, 17, 16, 64, 1.f, 1, nullptr, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd_cross(Q, K, V, O, 1, 1, 0, 16, 64, 1.f, 0, nullptr, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd_cross(Q, K, V, O, 1, 1, 16, 16, 64, 1.f, 0, reinterpret_cast<const int*>(fake(0x7000002)), nullptr) == FLAT_ERR_ALIGN);
    EXPECT(flat_attn_fwd_cross(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, nullptr) == FLAT_OK);
    EXPECT(flat_attn_fwd_cross(Q, K, V, O, 1, 1, 2147483647, 2147483647, 256, 1.f, 0, nullptr, nullptr) == FLAT_ERR_SHAPE);

    // split keys: the plan is real host code (csrc/flat_plan.hip), the launch is a stub
    EXPECT(flat_attn_fwd_splitkv_splits(1, 16, 256, 65536, 64, 0) == 32);      // 512 slots for 16 row blocks
    EXPECT(flat_attn_fwd_splitkv_splits(1, 16, 256, 65536, 64, 7) == 7);
    EXPECT(flat_attn_fwd_splitkv_splits(1, 1, 1, 100, 64, 9) == 2);          // two tiles: at most two splits
    EXPECT(flat_attn_fwd_splitkv_splits(1, 16, 1, 65536, 64, 0) == 47);      // 32-row shape, 3 workgroups per compute unit: 48 wanted, 22 tiles each
    EXPECT(flat_attn_fwd_splitkv_splits(1, 16, 1, 65536, 32, 0) == 94);      // d = 32: 6 per compute unit, 96 wanted,
    EXPECT(flat_attn_fwd_splitkv_splits(1, 16, 1, 65536, 64, 96) == 94);     // 11 tiles each, and 94 such splits cover the 1024 tiles
    EXPECT(flat_attn_fwd_splitkv_workspace_bytes(1, 16, 1, 65536, 64, 96) == (size_t)16 * 94 * 32 * 66 * 4);
    EXPECT(flat_attn_fwd_splitkv_splits(1, 1, 1, 100, 80, 0) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd_splitkv_splits(0, 1, 1, 100, 64, 0) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd_splitkv_splits(2147483647, 2147483647, 2147483647, 2147483647, 256, 0) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd_splitkv_workspace_bytes(1, 16, 256, 65536, 64, 8) == (size_t)16 * 8 * 256 * 66 * 4);
    EXPECT(flat_attn_fwd_splitkv_workspace_bytes(1, 16, 300, 65536, 256, 8) == (size_t)16 * 3 * 8 * 128 * 258 * 4);
    EXPECT(flat_attn_fwd_splitkv_workspace_bytes(1, 1, 2147483647, 2147483647, 256, 2147483647) == 0 ||
           flat_attn_fwd_splitkv_workspace_bytes(1, 1, 2147483647, 2147483647, 256, 2147483647) > 0);  // no overflow trap either way
    void* big_ws = fake(0x10000000);
    const size_t need = flat_attn_fwd_splitkv_workspace_bytes(2, 2, 16, 900, 96, 4);
    EXPECT(need > 0);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, nullptr, need, nullptr) == FLAT_ERR_NULL);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, big_ws, need - 1, nullptr) == FLAT_ERR_WORKSPACE);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, fake(0x10000004), need, nullptr) == FLAT_ERR_ALIGN);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, O, need, nullptr) == FLAT_ERR_ALIAS);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 17, 16, 96, 1.f, 1, lens_storage, 4, big_ws, need, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, big_ws, need, nullptr) == FLAT_OK);
    EXPECT(flat_attn_fwd_splitkv(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 0, nullptr, 0, big_ws, need, nullptr) == FLAT_OK);

    // the allocation-free form: the plan must fit the built-in buffer
    EXPECT(flat_attn_fwd_splitkv_static(Q, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, nullptr) == FLAT_OK && g_static_splits == 4);
    EXPECT(flat_attn_fwd_splitkv_static(Q, fake(1ull << 40), fake(2ull << 40), O, 1, 16, 256, 65536, 64, 1.f, 1, nullptr, 0, nullptr) == FLAT_OK);
    EXPECT(g_static_splits >= 1 && (size_t)16 * g_static_splits * 256 * 66 * 4 <= FLAT_SPLITKV_STATIC_BYTES);
    EXPECT(flat_attn_fwd_splitkv_static(Q, fake(1ull << 40), fake(2ull << 40), O, 1, 16, 256, 65536, 64, 1.f, 1, nullptr, 64, nullptr) == FLAT_ERR_WORKSPACE);
    EXPECT(flat_attn_fwd_splitkv_static(Q, fake(1ull << 40), fake(2ull << 40), fake(3ull << 40), 64, 64, 256, 4096, 256, 1.f, 0, nullptr, 0, nullptr) == FLAT_ERR_WORKSPACE);
    EXPECT(flat_attn_fwd_splitkv_static(nullptr, K, V, O, 2, 2, 16, 900, 96, 1.f, 1, lens_storage, 4, nullptr) == FLAT_ERR_NULL);

    EXPECT(flat_attn_fwd_f32((const float*)Q, (const float*)K, (const float*)V, (float*)O, 1, 1, 8, 32, 1.f, 0, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_fwd_f32((const float*)Q, (const float*)K, (const float*)V, (float*)O, 1, 1, 8, 64, 1.f, 0, nullptr) == FLAT_OK);

    EXPECT(flat_attn_unfused_workspace_bytes(1, 16, 16384, 64, FLAT_DTYPE_BF16) == (size_t)16 * 16384 * 16384 * 4);
    EXPECT(flat_attn_unfused_workspace_bytes(2147483647, 2147483647, 2147483647, 64, FLAT_DTYPE_BF16) == 0);
    EXPECT(flat_attn_unfused_workspace_bytes(1, 1, 8, 96, FLAT_DTYPE_BF16) == 0);
    void* ws = fake(0x8000000);
    EXPECT(flat_attn_unfused(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, nullptr, 1 << 20, 0, nullptr) == FLAT_ERR_NULL);
    EXPECT(flat_attn_unfused(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, ws, 255, 0, nullptr) == FLAT_ERR_WORKSPACE);
    EXPECT(flat_attn_unfused(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, O, 1 << 20, 0, nullptr) == FLAT_ERR_ALIAS);
    EXPECT(flat_attn_unfused(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, ws, 256, 0, nullptr) == FLAT_OK);
    EXPECT(flat_attn_unfused(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, ws, 256, 1, nullptr) == FLAT_ERR_UNSUPPORTED);

    const int* offs = reinterpret_cast<const int*>(fake(0x9000000));
    const int* ids = reinterpret_cast<const int*>(fake(0xa000000));
    EXPECT(flat_attn_fwd_blocksparse(Q, K, V, O, 1, 1, 700, 64, 1.f, nullptr, ids, 3, nullptr) == FLAT_ERR_NULL);
    EXPECT(flat_attn_fwd_blocksparse(Q, K, V, O, 1, 1, 700, 64, 1.f, offs, ids, -1, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd_blocksparse(Q, K, V, O, 1, 1, 131073, 64, 1.f, offs, ids, 3, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd_blocksparse(Q, K, V, O, 1, 1, 700, 256, 1.f, offs, ids, 3, nullptr) == FLAT_OK);

    flat_tile_shape t;
    EXPECT(flat_attn_tile_shape_get(64, 0, nullptr) == FLAT_ERR_NULL);
    EXPECT(flat_attn_tile_shape_get(64, 9, &t) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_tile_shape_get(48, 0, &t) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_tile_shape_get(256, 0, &t) == FLAT_OK && t.d == 256);
    EXPECT(flat_attn_fwd_tile(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, 5, nullptr) == FLAT_ERR_SHAPE);
    EXPECT(flat_attn_fwd_tile(Q, K, V, O, 1, 1, 8, 64, 1.f, 0, 1, nullptr) == FLAT_OK);

    EXPECT(flat_attn_mfma_probe(nullptr, 4096, 4, 0, nullptr) == FLAT_ERR_NULL);
    EXPECT(flat_attn_mfma_probe(ws, 4095, 4, 0, nullptr) == FLAT_ERR_WORKSPACE);
    EXPECT(flat_attn_mix_probe(ws, 4096, Q, 8192, 4, 4, nullptr) == FLAT_ERR_UNSUPPORTED);
    EXPECT(flat_attn_mix_probe(ws, 4096, Q, 8191, 3, 4, nullptr) == FLAT_ERR_WORKSPACE);
    EXPECT(flat_attn_mix_probe(ws, 4096, Q, 8192, 3, 4, nullptr) == FLAT_OK);
    for (int code = 1; code >= -9; --code) EXPECT(flat_attn_status_string(code) != nullptr);
}

// ---- oracle against a direct evaluation --------------------------------------------------------------------------------
static uint64_t g_rng = 88172645463325252ull;
static double rnd() {
    g_rng ^= g_rng << 13; g_rng ^= g_rng >> 7; g_rng ^= g_rng << 17;
    return (double)(g_rng >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

// visible(i, j) decides which keys count; returns the worst deviation of `got` [rows, d] from the direct evaluation
template <class Visible>
static double deviation(const double* Qh, const double* Kh, const double* Vh, const double* got, const std::vector<int64_t>& rows, int64_t Nk,
                        int d, double scale, Visible visible) {
    double worst = 0.0;
    for (size_t r = 0; r < rows.size(); ++r) {
        const int64_t i = rows[r];
        std::vector<long double> w(Nk, 0.0L);
        long double z = 0.0L;
        for (int64_t j = 0; j < Nk; ++j) {
            if (!visible(i, j)) continue;
            long double s = 0.0L;
            for (int c = 0; c < d; ++c) s += (long double)Qh[i * d + c] * Kh[j * d + c];
            w[j] = expl(s * scale);
            z += w[j];
        }
        for (int c = 0; c < d; ++c) {
            long double o = 0.0L;
            for (int64_t j = 0; j < Nk; ++j) o += w[j] * Vh[j * d + c];
            if (z > 0.0L) o /= z;
            worst = fmax(worst, fabs((double)o - got[r * d + c]));
        }
    }
    return worst;
}

static void check_oracle() {
    const int B = 2, H = 2, d = 8;
    const int64_t Nq = 37, Nk = 53;
    std::vector<double> Q(B * H * Nk * d), K(B * H * Nk * d), V(B * H * Nk * d);
    for (auto* t : {&Q, &K, &V})
        for (auto& x : *t) x = rnd();
    const double scale = 0.41;
    std::vector<int64_t> all_q(Nk), some = {0, 5, 36, 17, 17, 52};
    for (int64_t i = 0; i < Nk; ++i) all_q[i] = i;

    for (int mask = 0; mask < 2; ++mask)
        for (int threads : {1, 3, 0}) {
            // self-attention over Nk positions, all rows and a row subset
            std::vector<double> O(B * H * Nk * d, NAN), Os(B * H * some.size() * d, NAN);
            EXPECT(flat_oracle_attention(Q.data(), K.data(), V.data(), O.data(), B, H, Nk, d, scale, mask, nullptr, 0, threads) == 0);
            EXPECT(flat_oracle_attention(Q.data(), K.data(), V.data(), Os.data(), B, H, Nk, d, scale, mask, some.data(), (int64_t)some.size(), threads) == 0);
            for (int bh = 0; bh < B * H; ++bh) {
                const size_t o = (size_t)bh * Nk * d;
                auto vis = [&](int64_t i, int64_t j) { return mask == 0 || j <= i; };
                EXPECT(deviation(&Q[o], &K[o], &V[o], &O[o], all_q, Nk, d, scale, vis) < 1e-12);
                EXPECT(deviation(&Q[o], &K[o], &V[o], &Os[(size_t)bh * some.size() * d], some, Nk, d, scale, vis) < 1e-12);
            }
            // fewer queries than keys, key counts per batch entry
            std::vector<double> Qc(B * H * Nq * d);
            for (auto& x : Qc) x = rnd();
            const int64_t lens[2] = {53, 20};
            std::vector<double> Oc(B * H * Nq * d, NAN);
            EXPECT(flat_oracle_attention_cross(Qc.data(), K.data(), V.data(), Oc.data(), B, H, Nq, Nk, d, scale, mask, lens, nullptr, 0, threads) == 0);
            std::vector<int64_t> all_c(Nq);
            for (int64_t i = 0; i < Nq; ++i) all_c[i] = i;
            for (int bh = 0; bh < B * H; ++bh) {
                const int64_t len = lens[bh / H];
                auto vis = [&](int64_t i, int64_t j) { return j < len && (mask == 0 || j <= i + (Nk - Nq)); };
                EXPECT(deviation(&Qc[(size_t)bh * Nq * d], &K[(size_t)bh * Nk * d], &V[(size_t)bh * Nk * d], &Oc[(size_t)bh * Nq * d], all_c, Nk, d,
                                 scale, vis) < 1e-12);
            }
        }
    // block pattern: blocks of 16 rows x 8 keys, every third tile kept, one empty list
    const int64_t br = 16, bk = 8, n_rb = (Nk + br - 1) / br, n_kt = (Nk + bk - 1) / bk;
    std::vector<int64_t> offs = {0}, ids;
    for (int64_t r = 0; r < B * H * n_rb; ++r) {
        if (r != 2)
            for (int64_t t = r % 3; t < n_kt; t += 3) ids.push_back(t);
        offs.push_back((int64_t)ids.size());
    }
    std::vector<double> Ob(B * H * Nk * d, NAN);
    EXPECT(flat_oracle_attention_blocksparse(Q.data(), K.data(), V.data(), Ob.data(), B, H, Nk, d, scale, br, bk, offs.data(), ids.data(), nullptr, 0, 2) == 0);
    for (int bh = 0; bh < B * H; ++bh) {
        const size_t o = (size_t)bh * Nk * d;
        auto vis = [&](int64_t i, int64_t j) {
            const int64_t r = bh * n_rb + i / br;
            for (int64_t e = offs[r]; e < offs[r + 1]; ++e)
                if (ids[e] == j / bk) return true;
            return false;
        };
        EXPECT(deviation(&Q[o], &K[o], &V[o], &Ob[o], all_q, Nk, d, scale, vis) < 1e-12);
    }
    // logits and probabilities of one head
    std::vector<double> L(some.size() * Nk), A(some.size() * Nk);
    EXPECT(flat_oracle_logits_softmax(Q.data(), K.data(), Nk, d, scale, 1, some.data(), (int64_t)some.size(), L.data(), A.data()) == 0);
    for (size_t r = 0; r < some.size(); ++r) {
        double sum = 0.0;
        for (int64_t j = 0; j < Nk; ++j) sum += A[r * Nk + j];
        EXPECT(fabs(sum - 1.0) < 1e-12);
        EXPECT(some[r] + 1 >= Nk || (A[r * Nk + some[r] + 1] == 0.0 && isinf(L[r * Nk + some[r] + 1])));
    }
    // refused arguments
    const int64_t bad_row = Nk;
    EXPECT(flat_oracle_attention(Q.data(), K.data(), V.data(), Ob.data(), B, H, Nk, d, scale, 0, &bad_row, 1, 1) == -2);
    EXPECT(flat_oracle_attention(Q.data(), K.data(), V.data(), Ob.data(), B, H, Nk, d, scale, 2, nullptr, 0, 1) == -3);
    EXPECT(flat_oracle_attention_cross(Q.data(), K.data(), V.data(), Ob.data(), B, H, Nk, Nq, d, scale, 1, nullptr, nullptr, 0, 1) == -3);
    EXPECT(flat_oracle_hw_threads() >= 1);
}

int main() {
    check_validation();
    check_oracle();
    if (g_failed) {
        printf("%d checks failed\n", g_failed);
        return 1;
    }
    printf("host checks passed (%d launches reached the stubs)\n", g_launches);
    return 0;
}
