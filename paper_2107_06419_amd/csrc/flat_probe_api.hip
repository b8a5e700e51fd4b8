// C ABI of the probe library (include/flat_attn_probe.h): measurement aids only, built into a library of their
// own (libflat_attn_probe.so) so that the attention library carries nothing but attention.  Argument checks run
// before any HIP call, as in the attention library.
#include "../../include/flat_attn_probe.h"

#include <stdint.h>

#include "flat_launch.hpp"

namespace {
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}
}  // namespace

extern "C" {

size_t flat_attn_mfma_probe_sink_bytes(void) { return flat::mfma_probe_sink_bytes(); }

double flat_attn_mfma_probe_flops(int iters) { return iters > 0 ? flat::mfma_probe_flops(iters) : 0.0; }

int flat_attn_mfma_probe(void* sink, size_t sink_bytes, int iters, int random_operands, void* stream) {
    if (!sink) return FLAT_ERR_NULL;
    if (iters <= 0 || iters > (1 << 24)) return FLAT_ERR_SHAPE;
    if (!aligned16(sink)) return FLAT_ERR_ALIGN;
    if (sink_bytes < flat::mfma_probe_sink_bytes()) return FLAT_ERR_WORKSPACE;
    const hipError_t e = flat::launch_mfma_probe(static_cast<float*>(sink), iters, random_operands != 0,
                                                 static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

size_t flat_attn_mix_probe_sink_bytes(void) { return flat::mix_probe_sink_bytes(); }

size_t flat_attn_mix_probe_src_bytes(void) { return flat::mix_probe_src_bytes(); }

double flat_attn_mix_probe_flops(int iters) { return iters > 0 ? flat::mix_probe_flops(iters) : 0.0; }

int flat_attn_mix_probe(void* sink, size_t sink_bytes, const void* src, size_t src_bytes, int level, int iters, void* stream) {
    if (!sink) return FLAT_ERR_NULL;
    if (level < 0 || level > 3) return FLAT_ERR_UNSUPPORTED;
    if (iters <= 0 || iters > (1 << 20)) return FLAT_ERR_SHAPE;
    if (!aligned16(sink)) return FLAT_ERR_ALIGN;
    if (sink_bytes < flat::mix_probe_sink_bytes()) return FLAT_ERR_WORKSPACE;
    if (!src) return FLAT_ERR_NULL;
    if (!aligned16(src)) return FLAT_ERR_ALIGN;
    if (src_bytes < flat::mix_probe_src_bytes()) return FLAT_ERR_WORKSPACE;
    if (overlaps(sink, sink_bytes, src, src_bytes)) return FLAT_ERR_ALIAS;
    const hipError_t e = flat::launch_mix_probe(static_cast<float*>(sink), src, level, iters, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLAT_OK : FLAT_ERR_HIP;
}

}  // extern "C"
