/*
 * flat_attn_probe.h -- C ABI of the probe library (libflat_attn_probe.so) that accompanies the fused-attention
 * library for AMD MI355X (gfx950).  Nothing here computes attention: these are the measurement aids that put a
 * measured ceiling next to the published peak when the paper's utilisation metric (section 6, "Evaluation metrics":
 * ideal runtime = total computes / peak FLOPs) is reported.  Status codes, pointer and stream conventions are those
 * of flat_attn.h: device pointers, caller-owned buffers, enqueue-and-return, argument checks before any HIP call.
 */
#ifndef FLAT_ATTN_PROBE_H
#define FLAT_ATTN_PROBE_H

#include <stddef.h>

#include "flat_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid, not part of the attention path: a bf16 MFMA-only loop (the instruction both
 * contractions of the fused kernel run on) that shows what the matrix pipe sustains by itself on this
 * GPU.  The paper's utilisation metric (section 6, "Evaluation metrics": ideal runtime = total computes /
 * peak FLOPs) needs a peak; this gives the measured one next to the published one.
 *   sink: device, 16-byte aligned, at least flat_attn_mfma_probe_sink_bytes() bytes, overwritten.
 *   iters: rounds of four independent 32x32x16 MFMAs per wavefront (rounded up to a multiple of 4).
 *   random_operands: 0 = constant operands (1, 0); non-zero = pseudo-random operands in [-2, 2).
 * One launch performs flat_attn_mfma_probe_flops(iters) floating-point operations; the caller times it.
 */
size_t flat_attn_mfma_probe_sink_bytes(void);
double flat_attn_mfma_probe_flops(int iters);
int flat_attn_mfma_probe(void* sink, size_t sink_bytes, int iters, int random_operands, void* stream);

/*
 * Measurement aid, not part of the attention path: the instruction mix of one step of the fused d = 64 kernel
 * (16 MFMAs 32x32x16 bf16 for the Logit and Attend operators of section 2, and the 96 vector instructions of the
 * row softmax between them), looped on synthetic data.  It measures what that mix can sustain on this GPU when
 * nothing else is in the way, and what each part of the kernel's data movement takes from it:
 *   level 0: registers only;  1: + K and V operand fragments read from LDS every step;  2: + one workgroup
 *   barrier per 64-key tile;  3: + the K/V tiles streamed global -> LDS as the fused kernel streams them.
 *   sink: device, 16-byte aligned, at least flat_attn_mix_probe_sink_bytes() bytes, overwritten.
 *   src:  device, 16-byte aligned, at least flat_attn_mix_probe_src_bytes() bytes of finite bf16 values: every
 *         level takes its operands from it (the power an MFMA draws, and so the clock, depends on the data).
 *   iters: loop trips of 8 steps each, 1 .. 2^20.
 * One launch performs flat_attn_mix_probe_flops(iters) floating-point operations in its MFMAs; the caller times it.
 * Errors: FLAT_ERR_NULL, FLAT_ERR_UNSUPPORTED (level), FLAT_ERR_SHAPE (iters), FLAT_ERR_ALIGN, FLAT_ERR_WORKSPACE
 * (a buffer too small), FLAT_ERR_ALIAS, FLAT_ERR_HIP.
 */
size_t flat_attn_mix_probe_sink_bytes(void);
size_t flat_attn_mix_probe_src_bytes(void);
double flat_attn_mix_probe_flops(int iters);
int flat_attn_mix_probe(void* sink, size_t sink_bytes, const void* src, size_t src_bytes, int level, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLAT_ATTN_PROBE_H */
