/*
 * apt_hybrid_bench.h - measurement tooling of libapt_hybrid.so, kept apart from the product
 * interface (apt_hybrid.h): a variant of the attention call that records HIP events around its
 * item kernel, and two calibration kernels of known traffic / known flops.  bench.py and the
 * profiling runs use them; a serving caller needs none of them.
 */
#ifndef APT_HYBRID_BENCH_H
#define APT_HYBRID_BENCH_H

#include "apt_hybrid.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The same step as apt_hybrid_decode_attn (Eq. 1-3 over both cache kinds); in addition
 * the HIP events ev_begin and ev_end (hipEvent_t handles created by the caller with
 * timing enabled; either may be NULL) are recorded on `stream` immediately before and
 * after the item kernel (with APT_HIDDEN_ABSORBED: before the first and after the last of the
 * kernels that run ahead of the merge), so that a caller can time it apart from the merge.
 */
int apt_hybrid_decode_attn_timed(const apt_shape* s, const void* plan_host, void* plan_dev,
                                 const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                                 const void* W_K, const void* W_V, const void* W_packed,
                                 const void* b_K, const void* b_V, const int32_t* block_tables,
                                 void* out, void* workspace, size_t workspace_bytes, void* stream,
                                 void* ev_begin, void* ev_end);

/*
 * Plain device-to-device copy kernel of `bytes` bytes (multiple of 16; device
 * pointers, 16-byte aligned).  Exists so that hardware traffic counters can be
 * calibrated against a kernel of known traffic (reads `bytes`, writes `bytes`).
 */
int apt_copy_bytes(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Register-only MFMA loop (no memory traffic): n_workgroups workgroups of 256 threads, each wave
 * holding a 128 x 128 fp32 accumulator tile and issuing per iteration
 *   variant 0 / 2:  16 independent 32x32x16 MFMAs, fp16 / bf16  (iters * 16 * 32768 flops per wave)
 *   variant 1 / 3:  64 independent 16x16x32 MFMAs, fp16 / bf16  (iters * 64 * 16384 flops per wave)
 * random_operands = 0: constant operands; != 0: operands of magnitude ~1 with random mantissas and
 * signs, which is what the multipliers see with real data (the sustained clock under the board's
 * power limit depends on it).  `out` (device) receives n_workgroups * 256 floats.  Exists to measure
 * the rate the matrix pipes sustain on the device at hand, as context for the MFMA roofline fraction.
 */
int apt_probe_mfma(void* out, int n_workgroups, int iters, int random_operands, int variant, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* APT_HYBRID_BENCH_H */
