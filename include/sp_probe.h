/*
 * sp_probe.h -- measurement helpers of the benchmark (libspprobe.so), NOT part of the
 * SpecPrefill path: two kernels that only READ a per-layer bf16 K cache [T, H_kv, d] and do no
 * arithmetic, so that a benchmark run can state, next to sp_score's own bandwidth, what plain
 * reading of the same bytes achieves on the same device in the same run.
 *
 * All pointers in h_layers[] are DEVICE pointers (the array itself is HOST memory); d_sink is a
 * device buffer of at least 256 bytes that the kernels may write a few words to (so the reads
 * cannot be optimised away).  Both calls only enqueue one kernel on hip_stream; they allocate
 * nothing and never synchronise.  Return 0 on success, -1 on a bad argument, -6 if the launch
 * was refused.
 */
#ifndef SP_PROBE_H
#define SP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SP_PROBE_API __attribute__((visibility("default")))
#define SP_PROBE_MAX_LAYERS 128

/* The trivial streaming kernel: `blocks` workgroups of 256 lanes sweep every layer front to back
 * together (grid-stride, 16 bytes per lane per step).  bytes_per_layer must be a multiple of 16. */
SP_PROBE_API int sp_probe_read(const void* const* h_layers, int32_t L, size_t bytes_per_layer, int32_t blocks,
                               void* d_sink, void* hip_stream);

/* The single-pass scorer's own access pattern without its arithmetic: one persistent workgroup
 * of eight waves per compute unit (256 of them), every wave pulling 32-key x d tiles of ONE KV
 * head (256-byte pieces, k_token_stride apart) through a two-slot LDS ring with direct, non-temporal
 * global->LDS loads, layer by layer, four teams of 64 workgroups on two KV heads each -- the order in
 * which the team kernel of sp_score walks a 32K-token, 8-KV-head, head-dim-128 cache.
 * Only that shape is accepted: T = 32768, H_kv = 8, d = 128 (else -1). */
SP_PROBE_API int sp_probe_tiled(const void* const* h_layers, int32_t L, int32_t T, int32_t H_kv, int32_t d,
                                int64_t k_token_stride, int64_t k_head_stride, void* d_sink, void* hip_stream);

/* The same read with the loads' default cache policy instead of the non-temporal one: the difference between
 * the two is what the policy of the scorer's key loads is worth on this device.  Same arguments and errors. */
SP_PROBE_API int sp_probe_tiled_default_policy(const void* const* h_layers, int32_t L, int32_t T, int32_t H_kv, int32_t d,
                                               int64_t k_token_stride, int64_t k_head_stride, void* d_sink,
                                               void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SP_PROBE_H */
