/*
 * specprefill.h -- C ABI of the SpecPrefill token-importance path for AMD MI355X (gfx950).
 *
 * Method: "Speculative Prefill" (arXiv 2502.02789).  A draft model's stored queries
 * (the last prompt token and/or N look-ahead tokens) score every prompt token by
 * attention against the draft's K cache (Sec. 3.2 equation); scores are aggregated
 * over heads, layers and queries (Sec. 3.2.2), smoothed by 1-D average pooling and
 * cut to the top-k contiguous chunks (Sec. 3.2.3); kept tokens travel to the base
 * model with their ORIGINAL position ids (Sec. 3.2.4).  Algorithm 1 names these
 * steps compute_attention_score, aggregate_attention_score,
 * chunk_select_from_smoothed_attention and restore_pos_ids.
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers owned by the caller; everything else
 *     (the structs themselves, k_layers[], h_* arrays) is HOST memory.
 *   - The library allocates and frees no device memory; scratch space is the
 *     caller's workspace (size from the *_workspace_bytes query).  It never
 *     synchronises the stream: all work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream).
 *   - Return value: SP_OK (0) or a negative sp_status.  On an argument error
 *     nothing is launched and no output is written.
 *   - Sequence b owns prompt tokens [cu_seqlens[b], cu_seqlens[b+1]) of the flat
 *     token axis of length T = cu_seqlens[B]; empty sequences are allowed.
 *   - NaN/Inf in Q or K, and token ids outside [0, V), are precondition violations
 *     (undefined values, no fault for NaN/Inf; ids are NOT range-checked on device).
 *   - Calls that share a workspace must not overlap in time.
 *   - One-time set-up per device (kernel attributes, occupancy queries, the address of the
 *     library's static scratch) happens inside the first call made on that device, under a
 *     lock; that first call must not be made while the stream is being captured into a graph.
 */
#ifndef SPECPREFILL_H
#define SPECPREFILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SP_API __attribute__((visibility("default")))

typedef enum {
  SP_OK = 0,
  SP_EINVAL = -1,       /* a size, rate or enum is out of range                  */
  SP_ENULL = -2,        /* a required pointer is NULL                            */
  SP_EALIGN = -3,       /* a pointer or stride breaks the 16-byte alignment rule */
  SP_EWORKSPACE = -4,   /* workspace missing or smaller than *_workspace_bytes   */
  SP_EUNSUPPORTED = -5, /* valid request this build has no kernel for            */
  SP_ELAUNCH = -6,      /* the HIP runtime refused a launch                      */
  SP_ETIMEOUT = -7      /* a bounded device-side wait expired (see sp_score_check) */
} sp_status;

/* How per-layer values are combined (Sec. 3.2.2).  The paper takes the maximum over
 * heads AND layers; the alternative keeps the maximum over heads but averages layers. */
typedef enum { SP_LAYER_MAX = 0, SP_LAYER_MEAN = 1 } sp_layer_reduce;

/* How the K cache stores its elements.  SP_K_FP8_E4M3: one byte per element, OCP 8-bit floating point,
 * format E4M3 (1 sign, 4 exponent, 3 mantissa bits, bias 7, subnormals, no infinities, S.1111.111 = NaN,
 * largest finite value 448), and the key the paper's Sec. 3.2 equation sees is
 *     K_l[i, g, t] = d_k_scale[l * H_kv + g] * decode(byte)
 * (one fp32 scale per layer and KV head, as an engine with an 8-bit KV cache keeps them).  Every E4M3
 * value is a bf16 value, so the products with the bf16 queries are formed exactly as for a bf16 cache and
 * accumulated in fp32; the scale joins the logit scale.  Scores therefore meet the same tolerance against
 * the definition evaluated on the decoded keys as a bf16 cache does.  NaN codes are a precondition
 * violation like NaN in a bf16 cache. */
typedef enum { SP_K_BF16 = 0, SP_K_FP8_E4M3 = 1 } sp_k_dtype;

#define SP_MAX_LAYERS 128
#define SP_MAX_QUERIES 16

/* sp_score_args.flags */
#define SP_SCORE_EXCLUSIVE_DEVICE 1u /* The caller promises that nothing else runs on the GPU while
                                        sp_score runs (no other stream, no other process).  Only
                                        then may sp_score use its single-pass kernels, which read
                                        the K cache once but exchange softmax row statistics
                                        between workgroups that must all be resident together.
                                        Without the flag sp_score uses kernels that never wait for
                                        another workgroup (two passes over K or kept logits).
                                        If the promise is broken a bounded wait can expire; the
                                        affected scores are then NaN (see sp_score_check and
                                        sp_pool_select), never silently wrong. */
#define SP_SCORE_WORKSPACE_KEPT 2u   /* The caller promises that args->d_workspace was last written by
                                        an sp_score call with the same shape fields (B, T, N, L, H,
                                        H_kv, d, layer_reduce, paging) and SP_SCORE_EXCLUSIVE_DEVICE
                                        set that completed without SP_ETIMEOUT, and has not been
                                        touched since (not by sp_score_general or
                                        sp_score_pool_select either: they write it too).  A single-pass
                                        call leaves its exchange area ready for the next call, so
                                        the kernel that re-initialises it can then be skipped (a
                                        few microseconds per call in a serving loop that keeps its
                                        workspace).  The first call on a workspace, and the call
                                        after a time-out, must not set it.  Other kernels ignore
                                        it.  With a broken promise waits expire or scores are
                                        wrong. */

/* ---------------------------------------------------------------------------
 * sp_score: compute_attention_score + aggregate_attention_score (Algorithm 1),
 * i.e. for every prompt token i of sequence b
 *     s[l,h,n,i] = scale * <Q[l,b,n,h,:], K_l[i, h / (H/H_kv), :]>
 *     a[l,h,n,i] = exp(s[l,h,n,i] - logsumexp_{i' in sequence b} s[l,h,n,i'])   (Sec. 3.2 eq.)
 *     SP_LAYER_MAX : score[i] = mean_{n < n_valid[b]} max_{l,h} a               (Sec. 3.2.2)
 *     SP_LAYER_MEAN: score[i] = mean_{n < n_valid[b]} mean_l max_h a
 * The softmax runs over the prompt keys of the token's own sequence only.
 * Q and K are taken as stored by the draft model (already position-encoded) unless
 * rope_theta > 0 asks for the rotary encoding to be applied here.
 * --------------------------------------------------------------------------- */
typedef struct {
  int32_t B;                 /* sequences, >= 1                                           */
  int32_t N;                 /* query rows per sequence, 1..SP_MAX_QUERIES                */
  int32_t L;                 /* layers, 1..SP_MAX_LAYERS                                  */
  int32_t H;                 /* query heads                                               */
  int32_t H_kv;              /* key heads; H % H_kv == 0, H / H_kv <= 8                   */
  int32_t d;                 /* head dim: 64 or 128                                       */
  int64_t T;                 /* total prompt tokens = cu_seqlens[B], < 2^31               */
  const void* d_q;           /* bf16 [L, B, N, H, d] contiguous, 16-byte aligned          */
  const void* const* k_layers; /* HOST array of L device pointers; layer l holds bf16
                                  K_l[i, g, t] at element offset i*k_token_stride +
                                  g*k_head_stride + t (t contiguous); 16-byte aligned     */
  int64_t k_token_stride;    /* elements, multiple of 8                                   */
  int64_t k_head_stride;     /* elements, multiple of 8                                   */
  const int32_t* d_cu_seqlens; /* int32 [B+1], cu[0] = 0, non-decreasing, cu[B] = T       */
  const int32_t* d_n_valid;  /* int32 [B] with 1 <= n_valid[b] <= N, or NULL (= N): only the
                                first n_valid[b] query rows count (EOS validity, Sec. 3.3)  */
  float scale;               /* logit scale; the model's own attention uses 1/sqrt(d)     */
  int32_t layer_reduce;      /* sp_layer_reduce                                           */
  float rope_theta;          /* 0: Q and K are stored already position-encoded (what a serving
                                cache holds; the fast path).  > 0: Q and K are stored
                                un-rotated and are rotated here, rotate-half pairing
                                (t, t + d/2), angle pos * theta^(-2t/d): key i of a sequence
                                at position i, query row n of sequence b at d_q_pos[b*N+n];
                                cosine/sine in fp32 (angle formed in fp64), the two products
                                and their sum separate fp32 operations, rotated values
                                rounded to bf16 (nearest even): bit for bit what a cache
                                rotated that way would hold, then everything as for
                                rope_theta = 0.  Runs the two-pass kernels (the keys are
                                turned in registers on their way to the matrix cores; the
                                single-pass kernels take rotated caches only) and needs the
                                larger workspace the size query reports.                    */
  const int32_t* d_q_pos;    /* int32 [B, N] query positions if rope_theta > 0, else NULL  */
  float* d_scores;           /* out fp32 [T]                                              */
  float* d_lse;              /* out fp32 [L, B, N, H] row log-sum-exp, or NULL            */
  void* d_workspace;         /* device scratch, 256-byte aligned                          */
  size_t workspace_bytes;
  /* Paged K cache (Sec. 3.3: the draft's keys are fetched through the serving engine's slot
   * mapping).  d_block_table == NULL: token i of sequence b is row cu_seqlens[b] + i of every
   * layer, as described at k_layers.  Otherwise every layer is a pool of pages and token i of
   * sequence b is row (i % page_size) of page d_block_table[b*blocks_per_seq + i/page_size]:
   * element offset page*k_page_stride + (i % page_size)*k_token_stride + g*k_head_stride + t.
   * The table must cover every sequence and hold valid page numbers (not checked: a wrong
   * entry reads outside the pool).  Scores are still indexed by cu_seqlens[b] + i. */
  const int32_t* d_block_table; /* int32 [B, blocks_per_seq] page numbers, or NULL             */
  int32_t page_size;         /* tokens per page: a power of two >= 8 (ignored if not paged)   */
  int32_t blocks_per_seq;    /* row length of the table, >= 1                                 */
  int64_t k_page_stride;     /* elements, multiple of 8                                       */
  uint32_t flags;            /* SP_SCORE_* bits, 0 = none                                     */
  int32_t max_seqlen;        /* 0: nothing stated.  > 0: the caller's promise that no sequence has more
                                prompt tokens than this (the lengths themselves live on the device, where
                                the host side of sp_score cannot see them; with B == 1 the length is T and
                                nothing need be stated).  With it sp_score can take, for
                                batches of prompts of up to 8192 keys (4096 with 5..8 query rows per KV
                                head) whose KV heads carry at most eight query rows, a kernel that reads
                                the K cache once and keeps all logits of a sequence on chip.  A sequence
                                longer than promised is not scored: all of its scores (and its rows of
                                d_lse) are NaN, which sp_pool_select reports in band; never silently
                                wrong.  Nothing else depends on the promise.                            */
  int32_t k_dtype;           /* sp_k_dtype, 0 = bf16.  With SP_K_FP8_E4M3 the layers hold bytes: the strides
                                (token, head, page) still count ELEMENTS and must then be multiples of 16;
                                rope_theta must be 0 (SP_EUNSUPPORTED otherwise), and sp_score runs its
                                two-pass kernels (half the bytes per pass).                              */
  const float* d_k_scale;    /* fp32 [L, H_kv] scales of an SP_K_FP8_E4M3 cache, or NULL (all 1)          */
} sp_score_args;

/* Bytes of workspace sp_score needs for these shapes (pointers are not read).
 * Returns 0 if the shape fields are invalid (flags and max_seqlen are shape fields here: they
 * decide which kernels run).  The size grows with T: per-tile row statistics
 * (L*N*H*8 bytes per 64 tokens) always, plus, for batches whose KV heads have at most eight
 * query rows (H/H_kv * N <= 8), 16 or 32 bytes per token, layer and KV head of logits kept
 * between the two passes (0.7 GB for 167K tokens of a 32-layer, 8-KV-head model). */
SP_API size_t sp_score_workspace_bytes(const sp_score_args* args);

/* Enqueue the scoring on hip_stream.  Errors: SP_ENULL, SP_EINVAL (shape limits above),
 * SP_EALIGN, SP_EWORKSPACE, SP_ELAUNCH. */
SP_API sp_status sp_score(const sp_score_args* args, void* hip_stream);

/* Same contract and results as sp_score, but always runs the general two-pass kernels
 * (sp_score picks a faster single-pass kernel when the shape allows).  Meant for
 * cross-checking the two implementations of the Sec. 3.2 / 3.2.2 arithmetic. */
SP_API sp_status sp_score_general(const sp_score_args* args, void* hip_stream);

/* Optional post-check of the most recent sp_score call that used args->d_workspace.  The
 * single-pass kernels (SP_SCORE_EXCLUSIVE_DEVICE) exchange row statistics between workgroups
 * that must all be resident on the device at once.  Their waits are bounded: a workgroup whose
 * wait expired writes NaN for all of its tokens' scores and records the event in the workspace
 * instead of hanging.  This call SYNCHRONISES hip_stream (the only entry point that does), reads
 * that record and returns SP_ETIMEOUT if a wait expired, SP_OK otherwise.  Recovery: call
 * sp_score again without the flag (or sp_score_general). */
SP_API sp_status sp_score_check(const sp_score_args* args, void* hip_stream);

/* Upper bound on the polls one wave may spend waiting for other workgroups during one sp_score
 * call (process-wide, applies to later calls; default 65536, about 0.1 s).  0 makes every wait
 * give up at once, which turns every score of a single-pass call into NaN: that is how the
 * failure path is exercised without ever making a kernel hang.  Returns the previous value;
 * a negative argument only queries. */
SP_API int32_t sp_set_wait_budget(int32_t polls);

/* ---------------------------------------------------------------------------
 * sp_pool_select: chunk_select_from_smoothed_attention (Algorithm 1, Sec. 3.2.3).
 * Per sequence (length M): average-pool the scores with an odd window clipped to the
 * sequence (divisor = in-range count); split into ceil(M/chunk) contiguous chunks and
 * take each chunk's mean over its actual length; keep the
 * k = clamp(ceil(keep_rate * n_chunks - 1e-9), 1, n_chunks) best chunks (keep rate =
 * ratio of chunks, Sec. 4.1), equal scores resolved to the lower chunk index; emit the
 * tokens of the kept chunks in ascending order.  Arithmetic is fp64 on the fp32 input.
 * A NaN among the scores (sp_score writes NaN where a device-side wait expired) is reported
 * in band: cu_keep[0] = 0, cu_keep[1..B] = -1, and no kept index is written, so that neither
 * this call nor sp_gather after it hands on a keep set made from invalid scores.
 * --------------------------------------------------------------------------- */
typedef struct {
  int32_t B;
  int64_t T;
  const int32_t* d_cu_seqlens;  /* int32 [B+1]                                             */
  const float* d_scores;        /* fp32 [T]                                                */
  int32_t chunk;                /* >= 1                                                    */
  int32_t pool_window;          /* odd, >= 1 (1 = no smoothing)                            */
  double keep_rate;             /* in (0, 1]                                               */
  int32_t* d_kept_idx;          /* out int32 [kept_capacity]: flat token indices, ascending;
                                   entries at and beyond cu_keep[B] are left untouched     */
  int64_t kept_capacity;        /* >= number of kept tokens; T always suffices, see
                                   sp_keep_upper_bound.  Writes beyond it are suppressed.  */
  int32_t* d_cu_keep;           /* out int32 [B+1]: kept tokens of sequence b are
                                   kept_idx[cu_keep[b] .. cu_keep[b+1])                    */
  float* d_chunk_scores;        /* optional out fp32 [sum_b ceil(M_b/chunk)], NULL to skip */
  void* d_workspace;
  size_t workspace_bytes;
} sp_pool_select_args;

/* Host helper: an upper bound on the kept-token count from HOST sequence lengths
 * (sum over sequences of min(M_b, k_b * chunk)); -1 on invalid arguments. */
SP_API int64_t sp_keep_upper_bound(int32_t B, const int32_t* h_seqlens, int32_t chunk, double keep_rate);

SP_API size_t sp_pool_select_workspace_bytes(const sp_pool_select_args* args);
SP_API sp_status sp_pool_select(const sp_pool_select_args* args, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP-graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same operation and results as sp_pool_select, but
 * the scratch space is a fixed array inside the library's device image instead of a caller
 * workspace (d_workspace / workspace_bytes are ignored).  Limits: B <= SP_STATIC_MAX_SEQS and
 * T / chunk + B <= SP_STATIC_MAX_CHUNKS, else SP_EUNSUPPORTED.  Calls nothing that allocates.
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU race
 * (serialise them on one stream).  The array (SP_STATIC_SCRATCH_BYTES per GPU) lives until the
 * process ends. */
#define SP_STATIC_MAX_SEQS 4096
#define SP_STATIC_MAX_CHUNKS 131072
#define SP_STATIC_SCRATCH_BYTES (2u << 20)
SP_API sp_status sp_pool_select_static(const sp_pool_select_args* args, void* hip_stream);

/* ---------------------------------------------------------------------------
 * sp_score_pool_select: sp_score followed by sp_pool_select for ONE SHORT prompt, in a single
 * kernel launch (Sec. 3.2 equation, Sec. 3.2.2 and Sec. 3.2.3 in one go; the case of the paper's
 * variants without look-ahead on short contexts, Sec. 4.3, where the separate calls are bound by
 * their launches).  `score` and `select` are filled exactly as for the separate calls and must
 * describe the same prompt (select->B == score->B, select->T == score->T, select->d_scores ==
 * score->d_scores, select->d_cu_seqlens == score->d_cu_seqlens).  score->d_workspace must hold
 * sp_score_workspace_bytes(score) bytes as for sp_score (the logits pass through it; SP_EWORKSPACE
 * otherwise); select's workspace fields are ignored.  Outputs: everything the two calls write
 * (scores, optional lse, kept_idx, cu_keep, optional chunk_scores); scores agree with sp_score's
 * to the tolerance of fp32 summation order, the selection is sp_pool_select's on these scores.
 * The workgroups of the launch never wait for one another (the last one to finish its share
 * completes the call), so nothing depends on what else runs on the device; they do count their
 * arrivals in one word per device, so two of these calls must not overlap on one GPU.
 * Supported: B == 1, 1 <= T <= 2048, H/H_kv * N <= 16, L * H * N <= 4096, rope_theta == 0, a bf16 cache, no
 * block table, at most 2048 chunks; anything else returns SP_EUNSUPPORTED and launches nothing (use the
 * separate calls).  The part after the logits is done by one workgroup: the call pays while
 * L * H * N * T stays small (a few layers of a few thousand keys); the separate calls, which use
 * the whole device throughout, overtake it beyond that.
 * --------------------------------------------------------------------------- */
SP_API sp_status sp_score_pool_select(const sp_score_args* score, const sp_pool_select_args* select, void* hip_stream);

/* ---------------------------------------------------------------------------
 * sp_gather: restore_pos_ids (Algorithm 1, Sec. 3.2.4) plus the gathers the base
 * model's prefill needs.  For kept slot s of sequence b:
 *     kept_pos[s]  = kept_idx[s] - cu_seqlens[b]      (position in the ORIGINAL prompt)
 *     kept_ids[s]  = token_ids[kept_idx[s]]
 *     out_embed[s] = embed[kept_ids[s], :]
 *     decode_pos[b] = M_b   (the first decoded token sits at the full prompt length)
 * Integer outputs and copied rows are exact.
 * --------------------------------------------------------------------------- */
typedef struct {
  int32_t B;
  const int32_t* d_cu_seqlens;  /* int32 [B+1]                                            */
  const int32_t* d_cu_keep;     /* int32 [B+1] from sp_pool_select                        */
  const int32_t* d_kept_idx;    /* int32 [>= cu_keep[B]]                                  */
  const int32_t* d_token_ids;   /* int32 [T], or NULL (then d_kept_ids/d_embed unused)    */
  const void* d_embed;          /* bf16 [V, D] row-major, 16-byte aligned, or NULL        */
  int32_t V;
  int32_t D;                    /* multiple of 8 when d_embed != NULL                     */
  int32_t* d_kept_ids;          /* out int32 [kept_capacity], NULL iff d_token_ids NULL   */
  int32_t* d_kept_pos;          /* out int32 [kept_capacity]                              */
  int32_t* d_decode_pos;        /* out int32 [B]                                          */
  void* d_out_embed;            /* out bf16 [kept_capacity, D] or NULL to skip the rows   */
  int64_t kept_capacity;        /* slots at and beyond min(cu_keep[B], capacity) untouched */
} sp_gather_args;

SP_API sp_status sp_gather(const sp_gather_args* args, void* hip_stream);

/* Static, never-NULL description of a status code. */
SP_API const char* sp_strerror(sp_status status);

/* Library version as major*10000 + minor*100 + patch. */
SP_API int32_t sp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECPREFILL_H */
