/*
 * libarkv - ARKV per-layer KV-cache management around decode attention, for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer argument says whether it is HOST or DEVICE memory.  Tensors are dense,
 * row-major, in the index order written in brackets; "bf16" is the 16-bit brain float stored as
 * uint16_t.  hip_stream is a hipStream_t passed as void* (NULL = the default stream).  One cache
 * object must be driven from one stream at a time.  Every call returns 0 on success or a negative
 * ARKV_E* code; nothing throws.  Calls that take a stream are asynchronous on it unless stated.
 *
 * Notation (the paper's): L layers, B sequences, H_q query heads, H_kv KV heads, G = H_q / H_kv,
 * d head dimension, T prompt length, N cache limit in tokens per (sequence, kv-head), W protected
 * window.  A "unit" is one (layer, sequence, kv-head); units never interact during decode.
 */
#ifndef ARKV_H
#define ARKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ARKV_OK            0
#define ARKV_EINVAL       -1   /* bad argument (null pointer, shape, range) */
#define ARKV_ESTATE       -2   /* call out of order (decode before commit, commit twice, ...) */
#define ARKV_ENOMEM       -3   /* device or host allocation failed */
#define ARKV_EHIP         -4   /* a HIP runtime call failed; arkv_last_hip_error() has its text */
#define ARKV_EUNSUPPORTED -5   /* valid but not built (head_dim, group size, bit width) */
#define ARKV_ESCRATCH     -6   /* arkv_decode_step_static: the launch does not fit the static scratch array */

/* Token states (Sec. IV-B "Problem Formulation": full precision, quantized, evicted). */
#define ARKV_STATE_ORIGINAL  0
#define ARKV_STATE_QUANTIZED 1
#define ARKV_STATE_EVICTED   2

typedef struct arkv_cache arkv_cache;   /* opaque; the library owns all cache device memory */

/* Hyper-parameters (Sec. V "Main Results" gives the tuned values used as defaults). */
typedef struct {
  int32_t n_layers;         /* L */
  int32_t batch;            /* B */
  int32_t n_q_heads;        /* H_q, multiple of n_kv_heads; G in {1,2,4,8} */
  int32_t n_kv_heads;       /* H_kv */
  int32_t head_dim;         /* d: 64 or 128 */
  int32_t capacity_tokens;  /* N: cache limit per (sequence, kv-head), same for all layers (eq. 8 text) */
  int32_t window;           /* W: last W tokens always Original (eq. 10, last line); default 32 */
  float   alpha;            /* slack factor of Top-b, b = floor(alpha (N-W)) (eq. 10); default 0.75 */
  float   gamma;            /* weight of the variance in the heavy-hitter score (eq. 9); default 263.81 */
  float   tau[3];           /* temperatures of the OQ score (eq. 6); default 7.774, 5.407, 5.528 */
  int32_t quant_bits;       /* format of a Quantized token: 4 or 2 = uniform codes, groups of 32 channels, fp16
                             * scale and zero per group; 8 = fp8 E4M3 codes with one fp16 scale per K (V) row
                             * (Alg. 1 "Reconstruction Before Attention": x~ = q^ * s, per-token scale) */
  int32_t group_size;       /* channels per scale/zero pair: 32 */
  int32_t tailor_policy;    /* 0: tailor when the cache is full, keeping b = floor(alpha (N-W)) tokens (Sec. IV-F,
                               last paragraph: slack factor); 1: no slack, b = N-W-1, i.e. a tailor at every step once
                               the cache is full (Sec. IV-F first sentence read literally; stress timing) */
  int32_t budget_mode;      /* 0: the limit and the budgets are token counts (Sec. V: "512, 1024, 2048 tokens");
                               1: eq. 1 and eq. 8 in bytes: the limit is N*C_orig bytes per (sequence, kv-head),
                               a Quantized token is charged C_quant, so n_q = floor((b - n_o) C_orig / C_quant)
                               tokens fit where the token rule keeps b - n_o.  Tailors keep the token rule's
                               schedule (occupancy is booked as if every survivor were Original). */
} arkv_config;

/* Fills *cfg with the paper's tuned hyper-parameters, 4-bit groups of 32, and zero shapes. HOST. */
int arkv_config_default(arkv_config* cfg);

/* Allocates the pools of all layers on the current device (per unit: N bf16 K and V rows, b packed
 * rows, per-slot position / score accumulators, the latest queries per unit) and returns the cache in *out.
 * Synchronous.  ARKV_EINVAL: null pointers, non-positive shapes, W >= N - 1, alpha outside (0,1],
 * gamma < 0, group_size != 32.  ARKV_EUNSUPPORTED: head_dim not in {64,128}, G not in {1,2,4,8}, G*W > 512,
 * quant_bits not in {2,4,8}, N > 2^20 - 64 tokens, or pools of more than 2^21 - 32 rows per unit (byte budgets
 * keep up to C_orig / C_quant Quantized rows per Original row they replace). */
int arkv_cache_create(const arkv_config* cfg, arkv_cache** out);

/* Frees everything.  Synchronises the device first.  NULL is accepted. */
int arkv_cache_destroy(arkv_cache* cache);

/* Forgets the contents of one layer (layer >= 0) or of all layers (layer = -1) so that the prompt
 * of a new request can be scored and committed; keeps the memory. */
int arkv_cache_reset(arkv_cache* cache, int32_t layer);

/* Prefill scorer of one layer (Sec. IV-C, eqs. 2-5; Sec. IV-E eq. 9 for the accumulators).
 *   q_win  DEVICE bf16 [B][H_q][W][d]   queries of the last W prompt positions
 *   k      DEVICE bf16 [B][H_kv][T][d]  keys of the whole prompt (already position-encoded)
 *   stats  DEVICE float [B][3]          out: entropy, variance, kurtosis of the aggregated key
 *                                        distribution over keys [0, T-W), per sequence
 * Window query i (position T-W+i) attends causally to keys 0..T-W+i with
 * softmax(softmax_scale * q.k); the layer statistics use keys < T-W only.  As a side effect the
 * per-(kv-head, token) sums of attention and squared attention over the window are kept inside the
 * cache for arkv_prefill_commit.  Asynchronous, except that scratch is allocated on first use and when T grows
 * (an allocation may synchronise the device).
 * A prompt must be longer than the window: T <= W returns ARKV_EINVAL, because eqs. 3-5 are taken over the
 * keys outside the window and there are none.  Such a prompt needs no cache management until it has grown (below
 * the cache limit the method is plain attention, Sec. V-E); a caller can keep it outside the library and hand
 * over the first W + 1 or more tokens as the prompt.
 * ARKV_EINVAL: T <= W, bad layer.  ARKV_ESTATE: layer already committed. */
int arkv_prefill_stats(arkv_cache* cache, int32_t layer, const void* q_win, const void* k, int32_t T,
                       float softmax_scale, float* stats, void* hip_stream);

/* The same scorer for callers whose own attention kernel already produced the softmax normalisers of the window
 * rows: lse DEVICE float [B][H_q][W] = natural logarithm of the sum over the visible keys j <= T-W+i of
 * exp(softmax_scale * q.k), for window query i of every head (the per-row log-sum-exp that attention kernels
 * return).  The scorer then reads the keys once instead of twice (Sec. IV-C: eq. 2's rows are rows of the
 * prompt's attention).  Everything else as arkv_prefill_stats. */
int arkv_prefill_stats_lse(arkv_cache* cache, int32_t layer, const void* q_win, const void* k, int32_t T,
                           float softmax_scale, const float* lse, float* stats, void* hip_stream);

/* Causal self-attention of prompt queries with the scorer fused (Sec. IV-C: eq. 2's rows are the last W
 * rows of the prompt's causal attention).  ASYNC on hip_stream.
 * q [B][H_q][T_q][d] DEVICE bf16: the queries of positions [T - T_q, T); k, v [B][H_kv][T][d] DEVICE bf16: keys
 * and values of positions [0, T), already position-encoded; out [B][H_q][T_q][d] DEVICE bf16:
 * softmax(scale q k^T, causal) v.  A prompt may be fed in chunks: every call passes the keys so far and the new
 * chunk's queries.
 * stats == NULL: attention only.  stats != NULL ([B][3] DEVICE fp32, needs T_q >= W, T > W, layer not
 * committed): the call also does what arkv_prefill_stats does for the last W queries; the softmax maxima and
 * sums of those rows come out of the attention pass, so the scorer reads the keys once instead of twice.
 * Arithmetic: bf16 logits MFMA, probabilities and values as fp16 in the PV MFMA, fp32 accumulation; values
 * whose magnitude exceeds fp16's range (65504) are not supported.  All pointers 16-byte aligned.
 * ARKV_EINVAL / ARKV_ESTATE as for arkv_prefill_stats. */
int arkv_prefill_attention(arkv_cache* cache, int32_t layer, const void* q, const void* k, const void* v,
                           int32_t T_q, int32_t T, float softmax_scale, void* out, float* stats,
                           void* hip_stream);

/* OQ score and ratio (eqs. 6-7).  HOST, pure.  stats [L][B][3] -> rho [L][B]:
 * q = H^(1/tau1) V^(1/tau2) Kurt^(1/tau3), rho = q / max over the layers of the same sequence;
 * if every q of a sequence is 0, every rho of it is 1. */
int arkv_oq_ratio(const float* stats, int32_t n_layers, int32_t batch, const float tau[3], float* rho);

/* Token counts a tailor keeps (Alg. 1 "Assign origin budget", eq. 10).  HOST, pure.
 * b = min(floor(alpha (N-W)), N-W-1), or N-W-1 under tailor_policy 1; n_o = min(floor(rho (N-W)), b); n_q = b - n_o.
 * Under budget_mode 1 (needs head_dim and quant_bits): n_q = floor((b - n_o) C_orig / C_quant) and *b = n_o + n_q. */
int arkv_budget_counts(const arkv_config* cfg, float rho, int32_t* n_o, int32_t* n_q, int32_t* b);

/* Loads one layer's prompt into the cache and fixes the layer's budgets (Alg. 1, prefill phase).
 *   k, v  DEVICE bf16 [B][H_kv][T][d]  (the same k that was scored)
 *   rho   HOST float [B]               OQ ratio of this layer for every sequence
 * If T >= N the first tailor runs here on the window scores (Top-b, Top-B_o, quantise, evict).
 * Asynchronous on hip_stream (rho is read before the call returns; the budgets travel as launch arguments),
 * except that the first tailor's key scratch is allocated on first use and when T grows (an allocation may
 * synchronise the device).  The caller's k, v are not referenced after the stream has passed this call.
 * ARKV_ESTATE: the scorer (arkv_prefill_stats, _lse or arkv_prefill_attention with stats) has not run for this
 * layer with the same T, or the layer is already committed. */
int arkv_prefill_commit(arkv_cache* cache, int32_t layer, const void* k, const void* v, int32_t T,
                        const float* rho, void* hip_stream);

/* One decode step of one layer for the whole batch (Alg. 1, decoding phase + reconstruction).
 *   q             DEVICE bf16 [B][H_q][d]
 *   k_new, v_new  DEVICE bf16 [B][H_kv][d]   the token being generated (position T + step)
 *   out           DEVICE bf16 [B][H_q][d]    softmax(scale q.K~) V~ over every live token,
 *                                             K~/V~ = bf16 row (Original) or code*scale+zero (Quantized)
 * Appends the token as Original, attends (the new token included), adds each token's attention
 * probabilities to its running sums (eq. 9), and when the number of live tokens has reached N
 * runs the tailor (eq. 10): ranks tokens older than the W most recent by S = mean + gamma*variance,
 * keeps the top b, the top n_o of them in bf16 (a Quantized token is never promoted), quantises the
 * others in place, evicts the rest.  Never allocates, never synchronises.
 * ARKV_ESTATE: layer not committed, or an earlier step of it failed half way (ARKV_EHIP from a tailor launch):
 * such a layer refuses further steps until arkv_cache_reset. */
int arkv_decode_step(arkv_cache* cache, int32_t layer, const void* q, const void* k_new,
                     const void* v_new, float softmax_scale, void* out, void* hip_stream);

/* arkv_decode_step for callers that must not allocate device memory while they run (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same result bit for bit when the
 * split-K factor is the same.  The split-K partials and the units' tickets of the launch live in a 4 MiB array in
 * the library's static device memory (one per GPU, held until the process ends; its address is looked up by
 * arkv_cache_create on that GPU) instead of the cache's own buffers, and the call makes no hipMalloc / hipFree and
 * records no timing events.  Limits: B * H_kv <= 4096 units and B * H_kv * G * (d + 2) * 4 bytes <= 4 MiB - 16 KiB
 * (one split per unit must fit), else ARKV_ESCRATCH; the split-K factor is lowered to what fits (config of 32
 * units, G = 4, d = 128: up to 62 splits per unit).  Every call on a GPU shares that GPU's array: calls on
 * different streams (or different caches) that overlap in time on one GPU race; calls ordered on one stream do
 * not.  The tickets are zero between launches (the last workgroup of a unit clears its ticket); partials need
 * no clearing. */
int arkv_decode_step_static(arkv_cache* cache, int32_t layer, const void* q, const void* k_new,
                            const void* v_new, float softmax_scale, void* out, void* hip_stream);

/* The same for n consecutive, independent layers in one set of launches (benchmarks, graph capture).
 *   q [n][B][H_q][d], k_new/v_new [n][B][H_kv][d], out [n][B][H_q][d]  DEVICE bf16
 *   softmax_scale HOST float [n]
 * All n layers must be in the same state (same prompt length, same number of steps taken). */
int arkv_decode_step_layers(arkv_cache* cache, int32_t layer_begin, int32_t n, const void* q,
                            const void* k_new, const void* v_new, const float* softmax_scale,
                            void* out, void* hip_stream);

/* ---- observability and parity hooks: HOST outputs, synchronise the cache's last stream ---- */

/* Per unit of one layer, arrays [B][H_kv]: Original / Quantized token counts and live bytes
 * n_o*4d + n_q*C_q, C_q = 2*(d*bits/8 + 4*d/32) or 2*(d + 2) for fp8 rows (the left side of eq. 1 for that
 * unit), and the number of tokens
 * evicted so far (positions seen minus live tokens).  Any pointer may be NULL. */
int arkv_cache_counters(arkv_cache* cache, int32_t layer, int32_t* n_original, int32_t* n_quantized,
                        int32_t* n_evicted, int64_t* live_bytes);

/* Contents of one layer, per unit, tokens sorted by position.  max_tokens >= N, and at least the largest
 * number of live tokens of a unit (under budget_mode 1 a unit can hold more than N tokens: up to
 * W + n_o + n_q of arkv_budget_counts plus the steps since the last tailor; arkv_cache_counters gives the
 * counts); ARKV_EINVAL if a unit holds more.  Any output pointer may be NULL.  n_live [U]; pos, state [U][max_tokens]; s1, s2 [U][max_tokens] running sums of
 * attention and squared attention; rows_k, rows_v bf16 [U][max_tokens][d] (Original tokens, else 0);
 * codes_k, codes_v uint8 [U][max_tokens][d*bits/8] in canonical packing (channel c of a 4-bit row in
 * byte c/2 bits 4(c%2)..; of a 2-bit row in byte c/4 bits 2(c%4)..; of an fp8 row in byte c); scale_*,
 * zero_* fp16 bits [U][max_tokens][d/32], for fp8 rows [U][max_tokens][1] with zero_* = 0 (Quantized
 * tokens, else 0).  U = B*H_kv. */
int arkv_cache_export(arkv_cache* cache, int32_t layer, int32_t max_tokens, int32_t* n_live,
                      int32_t* pos, uint8_t* state, float* s1, float* s2,
                      uint16_t* rows_k, uint16_t* rows_v, uint8_t* codes_k, uint8_t* codes_v,
                      uint16_t* scale_k, uint16_t* zero_k, uint16_t* scale_v, uint16_t* zero_v);

/* Scores the latest tailor of this layer ranked on: per unit, count [U] eligible tokens with their
 * position and fp32 score S [U][max_tokens] in no particular order (count = -1: no tailor yet). */
int arkv_debug_last_tailor_scores(arkv_cache* cache, int32_t layer, int32_t max_tokens,
                                  int32_t* count, int32_t* pos, float* score);

/* fp32 attention output of the latest decode step of this layer, before rounding to bf16. [B][H_q][d] */
int arkv_debug_last_out_f32(arkv_cache* cache, int32_t layer, float* out);

/* Parity hook.  out_f32 DEVICE float [B][H_q][T_q][d] (caller-owned) or NULL: while set, every
 * arkv_prefill_attention on this cache also writes its output there before the rounding to bf16 (the bf16 output
 * is the round-to-nearest-even of these values); the buffer must be large enough for the T_q of those calls. */
int arkv_debug_prefill_attention_f32(arkv_cache* cache, float* out_f32);

/* Number of tailors run so far on this layer, the occupancy the trigger of the tailor counts (tokens per unit;
 * under budget_mode 1 the booked rows, i.e. every survivor counted as Original, which is an upper bound of the
 * live bytes / C_orig and not the number of live tokens: use arkv_cache_counters for those), and the position of
 * the latest token. */
int arkv_cache_progress(arkv_cache* cache, int32_t layer, int32_t* n_tailors, int32_t* n_live,
                        int32_t* position);

/* Measurement hook.  enable != 0: every later decode step brackets its attention kernel with HIP
 * events on the call's stream (a few microseconds of extra gap per step; off by default).
 * arkv_debug_attend_time synchronises, returns the summed duration in milliseconds and the number of
 * attention-kernel launches since the hook was enabled, and clears both. */
int arkv_debug_time_attend(arkv_cache* cache, int32_t enable);
int arkv_debug_attend_time(arkv_cache* cache, double* total_ms, int64_t* launches);

/* Measurement hook: launch shape of the kernels, for sweeps.  wg_target: workgroups a decode launch aims at
 * when it picks its split-K factor (default 512 = two per compute unit); packed_weight: cost of a packed row in
 * sixteenths of a bf16 row when rows are dealt to the splits (default: 10, or 16 for launches of at most 256
 * workgroups); prefill_chunk: keys per workgroup of the prefill scorer (multiple of 128, at most 8192; default:
 * 1024, halved while the grid would be small, or, with more than 256 query rows per kv-head, what makes the
 * grid one round of the chip; a value given here is taken as it is).  A value <= 0 leaves that setting as it
 * is.  Results do not depend on these beyond the order of floating-point additions.  ARKV_EINVAL: null cache,
 * packed_weight above 16, prefill_chunk not a multiple of 128 or above 8192. */
int arkv_debug_set_launch_shape(arkv_cache* cache, int32_t wg_target, int32_t packed_weight, int32_t prefill_chunk);

/* Parity hook, HOST, pure: the rows split `split` of `n_splits` owns in a decode launch over a unit with
 * n_original bf16 rows and n_quantized packed rows (a packed row weighs packed_weight sixteenths of a bf16
 * row; the last split is charged for appending the new token).  range[0..3] = first and one-past-last row of
 * the Original pool, then of the Quantized pool.  ARKV_EINVAL: null pointer, negative counts, n_splits not in
 * [1, 128], split outside [0, n_splits), packed_weight outside [1, 16]. */
int arkv_debug_split_range(int32_t n_original, int32_t n_quantized, int32_t packed_weight, int32_t n_splits,
                           int32_t split, int32_t* range);

/* Measurement hook of profiling builds (the library compiled with -DARKV_PHASE_TRACE, see the package's build
 * script; the product build returns ARKV_EUNSUPPORTED and its kernels carry none of this).  In such a build
 * thread 0 of every workgroup of the decode kernel stores the 100 MHz wall clock at its phase boundaries, and a
 * one-wave marker kernel is launched before and after the decode kernel.  Copies to HOST memory (synchronous):
 * which = 0: n_rows rows of 8 words, row = workgroup (unit-major, split-minor) of the latest decode launch:
 *   start, first tile requested, bf16 rows done, new token done, packed rows done, partial stored, end, and the
 *   XCC_ID hardware register (the XCD number is its low 4 bits); row 8190 holds the two markers' times in words 0 and 1;
 * which = 1: the same rows for the merge inside the unit's last workgroup: entered, loads issued, weights
 *   reduced, barrier passed, accumulated, stored (words 0..5; rows of other workgroups keep older values);
 * which = 2: 4 words of the latest prefill-attention launch: shader clock and wall clock at the start and at the
 *   end of workgroup (0, 0) (n_rows is ignored, pass 1).
 * ARKV_EINVAL: null pointer, which outside 0..2, n_rows outside 1..8192. */
int arkv_debug_phase_trace(int32_t which, unsigned long long* host_words, int32_t n_rows);

const char* arkv_strerror(int code);        /* static text for an ARKV_E* code */
const char* arkv_last_hip_error(void);      /* text of the HIP error behind the latest ARKV_EHIP */

#ifdef __cplusplus
}
#endif
#endif /* ARKV_H */
