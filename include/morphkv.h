/*
 * libmorphkv -- MorphKV's per-decode-step hot path on one MI355X (gfx950).
 *
 * What the path computes (paper: Section 3.1 Eq.1, Eq.3-7, Algorithm 1,
 * Section 3.3; Section 4 "Implementation" for the prompt-time selection):
 * every decode step, grouped-query attention of the new token over a
 * constant-size cache of C retained older tokens plus the R most recent ones;
 * the group-summed attention weights of that token are recorded as the newest
 * of R rows; the R rows are fused (sum, Eq.5, or max, Eq.6) into one score per
 * older token; the top-C older tokens are kept (Eq.7) and K/V are compacted in
 * fixed slots.  The same selection runs once over the whole prompt.
 *
 * Conventions
 *  - unit = one (layer, sequence, KV head); u = (layer*batch + b)*n_kv_heads + h;
 *    U = n_layers*batch*n_kv_heads independent caches (Section 3.3).
 *  - every function returns 0 on success or a negative MORPHKV_E* code; nothing
 *    throws or aborts.  morphkv_last_error() gives the text of the last failure
 *    on the calling thread.
 *  - ALL device buffers are caller-owned (sizes from morphkv_sizes); the handle
 *    is host memory only.  The library allocates no device memory, enqueues all
 *    work on the caller's stream, and never synchronises.
 *  - the layouts inside `cache`, `scores_ring` and `scratch` are private; read
 *    them through the export calls.
 *  - one handle must not be used from two streams at once: calls on it are
 *    ordered by the stream they are enqueued on.
 */
#ifndef MORPHKV_H
#define MORPHKV_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MORPHKV_OK 0
#define MORPHKV_EINVAL (-1) /* bad shape, flag, size or null pointer */
#define MORPHKV_ESTATE (-2) /* decode before prefill */
#define MORPHKV_EHIP (-3)   /* a HIP runtime call or kernel launch failed */

#define MORPHKV_FUSION_SUM 0 /* Eq.5 */
#define MORPHKV_FUSION_MAX 1 /* Eq.6 */
/* Comparison policy, not MorphKV: the score of an older token is the running sum of every weight later queries
 * gave it since it entered the cache, with no window (the accumulated attention score of H2O, Section 5
 * "Baselines"); the R most recent tokens are still always kept.  For run-time comparison on the same kernel. */
#define MORPHKV_FUSION_CUMSUM 2
#define MORPHKV_DTYPE_F32 0
#define MORPHKV_DTYPE_BF16 1

typedef struct morphkv_config {
  int32_t n_layers, batch;
  int32_t n_q_heads;      /* M  (Algorithm 1) */
  int32_t n_kv_heads;     /* M' ; M % M' == 0; group size G = M/M' must be 1..8 */
  int32_t head_dim;       /* d_h of Eq.1: 64 or 128 */
  int32_t C;              /* older tokens retained (Eq.3), >= 1 */
  int32_t R;              /* recent window (H1), 1..1024 */
  int32_t fusion;         /* MORPHKV_FUSION_* */
  int32_t dtype;          /* element type of q/K/V: MORPHKV_DTYPE_* */
  int32_t evict_every;    /* T of Appendix A.5, 1..64: selection runs at every T-th generation step of a sequence
                             (its T-th, 2T-th .. generated token); in between up to C+T-1 older tokens are held.
                             0 = comparison policy, not MorphKV: selection at the prompt only, every later token
                             is kept (SnapKV, Section 5 "Baselines"); needs max_new_tokens */
  int32_t max_prompt_len; /* largest Nmax that will be passed to prefill_select */
  float softmax_scale;    /* 0 -> 1/sqrt(head_dim) (Eq.1) */
  int32_t max_new_tokens; /* with evict_every == 0 or n_keep_all_layers > 0: decode steps the cache has room for
                             (the step after that returns MORPHKV_ESTATE); otherwise ignored */
  int32_t n_keep_all_layers; /* Appendix A.6 (selective layer retention): MorphKV is off in the first
                             n_keep_all_layers layers, which keep every token of the prompt and of the response
                             (max_prompt_len + max_new_tokens slots; attention only: nothing is recorded, fused or
                             selected there); the other layers run as configured above.  0..n_layers; bf16 only;
                             max_prompt_len + max_new_tokens + R <= 1048576 */
} morphkv_config;

typedef struct morphkv_handle morphkv_handle;

/* Bytes the caller must provide (device memory, 256-byte aligned) for a configuration. */
int morphkv_sizes(const morphkv_config *cfg, size_t *cache_bytes, size_t *ring_bytes, size_t *scratch_bytes);

/* Host-only handle over caller-owned DEVICE buffers of at least morphkv_sizes bytes.
 * The buffers need no initialisation; prefill_select writes all state.  They must
 * stay valid until morphkv_destroy.  Ownership stays with the caller.
 * MORPHKV_EINVAL if C + R is beyond what the decode kernels can hold (the reason is in morphkv_last_error): fp32
 * caches keep one weight per (query head, slot) in LDS (C + R up to about 9 k slots at 4 heads a group); bf16
 * caches beyond that run with several workgroups per unit, up to about 130 k slots at 4 heads a group; layers that
 * keep every token (n_keep_all_layers) have no such bound.
 * Environment variables, read by morphkv_sizes and here, override tuning choices and never change results:
 * MORPHKV_SPLIT_BPS (bf16: a positive value splits every unit over several workgroups of that many 32-slot blocks
 * each; unset or 0 = only units that one workgroup cannot hold are split),
 * MORPHKV_DECODE_THREADS (multiple of 64 in 128..1024: threads per unit in the decode kernel),
 * MORPHKV_DECODE_MIN_LDS (bytes of LDS to reserve per workgroup at least),
 * MORPHKV_KEEP_KERNEL ("split": layers that keep every token run in the split kernel instead of the kernel made for
 * them), MORPHKV_KEEP_SHARES (1..32: workgroups per unit of that kernel; unset = by the number of units in the
 * launch), MORPHKV_REBUILD_WAVES (1..16: how many waves of a unit's workgroup share the per-step rebuild of score aggregates;
 * rounding of sums may differ in the last bit between values, the retained sets stay within the tie tolerance) and
 * MORPHKV_CACHE_BUDGET_MB (bf16 caches; default 208: how much of the handle's K/V is read with ordinary loads
 * and so stays in the device's 256 MB memory-side cache from step to step; the rest is streamed with
 * non-temporal loads that leave that cache alone). */
int morphkv_create(morphkv_handle **h, const morphkv_config *cfg, void *cache, void *scores_ring, void *scratch);
int morphkv_destroy(morphkv_handle *h);

/* Selection over the prompt (Section 4 "Implementation"; Eq.4-7), once per batch.
 *  Q_window  device [L][B][M][R][d]   queries of the last min(R,N_b) prompt tokens of each
 *                                     sequence; row j = query of position N_b - min(R,N_b) + j
 *  K, V      device [L][B][M'][Nmax][d]  prompt keys/values, rows >= N_b are ignored padding
 *  prompt_len HOST  [B]               1 <= N_b <= Nmax <= cfg.max_prompt_len; read before the call returns and
 *                                     handed to the device as kernel arguments (no copy, no synchronisation:
 *                                     the call can be captured in a HIP graph)
 * For every unit: causal softmax rows of the window queries over the whole prompt, summed
 * over the group's heads (Algorithm 1), fused over the rows (Eq.5/6) for the older tokens
 * k < N_b - min(R,N_b), top-min(C, count) kept (ties keep the lower position), K/V gathered
 * into the cache, and the recorded rows seeded.  Inputs are only read. */
int morphkv_prefill_select(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                           const int32_t *prompt_len, int32_t Nmax, void *stream /* hipStream_t */);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): morphkv_prefill_select with the library's OWN workspace in
 * place of the handle's `scratch` buffer -- a static device array of MORPHKV_NOALLOC_SCRATCH_BYTES that every
 * GPU the library runs on holds until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine) and, like the other calls, only enqueues kernels on the stream.
 * Arguments, results and the state left behind are those of morphkv_prefill_select (same kernels).
 * MORPHKV_EINVAL, with the sizes in morphkv_last_error, if the configuration at this Nmax needs more workspace
 * than the array holds (what morphkv_sizes reports as scratch_bytes for max_prompt_len = Nmax).
 * All calls on one GPU share that array: two such calls that overlap in time on the same GPU (different streams
 * or threads) race; calls on one stream are ordered.  The array keeps the previous call's contents; nothing
 * in it has to start at zero (every field is written before it is read). */
#define MORPHKV_NOALLOC_SCRATCH_BYTES (16u << 20)
int morphkv_prefill_select_noalloc(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                                   const int32_t *prompt_len, int32_t Nmax, void *stream /* hipStream_t */);

/* The same when the prompt's own attention pass has already been run by the caller (Section 8 names fusing the
 * selection into that pass as future work): attention kernels return, per query row, the natural logarithm of the
 * sum of exp over its causal logits.
 *  lse_window device [L][B][M][R] fp32: that value for the window queries (row j as in Q_window, rows >= min(R,N_b)
 *             ignored), or NULL for the behaviour of morphkv_prefill_select.
 * The pass over the prompt that finds the rows' softmax statistics is then skipped; weights are
 * exp(logit - lse).  Everything else as morphkv_prefill_select. */
int morphkv_prefill_select_lse(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                               const float *lse_window, const int32_t *prompt_len, int32_t Nmax,
                               void *stream /* hipStream_t */);

/* The prompt's attention pass and the selection over the prompt in one call (Section 8 "future work": selection
 * fused with the attention kernel; Eq.1 at every prompt position with the token attending to itself, then Eq.4-7).
 * bf16 configurations only (MORPHKV_EINVAL otherwise).
 *  Q        device [L][B][M][Nmax][d]   queries of every prompt position (rows >= N_b are ignored padding)
 *  K, V     device [L][B][M'][Nmax][d]  as in morphkv_prefill_select
 *  O        device [L][B][M][Nmax][d]   bf16, written: O[i] = sum_{k<=i} softmax_k(scale q_i.k_k) v_k for i < N_b;
 *                                       rows >= N_b are left untouched
 *  lse      device [L][B][M][Nmax] fp32 or NULL: natural log of the sum of exp over each row's causal logits
 *  prompt_len HOST [B]
 * The weights that multiply V are rounded to bf16 (as the matrix cores take them), their sum is kept in fp32.
 * The window rows' normalisers go from the attention pass straight to the selection, whose own statistics pass
 * over the prompt is skipped, and the window queries are read in place from Q.  The state left behind is that
 * of morphkv_prefill_select on (the last R rows of Q, K, V).  Q, K, V, O 16-byte aligned; all caller-owned. */
int morphkv_prefill_attend_select(morphkv_handle *h, const void *Q, const void *K, const void *V, void *O,
                                  float *lse, const int32_t *prompt_len, int32_t Nmax,
                                  void *stream /* hipStream_t */);

/* One decode step for all units (Eq.1, Algorithm 1, Eq.7).
 *  q      device [L][B][M][d]    query of the new token
 *  k_new  device [L][B][M'][d]   its key   (enters the window after the step)
 *  v_new  device [L][B][M'][d]   its value
 *  out    device [L][B][M][d]    fp32 attention output over the resident cache plus the token itself
 * Inputs are only read; cache and scores_ring are updated in place.  Values are not checked: a query or key that
 * is not a number gives an output that is not one, and scores that are not numbers count as the largest (such a
 * step evicts by position alone); the cache keeps its structure -- C older tokens and the R most recent, every
 * position once -- whatever the values are. */
int morphkv_decode_step(morphkv_handle *h, const void *q, const void *k_new, const void *v_new, float *out,
                        void *stream /* hipStream_t */);

/* The same step for the units of ONE layer (Section 3.3: every layer's attention keeps its own cache; a
 * model calls this from inside layer `layer`'s attention, one call per layer per token):
 *  q      device [B][M][d],  k_new, v_new device [B][M'][d],  out device [B][M][d] fp32
 * of that layer alone.  Calls for different layers are independent; per layer they must come in token
 * order.  Whole-model and per-layer calls may be mixed as long as every layer sees every token once. */
int morphkv_decode_step_layer(morphkv_handle *h, int32_t layer, const void *q, const void *k_new, const void *v_new,
                              float *out, void *stream /* hipStream_t */);

/* Copies the retained positions to caller-owned DEVICE arrays (enqueued on the stream):
 *  pos    [U][Cs+R] int32, Cs = C+evict_every-1 (C+max_new_tokens when evict_every == 0): the position of the token
 *         each cache slot holds, -1 = free, in the cache's own order (a token keeps the slot it was written to
 *         until it is evicted: Eq.7 decides by position who is "older", not by slot).  A unit's window are its R
 *         largest positions, its older tokens all others.  With n_keep_all_layers > 0 the rows are max(Cs, Ck) + R
 *         long, Ck = max_prompt_len + max_new_tokens being the older-token capacity of a layer that keeps
 *         everything: a unit's row holds its own slots, then -1
 *  n_snap [U]      int32: older tokens currently held (tokens that are not among the R most recent) */
int morphkv_export_positions(morphkv_handle *h, int32_t *pos, int32_t *n_snap, void *stream);
/* evicted [U] int32 device: position evicted by the last decode step, -1 if none (with evict_every > 1:
 * the first of them). */
int morphkv_export_evicted(morphkv_handle *h, int32_t *evicted, void *stream);
/* evicted [U][evict_every] int32 device: every position evicted by the last decode step, -1 padded. */
int morphkv_export_evicted_list(morphkv_handle *h, int32_t *evicted, void *stream);

const char *morphkv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
