/*
 * CPU oracle for the MorphKV decode hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the path computes, written from
 * the paper (Section 3.1 Eq.1, Eq.4-7, Algorithm 1; Section 3.3 for GQA).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it;
 * the product library never links or calls it, and it shares no code with the
 * HIP path.  All pointers are HOST pointers.
 *
 * Parity status: attention/softmax, bookkeeping, fusion arithmetic, tie-break
 * and GQA aggregation are pinned by the CPU tests (dense attention, a
 * dict-based brute force, the paper's worked fusion numbers, closed forms).
 * The two comparison policies (running-sum score, selection at the prompt
 * only) are pinned by the same brute force.
 * End-task accuracy (the paper's tables) is "parity unpinned": it needs the
 * paper's models and datasets.
 *
 * Unit = one (layer, sequence, KV head): an independent cache (Section 3.3).
 * Unit index u = (layer * batch + b) * n_kv_heads + h.
 */
#ifndef MORPHKV_REF_H
#define MORPHKV_REF_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct morphkv_ref_config {
  int32_t n_layers, batch, n_q_heads, n_kv_heads, head_dim, C, R;
  int32_t fusion;         /* 0 = sum (Eq.5), 1 = max (Eq.6); 2 = comparison policy: running sum of every
                             recorded weight since the token entered the cache, no window (the accumulated
                             attention score of H2O, Section 2 / Section 5 "Baselines") */
  int32_t dtype;          /* element type of q/K/V inputs: 0 = fp32, 1 = bf16 bits */
  int32_t evict_every;    /* T of Appendix A.5: selection at every T-th generation step; 1 = at every step; 0 = comparison policy: selection at
                             the prompt only, every later token is kept (SnapKV, Section 5 "Baselines") */
  int32_t max_prompt_len; /* unused by the oracle; kept so one harness fills both structs */
  float softmax_scale;    /* 0 -> 1/sqrt(head_dim) (Eq.1) */
  int32_t max_new_tokens; /* with evict_every == 0: room for this many decode steps; else unused */
} morphkv_ref_config;

typedef struct morphkv_ref morphkv_ref;

#define MORPHKV_REF_OK 0
#define MORPHKV_REF_EINVAL (-1)
#define MORPHKV_REF_ESTATE (-2)

int morphkv_ref_create(morphkv_ref **h, const morphkv_ref_config *cfg);
int morphkv_ref_destroy(morphkv_ref *h);

/* Selection over the whole prompt (Section 4 "Implementation"; Eq.4-7).
 * Q_window [L][B][M][R][d]: row j = query of prompt position N_b - min(R,N_b) + j.
 * K, V [L][B][M'][Nmax][d].  prompt_len [B].
 * forced_pos: NULL, or [U][C] ascending positions (-1 padded) to retain instead
 * of the oracle's own top-C (used when a caller adopts another valid choice at
 * a near-tie); the scores are still computed and kept for prefill_scores. */
int morphkv_ref_prefill_select(morphkv_ref *h, const void *Q_window, const void *K, const void *V,
                               const int32_t *prompt_len, int32_t Nmax, const int32_t *forced_pos);
/* Fused score F[k] of every candidate k < N - min(R,N) of one unit, as of the last prefill.
 * Returns the candidate count (or <0); F may be NULL to query the count. */
int morphkv_ref_prefill_scores(morphkv_ref *h, int32_t unit, double *F, int32_t capacity);

/* One decode step in two halves.
 * begin: attention of the new token over the resident cache plus itself (Eq.1),
 *        out [L][B][M][d] fp64; records the group-summed weights as the newest
 *        row (Alg.1 aggregation); if the window is full, fuses the R rows into
 *        a score per candidate (Eq.4-6) and takes the oracle's own decision
 *        (Eq.7: keep top-C of C+1, ties keep the lower position).
 * commit: applies a decision per unit: evict_pos NULL = the oracle's own;
 *        otherwise evict_pos[u] = position to evict (must be a candidate),
 *        ignored for units where nothing is evicted this step. */
int morphkv_ref_decode_begin(morphkv_ref *h, const void *q, const void *k_new, const void *v_new, double *out);
int morphkv_ref_decode_commit(morphkv_ref *h, const int32_t *evict_pos);
int morphkv_ref_decode_step(morphkv_ref *h, const void *q, const void *k_new, const void *v_new, double *out);

/* After decode_begin: per unit the candidates of this step.
 * n_cand [U] (0 when nothing can be evicted), cand_pos / cand_F [U][C+T] (T = evict_every),
 * n_evict [U] (how many must go), choice [U][T] (oracle's own evictions, -1 padded). */
int morphkv_ref_candidates(morphkv_ref *h, int32_t *n_cand, int32_t *cand_pos, double *cand_F,
                           int32_t *n_evict, int32_t *choice);
/* multi-eviction commit for evict_every > 1: evict_pos [U][T], -1 padded. */
int morphkv_ref_decode_commit_multi(morphkv_ref *h, const int32_t *evict_pos);

/* Retained positions: pos [U][C+T-1+R], ascending snapshot positions then ascending
 * window positions, -1 padded at the end; n_snap [U]; n_win [U] (may be NULL). */
int morphkv_ref_export_positions(morphkv_ref *h, int32_t *pos, int32_t *n_snap, int32_t *n_win);
int morphkv_ref_row_stride(morphkv_ref *h); /* = C+T-1+R (C+max_new_tokens+R when evict_every == 0), the pos row length */

int morphkv_ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
