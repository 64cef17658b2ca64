/*
 * CPU oracle for the MorphKV decode hot path -- TEST INFRASTRUCTURE ONLY
 * (see morphkv_ref.h).  Plain C, fp64, one loop nest per equation; threads
 * (OpenMP) only across independent units.  Nothing here is tuned.
 *
 * Readings of the paper taken here (each is listed in the design notes):
 *  - the new token attends to itself as well as to the cache (Eq.1 is written
 *    over tokens j < i; the step is given k_new/v_new, as stock attention
 *    after a cache update would see them);
 *  - order inside a step: attend -> record the row -> the window slides (new
 *    token in, token p-R out) -> fuse the R rows of the new window -> select,
 *    so that between steps the cache is Top_C(F) plus the last R tokens
 *    (Eq.3, Eq.7);
 *  - recorded weights are used as recorded, never re-normalised (Section 4,
 *    "Implementation": profiles are appended and the oldest discarded);
 *  - weights on tokens that are still inside the window are recorded too,
 *    otherwise the token leaving the window would have no score (Eq.4);
 *  - GQA: sum over the M/M' query heads of a group, then fuse (Alg.1);
 *  - ties in Top_C keep the lower position;
 *  - fewer than C older tokens: keep all of them, nothing is evicted;
 *  - coarse eviction (Appendix A.5): selection runs only at every T-th
 *    generation step of a sequence (its T-th, 2T-th, ... generated token,
 *    whatever the prompt length); in between, tokens leaving the window are
 *    kept, so up to C+T-1 older tokens are resident.
 */
#include "morphkv_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t n_snap;   /* older ("distant") tokens held */
  int32_t next_pos; /* position of the next token to decode; -1 before prefill */
  double *Ks, *Vs;  /* [Cs][d] */
  int32_t *pos_s;   /* [Cs] */
  double *Kw, *Vw;  /* [R][d], slot = position mod R */
  int32_t *pos_w;   /* [R], -1 = empty */
  double *row;      /* [R][Cs+R] recorded group-summed weights; row index = query position mod R */
  int32_t *row_q;   /* [R] query position each row belongs to, -1 = none */
  /* pending decision between decode_begin and decode_commit */
  int pending;
  int32_t n_cand, n_evict;
  int32_t *cand_pos, *cand_col; /* [Cs+1] */
  double *cand_F;               /* [Cs+1] */
  int32_t *choice;              /* [T] */
  int32_t prompt_len;           /* N: generation steps are counted from here */
  /* running-sum policy (fusion 2) */
  double *cum;                  /* [Cs] sum of every weight recorded for the older token in the slot */
  double *S_last;               /* [Cs] what the query in flight adds to it */
  double *k_new, *v_new;        /* [d] staged new token */
  /* prefill scores kept for inspection */
  double *pf_F;
  int32_t pf_n;
} unit_t;

struct morphkv_ref {
  morphkv_ref_config c;
  int32_t G, U, Cs, W; /* group size, units, snapshot capacity C+T-1, row width Cs+R */
  double scale;
  unit_t *u;
};

static double ld(const void *base, size_t i, int dtype) {
  if (dtype == 0) return (double)((const float *)base)[i];
  uint32_t w = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 -> fp32 is exact */
  float f;
  memcpy(&f, &w, 4);
  return (double)f;
}

static double fuse2(int fusion, double a, double b) { return fusion == 1 ? (a > b ? a : b) : a + b; }

int morphkv_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

int morphkv_ref_create(morphkv_ref **out, const morphkv_ref_config *cfg) {
  if (!out || !cfg) return MORPHKV_REF_EINVAL;
  if (cfg->n_layers < 1 || cfg->batch < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads < 1) return MORPHKV_REF_EINVAL;
  if (cfg->n_q_heads % cfg->n_kv_heads) return MORPHKV_REF_EINVAL;
  if (cfg->head_dim < 1 || cfg->C < 1 || cfg->R < 1 || cfg->evict_every < 0) return MORPHKV_REF_EINVAL;
  if (cfg->evict_every == 0 && cfg->max_new_tokens < 1) return MORPHKV_REF_EINVAL;
  if (cfg->fusion < 0 || cfg->fusion > 2 || cfg->dtype < 0 || cfg->dtype > 1) return MORPHKV_REF_EINVAL;
  morphkv_ref *h = (morphkv_ref *)calloc(1, sizeof(*h));
  h->c = *cfg;
  h->G = cfg->n_q_heads / cfg->n_kv_heads;
  h->U = cfg->n_layers * cfg->batch * cfg->n_kv_heads;
  h->Cs = cfg->C + (cfg->evict_every >= 1 ? cfg->evict_every - 1 : cfg->max_new_tokens);
  h->W = h->Cs + cfg->R;
  h->scale = cfg->softmax_scale != 0.0f ? (double)cfg->softmax_scale : 1.0 / sqrt((double)cfg->head_dim);
  h->u = (unit_t *)calloc((size_t)h->U, sizeof(unit_t));
  const int d = cfg->head_dim, R = cfg->R, Cs = h->Cs;
  for (int i = 0; i < h->U; ++i) {
    unit_t *s = &h->u[i];
    s->next_pos = -1;
    s->Ks = (double *)calloc((size_t)Cs * d, sizeof(double));
    s->Vs = (double *)calloc((size_t)Cs * d, sizeof(double));
    s->pos_s = (int32_t *)calloc((size_t)Cs, sizeof(int32_t));
    s->Kw = (double *)calloc((size_t)R * d, sizeof(double));
    s->Vw = (double *)calloc((size_t)R * d, sizeof(double));
    s->pos_w = (int32_t *)calloc((size_t)R, sizeof(int32_t));
    s->row = (double *)calloc((size_t)R * h->W, sizeof(double));
    s->row_q = (int32_t *)calloc((size_t)R, sizeof(int32_t));
    s->cand_pos = (int32_t *)calloc((size_t)Cs + 1, sizeof(int32_t));
    s->cand_col = (int32_t *)calloc((size_t)Cs + 1, sizeof(int32_t));
    s->cand_F = (double *)calloc((size_t)Cs + 1, sizeof(double));
    s->choice = (int32_t *)calloc((size_t)(cfg->evict_every > 0 ? cfg->evict_every : 1), sizeof(int32_t));
    s->cum = (double *)calloc((size_t)Cs, sizeof(double));
    s->S_last = (double *)calloc((size_t)Cs, sizeof(double));
    s->k_new = (double *)calloc((size_t)d, sizeof(double));
    s->v_new = (double *)calloc((size_t)d, sizeof(double));
  }
  *out = h;
  return MORPHKV_REF_OK;
}

int morphkv_ref_destroy(morphkv_ref *h) {
  if (!h) return MORPHKV_REF_EINVAL;
  for (int i = 0; i < h->U; ++i) {
    unit_t *s = &h->u[i];
    free(s->Ks); free(s->Vs); free(s->pos_s); free(s->Kw); free(s->Vw); free(s->pos_w);
    free(s->row); free(s->row_q); free(s->cand_pos); free(s->cand_col); free(s->cand_F);
    free(s->choice); free(s->k_new); free(s->v_new); free(s->pf_F); free(s->cum); free(s->S_last);
  }
  free(h->u);
  free(h);
  return MORPHKV_REF_OK;
}

/* ---- selection helper: order candidates best-first: larger F first, ties -> lower position first ---- */
typedef struct { double F; int32_t pos; int32_t idx; } cand_t;
static int cand_cmp(const void *a, const void *b) {
  const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
  if (x->F > y->F) return -1;
  if (x->F < y->F) return 1;
  return (x->pos > y->pos) - (x->pos < y->pos);
}
static int i32_cmp(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

/* ---- prefill: window queries over the whole prompt, fuse, keep top-C (Eq.4-7) ---- */
static int prefill_unit(morphkv_ref *h, int l, int b, int kh, const void *Qw, const void *K, const void *V,
                        int32_t N, int32_t Nmax, const int32_t *forced) {
  const morphkv_ref_config *c = &h->c;
  const int d = c->head_dim, R = c->R, G = h->G, C = c->C, Cs = h->Cs, W = h->W, dt = c->dtype;
  unit_t *s = &h->u[(l * c->batch + b) * c->n_kv_heads + kh];
  const int Rw = N < R ? N : R;  /* window tokens */
  const int n_old = N - Rw;      /* candidates: positions [0, n_old) */
  const size_t kbase = ((size_t)(l * c->batch + b) * c->n_kv_heads + kh) * (size_t)Nmax * d;

  /* S[j][k] = sum over the group's heads of softmax_k(q_{g,j} . K_k * scale), k <= p_j (causal, self included) */
  double *S = (double *)calloc((size_t)Rw * N, sizeof(double));
  double *lg = (double *)malloc((size_t)N * sizeof(double));
  for (int j = 0; j < Rw; ++j) {
    const int pj = N - Rw + j;
    for (int g = 0; g < G; ++g) {
      const size_t qbase = ((((size_t)(l * c->batch + b) * c->n_q_heads + (kh * G + g)) * R) + j) * d;
      double m = -INFINITY;
      for (int k = 0; k <= pj; ++k) {
        double acc = 0.0;
        for (int e = 0; e < d; ++e) acc += ld(Qw, qbase + e, dt) * ld(K, kbase + (size_t)k * d + e, dt);
        lg[k] = acc * h->scale;
        if (lg[k] > m) m = lg[k];
      }
      double z = 0.0;
      for (int k = 0; k <= pj; ++k) { lg[k] = exp(lg[k] - m); z += lg[k]; }
      for (int k = 0; k <= pj; ++k) S[(size_t)j * N + k] += lg[k] / z;
    }
  }
  free(lg);

  /* F[k] = f(S_0[k], ..., S_{Rw-1}[k]) for the older tokens */
  free(s->pf_F);
  s->pf_F = (double *)malloc(sizeof(double) * (size_t)(n_old > 0 ? n_old : 1));
  s->pf_n = n_old;
  for (int k = 0; k < n_old; ++k) {
    double F = S[k];
    for (int j = 1; j < Rw; ++j) F = fuse2(c->fusion, F, S[(size_t)j * N + k]);
    s->pf_F[k] = F;
  }

  /* keep the min(C, n_old) best; ties keep the lower position */
  const int keep = n_old < C ? n_old : C;
  int32_t *kept = (int32_t *)malloc(sizeof(int32_t) * (size_t)(keep > 0 ? keep : 1));
  if (forced) {
    for (int i = 0; i < keep; ++i) {
      kept[i] = forced[i];
      if (kept[i] < 0 || kept[i] >= n_old) { free(kept); free(S); return MORPHKV_REF_EINVAL; }
    }
  } else {
    cand_t *cd = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n_old > 0 ? n_old : 1));
    for (int k = 0; k < n_old; ++k) { cd[k].F = s->pf_F[k]; cd[k].pos = k; cd[k].idx = k; }
    qsort(cd, (size_t)n_old, sizeof(cand_t), cand_cmp);
    for (int i = 0; i < keep; ++i) kept[i] = cd[i].pos;
    free(cd);
  }
  qsort(kept, (size_t)keep, sizeof(int32_t), i32_cmp);

  /* fill the cache */
  s->n_snap = keep;
  for (int i = 0; i < Cs; ++i) s->pos_s[i] = -1;
  for (int i = 0; i < keep; ++i) {
    s->pos_s[i] = kept[i];
    s->cum[i] = s->pf_F[kept[i]]; /* used by the running-sum policy only: there F is the sum over the rows */
    for (int e = 0; e < d; ++e) {
      s->Ks[(size_t)i * d + e] = ld(K, kbase + (size_t)kept[i] * d + e, dt);
      s->Vs[(size_t)i * d + e] = ld(V, kbase + (size_t)kept[i] * d + e, dt);
    }
  }
  for (int w = 0; w < R; ++w) s->pos_w[w] = -1;
  for (int k = n_old; k < N; ++k) {
    const int w = k % R;
    s->pos_w[w] = k;
    for (int e = 0; e < d; ++e) {
      s->Kw[(size_t)w * d + e] = ld(K, kbase + (size_t)k * d + e, dt);
      s->Vw[(size_t)w * d + e] = ld(V, kbase + (size_t)k * d + e, dt);
    }
  }
  /* the recorded rows of the window queries, restricted to what is resident */
  memset(s->row, 0, sizeof(double) * (size_t)R * W);
  for (int r = 0; r < R; ++r) s->row_q[r] = -1;
  for (int j = 0; j < Rw; ++j) {
    const int pj = N - Rw + j, r = pj % R;
    s->row_q[r] = pj;
    for (int i = 0; i < keep; ++i) s->row[(size_t)r * W + i] = S[(size_t)j * N + kept[i]];
    for (int k = n_old; k <= pj; ++k) s->row[(size_t)r * W + Cs + (k % R)] = S[(size_t)j * N + k];
  }
  s->next_pos = N;
  s->prompt_len = N;
  s->pending = 0;
  free(kept);
  free(S);
  return MORPHKV_REF_OK;
}

int morphkv_ref_prefill_select(morphkv_ref *h, const void *Qw, const void *K, const void *V,
                               const int32_t *prompt_len, int32_t Nmax, const int32_t *forced_pos) {
  if (!h || !Qw || !K || !V || !prompt_len) return MORPHKV_REF_EINVAL;
  const morphkv_ref_config *c = &h->c;
  for (int b = 0; b < c->batch; ++b)
    if (prompt_len[b] < 1 || prompt_len[b] > Nmax) return MORPHKV_REF_EINVAL;
  int rc = MORPHKV_REF_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int u = 0; u < h->U; ++u) {
    const int kh = u % c->n_kv_heads, lb = u / c->n_kv_heads, b = lb % c->batch, l = lb / c->batch;
    int r = prefill_unit(h, l, b, kh, Qw, K, V, prompt_len[b], Nmax,
                         forced_pos ? forced_pos + (size_t)u * c->C : NULL);
    if (r != MORPHKV_REF_OK) {
#pragma omp critical
      rc = r;
    }
  }
  return rc;
}

int morphkv_ref_prefill_scores(morphkv_ref *h, int32_t unit, double *F, int32_t capacity) {
  if (!h || unit < 0 || unit >= h->U) return MORPHKV_REF_EINVAL;
  unit_t *s = &h->u[unit];
  if (s->next_pos < 0) return MORPHKV_REF_ESTATE;
  if (F) {
    if (capacity < s->pf_n) return MORPHKV_REF_EINVAL;
    memcpy(F, s->pf_F, sizeof(double) * (size_t)s->pf_n);
  }
  return s->pf_n;
}

/* ---- decode, first half: Eq.1 over the resident cache + self; record; fuse; decide ---- */
static void decode_begin_unit(morphkv_ref *h, int l, int b, int kh, const void *q, const void *kn, const void *vn,
                              double *out) {
  const morphkv_ref_config *c = &h->c;
  const int d = c->head_dim, R = c->R, G = h->G, C = c->C, Cs = h->Cs, W = h->W, dt = c->dtype, T = c->evict_every;
  const int u = (l * c->batch + b) * c->n_kv_heads + kh;
  unit_t *s = &h->u[u];
  const int p = s->next_pos, w = p % R;
  const size_t nbase = (size_t)u * d;
  for (int e = 0; e < d; ++e) { s->k_new[e] = ld(kn, nbase + e, dt); s->v_new[e] = ld(vn, nbase + e, dt); }

  /* resident tokens: column index (in a recorded row), key, value */
  const int n_res_max = Cs + R;
  int32_t *col = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_res_max);
  const double **kp = (const double **)malloc(sizeof(double *) * (size_t)n_res_max);
  const double **vp = (const double **)malloc(sizeof(double *) * (size_t)n_res_max);
  int nr = 0;
  for (int i = 0; i < s->n_snap; ++i) { col[nr] = i; kp[nr] = s->Ks + (size_t)i * d; vp[nr] = s->Vs + (size_t)i * d; ++nr; }
  for (int x = 0; x < R; ++x)
    if (s->pos_w[x] >= 0) { col[nr] = Cs + x; kp[nr] = s->Kw + (size_t)x * d; vp[nr] = s->Vw + (size_t)x * d; ++nr; }

  double *S = (double *)calloc((size_t)nr + 1, sizeof(double)); /* group-summed weights */
  double *pr = (double *)malloc(sizeof(double) * ((size_t)nr + 1));
  for (int g = 0; g < G; ++g) {
    const size_t qbase = ((size_t)(l * c->batch + b) * c->n_q_heads + (kh * G + g)) * d;
    double m = -INFINITY;
    for (int j = 0; j <= nr; ++j) { /* j == nr is the new token itself */
      const double *kk = j < nr ? kp[j] : s->k_new;
      double acc = 0.0;
      for (int e = 0; e < d; ++e) acc += ld(q, qbase + e, dt) * kk[e];
      pr[j] = acc * h->scale;
      if (pr[j] > m) m = pr[j];
    }
    double z = 0.0;
    for (int j = 0; j <= nr; ++j) { pr[j] = exp(pr[j] - m); z += pr[j]; }
    for (int j = 0; j <= nr; ++j) pr[j] /= z;
    for (int e = 0; e < d; ++e) {
      double o = 0.0;
      for (int j = 0; j < nr; ++j) o += pr[j] * vp[j][e];
      o += pr[nr] * s->v_new[e];
      out[qbase + e] = o;
    }
    for (int j = 0; j < nr; ++j) S[j] += pr[j];
  }

  /* record the row of query p (the self weight has no column) */
  double *rw = s->row + (size_t)w * W;
  memset(rw, 0, sizeof(double) * (size_t)W);
  for (int j = 0; j < nr; ++j) rw[col[j]] = S[j];
  s->row_q[w] = p;
  for (int j = 0; j < nr; ++j)
    if (col[j] < Cs) s->S_last[col[j]] = S[j]; /* what this query adds to the running sums */

  /* the window slides: token p-R (slot w) becomes an older token.  Fuse and decide. */
  s->n_cand = 0;
  s->n_evict = 0;
  for (int i = 0; i < T; ++i) s->choice[i] = -1;
  const int demote = s->pos_w[w] >= 0; /* slot w holds token p-R */
  /* selection at every T-th generation step (Appendix A.5): token p is number p - N + 1 of the response */
  if (demote && T >= 1 && ((p - s->prompt_len + 1) % T) == 0 && s->n_snap + 1 > C) {
    int nc = 0;
    for (int i = 0; i < s->n_snap; ++i) { s->cand_pos[nc] = s->pos_s[i]; s->cand_col[nc] = i; ++nc; }
    s->cand_pos[nc] = s->pos_w[w]; s->cand_col[nc] = Cs + w; ++nc;
    for (int i = 0; i < nc; ++i) {
      int first = 1;
      double F = 0.0;
      for (int r = 0; r < R; ++r) {
        if (s->row_q[r] < 0 || s->row_q[r] <= p - R) continue; /* only rows of the window's queries */
        const double v = s->row[(size_t)r * W + s->cand_col[i]];
        F = first ? v : fuse2(c->fusion, F, v);
        first = 0;
      }
      /* running-sum policy: an older token's score is everything recorded for it so far; the token leaving
         the window has been seen by exactly the window's queries, whose rows were just summed */
      if (c->fusion == 2 && i < s->n_snap) F = s->cum[i] + s->S_last[i];
      s->cand_F[i] = F;
    }
    s->n_cand = nc;
    s->n_evict = nc - C;
    cand_t *cd = (cand_t *)malloc(sizeof(cand_t) * (size_t)nc);
    for (int i = 0; i < nc; ++i) { cd[i].F = s->cand_F[i]; cd[i].pos = s->cand_pos[i]; cd[i].idx = i; }
    qsort(cd, (size_t)nc, sizeof(cand_t), cand_cmp); /* best first; the last n_evict go */
    for (int i = 0; i < s->n_evict; ++i) s->choice[i] = cd[nc - 1 - i].pos;
    free(cd);
  }
  s->pending = 1;
  free(S); free(pr); free(col); free(kp); free(vp);
}

int morphkv_ref_decode_begin(morphkv_ref *h, const void *q, const void *k_new, const void *v_new, double *out) {
  if (!h || !q || !k_new || !v_new || !out) return MORPHKV_REF_EINVAL;
  const morphkv_ref_config *c = &h->c;
  for (int u = 0; u < h->U; ++u)
    if (h->u[u].next_pos < 0 || h->u[u].pending) return MORPHKV_REF_ESTATE;
#pragma omp parallel for schedule(dynamic, 1)
  for (int u = 0; u < h->U; ++u) {
    const int kh = u % c->n_kv_heads, lb = u / c->n_kv_heads, b = lb % c->batch, l = lb / c->batch;
    decode_begin_unit(h, l, b, kh, q, k_new, v_new, out);
  }
  return MORPHKV_REF_OK;
}

int morphkv_ref_candidates(morphkv_ref *h, int32_t *n_cand, int32_t *cand_pos, double *cand_F,
                           int32_t *n_evict, int32_t *choice) {
  if (!h) return MORPHKV_REF_EINVAL;
  const int stride = h->Cs + 1, T = h->c.evict_every;
  for (int u = 0; u < h->U; ++u) {
    unit_t *s = &h->u[u];
    if (!s->pending) return MORPHKV_REF_ESTATE;
    if (n_cand) n_cand[u] = s->n_cand;
    if (n_evict) n_evict[u] = s->n_evict;
    if (cand_pos) memcpy(cand_pos + (size_t)u * stride, s->cand_pos, sizeof(int32_t) * (size_t)s->n_cand);
    if (cand_F) memcpy(cand_F + (size_t)u * stride, s->cand_F, sizeof(double) * (size_t)s->n_cand);
    if (choice) memcpy(choice + (size_t)u * T, s->choice, sizeof(int32_t) * (size_t)T);
  }
  return MORPHKV_REF_OK;
}

/* ---- decode, second half: Eq.7 applied; new token enters the window ---- */
static int decode_commit_unit(morphkv_ref *h, int u, const int32_t *ev /* [T] or NULL */) {
  const morphkv_ref_config *c = &h->c;
  const int d = c->head_dim, R = c->R, Cs = h->Cs, W = h->W;
  unit_t *s = &h->u[u];
  const int p = s->next_pos, w = p % R;
  const int32_t *E = ev ? ev : s->choice;
  const int demote = s->pos_w[w] >= 0;
  for (int j = 0; j < s->n_snap; ++j) s->cum[j] += s->S_last[j];
  if (demote) {
    /* mark what goes */
    int drop_demoted = 0, n_marked = 0;
    char *gone = (char *)calloc((size_t)Cs, 1);
    for (int i = 0; i < s->n_evict; ++i) {
      const int32_t e = E[i];
      int found = 0;
      if (e == s->pos_w[w]) { if (!drop_demoted) { drop_demoted = 1; found = 1; } }
      else
        for (int j = 0; j < s->n_snap; ++j)
          if (s->pos_s[j] == e && !gone[j]) { gone[j] = 1; found = 1; break; }
      if (!found) { free(gone); return MORPHKV_REF_EINVAL; }
      ++n_marked;
    }
    /* compact the older tokens, order preserved; columns of the recorded rows move with them */
    int n = 0;
    for (int j = 0; j < s->n_snap; ++j) {
      if (gone[j]) continue;
      if (n != j) {
        s->pos_s[n] = s->pos_s[j];
        s->cum[n] = s->cum[j];
        memcpy(s->Ks + (size_t)n * d, s->Ks + (size_t)j * d, sizeof(double) * (size_t)d);
        memcpy(s->Vs + (size_t)n * d, s->Vs + (size_t)j * d, sizeof(double) * (size_t)d);
        for (int r = 0; r < R; ++r) s->row[(size_t)r * W + n] = s->row[(size_t)r * W + j];
      }
      ++n;
    }
    free(gone);
    if (!drop_demoted) { /* token p-R joins the older tokens */
      if (n >= Cs) return MORPHKV_REF_ESTATE;
      s->pos_s[n] = s->pos_w[w];
      memcpy(s->Ks + (size_t)n * d, s->Kw + (size_t)w * d, sizeof(double) * (size_t)d);
      memcpy(s->Vs + (size_t)n * d, s->Vw + (size_t)w * d, sizeof(double) * (size_t)d);
      s->cum[n] = 0.0;
      for (int r = 0; r < R; ++r) {
        s->row[(size_t)r * W + n] = s->row[(size_t)r * W + Cs + w];
        if (s->row_q[r] >= 0 && s->row_q[r] > p - R) s->cum[n] += s->row[(size_t)r * W + n];
      }
      ++n;
    }
    for (int j = n; j < Cs; ++j) s->pos_s[j] = -1;
    s->n_snap = n;
    (void)n_marked;
  }
  s->pos_w[w] = p;
  memcpy(s->Kw + (size_t)w * d, s->k_new, sizeof(double) * (size_t)d);
  memcpy(s->Vw + (size_t)w * d, s->v_new, sizeof(double) * (size_t)d);
  s->next_pos = p + 1;
  s->pending = 0;
  return MORPHKV_REF_OK;
}

int morphkv_ref_decode_commit_multi(morphkv_ref *h, const int32_t *evict_pos) {
  if (!h) return MORPHKV_REF_EINVAL;
  const int T = h->c.evict_every;
  for (int u = 0; u < h->U; ++u)
    if (!h->u[u].pending) return MORPHKV_REF_ESTATE;
  int rc = MORPHKV_REF_OK;
  for (int u = 0; u < h->U; ++u) {
    int r = decode_commit_unit(h, u, evict_pos ? evict_pos + (size_t)u * T : NULL);
    if (r != MORPHKV_REF_OK) rc = r;
  }
  return rc;
}

int morphkv_ref_decode_commit(morphkv_ref *h, const int32_t *evict_pos) {
  if (!h) return MORPHKV_REF_EINVAL;
  if (evict_pos && h->c.evict_every != 1) return MORPHKV_REF_EINVAL;
  return morphkv_ref_decode_commit_multi(h, evict_pos);
}

int morphkv_ref_decode_step(morphkv_ref *h, const void *q, const void *k_new, const void *v_new, double *out) {
  int rc = morphkv_ref_decode_begin(h, q, k_new, v_new, out);
  if (rc != MORPHKV_REF_OK) return rc;
  return morphkv_ref_decode_commit_multi(h, NULL);
}

int morphkv_ref_row_stride(morphkv_ref *h) { return h ? h->W : MORPHKV_REF_EINVAL; }

int morphkv_ref_export_positions(morphkv_ref *h, int32_t *pos, int32_t *n_snap, int32_t *n_win) {
  if (!h || !pos || !n_snap) return MORPHKV_REF_EINVAL;
  const int R = h->c.R, W = h->W;
  for (int u = 0; u < h->U; ++u) {
    unit_t *s = &h->u[u];
    int32_t *o = pos + (size_t)u * W;
    int n = 0;
    for (int j = 0; j < s->n_snap; ++j) o[n++] = s->pos_s[j];
    qsort(o, (size_t)n, sizeof(int32_t), i32_cmp);
    int nw = 0;
    for (int x = 0; x < R; ++x)
      if (s->pos_w[x] >= 0) { o[n + nw] = s->pos_w[x]; ++nw; }
    qsort(o + n, (size_t)nw, sizeof(int32_t), i32_cmp);
    for (int j = n + nw; j < W; ++j) o[j] = -1;
    n_snap[u] = s->n_snap;
    if (n_win) n_win[u] = nw;
  }
  return MORPHKV_REF_OK;
}
