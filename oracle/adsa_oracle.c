/*
 * CPU oracle for ADSA decode -- TEST INFRASTRUCTURE, see adsa_oracle.h for the
 * readings of the paper it fixes.  Plain C, one thread, fp64, no blocking, no
 * fusion: each function is the corresponding passage of the paper written out.
 */
#include "adsa_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

static int keep_largest_of(int mode) {
  return mode == ORC_SCORE_ATTN_MASS || mode == ORC_SCORE_EXT_LARGEST;
}

/* query heads per cache head (grouped-query attention); 0 means 1 */
static int32_t q_per_kv(const orc_cfg* c) { return c->q_per_kv > 1 ? c->q_per_kv : 1; }

int32_t orc_budget(const orc_cfg* c, int32_t s) {
  if (c->budget_den > 0) {
    int64_t L = (int64_t)c->grid_origin + s;
    return (int32_t)((L * c->budget_num) / c->budget_den);
  }
  return c->budget;
}

/* Section 4.1, Eq. 1: [prefix | previous | local]; local is the 2-D neighbourhood of
   the query token's own cell. */
int orc_classify(const orc_cfg* c, int32_t n_res, const int32_t* pos, int32_t s, int32_t* cls) {
  if (s < 0 || s > c->grid_h * c->grid_w) return -1;
  int32_t P = c->grid_origin, W = c->grid_w, R = c->win_rows_back, w = c->win_col_radius;
  int32_t jq = s - 1, r = 0, col = 0;
  if (s >= 1) { r = jq / W; col = jq % W; }
  for (int32_t i = 0; i < n_res; ++i) {
    if (pos[i] < c->n_keep_prefix) { cls[i] = ORC_PREFIX; continue; }
    if (pos[i] < P) { cls[i] = ORC_CANDIDATE; continue; }   /* unpinned condition token */
    if (s == 0) return -1;                                   /* image entry before any image step */
    int32_t j = pos[i] - P;
    if (j > jq) return -1;                                   /* entry from the future */
    int32_t rj = j / W, cj = j % W;
    int local = 0;
    if (c->win_recent_m > 0) {                               /* Section 4.1: the most recent m tokens */
      local = j > jq - c->win_recent_m;
    } else {
      if (rj == r) local = 1;                                /* current row so far */
      else if (rj >= r - R && rj <= r - 1 && abs(cj - col) <= w) local = 1;
    }
    cls[i] = local ? ORC_LOCAL : ORC_CANDIDATE;
  }
  return 0;
}

/* Eq. 2: S_ij = v_i.v_j / (|v_i||v_j|), S_ii = 0.  Eq. 3: S_i = mean over the other members. */
int orc_vcos(const orc_cfg* c, const float* V, int32_t n, const int32_t* slots, double* S) {
  int64_t dim = (int64_t)c->n_heads * c->head_dim;
  double* norm = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  if (!norm) return -1;
  for (int32_t a = 0; a < n; ++a) {
    const float* va = V + (int64_t)slots[a] * dim;
    double ss = 0.0;
    for (int64_t d = 0; d < dim; ++d) ss += (double)va[d] * (double)va[d];
    norm[a] = fmax(sqrt(ss), 1e-8);
  }
  for (int32_t a = 0; a < n; ++a) {
    const float* va = V + (int64_t)slots[a] * dim;
    double sum = 0.0;
    for (int32_t b = 0; b < n; ++b) {
      if (b == a) continue;                                  /* S_ii = 0 */
      const float* vb = V + (int64_t)slots[b] * dim;
      double dot = 0.0;
      for (int64_t d = 0; d < dim; ++d) dot += (double)va[d] * (double)vb[d];
      sum += dot / (norm[a] * norm[b]);
    }
    S[a] = (n > 1) ? sum / (double)(n - 1) : 0.0;
  }
  free(norm);
  return 0;
}

/* Eq. 4 by its definition for a sum objective: sort, take the first B.  Stable insertion
   sort on (priority, slot) so that equal scores keep ascending slot order. */
int orc_rank_keep(int32_t n, const int32_t* slots, const float* score, int keep_largest, int32_t B,
                  uint8_t* keep) {
  if (n <= 0) return 0;
  int32_t* order = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  if (!order) return -1;
  for (int32_t a = 0; a < n; ++a) {       /* slots[] is ascending, so index order == slot order */
    float sa = score[slots[a]];
    int32_t p = a;
    while (p > 0) {
      float sb = score[slots[order[p - 1]]];
      int before = keep_largest ? (sa > sb) : (sa < sb);    /* strict: ties stay in slot order */
      if (!before) break;
      order[p] = order[p - 1];
      --p;
    }
    order[p] = a;
  }
  int32_t nk = B < n ? (B < 0 ? 0 : B) : n;
  memset(keep, 0, (size_t)n);
  for (int32_t t = 0; t < nk; ++t) keep[order[t]] = 1;
  free(order);
  return nk;
}

int orc_select(const orc_cfg* c, int32_t n_res, const int32_t* pos, float* score, const float* V,
               int32_t s, int32_t* sel_idx, int32_t* sel_cnt) {
  int32_t* cls = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_res + 1));
  int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_res + 1));
  uint8_t* keep = (uint8_t*)malloc((size_t)(n_res + 1));
  if (!cls || !cand || !keep) return -1;
  int rc = orc_classify(c, n_res, pos, s, cls);
  if (rc) { free(cls); free(cand); free(keep); return rc; }
  int32_t nc = 0;
  for (int32_t i = 0; i < n_res; ++i) if (cls[i] == ORC_CANDIDATE) cand[nc++] = i;
  if (c->score_mode == ORC_SCORE_VCOS) {
    double* S = (double*)malloc(sizeof(double) * (size_t)(nc + 1));
    if (!S) return -1;
    orc_vcos(c, V, nc, cand, S);
    for (int32_t a = 0; a < nc; ++a) score[cand[a]] = (float)S[a];
    free(S);
  }
  orc_rank_keep(nc, cand, score, keep_largest_of(c->score_mode), orc_budget(c, s), keep);
  int32_t cnt = 0, a = 0;
  for (int32_t i = 0; i < n_res; ++i) {
    if (cls[i] == ORC_CANDIDATE) { if (keep[a]) sel_idx[cnt++] = i; ++a; }
    else sel_idx[cnt++] = i;
  }
  *sel_cnt = cnt;
  free(cls); free(cand); free(keep);
  return 0;
}

/* Eq. 5 gathers K_select, V_select; then scaled dot-product attention per head. */
int orc_attend(const orc_cfg* c, const float* K, const float* V, const float* q,
               const int32_t* sel_idx, int32_t sel_cnt, double* out, double* lse, double* probs) {
  int32_t h = c->n_heads, D = c->head_dim, G = q_per_kv(c);
  double scale = c->softmax_scale != 0.0 ? c->softmax_scale : 1.0 / sqrt((double)D);
  if (sel_cnt <= 0) return -1;
  double* z = (double*)malloc(sizeof(double) * (size_t)sel_cnt);
  if (!z) return -1;
  for (int32_t hh = 0; hh < h * G; ++hh) {               /* hh: query head; it reads cache head hh / G */
    const float* qh = q + (int64_t)hh * D;
    const int32_t hk = hh / G;
    double m = -INFINITY;
    for (int32_t t = 0; t < sel_cnt; ++t) {
      const float* kr = K + ((int64_t)sel_idx[t] * h + hk) * D;
      double dot = 0.0;
      for (int32_t d = 0; d < D; ++d) dot += (double)qh[d] * (double)kr[d];
      z[t] = dot * scale;
      if (z[t] > m) m = z[t];
    }
    double denom = 0.0;
    for (int32_t t = 0; t < sel_cnt; ++t) denom += exp(z[t] - m);
    for (int32_t d = 0; d < D; ++d) out[(int64_t)hh * D + d] = 0.0;
    for (int32_t t = 0; t < sel_cnt; ++t) {
      double p = exp(z[t] - m) / denom;
      if (probs) probs[(int64_t)hh * sel_cnt + t] = p;
      const float* vr = V + ((int64_t)sel_idx[t] * h + hk) * D;
      for (int32_t d = 0; d < D; ++d) out[(int64_t)hh * D + d] += p * (double)vr[d];
    }
    lse[hh] = m + log(denom);
  }
  free(z);
  return 0;
}

int orc_accumulate(const orc_cfg* c, float* score, const int32_t* sel_idx, int32_t sel_cnt,
                   const double* probs) {
  for (int32_t t = 0; t < sel_cnt; ++t) {
    double inc = 0.0;
    for (int32_t hh = 0; hh < c->n_heads * q_per_kv(c); ++hh) inc += probs[(int64_t)hh * sel_cnt + t];
    score[sel_idx[t]] = (float)((double)score[sel_idx[t]] + inc);
  }
  return 0;
}

/* stable removal of the slots with flag == 0 */
static void move_kept(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t n,
                      const uint8_t* flag, int32_t* keep_map, int32_t* n_out) {
  int64_t row = (int64_t)c->n_heads * c->head_dim;
  int32_t dst = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (!flag[i]) { keep_map[i] = -1; continue; }
    keep_map[i] = dst;
    if (dst != i) {
      memcpy(K + (int64_t)dst * row, K + (int64_t)i * row, sizeof(float) * (size_t)row);
      memcpy(V + (int64_t)dst * row, V + (int64_t)i * row, sizeof(float) * (size_t)row);
      pos[dst] = pos[i];
      score[dst] = score[i];
    }
    ++dst;
  }
  *n_out = dst;
}

int orc_evict_one(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t* n_res,
                  int32_t s, int32_t* keep_map, int32_t* did) {
  int32_t n = *n_res;
  *did = 0;
  if (s < 1 || s > c->grid_h * c->grid_w || n < c->cap) return 0;   /* not full: behave like the baseline */
  int32_t* cls = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 1));
  int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 1));
  uint8_t* keep = (uint8_t*)malloc((size_t)(n + 1));
  uint8_t* flag = (uint8_t*)malloc((size_t)(n + 1));
  if (!cls || !cand || !keep || !flag) return -1;
  /* partition for the token about to be inserted: it will be the newest member of the local region */
  int rc = orc_classify(c, n, pos, s, cls);
  if (rc) return rc;
  int32_t nc = 0;
  for (int32_t i = 0; i < n; ++i) { flag[i] = 1; if (cls[i] == ORC_CANDIDATE) cand[nc++] = i; }
  if (nc == 0) { free(cls); free(cand); free(keep); free(flag); return 0; }   /* nothing may go */
  if (c->score_mode == ORC_SCORE_VCOS) {
    double* S = (double*)malloc(sizeof(double) * (size_t)nc);
    if (!S) return -1;
    orc_vcos(c, V, nc, cand, S);
    for (int32_t a = 0; a < nc; ++a) score[cand[a]] = (float)S[a];
    free(S);
  }
  orc_rank_keep(nc, cand, score, keep_largest_of(c->score_mode), nc - 1, keep);   /* all but the last-ranked */
  for (int32_t a = 0; a < nc; ++a) flag[cand[a]] = keep[a];
  move_kept(c, K, V, pos, score, n, flag, keep_map, n_res);
  *did = 1;
  free(cls); free(cand); free(keep); free(flag);
  return 0;
}

int orc_compact(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t* n_res,
                int32_t s, int32_t* keep_map, int32_t* did) {
  int32_t W = c->grid_w, R = c->win_rows_back, P = c->grid_origin, n = *n_res;
  *did = 0;
  if (c->evict_when_full) return orc_evict_one(c, K, V, pos, score, n_res, s, keep_map, did);
  if (s < 1 || s > c->grid_h * W || (s - 1) % W != W - 1) return 0;
  int32_t r = (s - 1) / W;
  int32_t* rest = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 1));
  uint8_t* flag = (uint8_t*)malloc((size_t)(n + 1));
  uint8_t* keep = (uint8_t*)malloc((size_t)(n + 1));
  if (!rest || !flag || !keep) return -1;
  int32_t nr = 0;
  rest[0] = 0;
  for (int32_t i = 0; i < n; ++i) {
    int protect = 0;
    if (pos[i] < c->n_keep_prefix) protect = 1;
    else if (pos[i] >= P) {
      int32_t j = pos[i] - P, rj = j / W;
      if (c->win_recent_m > 0) {                             /* 1-D window (Section 4.1): the next row's queries */
        if (j > (s - 1) + 1 - c->win_recent_m) protect = 1;  /* s .. s+W-1 see j > query - m; the first reaches furthest back */
      } else if (rj >= r - R + 1 && rj <= r) protect = 1;    /* rows the next windows need */
    }
    flag[i] = (uint8_t)protect;
    if (!protect) rest[nr++] = i;
  }
  if (c->score_mode == ORC_SCORE_VCOS) {                     /* Section 4.2: Eq. 2-3 over the rest */
    double* S = (double*)malloc(sizeof(double) * (size_t)(nr + 1));
    if (!S) return -1;
    orc_vcos(c, V, nr, rest, S);
    for (int32_t a = 0; a < nr; ++a) score[rest[a]] = (float)S[a];
    free(S);
  }
  orc_rank_keep(nr, rest, score, keep_largest_of(c->score_mode), orc_budget(c, s), keep);
  for (int32_t a = 0; a < nr; ++a) flag[rest[a]] = keep[a];
  move_kept(c, K, V, pos, score, n, flag, keep_map, n_res);
  *did = 1;
  free(rest); free(flag); free(keep);
  return 0;
}

int orc_step(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t* n_res,
             int32_t s, const float* q, const float* k_new, const float* v_new,
             double* out, double* lse, int32_t* sel_idx, int32_t* sel_cnt,
             int32_t* keep_map, int32_t* did_compact) {
  int64_t row = (int64_t)c->n_heads * c->head_dim;
  if (s < 0 || s > c->grid_h * c->grid_w) return -1;
  *did_compact = 0;
  if (c->evict_when_full) {                                  /* Section 4.2: evict BEFORE inserting */
    int rc0 = orc_evict_one(c, K, V, pos, score, n_res, s, keep_map, did_compact);
    if (rc0) return rc0;
  }
  if (s >= 1) {                                              /* Section 4.2: append at the end */
    if (*n_res + 1 > c->cap) return -2;
    int32_t i = *n_res;
    memcpy(K + (int64_t)i * row, k_new, sizeof(float) * (size_t)row);
    memcpy(V + (int64_t)i * row, v_new, sizeof(float) * (size_t)row);
    pos[i] = c->grid_origin + s - 1;
    score[i] = 0.0f;
    *n_res = i + 1;
  }
  int rc = orc_select(c, *n_res, pos, score, V, s, sel_idx, sel_cnt);
  if (rc) return rc;
  double* probs = (double*)malloc(sizeof(double) * (size_t)c->n_heads * (size_t)q_per_kv(c) * (size_t)(*sel_cnt + 1));
  if (!probs) return -1;
  rc = orc_attend(c, K, V, q, sel_idx, *sel_cnt, out, lse, probs);
  if (!rc && c->score_mode == ORC_SCORE_ATTN_MASS)
    rc = orc_accumulate(c, score, sel_idx, *sel_cnt, probs);
  free(probs);
  if (rc) return rc;
  if (c->evict_when_full) return 0;
  return orc_compact(c, K, V, pos, score, n_res, s, keep_map, did_compact);
}
