/*
 * CPU oracle for Adaptive Dynamic Sparse Attention (ADSA) decode -- TEST INFRASTRUCTURE.
 *
 * A plain, slow, single-threaded, fp64 statement of what one ADSA decode step
 * computes, written from the paper (Section 4.1 "Adaptive Dynamic Sparse
 * Attention", Eq. 1-5, and Section 4.2 "Dynamic Sparse KV-Cache Updating").
 * It exists only so that tests, the smoke check and the benchmark's CPU
 * baseline have something independent to compare the HIP library against.
 * It shares no code, header, table or helper with the HIP path, and the
 * product never calls it.
 *
 * One call works on ONE sequence of ONE layer.  The cache is caller-owned:
 *   K, V    float [cap][n_heads][head_dim]   (values already rounded to the storage type)
 *   pos     int32 [cap]   absolute position of each resident slot, strictly ascending
 *   score   float [cap]   ranking score of each resident slot (fp32 storage)
 *   n_res   resident slots
 * All arithmetic is fp64; `score` is rounded to fp32 once per update because
 * fp32 is its storage type at the library boundary.
 *
 * Readings of the paper taken here (the paper is silent or inconsistent):
 *  - Partition (Eq. 1): PREFIX = positions < n_keep_prefix.  LOCAL is the 2-D
 *    neighbourhood the workload list prescribes, anchored at the query token's own
 *    grid cell (r,c): the current row so far, plus rows r-R..r-1 within +-w
 *    columns (no wrap-around).  With w >= W-1 it is the paper's 1-D "most
 *    recent m tokens".  Everything else is a CANDIDATE ("previous").
 *  - Eq. 2-4 range over the candidate set only: N = |candidates|, S_i is the
 *    mean over the other N-1 candidates (Eq. 3's "t" read as N), N = 1 gives 0.
 *    Zero-norm v: v/max(|v|, 1e-8).  The V vector of a token is the
 *    concatenation over heads (one selection shared by all heads).
 *  - Direction: keep the LOWEST mean cosine (Eq. 4 argmin; Section 4.2 evicts
 *    the most similar).  The sentence after Eq. 5 that says the least similar
 *    are discarded is taken as a slip.
 *  - Ties: the lower slot index is kept first (so Eq. 4's argmin is the
 *    lexicographically smallest optimal subset).  -0 == +0.
 *  - ATTN_MASS (not in the paper; the workload list's ranking): every attended
 *    slot gains the softmax probability it received, summed over heads in
 *    ascending head order; no decay; a new slot starts at 0.
 *  - Eviction runs when the query token closes a grid row (batched form of
 *    Section 4.2's evict-before-insert): keep PREFIX, the last R completed
 *    rows (every later window needs them), and the top min(B,|rest|) of the
 *    rest by the same ranking; survivors move to the front in order.
 *  - Budget B counts global tokens only; B = floor((P+s)*num/den) if den > 0.
 *  - Grouped-query attention (not in the paper, whose models have one query head per cache head):
 *    the usual definition, query head j attends with cache head floor(j/G); the selection stays one
 *    per sequence and ATTN_MASS sums the probabilities of all query heads.
 *  - evict_when_full (Section 4.2 as written): requires the 1-D window (win_recent_m > 0), for which
 *    a token that leaves the window never re-enters it, so evicting any candidate is safe.
 *  - 1-D window (win_recent_m > 0) with the per-row eviction: the local region is exempt from
 *    eviction like the prefix (Table 3: dropping it is catastrophic), so the row-end eviction keeps,
 *    instead of the last R rows, every token a window of the NEXT row contains: image tokens
 *    j > jq + 1 - m for the row-closing query jq (the next row's first query reaches back furthest).
 *
 * parity unpinned: the ATTN_MASS values themselves and the split of a context
 * length into prefix / window / budget are not in the paper; they are pinned
 * only by invariants (tests), not by a published number.
 */
#ifndef ADSA_ORACLE_H
#define ADSA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_PREFIX = 0, ORC_LOCAL = 1, ORC_CANDIDATE = 2 };
enum { ORC_SCORE_ATTN_MASS = 0, ORC_SCORE_VCOS = 1, ORC_SCORE_EXT_LARGEST = 2, ORC_SCORE_EXT_SMALLEST = 3 };

typedef struct {
  int32_t n_heads, head_dim;
  int32_t grid_h, grid_w;
  int32_t win_rows_back;   /* R */
  int32_t win_col_radius;  /* w */
  int32_t grid_origin;     /* P: absolute position of image token 0 */
  int32_t n_keep_prefix;   /* leading positions that are never dropped */
  int32_t budget;          /* B when budget_den == 0 */
  int32_t budget_num, budget_den;
  int32_t score_mode;
  int32_t cap;
  int32_t win_recent_m;    /* > 0: the paper's own 1-D window, local = the m most recent image tokens
                              (query included), instead of the 2-D neighbourhood */
  int32_t evict_when_full; /* 1: the paper's own cache policy (Section 4.2): when the cache holds `cap`
                              entries, evict the single most redundant candidate BEFORE inserting the
                              new token; 0: evict once per completed grid row */
  int32_t q_per_kv;        /* G > 1: grouped-query attention, n_heads*G query heads, query head j reads
                              cache head floor(j/G); 0 or 1: one query head per cache head */
  double  softmax_scale;   /* 0 => 1/sqrt(head_dim) */
} orc_cfg;

/* Eq. 1: class of every resident slot for the query of decode step s. */
int orc_classify(const orc_cfg* c, int32_t n_res, const int32_t* pos, int32_t s, int32_t* cls);

/* Eq. 2-3 literally: pairwise cosines of the listed V rows (dim = n_heads*head_dim), S_ii = 0,
   mean over the other members.  S is double [n]. */
int orc_vcos(const orc_cfg* c, const float* V, int32_t n, const int32_t* slots, double* S);

/* Eq. 4: from the listed slots keep min(B, n) by score (largest or smallest first),
   lower slot first among equals.  keep[n] gets 0/1.  Returns the number kept. */
int orc_rank_keep(int32_t n, const int32_t* slots, const float* score, int keep_largest, int32_t B,
                  uint8_t* keep);

/* Effective budget of step s. */
int32_t orc_budget(const orc_cfg* c, int32_t s);

/* Steps 2-4 of a decode step: the attended set PREFIX u LOCAL u GLOBAL, ascending slots.
   VCOS mode writes S_i (rounded to float) into score[] at candidate slots first. */
int orc_select(const orc_cfg* c, int32_t n_res, const int32_t* pos, float* score, const float* V,
               int32_t s, int32_t* sel_idx, int32_t* sel_cnt);

/* Eq. 5 + softmax attention over the listed slots, per query head (hq = n_heads * max(q_per_kv, 1)
   of them; q float [hq][D]).  out double [hq][D], lse double [hq], probs double [hq][sel_cnt] (may be NULL). */
int orc_attend(const orc_cfg* c, const float* K, const float* V, const float* q,
               const int32_t* sel_idx, int32_t sel_cnt, double* out, double* lse, double* probs);

/* ATTN_MASS update from probs [hq][sel_cnt]: every query head's probability counts. */
int orc_accumulate(const orc_cfg* c, float* score, const int32_t* sel_idx, int32_t sel_cnt,
                   const double* probs);

/* Section 4.2, per-row form: keep_map[i] = new slot or -1 for i < n_res; moves K,V,pos,score.
   No-op returning 0 with *did = 0 unless step s closes a grid row. */
int orc_compact(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t* n_res,
                int32_t s, int32_t* keep_map, int32_t* did);

/* Section 4.2 literally: if the cache is full (n_res == cap) and a token is about to be inserted
   (s >= 1), rank the candidates of the incoming query's partition (prefix and the m-1 most recent
   tokens are exempt), evict the ONE ranked last (highest mean cosine; among equals the highest slot),
   close the hole keeping the order.  keep_map as in orc_compact; *did = 1 if a token was evicted. */
int orc_evict_one(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t* n_res,
                  int32_t s, int32_t* keep_map, int32_t* did);

/* One whole decode step (append, select, attend, accumulate, row-end compact), or with
   evict_when_full: (evict one if full, append, select, attend, accumulate).
   Returns 0, or a negative code (-1 bad argument, -2 capacity overflow). */
int orc_step(const orc_cfg* c, float* K, float* V, int32_t* pos, float* score, int32_t* n_res,
             int32_t s, const float* q, const float* k_new, const float* v_new,
             double* out, double* lse, int32_t* sel_idx, int32_t* sel_cnt,
             int32_t* keep_map, int32_t* did_compact);

#ifdef __cplusplus
}
#endif
#endif
