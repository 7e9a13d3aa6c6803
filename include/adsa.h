/*
 * adsa.h -- C ABI of the MI355X (gfx950) ADSA decode library.
 *
 * One call processes ONE transformer layer for a batch of independent
 * sequences: the per-step decode attention of Adaptive Dynamic Sparse Attention
 * (paper Section 4.1) restricted to prefix + local window + globally ranked
 * tokens, and the dynamic KV-cache update that evicts and compacts
 * (Section 4.2).  Every entry point only ENQUEUES work on the caller's HIP
 * stream: no host synchronisation, no allocation, no global state (the
 * optional timing hook at the end of this file aside).  The library never
 * touches host memory behind the pointers it is given except `adsa_params`
 * (a host struct, read during the call).
 *
 * Pointers are DEVICE pointers owned by the caller unless marked [host].
 * Return value: ADSA_OK or a negative adsa_status; argument errors are found
 * on the host before anything is launched.  Conditions only the device can see
 * (a full cache, a malformed state) set `adsa_seq.status` of that sequence,
 * which the caller reads when it next synchronises; such a sequence is
 * skipped by every call until the caller clears the status, and its output
 * row is zero-filled.
 *
 * Cache layout.  Element (slot, head, d) of a sequence's K (same for V) lives
 * at  k + slot*kv_slot_stride + head*kv_head_stride + d  (strides in
 * elements).  [head][slot][D] (slot stride = head_dim, head stride >= cap*head_dim):
 * a head's rows are contiguous, one workgroup streams one head -- the fast
 * path; [slot][head][D] (slot stride = n_heads*head_dim, head stride =
 * head_dim) is supported too.  Base pointers must be 16-byte aligned and both
 * strides multiples of 16 bytes.
 *
 * Decode-step convention.  `step` = s = number of image tokens in the context
 * INCLUDING the query token; the query token is image token s-1, at grid cell
 * (row, col) = ((s-1) / grid_w, (s-1) % grid_w) and absolute position
 * grid_origin + s - 1.  s = 0 means the query is the last prefix token
 * (nothing is appended).  0 <= s <= grid_h*grid_w.  A sequence with step < 0
 * is inactive and skipped.
 */
#ifndef ADSA_H
#define ADSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADSA_VERSION 1
#define ADSA_MAX_CAP 8192      /* largest `cap` (slots per sequence) the select/compact kernels accept */
#define ADSA_STATIC_SCRATCH_BYTES (4u << 20)   /* built-in scratch of adsa_step_static, per GPU */

typedef enum {
  ADSA_OK = 0,
  ADSA_ERR_NULL = -1,          /* a required pointer is NULL */
  ADSA_ERR_SHAPE = -2,         /* a size or window parameter is out of range */
  ADSA_ERR_DTYPE = -3,         /* unknown dtype / score mode */
  ADSA_ERR_ALIGN = -4,         /* pointer or stride not 16-byte aligned */
  ADSA_ERR_CAPACITY = -5,      /* cap or sel_cap too small / above ADSA_MAX_CAP */
  ADSA_ERR_WORKSPACE = -6,     /* workspace missing or smaller than adsa_workspace_bytes() */
  ADSA_ERR_LAUNCH = -7,        /* the HIP runtime refused a launch */
  ADSA_ERR_UNSUPPORTED = -8,   /* valid request this build does not implement */
  ADSA_ERR_STATIC_SCRATCH = -9 /* adsa_step_static: these parameters need more than ADSA_STATIC_SCRATCH_BYTES */
} adsa_status;

typedef enum { ADSA_F32 = 0, ADSA_BF16 = 1 } adsa_dtype;

/* How the "previous" tokens are ranked for Eq. 4 (which K of them are kept). */
typedef enum {
  ADSA_SCORE_ATTN_MASS = 0,    /* accumulated softmax probability received so far; keep LARGEST */
  ADSA_SCORE_VCOS = 1,         /* mean pairwise cosine of V (Eq. 2-3) over the candidates; keep SMALLEST */
  ADSA_SCORE_EXT_LARGEST = 2,  /* caller-maintained score[]; keep largest */
  ADSA_SCORE_EXT_SMALLEST = 3, /* caller-maintained score[]; keep smallest */
  ADSA_SCORE_VCOS_FUSED = 4    /* the same Eq. 2-3 ranking as ADSA_SCORE_VCOS for ADSA_EVICT_REUSE_SLOT, without
                                  separate passes over V: the attention launch, which streams every resident
                                  V row anyway, also takes each row's squared norm and its dot product with
                                  the running sum u of the candidates' normalised V vectors (adsa_seq.vcos_u,
                                  kept up to date by adsa_compact: minus the evicted row, plus the row that
                                  leaves the local window next).  The next eviction ranks from those numbers.
                                  Needs [head][slot][D] caches, q_per_kv <= 1, win_recent_m >= 2 and
                                  16*n_heads*head_dim + cap bytes of LDS <= 64 KB (else ADSA_ERR_UNSUPPORTED).  Whenever the running state
                                  does not belong to the step at hand (first use, a cache edited by the
                                  caller) the call falls back to the two-pass computation, so results never
                                  depend on it being warm */
} adsa_score_mode;

/* When the dynamic cache evicts (Section 4.2). */
typedef enum {
  ADSA_EVICT_ROW_END = 0,      /* once per completed grid row: keep prefix + last R rows + top-B of the rest */
  ADSA_EVICT_WHEN_FULL = 1,    /* the paper's own rule: when n_res == cap and a token is about to be inserted,
                                  evict the ONE last-ranked candidate (most redundant) before the insertion;
                                  needs win_recent_m > 0 (a token that left a 1-D window is never local again).
                                  Attention then covers everything resident (Tables 1-2: context == KV cache):
                                  the budget fields are ignored.  The hole is closed: slots stay in position
                                  order, at the price of moving every row behind the hole */
  ADSA_EVICT_REUSE_SLOT = 2    /* the same rule and the same evicted token (among equal scores the newest
                                  position goes), but nothing moves: the evicted slot is recorded in
                                  adsa_seq.hole and the incoming token takes it.  From the first eviction on,
                                  slot order is no longer position order (pos[] says who lives where) */
} adsa_evict_policy;

/* Device-side per-sequence status bits (adsa_seq.status). */
#define ADSA_SEQ_OK            0
#define ADSA_SEQ_CACHE_FULL    1   /* append would exceed cap */
#define ADSA_SEQ_BAD_STATE     2   /* n_res/step out of range, or an entry newer than the query */
#define ADSA_SEQ_SEL_OVERFLOW  4   /* attended set larger than sel_cap */

/* Flags of adsa_select / adsa_attend / adsa_compact / adsa_step. */
#define ADSA_FLAG_NO_COMPACT    1u  /* caller guarantees no sequence closes a grid row in this step */
#define ADSA_FLAG_NO_ACCUMULATE 2u  /* adsa_attend: do not add attention mass to score[] */
#define ADSA_FLAG_PLAN_APPEND   4u  /* adsa_select: reserve slot n_res for the query token (pos, zero score,
                                       n_res += 1, pending_slot) and rank with it in place (it is always
                                       local); its K/V rows arrive with adsa_attend(ADSA_FLAG_APPEND).
                                       Once per decode step */
#define ADSA_FLAG_APPEND        8u  /* adsa_attend: write (k_new, v_new) into pending_slot while attending */
#define ADSA_FLAG_NEW_F32      32u  /* adsa_attend / adsa_step with a bf16 cache: k_new and v_new are fp32
                                       [n_seq][n_heads][head_dim]; each value is rounded to the nearest bf16
                                       (ties to even) once, as it enters the cache, and the launch attends the
                                       rounded row.  No effect with an fp32 cache */
#define ADSA_FLAG_ADVANCE      16u  /* adsa_attend / adsa_compact: step += 1 for every active sequence when
                                       the call is done; give it to the LAST call of a decode step only
                                       (adsa_compact tests the row end on the step before the increment) */

/* [host] Launch-wide parameters (Section 4.1's n, m, K and the problem shape). */
typedef struct adsa_params {
  int32_t n_seq;               /* sequences in this launch (>= 1) */
  int32_t n_heads;             /* key/value (cache) heads; the query has n_heads * max(q_per_kv, 1) heads */
  int32_t head_dim;            /* 64 or 128 */
  int32_t grid_h, grid_w;      /* image-token grid H x W, raster order */
  int32_t win_rows_back;       /* R: rows above the query's row that belong to the local window */
  int32_t win_col_radius;      /* w: column radius in those rows; w >= grid_w-1 gives the paper's
                                  1-D "most recent m tokens" window */
  int32_t sel_groups;          /* 1: one attended set per sequence shared by all heads.
                                  n_heads: one set, and one eviction history, PER (cache) HEAD (Eq. 4 does not say
                                  which).  Every (sequence, head) then is a sequence of one head: `seqs` holds
                                  n_seq * n_heads records, record b * n_heads + h describing head h of sequence b
                                  (k / v point at that head's first row, rows kv_slot_stride apart -- either cache
                                  nesting works, kv_head_stride is not used --, its own pos, score, n_res, step...);
                                  sel_idx, sel_cnt and keep_map carry one row per record ([n_seq][n_heads][...]);
                                  q, k_new, v_new, out, lse keep their layouts.  n_seq * n_heads <= 65535.
                                  Any other value: ADSA_ERR_UNSUPPORTED */
  int32_t dtype;               /* adsa_dtype of q, K, V, out */
  int32_t score_mode;          /* adsa_score_mode */
  int32_t cap;                 /* slots allocated per sequence (<= ADSA_MAX_CAP) */
  int32_t sel_cap;             /* entries per row of sel_idx */
  int64_t kv_slot_stride;      /* elements */
  int64_t kv_head_stride;      /* elements */
  float   softmax_scale;       /* 0 => 1/sqrt(head_dim) */
  int32_t win_recent_m;        /* > 0: the paper's own 1-D local region (Section 4.1), the m most recent image
                                  tokens incl. the query token, instead of the 2-D window (R, w ignored) */
  int32_t evict_policy;        /* adsa_evict_policy */
  int32_t q_per_kv;            /* G: query heads per cache head.  0 or 1: multi-head attention.  2..16:
                                  grouped-query attention, query head j reads cache head floor(j/G); bf16 only,
                                  one head's rows must span less than 4 GiB
                                  (cap * kv_slot_stride * 2 bytes: the kernel addresses them with 32-bit
                                  offsets), else ADSA_ERR_UNSUPPORTED */
} adsa_params;

/* Device array of n_seq entries (96 bytes each): the ragged per-sequence state.  The kernels read AND update
   n_res, step, status, compacted, so one launch serves sequences at different positions. */
typedef struct adsa_seq {
  void*    k;                  /* this sequence's K cache (dtype elements) */
  void*    v;                  /* this sequence's V cache */
  int32_t* pos;                /* [cap] absolute position of each resident slot, strictly ascending (under
                                  ADSA_EVICT_REUSE_SLOT only until the first eviction; always distinct) */
  float*   score;              /* [score_rows][cap] ranking score of each resident slot: the rank of slot i
                                  is the sum over rows (ascending, fp32) of score[row][i].
                                  ADSA_SCORE_ATTN_MASS: score_rows = n_heads, one accumulator per head
                                  (each head's workgroup updates only its own row).
                                  ADSA_SCORE_VCOS_FUSED: score_rows = 2*n_heads, rows 2h and 2h+1 hold head h's
                                  share of |v|^2 and of v.u per slot (written by the attention launch; not a
                                  rank by themselves).  Else score_rows = 1 */
  int32_t  n_res;              /* resident slots */
  int32_t  step;               /* s (see the decode-step convention above); < 0: inactive */
  int32_t  grid_origin;        /* P: absolute position of image token 0 (= prefix length) */
  int32_t  n_keep_prefix;      /* positions below this are pinned (never ranked, never evicted) */
  int32_t  budget;             /* B: global tokens kept, when budget_den == 0 */
  int32_t  budget_num;         /* else B = floor((P + s) * budget_num / budget_den) */
  int32_t  budget_den;
  int32_t  status;             /* ADSA_SEQ_* bits, set by the device, cleared by the caller */
  int32_t  compacted;          /* 1 if the last adsa_step/adsa_compact evicted+compacted this sequence */
  int32_t  pending_slot;       /* slot adsa_select(PLAN_APPEND) reserved for the query token, whose K/V rows
                                  the next adsa_attend(APPEND) fills; -1 if none.  Written by adsa_select */
  int32_t  hole;               /* ADSA_EVICT_REUSE_SLOT: 1 + the slot the last eviction freed, 0 if none (start
                                  with 0).  A freed slot still counts in n_res but is in no list; the next
                                  adsa_select(PLAN_APPEND) gives it to the query token and clears hole */
  int32_t  reserved;
  float*   vcos_u;             /* ADSA_SCORE_VCOS_FUSED: [n_heads*head_dim + 4] floats owned by the caller and
                                  maintained by the library: the running sum u, then two step tags (as floats)
                                  that say which step u and the score rows belong to.  Zero it when the cache
                                  or `step` is changed by hand.  NULL otherwise */
  int64_t  reserved2;
} adsa_seq;

/* Bytes of device scratch the entry points need for these parameters (0 if they are invalid). */
size_t adsa_workspace_bytes(const adsa_params* p);

/*
 * Prepare a workspace (256-byte aligned, >= adsa_workspace_bytes(p)) for use with parameters p:
 * zeroes the arrival counters at its head with a small fill kernel on `stream`.  Call it once
 * after allocating the workspace and again before using the same memory with different
 * parameters; every later call leaves the counters zero.  A workspace may be shared by calls
 * that are ordered on one stream, not by concurrent ones.
 */
int adsa_workspace_init(const adsa_params* p, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Eq. 1 + Eq. 4: partition every sequence's resident slots into prefix / local / candidate for
 * the query of its current `step`, rank the candidates, and write the attended set
 *   PREFIX u LOCAL u top-min(B, |candidates|)
 * as an ascending slot list.  Ties go to the lower slot; -0 == +0; NaN scores are a
 * precondition violation.  Reads seqs[].pos/score/n_res/step, writes pending_slot (and, with
 * ADSA_FLAG_PLAN_APPEND, pos / score / n_res of the reserved slot); VCOS mode first writes Eq. 3's
 * S_i into score[] at the candidate slots (reads V, needs the workspace; other modes accept a
 * NULL workspace).  The ranking does not depend on the query token's q/k/v, so one call may
 * cover the sequences of every layer of a model (n_seq = layers x batch) before the layers run.
 * flags: ADSA_FLAG_PLAN_APPEND.
 *   sel_idx  int32 [n_seq][sel_cap]   out
 *   sel_cnt  int32 [n_seq]            out
 */
int adsa_select(const adsa_params* p, adsa_seq* seqs, int32_t* sel_idx, int32_t* sel_cnt,
                uint32_t flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Eq. 5 + attention: per sequence and query head, softmax(q.K_sel^T * scale) V_sel over the slots
 * listed in sel_idx (gathered in place, never materialised), fp32 accumulation.  With
 * hq = n_heads * max(q_per_kv, 1) query heads:
 *   q    dtype [n_seq][hq][head_dim]
 *   out  dtype [n_seq][hq][head_dim]
 *   lse  float [n_seq][hq]   natural-log sum-exp of the scaled logits
 *   k_new, v_new  dtype [n_seq][n_heads][head_dim], only read with ADSA_FLAG_APPEND (else may be NULL)
 * For ADSA_SCORE_ATTN_MASS and unless ADSA_FLAG_NO_ACCUMULATE is set, score[slot] of every
 * attended slot gains, in row h of score[], the probability the query head(s) of cache head h gave it
 * (grouped queries: their sum in ascending head order).
 * ADSA_FLAG_APPEND (Section 4.2, new tokens go to the end of the cache): the row (k_new, v_new)
 * is written to the slot adsa_select(ADSA_FLAG_PLAN_APPEND) reserved (pending_slot >= 0), and that
 * slot is attended from k_new / v_new directly.
 * flags: ADSA_FLAG_NO_ACCUMULATE, ADSA_FLAG_APPEND, ADSA_FLAG_NEW_F32, ADSA_FLAG_ADVANCE.
 */
int adsa_attend(const adsa_params* p, adsa_seq* seqs, const void* q, const void* k_new,
                const void* v_new, const int32_t* sel_idx, const int32_t* sel_cnt, void* out,
                float* lse, uint32_t flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Section 4.2 in per-row form.  For every sequence whose query token closes a grid row
 * ((s-1) % grid_w == grid_w-1, s >= 1): keep the pinned prefix, the last R completed rows and
 * the top min(B, |rest|) of the rest by the same ranking as adsa_select; write
 *   keep_map int32 [n_seq][cap]: new slot of old slot i, or -1 (entries >= old n_res untouched)
 * move K, V, pos and every score row to the front in place, order preserved, and set n_res, compacted.
 * Other sequences are untouched (compacted = 0, keep_map row untouched).  Like adsa_select it
 * may cover every layer's sequences in one call.  flags: ADSA_FLAG_ADVANCE.
 * With ADSA_EVICT_WHEN_FULL / ADSA_EVICT_REUSE_SLOT the call acts instead on the sequences whose cache is full
 * (n_res == cap, step >= 1), BEFORE the step's adsa_select: it removes the one candidate ranked
 * last for the incoming query's partition (ties: the highest slot goes) and closes the hole.
 */
int adsa_compact(const adsa_params* p, adsa_seq* seqs, int32_t* keep_map, uint32_t flags,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * One whole decode step of one layer, in one call: adsa_select(PLAN_APPEND), adsa_attend(APPEND)
 * and, unless ADSA_FLAG_NO_COMPACT, adsa_compact in stream order, the last of them advancing: the query
 * token is appended at slot n_res (skipped when s == 0), the attended set is chosen and attended,
 * attention mass is accumulated (ATTN_MASS), sequences that closed a row are evicted+compacted,
 * and step += 1.  keep_map may be NULL only with ADSA_FLAG_NO_COMPACT.
 * With ADSA_EVICT_WHEN_FULL / ADSA_EVICT_REUSE_SLOT the order is the paper's: evict one if full, then
 * append/select/attend.
 */
int adsa_step(const adsa_params* p, adsa_seq* seqs, const void* q, const void* k_new,
              const void* v_new, void* out, float* lse, int32_t* sel_idx, int32_t* sel_cnt,
              int32_t* keep_map, uint32_t flags, void* workspace, size_t workspace_bytes,
              void* stream);

/*
 * adsa_step for callers that cannot allocate device memory or carry a workspace around: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same kernels and
 * same results as adsa_step, but the scratch memory is a built-in array of ADSA_STATIC_SCRATCH_BYTES that
 * every GPU the library runs on holds until the process ends; the call allocates nothing (its address is
 * looked up once per device, at the first call there).  Parameters whose adsa_workspace_bytes() exceeds
 * ADSA_STATIC_SCRATCH_BYTES are rejected with ADSA_ERR_STATIC_SCRATCH before anything is launched.
 * All calls on one GPU share the one array: calls ordered on one stream are fine, calls that may
 * overlap on the same GPU (different streams or host threads) race.
 */
int adsa_step_static(const adsa_params* p, adsa_seq* seqs, const void* q, const void* k_new,
                     const void* v_new, void* out, float* lse, int32_t* sel_idx, int32_t* sel_cnt,
                     int32_t* keep_map, uint32_t flags, void* stream);

/* Timing hook for benchmarks: when enabled, adsa_attend/adsa_step attach a start and a stop HIP
   event to every attention-kernel dispatch on the caller's stream.  adsa_profile_read
   synchronises those events and returns, through its arguments, the number of timed launches and
   their summed duration in milliseconds since the last adsa_profile_enable(1); [host] pointers.
   adsa_profile_enable(0) switches the hook off and destroys its events.  Process-wide state, not thread-safe. */
int adsa_profile_enable(int on);
int adsa_profile_read(int64_t* n_launches, double* total_ms);

const char* adsa_strerror(int code);
int adsa_version(void);

#ifdef __cplusplus
}
#endif
#endif
