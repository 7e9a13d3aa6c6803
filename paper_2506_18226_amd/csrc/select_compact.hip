// Partition + ranking kernels of the ADSA decode path (gfx950).
//
//  k_select        : Eq. 1 partition of the resident slots, Eq. 4 ranking of the candidates by an
//                    LDS-resident 4-pass MSB radix select with lowest-slot tie-break, and the
//                    ascending attended-slot list.  It can plan for the query token's append
//                    (Section 4.2: new tokens go to the end of the cache) that the attention
//                    launch performs, so the ranking never waits for the token's K/V.
//  k_compact_plan  : Section 4.2 in per-row form: keep flags (prefix, last R rows, top-B of the
//                    rest), ballot/prefix-sum keep map, in-place move of pos[] and score[]; or
//                    Section 4.2 as written (evict the one most redundant candidate when full), closing
//                    the hole in order or leaving it to the incoming token.
//  k_compact_move  : in-place, order-preserving move of the surviving K and V rows.
//
// One workgroup of 256 threads owns one sequence in the first two kernels; everything it ranks
// lives in LDS (keys 4 B/slot), so the score array is read from HBM exactly once.
#include "adsa_internal.h"
#include "adsa_partition.h"

namespace adsa {
namespace {

constexpr uint8_t kFixed = 0;      // prefix / local / protected row: always kept
constexpr uint8_t kSkip = 1;       // a freed slot (ADSA_EVICT_REUSE_SLOT): in no list
constexpr uint8_t kCand = 2;       // competes for the budget

// LDS of one ranking workgroup.  key[] and cls[] are sized by the launch's cap (dynamic LDS:
// 5 bytes per slot), so small caches leave room for many workgroups per CU.
struct RankShared {
  uint32_t hist[256];
  uint32_t wave_tot[kSelThreads / kWave];
  uint32_t bcast[4];
};

static size_t rank_lds_bytes(int cap) { return (size_t)cap * 4 + (((size_t)cap + 15) / 16) * 16; }

// Larger key == kept first.  -0 is folded into +0 so that they tie (IEEE equality).
__device__ __forceinline__ uint32_t order_key(float x, bool keep_largest) {
  if (x == 0.0f) x = 0.0f;
  uint32_t u = __float_as_uint(x);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return keep_largest ? u : ~u;
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    uint32_t o = __shfl_up(v, d, kWave);
    if (lane >= d) v += o;
  }
  return v;
}

// Exclusive prefix sum of one value per thread over the 256-thread workgroup; *total gets the sum.
__device__ __forceinline__ uint32_t block_excl_scan(RankShared& sh, uint32_t v, uint32_t* total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t incl = wave_incl_scan(v);
  __syncthreads();                                   // wave_tot may still be read from a previous scan
  if (lane == kWave - 1) sh.wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelThreads / kWave; ++w) {
    uint32_t t = sh.wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  *total = tot;
  return base + incl - v;
}

// Eq. 4 as a threshold: returns T and need_eq such that {key > T} plus the first need_eq slots
// with key == T (ascending slot) are exactly the `want` best candidates.
__device__ void radix_threshold(RankShared& sh, const uint32_t* key, const uint8_t* cls, int n, uint32_t n_cand,
                                uint32_t want, uint32_t* T_out, uint32_t* need_eq_out) {
  if (want == 0) { *T_out = 0xFFFFFFFFu; *need_eq_out = 0; return; }
  if (want >= n_cand) { *T_out = 0u; *need_eq_out = 0xFFFFFFFFu; return; }
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  uint32_t prefix = 0, mask = 0, remaining = want;
  for (int shift = 24; shift >= 0; shift -= 8) {
    sh.hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) {
      uint32_t k = key[i];
      if (cls[i] == kCand && (k & mask) == prefix) atomicAdd(&sh.hist[(k >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns digits 255-4l .. 252-4l; scan from the largest digit down
      uint32_t c[4];
      uint32_t local = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) { c[k] = sh.hist[255 - 4 * lane - k]; local += c[k]; }
      uint32_t incl = wave_incl_scan(local);
      unsigned long long hit = __ballot(incl >= remaining);
      int first = __ffsll((long long)hit) - 1;        // exists: remaining <= candidates under prefix
      if (lane == first) {
        uint32_t run = incl - local;
        int digit = 0;
        uint32_t rem = remaining;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if (run + c[k] >= remaining) { digit = 255 - 4 * lane - k; rem = remaining - run; break; }
          run += c[k];
        }
        sh.bcast[0] = (uint32_t)digit;
        sh.bcast[1] = rem;
      }
    }
    __syncthreads();
    prefix |= sh.bcast[0] << shift;
    mask |= 0xFFu << shift;
    remaining = sh.bcast[1];
    __syncthreads();
  }
  *T_out = prefix;
  *need_eq_out = remaining;
}

__device__ __forceinline__ int effective_budget(const adsa_seq& q, int s) {
  long long b = q.budget;
  if (q.budget_den > 0) b = ((long long)(q.grid_origin + s) * q.budget_num) / q.budget_den;
  if (b < 0) b = 0;
  if (b > ADSA_MAX_CAP) b = ADSA_MAX_CAP;
  return (int)b;
}

struct LaunchShape {
  int n_heads, head_dim, elem_bytes;
  int grid_h, grid_w, R, w;
  int cap, sel_cap, score_mode, score_rows, recent_m, evict_policy;
  long long slot_stride_b, head_stride_b;    // bytes
};

// Ranks of kRankSlots slots at once (4 when few workgroups run and memory latency is what counts, 1 when the launch
// fills the chip anyway and registers are better spent on occupancy): v[u] = sum over the score rows of slot idx[u], ascending row order, plain fp32
// adds (the order one slot at a time would use); slots with on[u] false give 0 and touch no memory.  The loads of all
// slots, and of the next batch of rows while one batch is added, are in flight together: a workgroup ranks its
// sequence in two or three memory round trips instead of one per slot and batch.
constexpr int kRankRows = 8;
template <int kRankSlots>
__device__ __forceinline__ void rank_values(const float* score, int rows, int cap, const int* idx, const bool* on, float* v) {
  float cur[kRankSlots][kRankRows], nxt[kRankSlots][kRankRows];
  auto load_rows = [&](int r0, float (&t)[kRankSlots][kRankRows]) {
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u)
#pragma unroll
      for (int k = 0; k < kRankRows; ++k)
        t[u][k] = (on[u] && r0 + k < rows) ? score[(size_t)(r0 + k) * cap + idx[u]] : 0.0f;
  };
#pragma unroll
  for (int u = 0; u < kRankSlots; ++u) v[u] = on[u] ? score[idx[u]] : 0.0f;
  if (rows > 1) load_rows(1, cur);
  for (int r = 1; r < rows; r += kRankRows) {
    if (r + kRankRows < rows) load_rows(r + kRankRows, nxt);
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u)
#pragma unroll
      for (int k = 0; k < kRankRows; ++k)
        if (r + k < rows) v[u] += cur[u][k];
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u)
#pragma unroll
      for (int k = 0; k < kRankRows; ++k) cur[u][k] = nxt[u][k];
  }
}

__device__ __forceinline__ bool keep_largest_of(int mode) {
  return mode == ADSA_SCORE_ATTN_MASS || mode == ADSA_SCORE_EXT_LARGEST;
}

template <int kRankSlots>
__global__ __launch_bounds__(kSelThreads) void k_select(LaunchShape L, adsa_seq* seqs, int32_t* sel_idx,
                                                       int32_t* sel_cnt, int plan_append) {
  __shared__ RankShared sh;
  extern __shared__ uint32_t s_rank_dyn[];
  uint32_t* key = s_rank_dyn;                                  // [cap] order-preserving keys
  uint8_t* cls = reinterpret_cast<uint8_t*>(s_rank_dyn + L.cap);   // [cap]
  __shared__ int s_bad;
  const int b = blockIdx.x, tid = threadIdx.x;
  adsa_seq& sq = seqs[b];
  const int s = sq.step;
  int n = sq.n_res;
  const int status_in = sq.status;
  if (tid == 0) s_bad = 0;
  __syncthreads();
  if (s < 0 || status_in != 0) { if (tid == 0) { sel_cnt[b] = 0; sq.pending_slot = -1; } return; }
  if (n < 0 || n > L.cap || s > L.grid_h * L.grid_w) {
    if (tid == 0) { sq.status = status_in | ADSA_SEQ_BAD_STATE; sel_cnt[b] = 0; sq.pending_slot = -1; }
    return;
  }
  // Section 4.2: the query token goes to the end of the cache (or, with ADSA_EVICT_REUSE_SLOT, into
  // the slot the last eviction freed).  When the append itself happens later in this step (inside
  // the attention launch), plan for it: that slot, always local, score 0.
  const int hole = L.evict_policy == ADSA_EVICT_REUSE_SLOT ? sq.hole - 1 : -1;     // freed slot or -1
  int slot_new = -1;
  if (plan_append && s >= 1) {
    if (hole >= 0 && hole < n) slot_new = hole;
    else {
      if (n + 1 > L.cap) {
        if (tid == 0) { sq.status = status_in | ADSA_SEQ_CACHE_FULL; sel_cnt[b] = 0; sq.pending_slot = -1; }
        return;
      }
      slot_new = n;
      n += 1;
    }
  }

  // ---- Eq. 1: partition, keys into LDS
  const QueryCell cell = make_query_cell(sq, s, L.grid_w, L.R, L.w, L.recent_m);
  const bool largest = keep_largest_of(L.score_mode);
  const bool ranked = L.evict_policy == ADSA_EVICT_ROW_END;
  uint32_t my_cand = 0;
  for (int i0 = tid; i0 < n; i0 += kRankSlots * kSelThreads) {
    int idx[kRankSlots], posv[kRankSlots];
    bool in[kRankSlots], planned[kRankSlots], rk[kRankSlots];
    float rv[kRankSlots];
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u) {
      const int i = i0 + u * kSelThreads;
      in[u] = i < n;
      idx[u] = in[u] ? i : n - 1;
      planned[u] = i == slot_new;                   // the slot the query token will occupy
      posv[u] = sq.pos[idx[u]];
      // (evict-one-when-full policies attend every candidate: their rank is never looked at)
      rk[u] = in[u] && ranked && !planned[u];
    }
    rank_values<kRankSlots>(sq.score, L.score_rows, L.cap, idx, rk, rv);
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u) {
      if (!in[u]) continue;
      const int i = idx[u];
      const bool freed = i == hole && !planned[u];  // evicted, not yet reused: nobody attends it
      const int c = (planned[u] || freed) ? 0 : select_class(cell, posv[u]);
      if (c < 0) s_bad = 1;
      cls[i] = freed ? kSkip : c == 1 ? kCand : kFixed;
      key[i] = order_key(rv[u], largest);
      my_cand += (c == 1);
    }
  }
  uint32_t n_cand;
  block_excl_scan(sh, my_cand, &n_cand);   // also orders the LDS writes above before the reads below
  if (s_bad) {
    if (tid == 0) { sq.status = status_in | ADSA_SEQ_BAD_STATE; sel_cnt[b] = 0; sq.pending_slot = -1; }
    return;
  }

  // ---- Eq. 4: threshold of the top-B candidates
  // the streaming policy attends everything resident (context == cache, Tables 1-2)
  const uint32_t B = L.evict_policy != ADSA_EVICT_ROW_END ? n_cand : (uint32_t)effective_budget(sq, s);
  uint32_t T, need_eq;
  radix_threshold(sh, key, cls, n, n_cand, B < n_cand ? B : n_cand, &T, &need_eq);

  // ---- ascending slot list: contiguous run of slots per thread, packed (kept | equal<<16) scan
  const int per = (n + kSelThreads - 1) / kSelThreads;
  const int lo = tid * per, hi = min(n, lo + per);
  uint32_t a = 0, e = 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t k = key[i];
    const uint8_t c = cls[i];
    a += (c == kFixed) || (c == kCand && k > T);
    e += c == kCand && (k == T);
  }
  uint32_t total;
  uint32_t ex = block_excl_scan(sh, a | (e << 16), &total);
  uint32_t a_run = ex & 0xFFFFu, e_run = ex >> 16;
  int32_t* out = sel_idx + (size_t)b * L.sel_cap;
  for (int i = lo; i < hi; ++i) {
    const uint32_t k = key[i];
    const uint8_t c = cls[i];
    bool take = (c == kFixed) || (c == kCand && k > T);
    const bool eq = c == kCand && (k == T);
    const uint32_t dest = a_run + min(e_run, need_eq);
    if (eq) { take = e_run < need_eq; ++e_run; } else if (take) ++a_run;
    if (take && dest < (uint32_t)L.sel_cap) out[dest] = i;
  }
  const uint32_t cnt = (total & 0xFFFFu) + min(total >> 16, need_eq);
  const bool ok = cnt <= (uint32_t)L.sel_cap;
  const bool reserve = ok && slot_new >= 0;          // commit the planned append: the slot now holds the query token
  if (reserve)
    for (int r = tid; r < L.score_rows; r += kSelThreads) sq.score[(size_t)r * L.cap + slot_new] = 0.0f;
  if (tid == 0) {
    if (!ok) { sq.status = status_in | ADSA_SEQ_SEL_OVERFLOW; sel_cnt[b] = 0; sq.pending_slot = -1; }
    else {
      sel_cnt[b] = (int32_t)cnt;
      sq.pending_slot = reserve ? slot_new : -1;
      if (reserve) {
        sq.pos[slot_new] = sq.grid_origin + s - 1;
        sq.n_res = n;
        if (slot_new == hole) sq.hole = 0;
      }
    }
  }
}

// plan[b] = { old n_res, first slot that moves, did compact, new n_res }
template <int kRankSlots>
__global__ __launch_bounds__(kSelThreads) void k_compact_plan(LaunchShape L, adsa_seq* seqs,
                                                             int32_t* keep_map, int32_t* plan,
                                                             int advance_step, const float* vcos_s) {
  __shared__ RankShared sh;
  extern __shared__ uint32_t s_rank_dyn[];
  uint32_t* key = s_rank_dyn;                                  // [cap] keys, later the keep map
  uint8_t* cls = reinterpret_cast<uint8_t*>(s_rank_dyn + L.cap);
  const int b = blockIdx.x, tid = threadIdx.x;
  adsa_seq& sq = seqs[b];
  const int s = sq.step, n = sq.n_res, W = L.grid_w;
  const bool active = s >= 0 && sq.status == 0;
  // per-row policy: act when the query token closed a grid row; streaming policy (Section 4.2 as
  // written): act when the cache is full and a token is about to be inserted
  const bool streaming = L.evict_policy != ADSA_EVICT_ROW_END;
  const bool reuse = L.evict_policy == ADSA_EVICT_REUSE_SLOT;
  const bool row_end = active && n >= 0 && n <= L.cap &&
                       (streaming ? (s >= 1 && s <= L.grid_h * W && n == L.cap && !(reuse && sq.hole != 0))
                                  : is_row_end(s, L.grid_h, W));
  if (!row_end) {
    if (tid == 0) {
      plan[4 * b + 0] = 0; plan[4 * b + 1] = 0; plan[4 * b + 2] = 0; plan[4 * b + 3] = n;
      if (active) { sq.compacted = 0; if (advance_step) sq.step = s + 1; }
    }
    return;
  }
  const QueryCell cell = make_query_cell(sq, s, W, L.R, L.w, L.recent_m);
  const bool largest = keep_largest_of(L.score_mode);
  uint32_t my_rest = 0;
  for (int i0 = tid; i0 < n; i0 += kRankSlots * kSelThreads) {
    int idx[kRankSlots], posv[kRankSlots];
    bool in[kRankSlots], rk[kRankSlots];
    float rv[kRankSlots];
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u) {
      const int i = i0 + u * kSelThreads;
      in[u] = i < n;
      idx[u] = in[u] ? i : n - 1;
      posv[u] = sq.pos[idx[u]];
      rk[u] = in[u] && L.score_mode != ADSA_SCORE_VCOS_FUSED;      // (fused form: keys of the candidates follow once N is known)
    }
    rank_values<kRankSlots>(sq.score, L.score_rows, L.cap, idx, rk, rv);
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u) {
      if (!in[u]) continue;
      const int i = idx[u];
      // streaming: the partition of the incoming query (its local region must survive)
      const int c = streaming ? (select_class(cell, posv[u]) == 1 ? 1 : 0) : evict_class(cell, posv[u]);
      cls[i] = c == 1 ? kCand : kFixed;
      key[i] = L.score_mode == ADSA_SCORE_VCOS_FUSED ? 0u : order_key(rv[u], largest);
      my_rest += (c == 1);
    }
  }
  uint32_t n_rest;
  block_excl_scan(sh, my_rest, &n_rest);
  if (L.score_mode == ADSA_SCORE_VCOS_FUSED) {
    // Eq. 3 from what the last attention launch left per (head, slot): S_i = (v^_i.u - v^_i.v^_i)/(N-1) with
    // |v_i|^2 and v_i.u summed over the heads' rows (ascending).  If those rows do not belong to this
    // step, the two-pass computation has just written S_i to the workspace instead.
    const float* tags = sq.vcos_u ? sq.vcos_u + (size_t)L.n_heads * L.head_dim : nullptr;
    const bool rows_ok = tags && tags[1] == (float)(s + 1);
    const float inv_nm1 = n_rest > 1 ? 1.0f / (float)(n_rest - 1) : 0.0f;
    for (int i = tid; i < n; i += kSelThreads) {
      if (cls[i] != kCand) continue;
      float S;
      if (rows_ok) {
        float ss = 0.0f, dot = 0.0f;
        for (int hh = 0; hh < L.n_heads; ++hh) {
          ss += sq.score[(size_t)(2 * hh) * L.cap + i];
          dot += sq.score[(size_t)(2 * hh + 1) * L.cap + i];
        }
        const float inv = 1.0f / fmaxf(sqrtf(ss), 1e-8f);
        S = (dot * inv - ss * inv * inv) * inv_nm1;
      } else {
        S = vcos_s[(size_t)b * L.cap + i];
      }
      key[i] = order_key(S, false);
    }
    __syncthreads();
  }
  if (reuse) {
    // Evict the candidate ranked last -- smallest key, among equals the newest position -- and leave
    // everything where it is: the freed slot goes to the incoming token.
    unsigned long long best = ~0ull;                  // (key, ~pos): the minimum is the victim
    int best_i = -1;
    for (int i = tid; i < n; i += kSelThreads) {
      if (cls[i] != kCand) continue;
      const unsigned long long v = ((unsigned long long)key[i] << 32) | (uint32_t)~(uint32_t)sq.pos[i];
      if (v < best) { best = v; best_i = i; }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const unsigned long long o = __shfl_xor(best, d, kWave);
      const int oi = __shfl_xor(best_i, d, kWave);
      if (o < best) { best = o; best_i = oi; }
    }
    __shared__ unsigned long long s_best[kSelThreads / kWave];
    __shared__ int s_best_i[kSelThreads / kWave];
    if ((tid & (kWave - 1)) == 0) { s_best[tid / kWave] = best; s_best_i[tid / kWave] = best_i; }
    __syncthreads();
    int victim = -1;
    unsigned long long vb = ~0ull;
#pragma unroll
    for (int w = 0; w < kSelThreads / kWave; ++w)
      if (s_best_i[w] >= 0 && s_best[w] < vb) { vb = s_best[w]; victim = s_best_i[w]; }
    int32_t* map = keep_map + (size_t)b * L.cap;
    if (victim >= 0)
      for (int i = tid; i < n; i += kSelThreads) map[i] = i == victim ? -1 : i;
    if (tid == 0) {
      plan[4 * b + 0] = n; plan[4 * b + 1] = n; plan[4 * b + 2] = 0; plan[4 * b + 3] = n;
      sq.compacted = victim >= 0 ? 1 : 0;
      if (victim >= 0) sq.hole = victim + 1;
      if (advance_step) sq.step = s + 1;
    }
    return;
  }
  uint32_t B = (uint32_t)effective_budget(sq, s);
  if (streaming) B = n_rest > 0 ? n_rest - 1 : 0;      // all candidates but the one ranked last
  uint32_t T, need_eq;
  radix_threshold(sh, key, cls, n, n_rest, B < n_rest ? B : n_rest, &T, &need_eq);

  const int per = (n + kSelThreads - 1) / kSelThreads;
  const int lo = tid * per, hi = min(n, lo + per);
  uint32_t a = 0, e = 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t k = key[i];
    const bool cand = cls[i] == kCand;
    a += (!cand) || (k > T);
    e += cand && (k == T);
  }
  uint32_t total;
  uint32_t ex = block_excl_scan(sh, a | (e << 16), &total);
  uint32_t a_run = ex & 0xFFFFu, e_run = ex >> 16;
  int32_t* map = keep_map + (size_t)b * L.cap;
  int my_first = n;
  for (int i = lo; i < hi; ++i) {
    const uint32_t k = key[i];
    const bool cand = cls[i] == kCand;
    bool take = (!cand) || (k > T);
    const bool eq = cand && (k == T);
    const uint32_t dest = a_run + min(e_run, need_eq);
    if (eq) { take = e_run < need_eq; ++e_run; } else if (take) ++a_run;
    const int32_t m = take ? (int32_t)dest : -1;
    map[i] = m;
    key[i] = (uint32_t)m;                 // own run only: no other thread reads key[i] any more
    if (m != i && i < my_first) my_first = i;
  }
  // first slot whose content changes (evicted or moved): everything before it stays put
  __syncthreads();
  if (tid == 0) sh.bcast[2] = (uint32_t)n;
  __syncthreads();
  atomicMin(&sh.bcast[2], (uint32_t)my_first);
  __syncthreads();
  const int first = (int)sh.bcast[2];
  const uint32_t n_new = (total & 0xFFFFu) + min(total >> 16, need_eq);

  // in-place, order-preserving move of pos[] and every score row: ascending tiles, load -> barrier ->
  // store.  A tile's destinations are <= its sources and below the next tile's sources; the rows are
  // independent arrays, so kRowBatch of them travel together (their loads overlap: the move costs one
  // memory round trip per tile and batch instead of one per tile and row).
  constexpr int kRowBatch = 8, kTileSlots = 4;       // a tile: kTileSlots slots per thread
  for (int base = (first / kSelThreads) * kSelThreads; base < n; base += kTileSlots * kSelThreads) {
    int m[kTileSlots], src[kTileSlots], pv[kTileSlots];
    bool mv[kTileSlots];
#pragma unroll
    for (int u = 0; u < kTileSlots; ++u) {
      const int i = base + u * kSelThreads + tid;
      m[u] = i < n ? (int)key[i] : -1;
      mv[u] = m[u] >= 0 && m[u] != i;
      src[u] = mv[u] ? i : 0;
      pv[u] = mv[u] ? sq.pos[i] : 0;
    }
    for (int r0 = 0; r0 < L.score_rows; r0 += kRowBatch) {
      float sv[kTileSlots][kRowBatch];
#pragma unroll
      for (int u = 0; u < kTileSlots; ++u)
#pragma unroll
        for (int k = 0; k < kRowBatch; ++k)
          sv[u][k] = (mv[u] && r0 + k < L.score_rows) ? sq.score[(size_t)(r0 + k) * L.cap + src[u]] : 0.0f;
      __syncthreads();
#pragma unroll
      for (int u = 0; u < kTileSlots; ++u) {
        if (!mv[u]) continue;
        if (r0 == 0) sq.pos[m[u]] = pv[u];
#pragma unroll
        for (int k = 0; k < kRowBatch; ++k)
          if (r0 + k < L.score_rows) sq.score[(size_t)(r0 + k) * L.cap + m[u]] = sv[u][k];
      }
    }
  }
  if (tid == 0) {
    plan[4 * b + 0] = n; plan[4 * b + 1] = first; plan[4 * b + 2] = 1; plan[4 * b + 3] = (int32_t)n_new;
    sq.n_res = (int32_t)n_new;
    sq.compacted = 1;
    if (advance_step) sq.step = s + 1;
  }
}

// grid = (row slices, 2 {K,V}, n_seq).  A workgroup owns a 16*lanes-byte column slice of every row
// of one cache and walks the rows in ascending tiles: load survivors -> barrier -> store.
template <int ROWS_PER_THREAD>
__global__ __launch_bounds__(kMoveThreads) void k_compact_move(LaunchShape L, const adsa_seq* seqs,
                                                              const int32_t* keep_map,
                                                              const int32_t* plan, int lanes_per_slice,
                                                              int slices_per_head) {
  const int b = blockIdx.z;
  if (plan[4 * b + 2] == 0) return;
  const int n_old = plan[4 * b + 0], first = plan[4 * b + 1];
  if (first >= n_old) return;
  const adsa_seq& sq = seqs[b];
  char* base = reinterpret_cast<char*>(blockIdx.y == 0 ? sq.k : sq.v);
  const int slice = blockIdx.x;
  const int head = slice / slices_per_head, part = slice - head * slices_per_head;
  base += (long long)head * L.head_stride_b + (long long)part * lanes_per_slice * 16;
  const int rows_per_pass = kMoveThreads / lanes_per_slice;
  const int row_in_pass = threadIdx.x / lanes_per_slice, lane = threadIdx.x % lanes_per_slice;
  const int32_t* map = keep_map + (size_t)b * L.cap;
  const int tile = rows_per_pass * ROWS_PER_THREAD;
  for (int t0 = (first / tile) * tile; t0 < n_old; t0 += tile) {
    uint4 val[ROWS_PER_THREAD];
    int dst[ROWS_PER_THREAD];
#pragma unroll
    for (int u = 0; u < ROWS_PER_THREAD; ++u) {
      const int i = t0 + u * rows_per_pass + row_in_pass;
      dst[u] = -1;
      if (i < n_old) {
        const int m = map[i];
        if (m >= 0 && m != i) {
          dst[u] = m;
          val[u] = reinterpret_cast<const uint4*>(base + (long long)i * L.slot_stride_b)[lane];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < ROWS_PER_THREAD; ++u)
      if (dst[u] >= 0) reinterpret_cast<uint4*>(base + (long long)dst[u] * L.slot_stride_b)[lane] = val[u];
  }
}

LaunchShape shape_of(const adsa_params& p) {
  LaunchShape L;
  L.n_heads = p.n_heads; L.head_dim = p.head_dim; L.elem_bytes = elem_bytes(p);
  L.grid_h = p.grid_h; L.grid_w = p.grid_w; L.R = p.win_rows_back; L.w = p.win_col_radius;
  L.cap = p.cap; L.sel_cap = p.sel_cap; L.score_mode = p.score_mode; L.score_rows = score_rows(p); L.recent_m = p.win_recent_m; L.evict_policy = p.evict_policy;
  L.slot_stride_b = (long long)p.kv_slot_stride * L.elem_bytes;
  L.head_stride_b = (long long)p.kv_head_stride * L.elem_bytes;
  return L;
}

}  // namespace

// from this many sequences per launch on the ranking kernels are throughput-bound (two workgroups per CU and more)
constexpr int kManySequences = 512;

hipError_t launch_select(const adsa_params& p, adsa_seq* seqs, int32_t* sel_idx, int32_t* sel_cnt,
                         bool plan_append, hipStream_t st) {
  if (p.n_seq >= kManySequences)
    hipLaunchKernelGGL(k_select<1>, dim3(p.n_seq), dim3(kSelThreads), rank_lds_bytes(p.cap), st, shape_of(p), seqs,
                       sel_idx, sel_cnt, plan_append ? 1 : 0);
  else
    hipLaunchKernelGGL(k_select<4>, dim3(p.n_seq), dim3(kSelThreads), rank_lds_bytes(p.cap), st, shape_of(p), seqs,
                       sel_idx, sel_cnt, plan_append ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_compact(const adsa_params& p, adsa_seq* seqs, int32_t* keep_map, char* ws,
                          const Workspace& w, bool advance_step, hipStream_t st) {
  int32_t* plan = reinterpret_cast<int32_t*>(ws + w.plan_off);
  LaunchShape L = shape_of(p);
  const float* vcos_s = p.score_mode == ADSA_SCORE_VCOS_FUSED ? reinterpret_cast<const float*>(ws + w.vcos_s_off) : nullptr;
  if (p.n_seq >= kManySequences)
    hipLaunchKernelGGL(k_compact_plan<1>, dim3(p.n_seq), dim3(kSelThreads), rank_lds_bytes(p.cap), st, L, seqs,
                       keep_map, plan, advance_step ? 1 : 0, vcos_s);
  else
    hipLaunchKernelGGL(k_compact_plan<4>, dim3(p.n_seq), dim3(kSelThreads), rank_lds_bytes(p.cap), st, L, seqs,
                       keep_map, plan, advance_step ? 1 : 0, vcos_s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.evict_policy == ADSA_EVICT_REUSE_SLOT) return e;     // slot reuse moves no row
  // one workgroup per 128-byte column slice of a head row (whole head row when it is narrower)
  const int head_bytes = p.head_dim * L.elem_bytes;
  const int slice_bytes = head_bytes < 128 ? head_bytes : 128;
  const int lanes = slice_bytes / 16, slices_per_head = head_bytes / slice_bytes;
  dim3 grid(p.n_heads * slices_per_head, 2, p.n_seq);
  hipLaunchKernelGGL(k_compact_move<4>, grid, dim3(kMoveThreads), 0, st, L, (const adsa_seq*)seqs,
                     (const int32_t*)keep_map, (const int32_t*)plan, lanes, slices_per_head);
  return hipGetLastError();
}

}  // namespace adsa
