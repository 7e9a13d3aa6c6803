// Gather flash-decode of the ADSA decode path (gfx950): Eq. 5's gather fused with softmax
// attention over the selected slots, plus the cache append (Section 4.2) and the per-head
// attention-mass update, in ONE launch.
//
//  k_attend<EB, D, HT, U, NW, VF, DIRECT> : grid (token chunk, head group, sequence), NW waves.
//    A 16-byte-per-lane streaming load of one wave covers RPW = 64 / (D*EB/16) rows of D
//    elements.  HT of them are different heads of one token ([slot][head][D] caches: HT = RPW, one
//    contiguous burst per token) or HT = 1 and they are RPW consecutive tokens of ONE head
//    ([head][slot][D] caches: a workgroup streams one head's rows back to back).  q.k is reduced
//    over the lanes of a row with DPP; every lane keeps an online-softmax state (m, l, acc) in
//    registers, fp32, log2 domain.  The lane groups of a wave merge in registers (DPP and 16-/32-lane
//    swaps), the waves through one small LDS record each.
//    With one chunk per (sequence, head group) -- the plan whenever that already fills the chip --
//    the workgroup writes out / lse itself and adds the probabilities it produced to its OWN
//    heads' rows of score[]: no workgroup ever talks to another one.
//    With several chunks, each writes a partial and the scaled logits to the workspace and the
//    LAST one to arrive (an arrival counter, nothing waits) merges them and updates the scores.
//    VF (ADSA_SCORE_VCOS_FUSED): every V row that streams through also yields its head's share of |v|^2
//    and of v.u (u = running sum of the candidates' normalised V, Eq. 2-3), stored per (head, slot): the
//    next eviction ranks from them instead of re-reading V.
#include <hip/hip_ext.h>

#include "adsa_internal.h"
#include "adsa_device.h"

namespace adsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Sum over the LPR consecutive lanes that hold one row; every lane of the group gets the sum.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x += dpp_f<0xB1>(x);            // quad_perm [1,0,3,2]
  x += dpp_f<0x4E>(x);            // quad_perm [2,3,0,1]
  x += dpp_f<0x141>(x);           // row_half_mirror: the other quad of the 8-lane group
  if (LPR >= 16) x += dpp_f<0x140>(x);   // row_mirror: the other half of the 16-lane row
  if (LPR >= 32) x += __shfl_xor(x, 16, kWave);
  return x;
}

template <int EB> struct Elems;
template <> struct Elems<2> {      // bf16: 8 values per 16-byte vector
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xFFFF0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xFFFF0000u);
  }
};
template <> struct Elems<4> {      // fp32: 4 values per 16-byte vector
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

// chunk c of a list of cnt (<= ADSA_MAX_CAP) tokens split evenly over nc (<= kMaxChunks) chunks
__device__ __forceinline__ int chunk_begin(int cnt, int c, int nc) { return (int)(((unsigned)cnt * (unsigned)c) / (unsigned)nc); }

// i / n for 0 <= i < 2^22, 1 <= n < 2^22, given r ~= 1/n: the float estimate is off by at most one
__device__ __forceinline__ int small_div(int i, int n, float r) {
  int qd = (int)((float)i * r);
  if (qd * n > i) --qd;
  else if ((qd + 1) * n <= i) ++qd;
  return qd;
}

struct AttendArgs {
  adsa_seq* seqs;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  const char* q;
  const char* k_new;
  const char* v_new;
  char* out;
  float* lse;
  float* logits;        // [n_seq][n_heads][lg_stride]   scaled logits, log2 units (split launches)
  float* part_ml;       // [n_seq][n_heads][n_chunks][2]
  float* part_acc;      // [n_seq][n_heads][n_chunks][D]
  int32_t* counters;    // [n_seq][n_hg]                 arrival counters, zero between launches
  int n_heads, n_hg, sel_cap, lg_stride, chunk_max, cap;
  int accumulate, append, advance;     // advance: step += 1 at the end
  int new_f32;                         // k_new / v_new are fp32 although the cache is bf16: round as they enter
  int vcos_fused;
  long long slot_stride_b, head_stride_b;
  float scale_log2;     // softmax scale * log2(e)
};

// score[row][slot] += 2^(z - lse2[row]) for `total` (row, token) pairs, loads batched so that the
// read-modify-write latencies overlap.  get(i, &row_local, &slot, &z) describes pair i.
template <typename Get>
__device__ __forceinline__ void add_mass(gfloat* score, int cap, int row0, const float* s_lse2, int total, Get get) {
  constexpr int B = 4;
  const int kAttThreads = blockDim.x;
  for (int i0 = threadIdx.x; i0 < total; i0 += kAttThreads * B) {
    gfloat* ptr[B];
    float inc[B], old[B];
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int i = i0 + u * kAttThreads;
      ptr[u] = nullptr; inc[u] = 0.0f; old[u] = 0.0f;
      if (i < total) {
        int sb, slot; float z;
        get(i, &sb, &slot, &z);
        ptr[u] = score + (size_t)(row0 + sb) * cap + slot;
        old[u] = *ptr[u];
        inc[u] = fast_exp2(z - s_lse2[sb]);
      }
    }
#pragma unroll
    for (int u = 0; u < B; ++u)
      if (ptr[u]) *ptr[u] = old[u] + inc[u];
  }
}

// DIRECT: the list of a (sequence, head group) is not split (grid.x == 1): the workgroup finishes its heads alone.
// The arguments the first round trip needs come first, as plain scalars: the build asks for leading kernel
// arguments to be preloaded into scalar registers at wave launch, so those loads can leave at once, without
// waiting for a scalar load of the argument block (which would also wait for the sequence record's).
template <int EB, int D, int HT, int U, int NW, bool VF, bool DIRECT>
__global__ __launch_bounds__(NW * kWave) void k_attend(adsa_seq* seqs_arg, const int32_t* sel_idx_arg, const int32_t* sel_cnt_arg,
                                                      const char* q_arg, const char* k_new_arg, const char* v_new_arg,
                                                      int heads_and_flags, int sel_cap_arg, AttendArgs A) {
  constexpr int kAttThreads = NW * kWave;           // the waves of the workgroup share one token chunk
  constexpr int EPL = Elems<EB>::N;                 // elements per lane
  constexpr int LPR = D / EPL;                      // lanes per row
  constexpr int RPW = kWave / LPR;                  // rows per wave-load
  constexpr int TT = RPW / HT;                      // tokens per wave-load
  constexpr int PF = 1024 / kAttThreads;            // score read-modify-writes a thread starts early
  extern __shared__ float s_logit[];                // logits tile [HT][chunk_max] ([2][chunk_max] for VF), then
                                                    // the chunk's slot list int [chunk_max]
  // merge: the lane groups of a wave meet in registers, the waves through these (one state per wave and head)
  __shared__ float s_wm[NW][HT], s_wl[NW][HT];
  __shared__ __attribute__((aligned(16))) float s_wacc[NW * HT * D];
  __shared__ float s_lse2[HT];
  __shared__ int s_ticket;

  const int chunk = DIRECT ? 0 : blockIdx.x, hg = blockIdx.y, b = blockIdx.z;
  const int n_chunks = DIRECT ? 1 : gridDim.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int sub = lane / LPR, dl = lane - sub * LPR;
  const int hs = sub % HT, ts = sub / HT;           // head and token of this lane's row within a wave-load
  const int head = hg * HT + hs;
  // (only 14 dwords of arguments are preloaded: the two flags the first trip needs ride on the head count)
  const int n_heads = heads_and_flags & 0xFFFF, sel_cap = sel_cap_arg;
  const bool head_ok = head < n_heads;
  const int head_c = head_ok ? head : n_heads - 1;
  const int heads_here = min(HT, n_heads - hg * HT);

  // ---- first round trip: everything that depends on the kernel arguments only -- the count, the
  // sequence record, q and (when the list is not split, so its chunk starts at 0) the first slots of
  // the loop and the slots whose score words this thread updates at the end.  The record and the
  // count are pinned here so that they cannot drift behind the count test below.
  ADSA_GLOBAL adsa_seq* const sqp = (ADSA_GLOBAL adsa_seq*)(seqs_arg + b);
  const int cnt_raw = ((const gint*)sel_cnt_arg)[b];
  gchar* const k_base = (gchar*)sqp->k;
  gchar* const v_base = (gchar*)sqp->v;
  gfloat* const score = (gfloat*)sqp->score;
  const int pending = sqp->pending_slot;
  gfloat* const u_state = VF ? (gfloat*)sqp->vcos_u : nullptr;
  const gint* idx = (const gint*)sel_idx_arg + (size_t)b * sel_cap;
  const size_t row_off = ((size_t)b * n_heads + head_c) * D * EB + dl * 16;
  const gchar* const q_g = (const gchar*)q_arg;
  const gchar* const k_new_g = (const gchar*)k_new_arg;
  const gchar* const v_new_g = (const gchar*)v_new_arg;
  gchar* const out_g = (gchar*)A.out;
  gfloat* const lse_g = (gfloat*)A.lse;
  const uint4 qr = load16(q_g + row_off);
  // The wave takes the TT-token units wave, wave + NW, ... of the chunk, in that order; unit number k of the
  // wave holds, for this lane, token (wave + k * NW) * TT + ts.  slot_a[u]: slot of unit u; slot_nx[u]: of the unit
  // that takes ring position u next.  pf_slot: the whole list (its first PF * threads entries), one entry per
  // thread and round: staged in LDS below so that the loop finds its slots there instead of in global memory.
  // (These loads need nothing but preloaded arguments: they leave before anything waits for a scalar load.)
  int slot_a[U], slot_nx[U];
  int pf_slot[PF];
  if constexpr (DIRECT) {
#pragma unroll
    for (int u = 0; u < U; ++u) slot_a[u] = idx[min((wave + u * NW) * TT + ts, sel_cap - 1)];
#pragma unroll
    for (int k = 0; k < PF; ++k) pf_slot[k] = idx[min(tid + k * kAttThreads, sel_cap - 1)];
  }
  // the query token's own K/V row (Section 4.2 append), as this launch attends and stores it: every lane keeps
  // its 16-byte piece in registers; fp32 rows of a bf16 cache are rounded once, here
  const bool append = (heads_and_flags & 0x10000) != 0, new_f32 = (heads_and_flags & 0x20000) != 0;
  uint4 nk = make_uint4(0u, 0u, 0u, 0u), nv = nk;
  if (append) {
    if (EB == 2 && new_f32) {
      const size_t off32 = ((size_t)b * n_heads + head_c) * D * 4 + dl * 32;
      nk = pack8_bf16(k_new_g + off32);
      nv = pack8_bf16(v_new_g + off32);
    } else {
      nk = load16(k_new_g + row_off);
      nv = load16(v_new_g + row_off);
    }
  }
  pin_uniform(cnt_raw); pin_uniform(k_base); pin_uniform(v_base); pin_uniform(score); pin_uniform(pending);
  if constexpr (VF) pin_uniform(u_state);
  // (the remaining arguments the loop needs: fetched in the same batch of scalar loads, not after it)
  pin_uniform(A.cap); pin_uniform(A.chunk_max); pin_uniform(A.slot_stride_b); pin_uniform(A.head_stride_b);
  pin_uniform(A.scale_log2); pin_uniform(A.accumulate);

  const int cnt = min(cnt_raw, sel_cap);
  if (cnt <= 0) {                                   // inactive or rejected sequence: zero-filled row
    if (chunk == 0) {
      for (int o = tid; o < HT * D; o += kAttThreads) {
        const int hd = hg * HT + o / D;
        if (hd < A.n_heads) {
          const size_t oi = ((size_t)b * A.n_heads + hd) * D + (o % D);
          if (EB == 4) reinterpret_cast<gfloat*>(out_g)[oi] = 0.0f;
          else reinterpret_cast<ADSA_GLOBAL uint16_t*>(out_g)[oi] = 0;
          if (o % D == 0) lse_g[(size_t)b * A.n_heads + hd] = 0.0f;
        }
      }
    }
    return;
  }
  const int t_begin = DIRECT ? 0 : chunk_begin(cnt, chunk, n_chunks);
  const int t_end = DIRECT ? cnt : chunk_begin(cnt, chunk + 1, n_chunks);
  if (t_begin >= t_end) return;                     // fewer tokens than chunks
  const int len = t_end - t_begin;
  const float inv_len = 1.0f / (float)len;
  int* const s_idx = reinterpret_cast<int*>(s_logit + (VF ? 2 : HT) * A.chunk_max);   // the chunk's slot list (filled below)
  if constexpr (!DIRECT) {
#pragma unroll
    for (int u = 0; u < U; ++u) slot_a[u] = idx[t_begin + min((wave + u * NW) * TT + ts, len - 1)];
  }
  // the slot adsa_select reserved for the query token (Section 4.2 append), if this launch fills it
  const int new_slot = (append && pending < A.cap) ? pending : -1;

  const int n_pairs = heads_here * len;
  float pf_old[PF];
  float qf[EPL];
  Elems<EB>::unpack(qr, qf);
#pragma unroll
  for (int e = 0; e < EPL; ++e) qf[e] *= A.scale_log2;
  const long long lane_off = (long long)head_c * A.head_stride_b + dl * 16;
  gchar* kb = k_base + lane_off;
  gchar* vb = v_base + lane_off;
  // VF: this lane's columns of u for its head, and the two score rows of the head
  float uf[EPL];
  gfloat* vrows = nullptr;
  bool vf_on = false;
  if constexpr (VF) {
    vf_on = u_state != nullptr && head_ok;
#pragma unroll
    for (int e = 0; e < EPL; ++e) uf[e] = vf_on ? u_state[(size_t)head_c * D + dl * EPL + e] : 0.0f;
    vrows = score + (size_t)(2 * head_c) * A.cap;
  }

  float m = -INFINITY, l = 0.0f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.0f;

  // Rolling gather: U units (row pairs per lane) are in flight per wave; as soon as the oldest has arrived it is
  // folded into the lane's online-softmax state and its registers are given to the next unit's loads, so the
  // number of outstanding requests stays constant instead of draining once per batch.
  {
    const int n_units = (len + TT - 1) / TT;
    const int n_mine = n_units > wave ? (n_units - wave + NW - 1) / NW : 0;       // units of this wave
    uint4 kr[U], vr[U];
    int tok[U];                                     // token (chunk-relative) in flight at ring position u; >= len: none
    bool fresh[U];                                  // ring position u stands for the query token's own row
#pragma unroll
    for (int u = 0; u < U; ++u) { kr[u] = make_uint4(0u, 0u, 0u, 0u); vr[u] = kr[u]; tok[u] = len; fresh[u] = false; }
    auto issue = [&](int u, int slot_raw, int token) {
      const int slot = min(max(slot_raw, 0), A.cap - 1);      // never touch memory outside the cache
      const long long off = (long long)slot * A.slot_stride_b;
      const bool is_new = slot == new_slot;         // the query token itself: its row is in registers (nk, nv)
      const bool live = token < len && !is_new;     // else (also past the end of the chunk) re-read q's row: cached
      kr[u] = load_stream16(live ? kb + off : q_g + row_off);
      vr[u] = load_stream16(live ? vb + off : q_g + row_off);
      tok[u] = token;
      fresh[u] = is_new;
    };
    auto fold = [&](int u) {
      const bool on = tok[u] < len;
      const uint4 kx = fresh[u] ? nk : kr[u], vx = fresh[u] ? nv : vr[u];
      float kf[EPL];
      Elems<EB>::unpack(kx, kf);
      float d = 0.0f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kf[e], d);
      d = row_sum<LPR>(d);
      const float z = on ? d : -INFINITY;
      if (A.accumulate && dl == 0 && on) s_logit[hs * A.chunk_max + tok[u]] = z;
      const float m_new = fmaxf(m, z);
      const float corr = (m == -INFINITY) ? 0.0f : fast_exp2(m - m_new);     // (l and acc are 0 while m is -inf)
      const float pr = on ? fast_exp2(z - m_new) : 0.0f;
      float vf[EPL];
      Elems<EB>::unpack(vx, vf);
      l = fmaf(l, corr, pr);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = fmaf(acc[e], corr, pr * vf[e]);
      m = m_new;
      if constexpr (VF) {                           // Eq. 2-3 bookkeeping of this row: |v_h|^2 and v_h . u_h
        float dv = 0.0f, sv = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) { dv = fmaf(vf[e], uf[e], dv); sv = fmaf(vf[e], vf[e], sv); }
        dv = row_sum<LPR>(dv);
        sv = row_sum<LPR>(sv);
        if (dl == 0 && on) { s_logit[tok[u]] = sv; s_logit[A.chunk_max + tok[u]] = dv; }
      }
      // the state is demanded HERE, and no memory access may cross: the unit is folded completely before the
      // loads that reuse its ring position are issued, and no later unit's arithmetic is pulled in front of it
      // (left to itself the compiler gathers all the logits of a trip first and so waits for the whole ring)
      static_assert(EPL == 4 || EPL == 8, "elements per lane");
      if constexpr (EPL == 8)
        asm volatile("" : "+v"(m), "+v"(l), "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]),
                     "+v"(acc[5]), "+v"(acc[6]), "+v"(acc[7]) : : "memory");
      else
        asm volatile("" : "+v"(m), "+v"(l), "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]) : : "memory");
    };
    // unit k of the wave lives at ring position k % U: units 0 .. U-1 are requested here, trip t folds units
    // tU .. tU+U-1 and requests the units one ring revolution later, the last trip only folds.  (Units past
    // the wave's last one re-read the q row, which is cached by then.)
    auto refill = [&](int u, int k, int slot_raw) { // ring position u <- unit k; fetch the slot of unit k + U
      const int token = (wave + k * NW) * TT + ts;
      issue(u, slot_raw, token);
      slot_nx[u] = s_idx[min(token + U * NW * TT, len - 1)];
      asm volatile("" : : : "memory");             // requests leave in ring order (the wait counts rely on it)
      __builtin_amdgcn_sched_barrier(0);            // ... and before the next unit's arithmetic, which waits for ITS rows
    };
    const int n_trips = (n_mine + U - 1) / U;
    // The first revolution's rows are requested at once, from the slots the first round trip brought in registers ...
#pragma unroll
    for (int u = 0; u < U; ++u) {
      issue(u, slot_a[u], (wave + u * NW) * TT + ts);
      asm volatile("" : : : "memory");
      __builtin_amdgcn_sched_barrier(0);
    }
    // ... and while they are on their way the chunk's slot list goes to LDS (clamped to the cache: nothing below
    // ever leaves it), where the later revolutions and the score update find it
    if constexpr (DIRECT) {
#pragma unroll
      for (int k = 0; k < PF; ++k) {
        const int j = tid + k * kAttThreads;
        if (j < len) s_idx[j] = min(max(pf_slot[k], 0), A.cap - 1);
      }
      for (int j = tid + PF * kAttThreads; j < len; j += kAttThreads) s_idx[j] = min(max(idx[j], 0), A.cap - 1);
    } else {
      for (int j = tid; j < len; j += kAttThreads) s_idx[j] = min(max(idx[t_begin + j], 0), A.cap - 1);
    }
    __syncthreads();
    // pair i of the final score update is (head i / len, token i % len); start the first PF reads now
    if (DIRECT && A.accumulate) {
#pragma unroll
      for (int k = 0; k < PF; ++k) {
        const int i = tid + k * kAttThreads;
        pf_old[k] = 0.0f;
        if (i < n_pairs) {
          int sb = 0, j = i;
          if constexpr (HT > 1) { sb = small_div(i, len, inv_len); j = i - sb * len; }   // several heads per workgroup
          pf_slot[k] = s_idx[j];
          pf_old[k] = score[(size_t)(hg * HT + sb) * A.cap + pf_slot[k]];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) slot_nx[u] = s_idx[min((wave + (u + U) * NW) * TT + ts, len - 1)];
    asm volatile("" : : : "memory");
    __builtin_amdgcn_sched_barrier(0);
    int k_next = U;
    for (int trip = 1; trip < n_trips; ++trip) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        fold(u);
        refill(u, k_next + u, slot_nx[u]);
      }
      k_next += U;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) fold(u);
  }
  // ---- merge, step 1 (registers): the TT lane groups of a wave that worked on the same head bring their
  // states to the wave's maximum and add them up across lanes; every lane ends up with the wave's state.
  if constexpr (TT > 1) {
    float M = m;
#pragma unroll
    for (int x = LPR * HT; x < kWave; x <<= 1)
      M = x == 8 ? xor_max<8>(M) : x == 16 ? xor_max<16>(M) : xor_max<32>(M);
    const float sc = (m == -INFINITY) ? 0.0f : fast_exp2(m - M);     // a group that saw no token weighs 0
    l *= sc;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= sc;
#pragma unroll
    for (int x = LPR * HT; x < kWave; x <<= 1) {
      l = x == 8 ? xor_sum<8>(l) : x == 16 ? xor_sum<16>(l) : xor_sum<32>(l);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = x == 8 ? xor_sum<8>(acc[e]) : x == 16 ? xor_sum<16>(acc[e]) : xor_sum<32>(acc[e]);
    }
    m = M;
  }
  // ---- step 2 (LDS): one state per (wave, head); after ONE barrier every thread works out the
  // normalisers it needs itself, the first HT*D threads each finish one output element
  if (ts == 0) {
    if (dl == 0) { s_wm[wave][hs] = m; s_wl[wave][hs] = l; }
    float4* dst = reinterpret_cast<float4*>(&s_wacc[(wave * HT + hs) * D + dl * EPL]);
#pragma unroll
    for (int e = 0; e < EPL; e += 4) dst[e / 4] = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
  }
  __syncthreads();
  // Section 4.2: the query token's row enters the cache (nothing in this launch reads it from there)
  if (new_slot >= 0 && chunk == n_chunks - 1 && wave == 0 && ts == 0 && head_ok) {
    const long long off = (long long)new_slot * A.slot_stride_b;
    store16(kb + off, nk);
    store16(vb + off, nv);
  }
  for (int o = tid; o < heads_here * D; o += kAttThreads) {
    const int sb = o / D, d = o - sb * D;
    float mw[NW], M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) { mw[w] = s_wm[w][sb]; M = fmaxf(M, mw[w]); }
    float L = 0.0f, a = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wgt = (mw[w] == -INFINITY) ? 0.0f : fast_exp2(mw[w] - M);      // empty wave: weight 0
      L = fmaf(s_wl[w][sb], wgt, L);
      a = fmaf(s_wacc[(w * HT + sb) * D + d], wgt, a);
    }
    const int hd = hg * HT + sb;
    if constexpr (DIRECT) {
      const float val = __fdividef(a, L);
      const size_t oi = ((size_t)b * A.n_heads + hd) * D + d;
      if (EB == 4) reinterpret_cast<gfloat*>(out_g)[oi] = val;
      else reinterpret_cast<ADSA_GLOBAL uint16_t*>(out_g)[oi] = (uint16_t)f32_to_bf16_rne(val);
      if (d == 0) lse_g[(size_t)b * A.n_heads + hd] = (M + __log2f(L)) * kLn2;
    } else {
      const size_t pidx = ((size_t)b * A.n_heads + hd) * n_chunks + chunk;
      st_dev(A.part_acc + pidx * D + d, a);
      if (d == 0) st_dev2(A.part_ml + pidx * 2, M, L);
    }
  }

  if constexpr (VF) {
    // |v_h|^2 and v_h.u_h of this chunk's tokens, left in LDS by the loop (the barrier above ordered them)
    if (vf_on) {
      int j0 = tid;
      if constexpr (DIRECT) {                       // the first slots were fetched before the loop
#pragma unroll
        for (int k = 0; k < PF; ++k) {
          const int j = tid + k * kAttThreads;
          if (j < len) {
            const int slot = min(max(pf_slot[k], 0), A.cap - 1);
            vrows[slot] = s_logit[j];
            vrows[A.cap + slot] = s_logit[A.chunk_max + j];
          }
        }
        j0 = tid + PF * kAttThreads;
      }
      for (int j = j0; j < len; j += kAttThreads) {
        const int slot = s_idx[j];
        vrows[slot] = s_logit[j];
        vrows[A.cap + slot] = s_logit[A.chunk_max + j];
      }
    }
  }
  if constexpr (DIRECT) {
    // -------- per-head attention mass: score[head][slot] += p, from the logits still in LDS
    if (A.accumulate) {
      // log2-domain log-sum-exp of the head(s): one head -> every thread redoes the few operations itself
      float lse2_0 = 0.0f;
      if constexpr (HT == 1) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, s_wm[w][0]);
        float L = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const float mp = s_wm[w][0];
          L = fmaf(s_wl[w][0], (mp == -INFINITY) ? 0.0f : fast_exp2(mp - M), L);
        }
        lse2_0 = M + __log2f(L);
      } else {
        if (tid < heads_here) {
          float M = -INFINITY;
#pragma unroll
          for (int w = 0; w < NW; ++w) M = fmaxf(M, s_wm[w][tid]);
          float L = 0.0f;
#pragma unroll
          for (int w = 0; w < NW; ++w) {
            const float mp = s_wm[w][tid];
            L = fmaf(s_wl[w][tid], (mp == -INFINITY) ? 0.0f : fast_exp2(mp - M), L);
          }
          s_lse2[tid] = M + __log2f(L);
        }
        __syncthreads();
      }
#pragma unroll
      for (int k = 0; k < PF; ++k) {                // reads were started before the loop
        const int i = tid + k * kAttThreads;
        if (i < n_pairs) {
          int sb = 0, j = i;
          float lse2 = lse2_0;
          if constexpr (HT > 1) { sb = small_div(i, len, inv_len); j = i - sb * len; lse2 = s_lse2[sb]; }
          gfloat* sp = score + (size_t)(hg * HT + sb) * A.cap + pf_slot[k];
          const float sv_new = pf_old[k] + fast_exp2(s_logit[sb * A.chunk_max + j] - lse2);
          *sp = sv_new;
        }
      }
      if (n_pairs > PF * kAttThreads) {             // rare long lists
        if constexpr (HT == 1) {
          if (tid == 0) s_lse2[0] = lse2_0;
          __syncthreads();
        }
        const int cm = A.chunk_max;
        add_mass(score, A.cap, hg * HT, s_lse2, n_pairs - PF * kAttThreads, [=](int i, int* sb, int* slot, float* z) {
          const int ii = i + PF * kAttThreads;
          *sb = HT == 1 ? 0 : small_div(ii, len, inv_len); const int j = ii - *sb * len;
          *slot = s_idx[j]; *z = s_logit[*sb * cm + j];
        });
      }
    }
    // last act on a sequence (one thread; no other workgroup reads step): VF marks the score rows as the
    // next step's if u was (tags kept as floats behind u); then the step may advance.  (Written out here:
    // handing the kernel's argument struct to a helper by reference made every variant slower.)
    if (hg == 0 && tid == 0) {
      if constexpr (VF) {
        if (u_state) {
          gfloat* tags = u_state + (size_t)A.n_heads * D;
          const float want = (float)(sqp->step + 2);
          tags[1] = tags[0] == want ? want : 0.0f;
        }
      }
      if (A.advance) sqp->step = sqp->step + 1;
    }
    return;
  } else {
    // -------- several chunks: publish logits, arrive, and let the last workgroup finish the group.
    // Hand-off between workgroups (possibly on different XCDs, whose L2s are not coherent with each
    // other): partials and logits are written with device-scope atomic stores (written through, never
    // left dirty in an L2); every thread waits until its own stores have completed, the barrier
    // collects the workgroup, and one thread bumps the arrival counter with a device-scope
    // release/acquire read-modify-write.  The workgroup that draws the last ticket reads the partials
    // with device-scope atomic loads, issued after the barrier that follows its acquire.
    if (A.accumulate) {
      for (int i = tid; i < heads_here * len; i += kAttThreads) {
        const int sb = HT == 1 ? 0 : small_div(i, len, inv_len), j = i - sb * len;
        st_dev(A.logits + ((size_t)b * A.n_heads + hg * HT + sb) * A.lg_stride + t_begin + j, s_logit[sb * A.chunk_max + j]);
      }
    }
    const int n_nonempty = min(cnt, n_chunks);
    int32_t* ctr = A.counters + (size_t)b * A.n_hg + hg;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this thread's stores have completed ...
    __syncthreads();                                          // ... and so have everybody's, before thread 0 announces them
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != n_nonempty - 1) return;
    if (tid == 0) *ctr = 0;                         // ready for the next launch

    const bool all_full = cnt >= n_chunks;          // else only `cnt` scattered chunks hold a token
    for (int o = tid; o < heads_here * D; o += kAttThreads) {
      const int sb = o / D, d = o - sb * D;
      const int hd = hg * HT + sb;
      const size_t pbase = ((size_t)b * A.n_heads + hd) * n_chunks;
      float mc[kMaxChunks], lc[kMaxChunks], ac[kMaxChunks];
#pragma unroll
      for (int c = 0; c < kMaxChunks; ++c) {        // all loads in flight together
        const bool on = c < n_chunks && (all_full || chunk_begin(cnt, c, n_chunks) < chunk_begin(cnt, c + 1, n_chunks));
        mc[c] = on ? ld_dev(A.part_ml + (pbase + c) * 2) : -INFINITY;
        lc[c] = on ? ld_dev(A.part_ml + (pbase + c) * 2 + 1) : 0.0f;
        ac[c] = on ? ld_dev(A.part_acc + (pbase + c) * D + d) : 0.0f;
      }
      float Mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < kMaxChunks; ++c) Mx = fmaxf(Mx, mc[c]);
      float Lx = 0.0f, a = 0.0f;
#pragma unroll
      for (int c = 0; c < kMaxChunks; ++c) {
        const float wgt = (mc[c] == -INFINITY) ? 0.0f : fast_exp2(mc[c] - Mx);
        Lx = fmaf(lc[c], wgt, Lx);
        a = fmaf(ac[c], wgt, a);
      }
      const float val = __fdividef(a, Lx);
      const size_t oi = ((size_t)b * A.n_heads + hd) * D + d;
      if (EB == 4) reinterpret_cast<gfloat*>(out_g)[oi] = val;
      else reinterpret_cast<ADSA_GLOBAL uint16_t*>(out_g)[oi] = (uint16_t)f32_to_bf16_rne(val);
      if (d == 0) {
        const float lse2 = Mx + __log2f(Lx);
        lse_g[(size_t)b * A.n_heads + hd] = lse2 * kLn2;
        s_lse2[sb] = lse2;
      }
    }
    if (A.accumulate) {
      __syncthreads();
      const float* lg = A.logits + ((size_t)b * A.n_heads + hg * HT) * A.lg_stride;
      const int lgs = A.lg_stride, cap = A.cap;
      const float inv_cnt = 1.0f / (float)cnt;
      add_mass(score, A.cap, hg * HT, s_lse2, heads_here * cnt, [=](int i, int* sb, int* slot, float* z) {
        *sb = HT == 1 ? 0 : small_div(i, cnt, inv_cnt); const int j = i - *sb * cnt;
        *slot = min(max(idx[j], 0), cap - 1); *z = ld_dev(lg + (size_t)*sb * lgs + j);
      });
    }
    if (hg == 0 && tid == 0) {
      if constexpr (VF) {
        if (u_state) {
          gfloat* tags = u_state + (size_t)A.n_heads * D;
          const float want = (float)(sqp->step + 2);
          tags[1] = tags[0] == want ? want : 0.0f;
        }
      }
      if (A.advance) sqp->step = sqp->step + 1;
    }
  }
}

template <int EB, int D, int HT, int NW, bool VF, bool DIRECT>
hipError_t launch_attend_w(const AttendArgs& A, const AttendPlan& plan, int n_seq, hipStream_t st,
                           hipEvent_t ev_start, hipEvent_t ev_stop) {
  // row pairs in flight per lane: 2, 3, 6 and 8 were measured slower on 4-wave workgroups; 16-wave workgroups
  // (at most 128 registers per lane: the kernel needs < 100) run the same within 1 % with 2 or 4
  constexpr int U = 4;
  const size_t lds = (size_t)((VF ? 2 : HT) + 1) * plan.chunk_max * sizeof(float);      // logits rows + the slot list
  dim3 grid(plan.n_chunks, plan.n_head_groups, n_seq);
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL((k_attend<EB, D, HT, U, NW, VF, DIRECT>), grid, dim3(NW * kWave), (uint32_t)lds, st, ev_start, ev_stop, 0,
                          A.seqs, A.sel_idx, A.sel_cnt, A.q, A.k_new, A.v_new,
                          A.n_heads | (A.append ? 0x10000 : 0) | (A.new_f32 ? 0x20000 : 0), A.sel_cap, A);
  else
    hipLaunchKernelGGL((k_attend<EB, D, HT, U, NW, VF, DIRECT>), grid, dim3(NW * kWave), lds, st,
                       A.seqs, A.sel_idx, A.sel_cnt, A.q, A.k_new, A.v_new,
                          A.n_heads | (A.append ? 0x10000 : 0) | (A.new_f32 ? 0x20000 : 0), A.sel_cap, A);
  return hipGetLastError();
}

template <int EB, int D, int HT, bool VF>
hipError_t launch_attend_v(const AttendArgs& A, const AttendPlan& plan, int n_seq, hipStream_t st,
                           hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (plan.n_chunks > 1)       // split lists always run with 4-wave workgroups
    return launch_attend_w<EB, D, HT, 4, VF, false>(A, plan, n_seq, st, ev_start, ev_stop);
  if (plan.waves == 16) return launch_attend_w<EB, D, HT, 16, VF, true>(A, plan, n_seq, st, ev_start, ev_stop);
  if (plan.waves == 8) return launch_attend_w<EB, D, HT, 8, VF, true>(A, plan, n_seq, st, ev_start, ev_stop);
  return launch_attend_w<EB, D, HT, 4, VF, true>(A, plan, n_seq, st, ev_start, ev_stop);
}

template <int EB, int D, int HT>
hipError_t launch_attend_t(const AttendArgs& A, const AttendPlan& plan, int n_seq, hipStream_t st,
                           hipEvent_t ev_start, hipEvent_t ev_stop) {
  if constexpr (HT == 1) {
    if (A.vcos_fused) return launch_attend_v<EB, D, HT, true>(A, plan, n_seq, st, ev_start, ev_stop);
  }
  return launch_attend_v<EB, D, HT, false>(A, plan, n_seq, st, ev_start, ev_stop);
}

__global__ void k_zero_words(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

}  // namespace

AttendPlan make_attend_plan(const adsa_params& p) {
  AttendPlan a;
  const int epl = 16 / elem_bytes(p);
  a.lanes_per_row = p.head_dim / epl;
  const int rpw = kWave / a.lanes_per_row;
  // [slot][head][D]: a wave-load takes rpw heads of one token; [head][slot][D]: rpw tokens of one head
  a.head_major = p.kv_slot_stride < p.kv_head_stride;
  if (p.q_per_kv > 1) {      // grouped queries: one workgroup per (sequence, cache head, chunk of whole 16-token tiles)
    a.heads_per_group = 1;
    a.n_head_groups = p.n_heads;
    const long long wgs = (long long)p.n_seq * p.n_heads;
    a.waves = wgs >= 512 ? 4 : 8;
    // Lists are split only when they must be (the logits of a whole list, all G queries, do not fit in LDS even
    // with 4 waves) or when it was measured to pay: long lists (>= 2560 slots) of at most 32 (sequence, cache head)
    // pairs.  The hand-off between workgroups costs a release/acquire at device scope per workgroup, which grows
    // with the number of workgroups: 88 pairs x 16 chunks of 2800-token lists took 82 us, unsplit 42 us; one
    // sequence (8 pairs) 25 us against 41 us.  Hence: as many chunks as fit the LDS limit, and more only while the
    // launch stays near 128 workgroups.
    int nc = 1;
    const bool must = gqa_lds_bytes(p, 4, 1) > kGqaMaxLds;
    if (must || (p.sel_cap >= 2560 && wgs <= 32)) {
      while (nc < kMaxChunks && gqa_lds_bytes(p, 4, nc) > kGqaMaxLds) ++nc;
      int more = (int)((128 + wgs - 1) / wgs);
      if (more > p.sel_cap / 160) more = p.sel_cap / 160;
      if (more > kMaxChunks) more = kMaxChunks;
      if (nc < more) nc = more;
    }
    while (nc == 1 && a.waves > 4 && gqa_lds_bytes(p, a.waves, 1) > kGqaMaxLds) a.waves /= 2;
    if (nc > 1) a.waves = 4;
    a.n_chunks = nc;
    a.chunk_max = gqa_logit_stride(p, nc);
    return a;
  }
  a.heads_per_group = a.head_major ? 1 : rpw;
  a.n_head_groups = (p.n_heads + a.heads_per_group - 1) / a.heads_per_group;
  // One workgroup per (sequence, head group) whenever there are enough of them to keep ~16 MB of
  // loads in flight chip-wide: 4 waves each from 512 pairs up, 8 or 16 waves for fewer (HBM is shared,
  // so a CU holding two workgroups is no slower per byte).  Only tiny batches split the list, until
  // ~768 workgroups, never below 32 tokens per chunk.
  const long long pairs = (long long)p.n_seq * a.n_head_groups;
  a.waves = pairs >= 512 ? 4 : pairs >= 256 ? 8 : pairs >= 96 ? 16 : 4;
  int nc = 1;
  if (pairs < 96) {
    nc = (int)((768 + pairs - 1) / pairs);
    int max_by_len = p.sel_cap / 32;
    if (max_by_len < 1) max_by_len = 1;
    if (nc > max_by_len) nc = max_by_len;
    if (nc > kMaxChunks) nc = kMaxChunks;
  }
  // the logits tile [heads_per_group][chunk] must fit in LDS next to the merge buffers
  const int lds_rows = (p.score_mode == ADSA_SCORE_VCOS_FUSED ? 2 : a.heads_per_group) + 1;   // words of LDS per token
  while (nc < kMaxChunks && (size_t)lds_rows * ((p.sel_cap + nc - 1) / nc + 1) * sizeof(float) > 40 * 1024) ++nc;
  if (nc > 1) a.waves = 4;      // split lists run as 4-wave workgroups (more of them instead of wider ones)
  a.n_chunks = nc;
  a.chunk_max = (p.sel_cap + nc - 1) / nc + 1;
  return a;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Workspace make_workspace(const adsa_params& p, const AttendPlan& plan) {
  Workspace w;
  size_t off = 0;
  const bool split = plan.n_chunks > 1;
  const size_t hq = (size_t)p.n_heads * (p.q_per_kv > 1 ? p.q_per_kv : 1);      // rows of out / logits / partials per sequence
  w.lg_stride = p.q_per_kv > 1 ? gqa_global_logit_stride(p) : (int)align_up((size_t)p.sel_cap, 4);
  w.counters_off = off;
  off = align_up(off + sizeof(int32_t) * (size_t)p.n_seq * plan.n_head_groups, 256);
  w.persistent_bytes = off;     // must stay zero between launches
  w.logits_off = off;
  if (split) off = align_up(off + sizeof(float) * (size_t)p.n_seq * hq * w.lg_stride, 256);
  w.part_ml_off = off;
  if (split) off = align_up(off + sizeof(float) * (size_t)p.n_seq * hq * plan.n_chunks * 2, 256);
  w.part_acc_off = off;
  if (split) off = align_up(off + sizeof(float) * (size_t)p.n_seq * hq * plan.n_chunks * p.head_dim, 256);
  w.plan_off = off;
  off = align_up(off + sizeof(int32_t) * (size_t)p.n_seq * 4, 256);
  w.vcos_off = off;
  w.vcos_u_off = off;
  w.vcos_s_off = off;
  if (is_vcos(p)) {
    off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.cap, 256);
    w.vcos_u_off = off;
    off = align_up(off + sizeof(float) * (size_t)p.n_seq * vcos_tiles(p.cap) * p.n_heads * p.head_dim, 256);
    w.vcos_s_off = off;
    if (p.score_mode == ADSA_SCORE_VCOS_FUSED) off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.cap, 256);
  }
  w.total = off;
  return w;
}

hipError_t launch_workspace_init(char* ws, const Workspace& w, hipStream_t st) {
  const size_t words = w.persistent_bytes / 4;
  hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(ws + w.counters_off), words);
  return hipGetLastError();
}

hipError_t launch_attend(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                         const void* k_new, const void* v_new, const int32_t* sel_idx, const int32_t* sel_cnt,
                         void* out, float* lse, char* ws, const Workspace& w, bool accumulate, bool append,
                         bool advance, bool new_f32, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (p.q_per_kv > 1)
    return launch_attend_gqa(p, plan, seqs, q, k_new, v_new, sel_idx, sel_cnt, out, lse, ws, w, accumulate, append,
                             advance, new_f32, st, ev_start, ev_stop);
  AttendArgs A;
  A.seqs = seqs; A.q = (const char*)q; A.k_new = (const char*)k_new; A.v_new = (const char*)v_new;
  A.sel_idx = sel_idx; A.sel_cnt = sel_cnt; A.out = (char*)out; A.lse = lse;
  A.logits = reinterpret_cast<float*>(ws + w.logits_off);
  A.part_ml = reinterpret_cast<float*>(ws + w.part_ml_off);
  A.part_acc = reinterpret_cast<float*>(ws + w.part_acc_off);
  A.counters = reinterpret_cast<int32_t*>(ws + w.counters_off);
  A.n_heads = p.n_heads; A.n_hg = plan.n_head_groups; A.sel_cap = p.sel_cap; A.lg_stride = w.lg_stride;
  A.chunk_max = plan.chunk_max; A.cap = p.cap;
  A.accumulate = accumulate ? 1 : 0; A.append = append ? 1 : 0; A.advance = advance ? 1 : 0;
  A.new_f32 = (new_f32 && append) ? 1 : 0;
  A.vcos_fused = p.score_mode == ADSA_SCORE_VCOS_FUSED ? 1 : 0;
  const int eb = elem_bytes(p);
  A.slot_stride_b = (long long)p.kv_slot_stride * eb;
  A.head_stride_b = (long long)p.kv_head_stride * eb;
  const float scale = p.softmax_scale != 0.0f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  A.scale_log2 = scale * kLog2e;
  const int key = eb * 1000 + p.head_dim;
  if (plan.head_major) {
    if (key == 2064) return launch_attend_t<2, 64, 1>(A, plan, p.n_seq, st, ev_start, ev_stop);
    if (key == 2128) return launch_attend_t<2, 128, 1>(A, plan, p.n_seq, st, ev_start, ev_stop);
    if (key == 4064) return launch_attend_t<4, 64, 1>(A, plan, p.n_seq, st, ev_start, ev_stop);
    if (key == 4128) return launch_attend_t<4, 128, 1>(A, plan, p.n_seq, st, ev_start, ev_stop);
  } else {
    if (key == 2064) return launch_attend_t<2, 64, 8>(A, plan, p.n_seq, st, ev_start, ev_stop);
    if (key == 2128) return launch_attend_t<2, 128, 4>(A, plan, p.n_seq, st, ev_start, ev_stop);
    if (key == 4064) return launch_attend_t<4, 64, 4>(A, plan, p.n_seq, st, ev_start, ev_stop);
    if (key == 4128) return launch_attend_t<4, 128, 2>(A, plan, p.n_seq, st, ev_start, ev_stop);
  }
  return hipErrorInvalidValue;
}

}  // namespace adsa
