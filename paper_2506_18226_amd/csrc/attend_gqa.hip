// Grouped-query gather flash-decode of the ADSA decode path (gfx950): Eq. 5's gather + softmax
// attention when G = 2..16 query heads share one cache head.  Every K/V row read from HBM now
// meets G queries, so the two products are small dense contractions and run on the matrix cores
// (v_mfma_f32_16x16x16_bf16, fp32 accumulation); the kernel is still bound by the HBM stream.
//
//  k_attend_gqa<D, NW> : grid (cache head, sequence), NW waves.  The list is cut into 16-token tiles,
//  dealt round-robin to the waves of the workgroup (a fixed assignment: results are reproducible bit
//  for bit; claiming tiles from a counter was measured no faster), and each wave runs its own online
//  softmax:
//    S[t][g] = K[t] . q[g]   K rows are fetched with coalesced 16-byte loads and staged through a
//            wave-private LDS tile (the MFMA operand layout wants lane%16 = token; a global load in
//            that shape would touch 16 rows per quarter wave), then multiplied with the G (<= 16)
//            query rows held in registers.  The product comes out with lane%16 = query and 4
//            consecutive tokens per lane: exactly the operand layout of the next product, so the
//            probabilities never leave the registers.  The scaled logits (log2 units) are also kept
//            in LDS, [G][list], for the score update.
//    out[g][:] += 2^(S - m[g]) V[t]   V rows come straight from HBM in operand layout: a lane loads the
//            same D/16 columns of 4 tokens and transposes the 4 x D/16 block in registers (the
//            contraction runs over tokens).  P is split into two bf16 halves (hi + lo) so that the
//            product carries ~16 mantissa bits of the probabilities.  When a query's running maximum
//            m[g] grows, the accumulators are rescaled (factors fetched across lanes).
//    Each wave keeps a small ring of tiles in flight: it waits for the OLDEST tile's K rows only (in-order wait
//    counts; a tile is always requested as its K loads followed by its V loads, with no branch in between),
//    multiplies it and refills its registers with the tile one ring revolution later.  Loads take a uniform base
//    and a 32-bit lane offset; the query token's own slot is read like any other and replaced from registers.
//    The first round trip (count, sequence record, q, slot list, the query token's row) depends on preloaded
//    kernel arguments only, and leaves before anything waits for a scalar load.
//    At the end the waves' (m, l, partial out) are merged through LDS in wave order, the workgroup writes
//    out / lse for its G query heads and adds the probabilities of all G queries, summed in ascending head
//    order, to its OWN cache head's row of score[]: no workgroup talks to another.
#include <hip/hip_ext.h>

#include "adsa_internal.h"
#include "adsa_device.h"

namespace adsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ s16x4 as_bf16x4(uint32_t lo, uint32_t hi) {
  const u32x2 v = {lo, hi};
  return __builtin_bit_cast(s16x4, v);
}

__device__ __forceinline__ f32x4 mfma_bf16(s16x4 a, s16x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}

// Lanes of one wave hand data to each other through LDS: LDS instructions of a wave execute in
// issue order, so only the compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// c ? a : b by components (a ternary on the structs themselves would select between their ADDRESSES and
// keep both in memory)
__device__ __forceinline__ uint4 pick16(bool c, const uint4& a, const uint4& b) {
  return make_uint4(c ? a.x : b.x, c ? a.y : b.y, c ? a.z : b.z, c ? a.w : b.w);
}

// 2 or 4 dwords of a V row: streaming (nontemporal) or plain
template <int W, bool stream>
__device__ __forceinline__ void vload(const gchar* p, uint32_t* w) {
  if constexpr (W == 2) {
    u32x2 v;
    if constexpr (stream) v = __builtin_nontemporal_load(reinterpret_cast<const ADSA_GLOBAL u32x2*>(p));
    else v = *reinterpret_cast<const ADSA_GLOBAL u32x2*>(p);
    w[0] = v.x; w[1] = v.y;
  } else {
    uint4 v;
    if constexpr (stream) v = load_stream16(p);
    else v = load16(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
}

struct GqaArgs {
  adsa_seq* seqs;
  const char* q;
  const char* k_new;
  const char* v_new;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  char* out;
  float* lse;
  float* logits;        // [n_seq][n_heads * G][lg_global]  scaled logits, log2 units (split launches)
  float* part_ml;       // [n_seq][n_heads * G][n_chunks][2]
  float* part_acc;      // [n_seq][n_heads * G][n_chunks][D]
  int32_t* counters;    // [n_seq][n_heads]                 arrival counters, zero between launches
  int lg_global;        // row stride of logits
  int n_heads, G, sel_cap, lg_stride, cap, stage_b;
  int accumulate, append, advance;
  int new_f32;          // k_new / v_new are fp32 although the cache is bf16: round as they enter
  long long slot_stride_b, head_stride_b;
  float scale_log2;
};

// The arguments the first round trip needs come first, as plain scalars (the build asks for leading kernel
// arguments to be preloaded into scalar registers at wave launch): the vector loads of that trip then leave
// without waiting for a scalar load of the argument block.  Only 14 dwords are preloaded, so the group size and
// the two append flags ride on the head count: heads | G << 16 | append << 24 | new_f32 << 25.
// SPLIT: the list of a (sequence, cache head) is cut into gridDim.z chunks of whole 16-token tiles, one workgroup
// each; every workgroup leaves a partial and its logits in the workspace and the LAST one to arrive merges them, in
// chunk order (an arrival counter; nothing waits).
template <int D, int NW, bool SPLIT>
__global__ __launch_bounds__(NW * kWave) void k_attend_gqa(adsa_seq* seqs_arg, const int32_t* sel_idx_arg, const int32_t* sel_cnt_arg,
                                                          const char* q_arg, const char* k_new_arg, const char* v_new_arg,
                                                          int heads_g_flags, int sel_cap_arg, GqaArgs A) {
  constexpr int T = NW * kWave;
  constexpr int ROWB = D * 2 + 16;          // bytes of a staged K row (padded against bank conflicts)
  constexpr int LPR = D / 8;                // lanes per K row with 16-byte loads
  constexpr int RPL = kWave / LPR;          // rows per wave-load
  constexpr int LT = 16 / RPL;              // wave-loads per 16-token tile
  constexpr int NC = D / 16;                // 16-wide chunks of the q.k contraction
  constexpr int EV = D / 16;                // V columns a lane holds per token
  constexpr int VW = EV / 2;                // dwords of V a lane loads per token
  constexpr int R = D == 64 ? 4 : 2;        // tiles in flight per wave (a ring: the oldest is multiplied, then refilled;
                                            // 1, 2 and 3 were measured within 1 % of each other on 8 x 128 x 8-wave lists)
  constexpr int PF = 2048 / T;              // slot-list entries a thread fetches in the first round trip
  extern __shared__ __align__(16) char smem[];
  __shared__ float s_wm[NW][16], s_wl[NW][16], s_lse2[16], s_m[16], s_l[16];
  __shared__ int s_ticket;

  const int hk = blockIdx.x, b = blockIdx.y;
  const int chunk = SPLIT ? blockIdx.z : 0, n_chunks = SPLIT ? gridDim.z : 1;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int r = lane & 15, kg = lane >> 4;                 // matrix-operand role of this lane
  const int n_heads = heads_g_flags & 0xFFFF, G = (heads_g_flags >> 16) & 0xFF, sel_cap = sel_cap_arg;
  const bool append = (heads_g_flags & (1 << 24)) != 0, cvt = (heads_g_flags & (1 << 25)) != 0;
  const int HQ = n_heads * G;

  // ---- first round trip: the count and the sequence record (scalar loads), q, the whole slot list (one entry per
  // thread and round) and the query token's own K/V row as this launch attends and stores it -- everything that
  // depends on the kernel arguments only.  The record and the count are pinned so that they cannot drift behind
  // the count test below, into a second, dependent trip.
  ADSA_GLOBAL adsa_seq* const sqp = (ADSA_GLOBAL adsa_seq*)(seqs_arg + b);
  const int cnt_raw = ((const gint*)sel_cnt_arg)[b];
  gchar* const k_rec = (gchar*)sqp->k;
  gchar* const v_rec = (gchar*)sqp->v;
  gfloat* const score_rec = (gfloat*)sqp->score;
  const int pending = sqp->pending_slot;
  const gint* const idx = (const gint*)sel_idx_arg + (size_t)b * sel_cap;
  const gchar* const q_g = (const gchar*)q_arg;
  // q as the B operand of the first product: lane (g = r, kg) holds columns [D/4*kg, D/4*(kg+1)) of query g
  const gchar* const q_row0 = q_g + ((size_t)b * HQ + (size_t)hk * G) * D * 2;        // query 0 of this cache head
  uint4 qx[NC / 2];
#pragma unroll
  for (int c2 = 0; c2 < NC / 2; ++c2) qx[c2] = load16(q_row0 + ((size_t)min(r, G - 1) * D + (D / 4) * kg) * 2 + c2 * 16);
  int pf_slot[PF];                                   // (a chunk of a split list starts where the count says: fetched below)
  if constexpr (!SPLIT) {
#pragma unroll
    for (int k = 0; k < PF; ++k) pf_slot[k] = idx[min(tid + k * T, sel_cap - 1)];
  }
  // the query token's row (Section 4.2 append); fp32 rows are rounded once, here: every lane keeps the pieces of
  // the rounded row it would load from the cache (K: 16 bytes at ld_piece, V: its EV columns)
  const int ld_row = lane / LPR, ld_piece = lane - ld_row * LPR;
  const size_t new_row = ((size_t)b * n_heads + hk) * D;
  uint4 nk = make_uint4(0u, 0u, 0u, 0u);
  uint32_t nv[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) nv[i] = 0u;
  if (append) {
    const gchar* const kn = (const gchar*)k_new_arg;
    const gchar* const vn = (const gchar*)v_new_arg;
    if (cvt) {
      nk = pack8_bf16(kn + (new_row + ld_piece * 8) * 4);
      if constexpr (EV == 8) {
        const uint4 x = pack8_bf16(vn + (new_row + r * 8) * 4);
        nv[0] = x.x; nv[1] = x.y; nv[2] = x.z; nv[3] = x.w;
      } else {
        const uint4 x = load16(vn + (new_row + r * 4) * 4);
        nv[0] = f32_to_bf16_rne(__uint_as_float(x.x)) | (f32_to_bf16_rne(__uint_as_float(x.y)) << 16);
        nv[1] = f32_to_bf16_rne(__uint_as_float(x.z)) | (f32_to_bf16_rne(__uint_as_float(x.w)) << 16);
      }
    } else {
      nk = load16(kn + new_row * 2 + ld_piece * 16);
      vload<VW, false>(vn + new_row * 2 + r * (EV * 2), nv);
    }
  }
  pin_uniform(cnt_raw); pin_uniform(k_rec); pin_uniform(v_rec); pin_uniform(score_rec); pin_uniform(pending);
  // (the remaining arguments: fetched in the same batch of scalar loads, not after it)
  pin_uniform(A.cap); pin_uniform(A.lg_stride); pin_uniform(A.stage_b); pin_uniform(A.slot_stride_b);
  pin_uniform(A.head_stride_b); pin_uniform(A.scale_log2); pin_uniform(A.accumulate);

  const int lgs = A.lg_stride;
  float* const s_logit = reinterpret_cast<float*>(smem);                 // [G][lgs]
  int* const s_slot = reinterpret_cast<int*>(s_logit + (size_t)G * lgs); // [lgs]
  char* const s_stage = reinterpret_cast<char*>(s_slot + lgs);           // [NW][stage_b]: K tile [16][ROWB], later partial out [G][D]
  gchar* const k_base = k_rec + (long long)hk * A.head_stride_b;
  gchar* const v_base = v_rec + (long long)hk * A.head_stride_b;
  gfloat* const score = score_rec + (size_t)hk * A.cap;
  ADSA_GLOBAL uint16_t* const out = reinterpret_cast<ADSA_GLOBAL uint16_t*>((gchar*)A.out) + ((size_t)b * HQ + (size_t)hk * G) * D;
  gfloat* const lse = (gfloat*)A.lse + (size_t)b * HQ + (size_t)hk * G;

  const int cnt = min(cnt_raw, sel_cap);
  if (cnt <= 0) {                                    // inactive or rejected sequence: zero-filled rows
    if (chunk == 0) {
      for (int o = tid; o < G * D; o += T) {
        out[o] = 0;
        if (o % D == 0) lse[o / D] = 0.0f;
      }
    }
    return;
  }
  // this workgroup's tiles of the list: all of them, or chunk `chunk` of n_chunks (whole tiles; the last chunk is
  // never empty, chunks beyond the number of tiles are)
  const int tiles_all = (cnt + 15) / 16;
  const int tile_begin = SPLIT ? (int)(((unsigned)tiles_all * (unsigned)chunk) / (unsigned)n_chunks) : 0;
  const int tile_end = SPLIT ? (int)(((unsigned)tiles_all * (unsigned)(chunk + 1)) / (unsigned)n_chunks) : tiles_all;
  if (tile_begin >= tile_end) return;
  const int t_begin = tile_begin * 16;
  const int len = min(cnt, tile_end * 16) - t_begin;           // tokens of this workgroup, numbered from 0 below
  const int n_tiles = tile_end - tile_begin;
  // slots of the list, clamped into the cache, go to LDS (readers clamp their list position to the last token)
  if constexpr (!SPLIT) {
#pragma unroll
    for (int k = 0; k < PF; ++k) {
      const int j = tid + k * T;
      if (j < len) s_slot[j] = min(max(pf_slot[k], 0), A.cap - 1);
    }
    for (int j = tid + PF * T; j < len; j += T) s_slot[j] = min(max(idx[j], 0), A.cap - 1);
  } else {
    for (int j = tid; j < len; j += T) s_slot[j] = min(max(idx[t_begin + j], 0), A.cap - 1);
  }
  s16x4 qb[NC];
#pragma unroll
  for (int c2 = 0; c2 < NC / 2; ++c2) {
    const uint4 x = r < G ? qx[c2] : make_uint4(0u, 0u, 0u, 0u);
    qb[2 * c2] = as_bf16x4(x.x, x.y);
    qb[2 * c2 + 1] = as_bf16x4(x.z, x.w);
  }
  const int new_slot = (append && pending >= 0 && pending < A.cap) ? pending : -1;
  __syncthreads();

  // (the lambdas below work on copies: they capture by reference, and a reference to the kernel's argument
  //  struct was measured to cost time in the multi-head kernel)
  const long long slot_stride_b = A.slot_stride_b;
  const float scale_log2 = A.scale_log2;
  const bool keep_logits = A.accumulate != 0;
  char* const stage = s_stage + wave * A.stage_b;    // LDS this wave owns

  // Ring of R tiles per wave.  Ring position u holds unit k of the wave, i.e. tile wave + k * NW, for k = u, u + R, ...
  // A tile is requested as LT K loads followed by 4 V loads per lane, always in that order and with no branch in
  // between, so that "the oldest K rows have arrived" is one in-order wait count.
  uint4 kr[R][LT];
  uint32_t vr[R][4][VW];
  uint32_t fresh[R];                                 // bit l: K load l, bit 8 + i: V load i stands for the query token's own row
  // byte offsets inside one head's rows fit 32 bits (cap <= 8192 slots, rows at most 64 KB apart): the loads then
  // take a uniform base and a 32-bit lane offset, two instructions of address arithmetic instead of a 64-bit product
  const uint32_t stride32 = (uint32_t)slot_stride_b;
  const uint32_t k_lane_off = (uint32_t)ld_piece * 16u, v_lane_off = (uint32_t)r * (EV * 2);
  auto issue = [&](int u, int tile) {
    int slot_k[LT], slot_v[4];                       // all slots of the tile first: one LDS round trip, then the loads
#pragma unroll
    for (int l = 0; l < LT; ++l) slot_k[l] = s_slot[min(tile * 16 + l * RPL + ld_row, len - 1)];   // (tiles past the end re-read the last row)
#pragma unroll
    for (int i = 0; i < 4; ++i) slot_v[i] = s_slot[min(tile * 16 + 4 * kg + i, len - 1)];
    // The query token's own slot is read like any other (valid memory of the cache; the row is stored at the end of
    // this launch) and what arrives is replaced by the row held in registers when the tile is multiplied.
    uint32_t f = 0u;
#pragma unroll
    for (int l = 0; l < LT; ++l) {
      kr[u][l] = load_stream16(k_base + ((uint32_t)slot_k[l] * stride32 + k_lane_off));
      f |= slot_k[l] == new_slot ? (1u << l) : 0u;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      vload<VW, true>(v_base + ((uint32_t)slot_v[i] * stride32 + v_lane_off), vr[u][i]);
      f |= slot_v[i] == new_slot ? (1u << (8 + i)) : 0u;
    }
    fresh[u] = f;
    asm volatile("" : : : "memory");                 // requests leave in ring order (the wait counts rely on it)
    __builtin_amdgcn_sched_barrier(0);               // ... and before the next tile's arithmetic, which waits for ITS rows
  };

  float m_run = -INFINITY, l_lane = 0.0f;            // online softmax of query g = r (l: this lane's tokens only)
  f32x4 acc[EV];                                     // acc[j][i] = partial out[g = 4*kg + i][d = EV*r + j]
#pragma unroll
  for (int j = 0; j < EV; ++j) acc[j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  auto fold = [&](int u, int tile) {
    if (__any(fresh[u] != 0u)) {                     // (rare) the tile holds the query token: its row comes from registers
#pragma unroll
      for (int l = 0; l < LT; ++l) kr[u][l] = pick16(((fresh[u] >> l) & 1u) != 0, nk, kr[u][l]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int w2 = 0; w2 < VW; ++w2) vr[u][i][w2] = (fresh[u] >> (8 + i)) & 1u ? nv[w2] : vr[u][i][w2];
      }
    }
    wave_lds_sync();                                 // the previous tile's operand reads are issued
#pragma unroll
    for (int l = 0; l < LT; ++l)
      *reinterpret_cast<uint4*>(stage + (l * RPL + ld_row) * ROWB + ld_piece * 16) = kr[u][l];
    wave_lds_sync();
    const char* rowp = stage + r * ROWB + kg * (D / 2);     // token r of the tile, this lane's columns
    f32x4 s4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int c2 = 0; c2 < NC / 2; ++c2) {
      const uint4 x = *reinterpret_cast<const uint4*>(rowp + c2 * 16);
      s4 = mfma_bf16(as_bf16x4(x.x, x.y), qb[2 * c2], s4);
      s4 = mfma_bf16(as_bf16x4(x.z, x.w), qb[2 * c2 + 1], s4);
    }
    // s4[i] = q[g = r] . K[token tile*16 + 4*kg + i]
    const int t0 = tile * 16 + 4 * kg;
    float z[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) z[i] = (t0 + i < len) ? s4[i] * scale_log2 : -INFINITY;
    if (keep_logits && r < G)
      *reinterpret_cast<float4*>(s_logit + (size_t)r * lgs + t0) = make_float4(z[0], z[1], z[2], z[3]);
    float tm = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
    tm = xor_max<32>(xor_max<16>(tm));               // maximum of query r over the tile (its first token is valid)
    const float m_new = fmaxf(m_run, tm);
    if (__any(m_new > m_run)) {                      // some query's maximum grew: rescale what was summed so far
      const float c = fast_exp2(m_run - m_new);      // 0 for the first tile
      l_lane *= c;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float ci = __shfl(c, 4 * kg + i, kWave);     // factor of query 4*kg + i
#pragma unroll
        for (int j = 0; j < EV; ++j) acc[j][i] *= ci;
      }
      m_run = m_new;
    }
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float p = fast_exp2(z[i] - m_run);
      if (r >= G) p = 0.0f;
      l_lane += p;
      hi[i] = __float_as_uint(p) & 0xFFFF0000u;
      lo[i] = __float_as_uint(p - __uint_as_float(hi[i])) >> 16;     // exact difference, truncated
    }
    const s16x4 a_hi = as_bf16x4((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]);
    const s16x4 a_lo = as_bf16x4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
#pragma unroll
    for (int w2 = 0; w2 < VW; ++w2) {
      const uint32_t r0 = vr[u][0][w2], r1 = vr[u][1][w2], r2 = vr[u][2][w2], r3 = vr[u][3][w2];
      // columns 2*w2 (low halves) and 2*w2+1 (high halves) of the 4 tokens
      const s16x4 b_even = as_bf16x4((r0 & 0xFFFFu) | (r1 << 16), (r2 & 0xFFFFu) | (r3 << 16));
      const s16x4 b_odd = as_bf16x4((r0 >> 16) | (r1 & 0xFFFF0000u), (r2 >> 16) | (r3 & 0xFFFF0000u));
      acc[2 * w2] = mfma_bf16(a_hi, b_even, acc[2 * w2]);
      acc[2 * w2] = mfma_bf16(a_lo, b_even, acc[2 * w2]);
      acc[2 * w2 + 1] = mfma_bf16(a_hi, b_odd, acc[2 * w2 + 1]);
      acc[2 * w2 + 1] = mfma_bf16(a_lo, b_odd, acc[2 * w2 + 1]);
    }
    // the tile is multiplied completely before the loads that reuse its ring position are issued
    asm volatile("" : "+v"(m_run), "+v"(l_lane) : : "memory");
  };

  {
    // wave w takes tiles w, w + NW, ...: a fixed assignment, so results are reproducible bit for bit.  Units
    // 0 .. R-1 are requested here; trip t multiplies units (t-1)R .. tR-1 (all of them real tiles) and requests
    // the units one ring revolution later; the last trip only multiplies, and skips ring positions without a tile.
    const int n_mine = n_tiles > wave ? (n_tiles - wave + NW - 1) / NW : 0;
    const int n_trips = (n_mine + R - 1) / R;
#pragma unroll
    for (int u = 0; u < R; ++u) issue(u, wave + u * NW);
    int k0 = 0;                                      // unit at ring position 0
    for (int trip = 1; trip < n_trips; ++trip) {
#pragma unroll
      for (int u = 0; u < R; ++u) {
        fold(u, wave + (k0 + u) * NW);
        issue(u, wave + (k0 + R + u) * NW);
      }
      k0 += R;
    }
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int tile = wave + (k0 + u) * NW;
      if (tile < n_tiles) fold(u, tile);             // wave-uniform
    }
  }
  l_lane = xor_sum<32>(xor_sum<16>(l_lane));
  if (lane < 16) { s_wm[wave][lane] = m_run; s_wl[wave][lane] = l_lane; }
  // one slab of partial outputs per wave, merged below with the waves' softmax weights
  wave_lds_sync();                                   // (the slab reuses the wave's K tile)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int g = 4 * kg + i;
    if (g < G) {
      float* dst = reinterpret_cast<float*>(stage) + (size_t)g * D + EV * r;
#pragma unroll
      for (int j = 0; j < EV; ++j) dst[j] = acc[j][i];
    }
  }
  __syncthreads();
  // Softmax weights of the waves, per query: s_wm[w][g] becomes wave w's weight 2^(m_w - M).  No global
  // store has been issued so far, so the two barriers here wait for LDS traffic only; every store of
  // the kernel follows the last barrier and is acknowledged once, at the end.
  if (tid < 16) {
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, s_wm[w][tid]);
    float L = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float mw = s_wm[w][tid];
      const float wgt = (mw == -INFINITY) ? 0.0f : fast_exp2(mw - M);      // a wave that saw no tile: weight 0
      L = fmaf(s_wl[w][tid], wgt, L);
      s_wm[w][tid] = wgt;
    }
    s_lse2[tid] = M + __log2f(L);
    s_m[tid] = M; s_l[tid] = L;
    s_wl[0][tid] = 1.0f / L;
  }
  __syncthreads();
  const size_t hq0 = (size_t)b * HQ + (size_t)hk * G;           // first query head of this cache head
  for (int o = tid; o < G * D; o += T) {
    const int g = o / D, d = o - g * D;
    float a = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) a = fmaf(reinterpret_cast<const float*>(s_stage + w * A.stage_b)[o], s_wm[w][g], a);
    if constexpr (!SPLIT) {
      out[o] = (uint16_t)f32_to_bf16_rne(a * s_wl[0][g]);
      if (d == 0) lse[g] = s_lse2[g] * kLn2;
    } else {                                         // this chunk's partial, relative to its own maximum
      const size_t pidx = (hq0 + g) * n_chunks + chunk;
      st_dev(A.part_acc + pidx * D + d, a);
      if (d == 0) st_dev2(A.part_ml + pidx * 2, s_m[g], s_l[g]);
    }
  }
  // Section 4.2 append: this cache head's rows of the new token, from the registers that attended them
  if (new_slot >= 0 && wave == 0 && chunk == n_chunks - 1) {
    const long long off = (long long)new_slot * slot_stride_b;
    if (ld_row == 0) store16(k_base + off + ld_piece * 16, nk);
    if (kg == 0) {
      if constexpr (VW == 4) store16(v_base + off + r * 16, make_uint4(nv[0], nv[1], nv[2], nv[3]));
      else {
        u32x2 v; v.x = nv[0]; v.y = nv[1];
        *reinterpret_cast<ADSA_GLOBAL u32x2*>(v_base + off + r * 8) = v;
      }
    }
  }

  if constexpr (!SPLIT) {
    // ---------------- attention mass of this cache head: sum over its G queries, ascending
    // Each (cache head, slot) word is touched by exactly one thread of one workgroup per launch, so a
    // no-return hardware add gives the same fp32 sum as a load + store, without waiting for the load
    // (requesting the old values before the loop and storing plainly was measured: not faster).
    if (A.accumulate) {
      for (int t = tid; t < len; t += T) {
        float inc = 0.0f;
        for (int g = 0; g < G; ++g) inc += fast_exp2(s_logit[(size_t)g * lgs + t] - s_lse2[g]);
        unsafeAtomicAdd((float*)(score + s_slot[t]), inc);
      }
    }
    if (hk == 0 && tid == 0 && A.advance) sqp->step = sqp->step + 1;     // no other workgroup reads step
  } else {
    // ---------------- several chunks: publish the logits, arrive, and let the last workgroup finish the cache head.
    // Partials and logits are written with device-scope atomic stores (written through to where all XCDs agree);
    // every thread waits until its own stores have completed, the barrier collects the workgroup, one thread bumps
    // the arrival counter with a device-scope release/acquire read-modify-write, and the workgroup that draws the
    // last ticket reads everything back with device-scope atomic loads after the barrier that follows its acquire.
    const int lgG = A.lg_global;
    if (keep_logits) {
      for (int i = tid; i < G * len; i += T) {
        const int g = i / len, t = i - g * len;
        st_dev(A.logits + (hq0 + g) * lgG + t_begin + t, s_logit[(size_t)g * lgs + t]);
      }
    }
    const int n_nonempty = min(tiles_all, n_chunks);
    int32_t* ctr = A.counters + (size_t)b * n_heads + hk;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != n_nonempty - 1) return;
    if (tid == 0) *ctr = 0;                          // ready for the next launch
    for (int o = tid; o < G * D; o += T) {
      const int g = o / D, d = o - g * D;
      const size_t pbase = (hq0 + g) * n_chunks;
      float mc[kMaxChunks], lc[kMaxChunks], ac[kMaxChunks];
#pragma unroll
      for (int c = 0; c < kMaxChunks; ++c) {         // all loads in flight together
        const bool on = c < n_chunks && ((unsigned)tiles_all * (unsigned)c) / (unsigned)n_chunks <
                                            ((unsigned)tiles_all * (unsigned)(c + 1)) / (unsigned)n_chunks;
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
      out[o] = (uint16_t)f32_to_bf16_rne(__fdividef(a, Lx));
      if (d == 0) {
        const float lse2 = Mx + __log2f(Lx);
        lse[g] = lse2 * kLn2;
        s_lse2[g] = lse2;
      }
    }
    if (A.accumulate) {
      __syncthreads();
      for (int t0 = tid; t0 < cnt; t0 += 2 * T) {     // two tokens per thread and trip: all their logits in flight together
        float z[2][16];
        int slot[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int t = min(t0 + u * T, cnt - 1);
#pragma unroll
          for (int g = 0; g < 16; ++g) z[u][g] = g < G ? ld_dev(A.logits + (hq0 + g) * lgG + t) : 0.0f;
          slot[u] = min(max(idx[t], 0), A.cap - 1);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          if (t0 + u * T >= cnt) continue;
          float inc = 0.0f;
#pragma unroll
          for (int g = 0; g < 16; ++g)
            if (g < G) inc += fast_exp2(z[u][g] - s_lse2[g]);
          unsafeAtomicAdd((float*)(score + slot[u]), inc);
        }
      }
    }
    if (hk == 0 && tid == 0 && A.advance) sqp->step = sqp->step + 1;
  }
}

template <int D, int NW, bool SPLIT>
hipError_t launch_gqa_w(const GqaArgs& A, int n_seq, int n_chunks, size_t lds, hipStream_t st, hipEvent_t ev_start,
                        hipEvent_t ev_stop) {
  dim3 grid(A.n_heads, n_seq, n_chunks);     // (lists that need more than 64 KB of LDS: see gqa_prepare_kernels)
  const int hgf = A.n_heads | (A.G << 16) | (A.append ? 1 << 24 : 0) | (A.new_f32 ? 1 << 25 : 0);
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL((k_attend_gqa<D, NW, SPLIT>), grid, dim3(NW * kWave), (uint32_t)lds, st, ev_start, ev_stop, 0,
                          A.seqs, A.sel_idx, A.sel_cnt, A.q, A.k_new, A.v_new, hgf, A.sel_cap, A);
  else
    hipLaunchKernelGGL((k_attend_gqa<D, NW, SPLIT>), grid, dim3(NW * kWave), lds, st,
                       A.seqs, A.sel_idx, A.sel_cnt, A.q, A.k_new, A.v_new, hgf, A.sel_cap, A);
  return hipGetLastError();
}

template <int D>
hipError_t launch_gqa_d(const GqaArgs& A, const AttendPlan& plan, int n_seq, size_t lds, hipStream_t st, hipEvent_t e0,
                        hipEvent_t e1) {
  if (plan.n_chunks > 1) return launch_gqa_w<D, 4, true>(A, n_seq, plan.n_chunks, lds, st, e0, e1);     // split lists: 4 waves
  if (plan.waves == 8) return launch_gqa_w<D, 8, false>(A, n_seq, 1, lds, st, e0, e1);
  return launch_gqa_w<D, 4, false>(A, n_seq, 1, lds, st, e0, e1);
}

}  // namespace

// Dynamic LDS above the default 64 KB per-launch limit has to be allowed per kernel, once per device; that is done
// here, at the library's first use of a device, not next to a launch (where it would also sit inside a captured graph).
hipError_t gqa_prepare_kernels() {
  const int lim = (int)kGqaMaxLds;
  const void* kernels[] = {
      reinterpret_cast<const void*>(&k_attend_gqa<64, 4, false>), reinterpret_cast<const void*>(&k_attend_gqa<64, 8, false>),
      reinterpret_cast<const void*>(&k_attend_gqa<128, 4, false>), reinterpret_cast<const void*>(&k_attend_gqa<128, 8, false>),
      reinterpret_cast<const void*>(&k_attend_gqa<64, 4, true>), reinterpret_cast<const void*>(&k_attend_gqa<128, 4, true>)};
  for (const void* k : kernels) {
    const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}


// row stride of the logits one workgroup keeps in LDS: the tokens of its chunk (whole tiles) + one tile of slack
int gqa_logit_stride(const adsa_params& p, int n_chunks) {
  const int tiles = (p.sel_cap + 15) / 16;
  return ((tiles + n_chunks - 1) / n_chunks) * 16 + 16;
}
// row stride of the logits in the workspace (split launches)
int gqa_global_logit_stride(const adsa_params& p) { return (p.sel_cap + 15) / 16 * 16 + 16; }

// LDS each wave owns: a staged K tile [16][D*2+16 bytes], reused for its partial output [G][D] floats
static size_t gqa_stage_bytes(const adsa_params& p) {
  const size_t tile = (size_t)16 * (p.head_dim * 2 + 16), part = (size_t)p.q_per_kv * p.head_dim * sizeof(float);
  return tile > part ? tile : part;
}

size_t gqa_lds_bytes(const adsa_params& p, int waves, int n_chunks) {
  const size_t lgs = (size_t)gqa_logit_stride(p, n_chunks);
  return ((size_t)p.q_per_kv + 1) * lgs * sizeof(float) + (size_t)waves * gqa_stage_bytes(p);
}

hipError_t launch_attend_gqa(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                             const void* k_new, const void* v_new, const int32_t* sel_idx,
                             const int32_t* sel_cnt, void* out, float* lse, char* ws, const Workspace& w,
                             bool accumulate, bool append, bool advance, bool new_f32, hipStream_t st,
                             hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (p.dtype != ADSA_BF16 || p.q_per_kv < 2 || p.q_per_kv > 16) return hipErrorInvalidValue;
  if (plan.n_chunks < 1 || plan.n_chunks > kMaxChunks) return hipErrorInvalidValue;
  GqaArgs A;
  A.seqs = seqs; A.q = (const char*)q; A.k_new = (const char*)k_new; A.v_new = (const char*)v_new;
  A.sel_idx = sel_idx; A.sel_cnt = sel_cnt; A.out = (char*)out; A.lse = lse;
  A.logits = reinterpret_cast<float*>(ws + w.logits_off);
  A.part_ml = reinterpret_cast<float*>(ws + w.part_ml_off);
  A.part_acc = reinterpret_cast<float*>(ws + w.part_acc_off);
  A.counters = reinterpret_cast<int32_t*>(ws + w.counters_off);
  A.lg_global = gqa_global_logit_stride(p);
  A.n_heads = p.n_heads; A.G = p.q_per_kv; A.sel_cap = p.sel_cap; A.lg_stride = gqa_logit_stride(p, plan.n_chunks);
  A.cap = p.cap; A.stage_b = (int)gqa_stage_bytes(p);
  A.accumulate = accumulate ? 1 : 0; A.append = append ? 1 : 0; A.advance = advance ? 1 : 0;
  A.new_f32 = (new_f32 && append) ? 1 : 0;
  A.slot_stride_b = (long long)p.kv_slot_stride * 2;
  A.head_stride_b = (long long)p.kv_head_stride * 2;
  const float scale = p.softmax_scale != 0.0f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  A.scale_log2 = scale * kLog2e;
  const size_t lds = gqa_lds_bytes(p, plan.waves, plan.n_chunks);
  if (lds > kGqaMaxLds) return hipErrorInvalidValue;
  if (p.head_dim == 64) return launch_gqa_d<64>(A, plan, p.n_seq, lds, st, ev_start, ev_stop);
  if (p.head_dim == 128) return launch_gqa_d<128>(A, plan, p.n_seq, lds, st, ev_start, ev_stop);
  return hipErrorInvalidValue;
}

}  // namespace adsa
