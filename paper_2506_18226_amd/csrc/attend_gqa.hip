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
//    K and V of the next tiles are in flight while the current ones are multiplied.
//    At the end the waves' (m, l, partial out) are merged through LDS in wave order, the workgroup writes out / lse for its G query heads and adds the
//    probabilities of all G queries, summed in ascending head order, to its OWN cache head's row of
//    score[]: no workgroup talks to another.
#include <hip/hip_ext.h>

#include "adsa_internal.h"

namespace adsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

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

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// n consecutive fp32 values (n = 4 or 8) -> bf16, round to nearest even, packed two per dword
__device__ __forceinline__ void pack_bf16(const float* f, int n, uint32_t* w) {
  for (int i = 0; i < n / 2; ++i) w[i] = f32_to_bf16_rne(f[2 * i]) | (f32_to_bf16_rne(f[2 * i + 1]) << 16);
}

template <int BYTES> struct VLoad;
template <> struct VLoad<8> {
  static constexpr int W = 2;
  static __device__ __forceinline__ void load(const char* p, uint32_t* w) {
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    w[0] = v.x; w[1] = v.y;
  }
};
template <> struct VLoad<16> {
  static constexpr int W = 4;
  static __device__ __forceinline__ void load(const char* p, uint32_t* w) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
};

struct GqaArgs {
  adsa_seq* seqs;
  const char* q;
  const char* k_new;
  const char* v_new;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  char* out;
  float* lse;
  int n_heads, G, sel_cap, lg_stride, cap, stage_b;
  int accumulate, append, advance;
  int new_f32;          // k_new / v_new are fp32 although the cache is bf16: round as they enter
  long long slot_stride_b, head_stride_b;
  float scale_log2;
};

template <int D, int NW>
__global__ __launch_bounds__(NW * kWave) void k_attend_gqa(GqaArgs A) {
  constexpr int T = NW * kWave;
  constexpr int ROWB = D * 2 + 16;          // bytes of a staged K row (padded against bank conflicts)
  constexpr int LPR = D / 8;                // lanes per K row with 16-byte loads
  constexpr int RPL = kWave / LPR;          // rows per wave-load
  constexpr int LT = 16 / RPL;              // wave-loads per 16-token tile
  constexpr int NC = D / 16;                // 16-wide chunks of the q.k contraction
  constexpr int EV = D / 16;                // V columns a lane holds per token
  constexpr int UT = D == 64 ? 2 : 1;       // 16-token tiles per pipeline stage (two stages in flight)
  constexpr int VW = VLoad<EV * 2>::W;      // dwords of V a lane loads per token
  extern __shared__ __align__(16) char smem[];
  __shared__ float s_wm[NW][16], s_wl[NW][16], s_lse2[16];

  const int hk = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int r = lane & 15, kg = lane >> 4;                 // matrix-operand role of this lane
  const int G = A.G, lgs = A.lg_stride, HQ = A.n_heads * G;
  float* const s_logit = reinterpret_cast<float*>(smem);                 // [G][lgs]
  int* const s_slot = reinterpret_cast<int*>(s_logit + (size_t)G * lgs); // [lgs]
  char* const s_stage = reinterpret_cast<char*>(s_slot + lgs);           // [NW][stage_b]: K tile [16][ROWB], later partial out [G][D]

  // One round trip brings everything the first K loads depend on: the sequence record, the count, q,
  // and the whole slot list (its address and extent do not depend on the count).
  adsa_seq& sq = A.seqs[b];
  const int cnt_raw = A.sel_cnt[b];
  char* const k_base = reinterpret_cast<char*>(sq.k) + (long long)hk * A.head_stride_b;
  char* const v_base = reinterpret_cast<char*>(sq.v) + (long long)hk * A.head_stride_b;
  float* const score = sq.score + (size_t)hk * A.cap;
  const int pending = sq.pending_slot;
  const int32_t* idx = A.sel_idx + (size_t)b * A.sel_cap;
  uint16_t* const out = reinterpret_cast<uint16_t*>(A.out) + ((size_t)b * HQ + (size_t)hk * G) * D;
  float* const lse = A.lse + (size_t)b * HQ + (size_t)hk * G;
  // slots of the list, clamped into the cache (entries past the count are never used: readers clamp
  // their list position to the last token)
  for (int t = tid; t < A.sel_cap; t += T) s_slot[t] = min(max(idx[t], 0), A.cap - 1);
  // q as the B operand of pass 1: lane (g = r, kg) holds columns [D/4*kg, D/4*(kg+1)) of query g
  s16x4 qb[NC];
  {
    const char* qp = A.q + (((size_t)b * HQ + (size_t)hk * G + min(r, G - 1)) * D + (D / 4) * kg) * 2;
#pragma unroll
    for (int c2 = 0; c2 < NC / 2; ++c2) {
      uint4 x = *reinterpret_cast<const uint4*>(qp + c2 * 16);
      if (r >= G) x = make_uint4(0u, 0u, 0u, 0u);
      qb[2 * c2] = as_bf16x4(x.x, x.y);
      qb[2 * c2 + 1] = as_bf16x4(x.z, x.w);
    }
  }
  const int cnt = min(cnt_raw, A.sel_cap);
  if (cnt <= 0) {                                    // inactive or rejected sequence: zero-filled rows
    for (int o = tid; o < G * D; o += T) {
      out[o] = 0;
      if (o % D == 0) lse[o / D] = 0.0f;
    }
    return;
  }
  const int len = cnt;
  const int n_tiles = (len + 15) / 16;
  const int new_slot = (A.append && pending >= 0 && pending < A.cap) ? pending : -1;
  // the new token's row as this launch attends it; fp32 rows are rounded once, here: every lane keeps
  // the pieces of the rounded row it would load (K: 16 bytes at ld_piece, V: its EV columns)
  const bool cvt = A.new_f32 && new_slot >= 0;
  const size_t new_row = ((size_t)b * A.n_heads + hk) * D;
  const char* const kn = cvt ? k_base : A.k_new + new_row * 2;     // (cvt: any valid row; the value is replaced)
  const char* const vn = cvt ? v_base : A.v_new + new_row * 2;
  const int ld_row = lane / LPR, ld_piece = lane - ld_row * LPR;
  uint32_t nk[4] = {0u, 0u, 0u, 0u}, nv[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) nv[i] = 0u;
  if (cvt) {
    const float* k32 = reinterpret_cast<const float*>(A.k_new) + new_row;
    const float* v32 = reinterpret_cast<const float*>(A.v_new) + new_row;
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = k32[ld_piece * 8 + i];
    pack_bf16(t, 8, nk);
#pragma unroll
    for (int i = 0; i < EV; ++i) t[i] = v32[r * EV + i];
    pack_bf16(t, EV, nv);
  }
  __syncthreads();

  // (the lambdas below work on copies: they capture by reference, and a reference to the kernel's argument
  //  struct was measured to cost time in the multi-head kernel)
  const long long slot_stride_b = A.slot_stride_b;
  const float scale_log2 = A.scale_log2;
  const bool keep_logits = A.accumulate != 0;
  const int stage_b = A.stage_b;                     // bytes of LDS each wave owns
  char* const stage = s_stage + wave * stage_b;
  struct Stage { uint4 k[UT][LT]; uint32_t v[UT][4][VW]; };

  auto load = [&](Stage& st, int sid) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      const int tile = sid * UT + ut;
      if (tile < n_tiles) {                          // wave-uniform
#pragma unroll
        for (int u = 0; u < LT; ++u) {
          const int slot = s_slot[min(tile * 16 + u * RPL + ld_row, len - 1)];
          const char* p = (slot == new_slot) ? kn : k_base + (long long)slot * slot_stride_b;
          const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + ld_piece * 16));
          st.k[ut][u] = (cvt && slot == new_slot) ? make_uint4(nk[0], nk[1], nk[2], nk[3]) : make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int slot = s_slot[min(tile * 16 + 4 * kg + i, len - 1)];
          const char* p = (slot == new_slot) ? vn : v_base + (long long)slot * slot_stride_b;
          VLoad<EV * 2>::load(p + r * (EV * 2), st.v[ut][i]);
          if (cvt && slot == new_slot) {
#pragma unroll
            for (int w2 = 0; w2 < VW; ++w2) st.v[ut][i][w2] = nv[w2];
          }
        }
      }
    }
  };

  float m_run = -INFINITY, l_lane = 0.0f;            // online softmax of query g = r (l: this lane's tokens only)
  f32x4 acc[EV];                                     // acc[j][i] = partial out[g = 4*kg + i][d = EV*r + j]
#pragma unroll
  for (int j = 0; j < EV; ++j) acc[j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  auto mul = [&](const Stage& st, int sid) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      const int tile = sid * UT + ut;
      if (tile < n_tiles) {
        wave_lds_sync();                             // the previous tile's operand reads are issued
#pragma unroll
        for (int u = 0; u < LT; ++u)
          *reinterpret_cast<uint4*>(stage + (u * RPL + ld_row) * ROWB + ld_piece * 16) = st.k[ut][u];
        wave_lds_sync();
        const char* rowp = stage + r * ROWB + kg * (D / 2);   // token r of the tile, this lane's columns
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
        tm = fmaxf(tm, __shfl_xor(tm, 16, kWave));
        tm = fmaxf(tm, __shfl_xor(tm, 32, kWave));   // maximum of query r over the tile (its first token is valid)
        const float m_new = fmaxf(m_run, tm);
        if (__any(m_new > m_run)) {                  // some query's maximum grew: rescale what was summed so far
          const float c = fast_exp2(m_run - m_new);  // 0 for the first tile
          l_lane *= c;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float ci = __shfl(c, 4 * kg + i, kWave);   // factor of query 4*kg + i
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
          const uint32_t r0 = st.v[ut][0][w2], r1 = st.v[ut][1][w2], r2 = st.v[ut][2][w2], r3 = st.v[ut][3][w2];
          // columns 2*w2 (low halves) and 2*w2+1 (high halves) of the 4 tokens
          const s16x4 b_even = as_bf16x4((r0 & 0xFFFFu) | (r1 << 16), (r2 & 0xFFFFu) | (r3 << 16));
          const s16x4 b_odd = as_bf16x4((r0 >> 16) | (r1 & 0xFFFF0000u), (r2 >> 16) | (r3 & 0xFFFF0000u));
          acc[2 * w2] = mfma_bf16(a_hi, b_even, acc[2 * w2]);
          acc[2 * w2] = mfma_bf16(a_lo, b_even, acc[2 * w2]);
          acc[2 * w2 + 1] = mfma_bf16(a_hi, b_odd, acc[2 * w2 + 1]);
          acc[2 * w2 + 1] = mfma_bf16(a_lo, b_odd, acc[2 * w2 + 1]);
        }
      }
    }
  };

  {
    Stage sa, sb;
    // wave w takes stages w, w + NW, ...: a fixed assignment, so results are reproducible bit for bit
    int ia = wave, ib = wave + NW;
    load(sa, ia);
    load(sb, ib);
    while (ia * UT < n_tiles) {
      mul(sa, ia);
      ia += 2 * NW;
      load(sa, ia);
      if (ib * UT >= n_tiles) break;
      mul(sb, ib);
      ib += 2 * NW;
      load(sb, ib);
    }
  }
  l_lane += __shfl_xor(l_lane, 16, kWave);
  l_lane += __shfl_xor(l_lane, 32, kWave);
  if (lane < 16) { s_wm[wave][lane] = m_run; s_wl[wave][lane] = l_lane; }
  // one slab of partial outputs per wave, merged below with the waves' softmax weights
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int g = 4 * kg + i;
    if (g < G) {
      float* dst = reinterpret_cast<float*>(s_stage + wave * stage_b) + (size_t)g * D + EV * r;
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
    s_wl[0][tid] = 1.0f / L;
  }
  __syncthreads();
  for (int o = tid; o < G * D; o += T) {
    const int g = o / D, d = o - g * D;
    float a = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) a = fmaf(reinterpret_cast<const float*>(s_stage + w * stage_b)[o], s_wm[w][g], a);
    out[o] = (uint16_t)f32_to_bf16_rne(a * s_wl[0][g]);
    if (d == 0) lse[g] = s_lse2[g] * kLn2;
  }
  if (new_slot >= 0 && tid < D / 8) {                // Section 4.2 append: this cache head's rows of the new token
    const long long off = (long long)new_slot * A.slot_stride_b + tid * 16;
    if (cvt) {
      float t[8];
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = reinterpret_cast<const float*>(A.k_new)[new_row + tid * 8 + i];
      pack_bf16(t, 8, w);
      *reinterpret_cast<uint4*>(k_base + off) = make_uint4(w[0], w[1], w[2], w[3]);
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = reinterpret_cast<const float*>(A.v_new)[new_row + tid * 8 + i];
      pack_bf16(t, 8, w);
      *reinterpret_cast<uint4*>(v_base + off) = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
      *reinterpret_cast<uint4*>(k_base + off) = *reinterpret_cast<const uint4*>(kn + tid * 16);
      *reinterpret_cast<uint4*>(v_base + off) = *reinterpret_cast<const uint4*>(vn + tid * 16);
    }
  }

  // ---------------- attention mass of this cache head: sum over its G queries, ascending
  // Each (cache head, slot) word is touched by exactly one thread of one workgroup per launch, so a
  // no-return hardware add gives the same fp32 sum as a load + store, without waiting for the load.
  if (A.accumulate) {
    for (int t = tid; t < len; t += T) {
      float inc = 0.0f;
      for (int g = 0; g < G; ++g) inc += fast_exp2(s_logit[(size_t)g * lgs + t] - s_lse2[g]);
      unsafeAtomicAdd(score + s_slot[t], inc);
    }
  }
  if (hk == 0 && tid == 0 && A.advance) sq.step = sq.step + 1;     // no other workgroup reads step
}

template <int D, int NW>
hipError_t launch_gqa_w(const GqaArgs& A, int n_seq, size_t lds, hipStream_t st, hipEvent_t ev_start,
                        hipEvent_t ev_stop) {
  dim3 grid(A.n_heads, n_seq);     // (lists that need more than 64 KB of LDS: see gqa_prepare_kernels)
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL((k_attend_gqa<D, NW>), grid, dim3(NW * kWave), (uint32_t)lds, st, ev_start, ev_stop, 0, A);
  else
    hipLaunchKernelGGL((k_attend_gqa<D, NW>), grid, dim3(NW * kWave), lds, st, A);
  return hipGetLastError();
}

template <int D>
hipError_t launch_gqa_d(const GqaArgs& A, int waves, int n_seq, size_t lds, hipStream_t st, hipEvent_t e0,
                        hipEvent_t e1) {
  if (waves == 8) return launch_gqa_w<D, 8>(A, n_seq, lds, st, e0, e1);
  return launch_gqa_w<D, 4>(A, n_seq, lds, st, e0, e1);
}

}  // namespace

// Dynamic LDS above the default 64 KB per-launch limit has to be allowed per kernel, once per device; that is done
// here, at the library's first use of a device, not next to a launch (where it would also sit inside a captured graph).
hipError_t gqa_prepare_kernels() {
  const int lim = (int)kGqaMaxLds;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attend_gqa<64, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, lim);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attend_gqa<64, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, lim);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attend_gqa<128, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, lim);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attend_gqa<128, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, lim);
  return e;
}


int gqa_logit_stride(const adsa_params& p) { return (p.sel_cap + 15) / 16 * 16 + 16; }

// LDS each wave owns: a staged K tile [16][D*2+16 bytes], reused for its partial output [G][D] floats
static size_t gqa_stage_bytes(const adsa_params& p) {
  const size_t tile = (size_t)16 * (p.head_dim * 2 + 16), part = (size_t)p.q_per_kv * p.head_dim * sizeof(float);
  return tile > part ? tile : part;
}

size_t gqa_lds_bytes(const adsa_params& p, int waves) {
  const size_t lgs = (size_t)gqa_logit_stride(p);
  return ((size_t)p.q_per_kv + 1) * lgs * sizeof(float) + (size_t)waves * gqa_stage_bytes(p);
}

hipError_t launch_attend_gqa(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                             const void* k_new, const void* v_new, const int32_t* sel_idx,
                             const int32_t* sel_cnt, void* out, float* lse, bool accumulate, bool append,
                             bool advance, bool new_f32, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (p.dtype != ADSA_BF16 || p.q_per_kv < 2 || p.q_per_kv > 16) return hipErrorInvalidValue;
  GqaArgs A;
  A.seqs = seqs; A.q = (const char*)q; A.k_new = (const char*)k_new; A.v_new = (const char*)v_new;
  A.sel_idx = sel_idx; A.sel_cnt = sel_cnt; A.out = (char*)out; A.lse = lse;
  A.n_heads = p.n_heads; A.G = p.q_per_kv; A.sel_cap = p.sel_cap; A.lg_stride = gqa_logit_stride(p);
  A.cap = p.cap; A.stage_b = (int)gqa_stage_bytes(p);
  A.accumulate = accumulate ? 1 : 0; A.append = append ? 1 : 0; A.advance = advance ? 1 : 0;
  A.new_f32 = (new_f32 && append) ? 1 : 0;
  A.slot_stride_b = (long long)p.kv_slot_stride * 2;
  A.head_stride_b = (long long)p.kv_head_stride * 2;
  const float scale = p.softmax_scale != 0.0f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  A.scale_log2 = scale * kLog2e;
  const size_t lds = gqa_lds_bytes(p, plan.waves);
  if (lds > kGqaMaxLds) return hipErrorInvalidValue;
  if (p.head_dim == 64) return launch_gqa_d<64>(A, plan.waves, p.n_seq, lds, st, ev_start, ev_stop);
  if (p.head_dim == 128) return launch_gqa_d<128>(A, plan.waves, p.n_seq, lds, st, ev_start, ev_stop);
  return hipErrorInvalidValue;
}

}  // namespace adsa
