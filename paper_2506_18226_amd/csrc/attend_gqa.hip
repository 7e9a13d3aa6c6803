// Grouped-query gather flash-decode of the ADSA decode path (gfx950): Eq. 5's gather + softmax
// attention when G = 2..16 query heads share one cache head.  Every K/V row read from HBM now
// meets G queries, so the two products are small dense contractions and run on the matrix cores
// (v_mfma_f32_16x16x16_bf16, fp32 accumulation); the kernel is still bound by the HBM stream.
//
//  k_attend_gqa<D, NW> : grid (cache head, sequence), NW waves.  Two passes over the list:
//    pass 1  S[t][g] = K[t] . q[g]   per 16-token tile: rows are fetched with coalesced 16-byte
//            loads, staged through a wave-private LDS tile (the MFMA operand layout wants lane%16 =
//            token, a global load in that shape would touch 16 rows per quarter wave), multiplied
//            with the G (<= 16) query rows held in registers, scaled to log2 units and kept in LDS
//            as the logits [G][list]; per-query maxima are merged over lanes and waves.
//    pass 2  out[g][:] = sum_t 2^(S - max) V[t]   V rows come straight from HBM in operand layout:
//            a lane loads the same D/16 columns of 4 tokens and transposes the 4 x D/16 block in
//            registers (the contraction runs over tokens).  P is split into two bf16 halves
//            (hi + lo) so that the product carries ~16 mantissa bits of the probabilities.
//    Both passes are software-pipelined (the next stage's rows are in flight while the current one is
//    multiplied) and the first V rows are requested before the barrier between the passes.
//    The waves' partial outputs are added in wave order through LDS (deterministic), the workgroup
//    writes out / lse for its G query heads and adds the probabilities of all G queries, summed in
//    ascending head order, to its OWN cache head's row of score[]: no workgroup talks to another.
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
  constexpr int UT = (D == 64 ? 4 : 2) / (NW == 16 ? 2 : 1);   // tiles per pipeline stage (two stages in flight)
  constexpr int PF = (1024 / T) > 0 ? (1024 / T) : 1;
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

  adsa_seq& sq = A.seqs[b];
  const int cnt = min(A.sel_cnt[b], A.sel_cap);
  char* const k_base = reinterpret_cast<char*>(sq.k) + (long long)hk * A.head_stride_b;
  char* const v_base = reinterpret_cast<char*>(sq.v) + (long long)hk * A.head_stride_b;
  float* const score = sq.score + (size_t)hk * A.cap;
  const int pending = sq.pending_slot;
  const int32_t* idx = A.sel_idx + (size_t)b * A.sel_cap;
  uint16_t* const out = reinterpret_cast<uint16_t*>(A.out) + ((size_t)b * HQ + (size_t)hk * G) * D;
  float* const lse = A.lse + (size_t)b * HQ + (size_t)hk * G;

  if (cnt <= 0) {                                    // inactive or rejected sequence: zero-filled rows
    for (int o = tid; o < G * D; o += T) {
      out[o] = 0;
      if (o % D == 0) lse[o / D] = 0.0f;
    }
    return;
  }
  const int len = cnt;
  const int n_tiles = (len + 15) / 16, padded = n_tiles * 16;
  const int new_slot = (A.append && pending >= 0 && pending < A.cap) ? pending : -1;
  const char* const kn = A.k_new + ((size_t)b * A.n_heads + hk) * D * 2;
  const char* const vn = A.v_new + ((size_t)b * A.n_heads + hk) * D * 2;

  // slots of the list, clamped into the cache; the ragged tail repeats the last token's slot
  for (int t = tid; t < padded; t += T) s_slot[t] = min(max(idx[min(t, len - 1)], 0), A.cap - 1);

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
  if (new_slot >= 0 && tid < D / 8) {                // Section 4.2 append: this cache head's rows of the new token
    const long long off = (long long)new_slot * A.slot_stride_b + tid * 16;
    *reinterpret_cast<uint4*>(k_base + off) = *reinterpret_cast<const uint4*>(kn + tid * 16);
    *reinterpret_cast<uint4*>(v_base + off) = *reinterpret_cast<const uint4*>(vn + tid * 16);
  }
  __syncthreads();

  // the first PF score words this thread will update at the end: start the reads now
  int pf_slot[PF];
  float pf_old[PF];
#pragma unroll
  for (int k = 0; k < PF; ++k) {
    const int t = tid + k * T;
    pf_slot[k] = s_slot[min(t, padded - 1)];
    pf_old[k] = (A.accumulate && t < len) ? score[pf_slot[k]] : 0.0f;
  }

  // every wave takes an even, contiguous share of the list's 16-token tiles and walks it UT tiles at
  // a time, the loads of the next stage in flight while the current one is multiplied
  const int tb = (int)(((long long)n_tiles * wave) / NW), te = (int)(((long long)n_tiles * (wave + 1)) / NW);
  const int stage_b = A.stage_b;                     // bytes of LDS each wave owns
  char* const stage = s_stage + wave * stage_b;
  const int ld_row = lane / LPR, ld_piece = lane - ld_row * LPR;

  auto load_k = [&](uint4 (&buf)[UT][LT], int tile0) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      if (tile0 + ut < te) {                         // wave-uniform
#pragma unroll
        for (int u = 0; u < LT; ++u) {
          const int slot = s_slot[(tile0 + ut) * 16 + u * RPL + ld_row];
          const char* p = (slot == new_slot) ? kn : k_base + (long long)slot * A.slot_stride_b;
          const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + ld_piece * 16));
          buf[ut][u] = make_uint4(v.x, v.y, v.z, v.w);
        }
      }
    }
  };
  float m_lane = -INFINITY;
  auto mul_k = [&](const uint4 (&buf)[UT][LT], int tile0) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      const int tile = tile0 + ut;
      if (tile < te) {
        wave_lds_sync();                             // the previous tile's operand reads are issued
#pragma unroll
        for (int u = 0; u < LT; ++u)
          *reinterpret_cast<uint4*>(stage + (u * RPL + ld_row) * ROWB + ld_piece * 16) = buf[ut][u];
        wave_lds_sync();
        const char* rowp = stage + r * ROWB + kg * (D / 2);   // token r of the tile, this lane's columns
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int c2 = 0; c2 < NC / 2; ++c2) {
          const uint4 x = *reinterpret_cast<const uint4*>(rowp + c2 * 16);
          acc = mfma_bf16(as_bf16x4(x.x, x.y), qb[2 * c2], acc);
          acc = mfma_bf16(as_bf16x4(x.z, x.w), qb[2 * c2 + 1], acc);
        }
        // acc[i] = q[g = r] . K[token tile*16 + 4*kg + i]
        const int t0 = tile * 16 + 4 * kg;
        float4 z;
        z.x = (t0 + 0 < len) ? acc[0] * A.scale_log2 : -INFINITY;
        z.y = (t0 + 1 < len) ? acc[1] * A.scale_log2 : -INFINITY;
        z.z = (t0 + 2 < len) ? acc[2] * A.scale_log2 : -INFINITY;
        z.w = (t0 + 3 < len) ? acc[3] * A.scale_log2 : -INFINITY;
        if (r < G) {
          *reinterpret_cast<float4*>(s_logit + (size_t)r * lgs + t0) = z;
          m_lane = fmaxf(m_lane, fmaxf(fmaxf(z.x, z.y), fmaxf(z.z, z.w)));
        }
      }
    }
  };
  typedef uint32_t VTile[UT][4][VLoad<EV * 2>::W];
  auto load_v = [&](VTile& buf, int tile0) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      if (tile0 + ut < te) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int slot = s_slot[(tile0 + ut) * 16 + 4 * kg + i];
          const char* p = (slot == new_slot) ? vn : v_base + (long long)slot * A.slot_stride_b;
          VLoad<EV * 2>::load(p + r * (EV * 2), buf[ut][i]);
        }
      }
    }
  };

  // ---------------- pass 1: logits
  {
    uint4 ka[UT][LT], kb[UT][LT];
    if (tb < te) load_k(ka, tb);
    for (int t0 = tb; t0 < te; t0 += 2 * UT) {
      if (t0 + UT < te) load_k(kb, t0 + UT);
      mul_k(ka, t0);
      if (t0 + UT < te) {
        if (t0 + 2 * UT < te) load_k(ka, t0 + 2 * UT);
        mul_k(kb, t0 + UT);
      }
    }
  }
  VTile va, vb;
  if (tb < te) load_v(va, tb);                        // the first V rows travel while the maxima are merged
  m_lane = fmaxf(m_lane, __shfl_xor(m_lane, 16, kWave));
  m_lane = fmaxf(m_lane, __shfl_xor(m_lane, 32, kWave));
  if (lane < 16) s_wm[wave][lane] = m_lane;
  __syncthreads();

  // ---------------- pass 2: probabilities x V
  float Mg = -INFINITY;                               // maximum of query g = r
#pragma unroll
  for (int w = 0; w < NW; ++w) Mg = fmaxf(Mg, s_wm[w][r]);
  f32x4 acc[EV];
#pragma unroll
  for (int j = 0; j < EV; ++j) acc[j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  float l_lane = 0.0f;
  const float* const lrow = s_logit + (size_t)min(r, G - 1) * lgs + 4 * kg;
  auto mul_v = [&](const VTile& buf, int tile0) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      const int tile = tile0 + ut;
      if (tile < te) {
        const float4 z = *reinterpret_cast<const float4*>(lrow + tile * 16);
        float p[4];
        p[0] = fast_exp2(z.x - Mg); p[1] = fast_exp2(z.y - Mg);
        p[2] = fast_exp2(z.z - Mg); p[3] = fast_exp2(z.w - Mg);
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (r >= G) p[i] = 0.0f;
          l_lane += p[i];
          hi[i] = __float_as_uint(p[i]) & 0xFFFF0000u;
          lo[i] = __float_as_uint(p[i] - __uint_as_float(hi[i])) >> 16;   // exact difference, truncated
        }
        const s16x4 a_hi = as_bf16x4((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]);
        const s16x4 a_lo = as_bf16x4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
#pragma unroll
        for (int w2 = 0; w2 < VLoad<EV * 2>::W; ++w2) {
          const uint32_t r0 = buf[ut][0][w2], r1 = buf[ut][1][w2], r2 = buf[ut][2][w2], r3 = buf[ut][3][w2];
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
  for (int t0 = tb; t0 < te; t0 += 2 * UT) {
    if (t0 + UT < te) load_v(vb, t0 + UT);
    mul_v(va, t0);
    if (t0 + UT < te) {
      if (t0 + 2 * UT < te) load_v(va, t0 + 2 * UT);
      mul_v(vb, t0 + UT);
    }
  }
  l_lane += __shfl_xor(l_lane, 16, kWave);
  l_lane += __shfl_xor(l_lane, 32, kWave);
  if (lane < 16) s_wl[wave][lane] = l_lane;

  // acc[j][i] = this wave's partial out[g = 4*kg + i][d = EV*r + j]: one slab per wave, summed in wave order below
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
  for (int o = tid; o < G * D; o += T) {
    const int g = o / D, d = o - g * D;
    float L = 0.0f, M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) { L += s_wl[w][g]; M = fmaxf(M, s_wm[w][g]); }
    float a = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) a += reinterpret_cast<const float*>(s_stage + w * stage_b)[o];
    out[o] = (uint16_t)f32_to_bf16_rne(a / L);
    if (d == 0) {
      const float lse2 = M + __log2f(L);
      lse[g] = lse2 * kLn2;
      s_lse2[g] = lse2;
    }
  }

  // ---------------- attention mass of this cache head: sum over its G queries, ascending
  if (A.accumulate) {
    __syncthreads();
#pragma unroll
    for (int k = 0; k < PF; ++k) {
      const int t = tid + k * T;
      if (t < len) {
        float inc = 0.0f;
        for (int g = 0; g < G; ++g) inc += fast_exp2(s_logit[(size_t)g * lgs + t] - s_lse2[g]);
        score[pf_slot[k]] = pf_old[k] + inc;
      }
    }
    for (int t = tid + PF * T; t < len; t += T) {
      float inc = 0.0f;
      for (int g = 0; g < G; ++g) inc += fast_exp2(s_logit[(size_t)g * lgs + t] - s_lse2[g]);
      float* sp = score + s_slot[t];
      *sp = *sp + inc;
    }
  }
  if (hk == 0 && tid == 0 && A.advance) sq.step = sq.step + 1;     // no other workgroup reads step
}

template <int D, int NW>
hipError_t launch_gqa_w(const GqaArgs& A, int n_seq, size_t lds, hipStream_t st, hipEvent_t ev_start,
                        hipEvent_t ev_stop) {
  static size_t lds_allowed = 48 * 1024;       // raise the per-launch LDS limit once per kernel and size
  if (lds > lds_allowed) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attend_gqa<D, NW>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_allowed = lds;
  }
  dim3 grid(A.n_heads, n_seq);
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL((k_attend_gqa<D, NW>), grid, dim3(NW * kWave), (uint32_t)lds, st, ev_start, ev_stop, 0, A);
  else
    hipLaunchKernelGGL((k_attend_gqa<D, NW>), grid, dim3(NW * kWave), lds, st, A);
  return hipGetLastError();
}

template <int D>
hipError_t launch_gqa_d(const GqaArgs& A, int waves, int n_seq, size_t lds, hipStream_t st, hipEvent_t e0,
                        hipEvent_t e1) {
  if (waves == 16) return launch_gqa_w<D, 16>(A, n_seq, lds, st, e0, e1);
  if (waves == 8) return launch_gqa_w<D, 8>(A, n_seq, lds, st, e0, e1);
  return launch_gqa_w<D, 4>(A, n_seq, lds, st, e0, e1);
}

}  // namespace

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
                             bool advance, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (p.dtype != ADSA_BF16 || p.q_per_kv < 2 || p.q_per_kv > 16) return hipErrorInvalidValue;
  GqaArgs A;
  A.seqs = seqs; A.q = (const char*)q; A.k_new = (const char*)k_new; A.v_new = (const char*)v_new;
  A.sel_idx = sel_idx; A.sel_cnt = sel_cnt; A.out = (char*)out; A.lse = lse;
  A.n_heads = p.n_heads; A.G = p.q_per_kv; A.sel_cap = p.sel_cap; A.lg_stride = gqa_logit_stride(p);
  A.cap = p.cap; A.stage_b = (int)gqa_stage_bytes(p);
  A.accumulate = accumulate ? 1 : 0; A.append = append ? 1 : 0; A.advance = advance ? 1 : 0;
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
