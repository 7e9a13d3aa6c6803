// Gather flash-decode of the ADSA decode path (gfx950): Eq. 5's gather fused with softmax
// attention over the selected slots, split over the index list.
//
//  k_attend  : grid (token chunk, head group, sequence).  Every sequence splits ITS OWN attended
//              count evenly over the chunks.  A wave reads one token's rows for `heads_per_wave`
//              heads with a single 16-byte-per-lane load (1 KiB contiguous in [slot][head][D]
//              layout), reduces q.k over the lanes of a row with DPP, and keeps an online-softmax
//              state (m, l, acc) in registers, fp32, log2 domain.  The four waves of a workgroup
//              interleave the chunk's tokens and merge through LDS; one partial per
//              (sequence, head, chunk) goes to the workspace together with the scaled logits.
//  k_combine : merges the chunk partials into out / lse and (ATTN_MASS) adds the probability each
//              attended slot received, summed over heads in ascending order, to score[].
#include "adsa_internal.h"

namespace adsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

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

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

struct AttendArgs {
  const adsa_seq* seqs;
  const char* q;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  float* logits;        // [n_seq][n_heads][sel_cap]
  float* part_ml;       // [n_seq][n_heads][n_chunks][2]
  float* part_acc;      // [n_seq][n_heads][n_chunks][D]
  int n_heads, sel_cap, chunk_max, want_logits, cap;
  long long slot_stride_b, head_stride_b;
  float scale_log2;     // softmax scale * log2(e)
};

template <int EB, int D, int U>
__global__ __launch_bounds__(kAttThreads) void k_attend(AttendArgs A) {
  constexpr int EPL = Elems<EB>::N;                 // elements per lane
  constexpr int LPR = D / EPL;                      // lanes per row
  constexpr int HPW = kWave / LPR;                  // heads per wave
  extern __shared__ float s_dyn[];                  // logits tile [HPW][chunk_max]
  __shared__ float s_m[kAttWaves][HPW], s_l[kAttWaves][HPW];
  __shared__ float s_acc[kAttWaves][kWave][EPL];

  const int chunk = blockIdx.x, hg = blockIdx.y, b = blockIdx.z, n_chunks = gridDim.x;
  const int cnt = min(A.sel_cnt[b], A.sel_cap);
  if (cnt <= 0) return;
  const int t_begin = (int)(((long long)cnt * chunk) / n_chunks);
  const int t_end = (int)(((long long)cnt * (chunk + 1)) / n_chunks);
  if (t_begin >= t_end) return;                     // fewer tokens than chunks

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int sub = lane / LPR, dl = lane - sub * LPR;
  const int head = hg * HPW + sub;
  const bool head_ok = head < A.n_heads;
  const int head_c = head_ok ? head : A.n_heads - 1;

  const adsa_seq& sq = A.seqs[b];
  float qf[EPL];
  {
    const uint4 qr = reinterpret_cast<const uint4*>(A.q + ((size_t)b * A.n_heads + head_c) * D * EB)[dl];
    Elems<EB>::unpack(qr, qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] *= A.scale_log2;
  }
  const char* kb = reinterpret_cast<const char*>(sq.k) + (long long)head_c * A.head_stride_b + dl * 16;
  const char* vb = reinterpret_cast<const char*>(sq.v) + (long long)head_c * A.head_stride_b + dl * 16;
  const int32_t* idx = A.sel_idx + (size_t)b * A.sel_cap;

  float m = -INFINITY, l = 0.0f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.0f;

  for (int t = t_begin + wave * U; t < t_end; t += kAttWaves * U) {
    uint4 kr[U], vr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tt = min(t + u, t_end - 1);         // wave-uniform: scalar index load
      const int slot = min(max(idx[tt], 0), A.cap - 1);   // never read outside the cache
      const long long off = (long long)slot * A.slot_stride_b;
      kr[u] = *reinterpret_cast<const uint4*>(kb + off);
      vr[u] = *reinterpret_cast<const uint4*>(vb + off);
    }
    float z[U];
    float m_new = m;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      Elems<EB>::unpack(kr[u], kf);
      float d = 0.0f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kf[e], d);
      d = row_sum<LPR>(d);
      z[u] = (t + u < t_end) ? d : -INFINITY;
      m_new = fmaxf(m_new, z[u]);
    }
    if (A.want_logits && dl == 0) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (t + u < t_end) s_dyn[sub * A.chunk_max + (t + u - t_begin)] = z[u];
    }
    const float corr = fast_exp2(m - m_new);
    l *= corr;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= corr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float pr = fast_exp2(z[u] - m_new);
      float vf[EPL];
      Elems<EB>::unpack(vr[u], vf);
      l += pr;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = fmaf(pr, vf[e], acc[e]);
    }
    m = m_new;
  }

  // merge the four waves through LDS
  if (dl == 0) { s_m[wave][sub] = m; s_l[wave][sub] = l; }
#pragma unroll
  for (int e = 0; e < EPL; ++e) s_acc[wave][lane][e] = acc[e];
  __syncthreads();
  if (wave == 0 && head_ok) {
    float M = s_m[0][sub];
#pragma unroll
    for (int w = 1; w < kAttWaves; ++w) M = fmaxf(M, s_m[w][sub]);
    float lt = 0.0f, at[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) at[e] = 0.0f;
#pragma unroll
    for (int w = 0; w < kAttWaves; ++w) {
      const float wgt = fast_exp2(s_m[w][sub] - M);   // a wave without tokens has m = -inf -> 0
      lt = fmaf(s_l[w][sub], wgt, lt);
#pragma unroll
      for (int e = 0; e < EPL; ++e) at[e] = fmaf(s_acc[w][lane][e], wgt, at[e]);
    }
    const size_t pidx = ((size_t)b * A.n_heads + head) * n_chunks + chunk;
    if (dl == 0) { A.part_ml[pidx * 2] = M; A.part_ml[pidx * 2 + 1] = lt; }
    float* pa = A.part_acc + pidx * D + dl * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4)
      *reinterpret_cast<float4*>(pa + e) = make_float4(at[e], at[e + 1], at[e + 2], at[e + 3]);
  }
  if (A.want_logits) {
    const int len = t_end - t_begin;
    for (int i = tid; i < HPW * len; i += kAttThreads) {
      const int sb = i / len, j = i - sb * len;
      const int hd = hg * HPW + sb;
      if (hd < A.n_heads)
        A.logits[((size_t)b * A.n_heads + hd) * A.sel_cap + t_begin + j] = s_dyn[sb * A.chunk_max + j];
    }
  }
}

struct CombineArgs {
  adsa_seq* seqs;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  const float* logits;
  const float* part_ml;
  const float* part_acc;
  char* out;
  float* lse;
  int n_heads, head_dim, sel_cap, n_chunks, elem_bytes, accumulate, advance_step, cap;
};

constexpr int kCombineThreads = 256;
constexpr int kMaxHeads = 256;

__global__ __launch_bounds__(kCombineThreads) void k_combine(CombineArgs A) {
  __shared__ float s_lse2[kMaxHeads];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int cnt = min(A.sel_cnt[b], A.sel_cap);
  const int h = A.n_heads, D = A.head_dim, nc = A.n_chunks;
  adsa_seq& sq = A.seqs[b];
  const bool active = sq.step >= 0 && sq.status == 0;
  for (int o = tid; o < h * D; o += kCombineThreads) {
    const int head = o / D, d = o - head * D;
    float val = 0.0f, lse2 = 0.0f;
    if (cnt > 0) {
      const size_t pbase = ((size_t)b * h + head) * nc;
      float M = -INFINITY;
      for (int c = 0; c < nc; ++c) {
        const bool nonempty = ((long long)cnt * c) / nc < ((long long)cnt * (c + 1)) / nc;
        if (nonempty) M = fmaxf(M, A.part_ml[(pbase + c) * 2]);
      }
      float L = 0.0f, a = 0.0f;
      for (int c = 0; c < nc; ++c) {
        const bool nonempty = ((long long)cnt * c) / nc < ((long long)cnt * (c + 1)) / nc;
        if (!nonempty) continue;
        const float wgt = fast_exp2(A.part_ml[(pbase + c) * 2] - M);
        L = fmaf(A.part_ml[(pbase + c) * 2 + 1], wgt, L);
        a = fmaf(A.part_acc[(pbase + c) * D + d], wgt, a);
      }
      val = a / L;
      lse2 = M + __log2f(L);
    }
    const size_t oi = ((size_t)b * h + head) * D + d;
    if (A.elem_bytes == 4) reinterpret_cast<float*>(A.out)[oi] = val;
    else reinterpret_cast<uint16_t*>(A.out)[oi] = (uint16_t)f32_to_bf16_rne(val);
    if (d == 0) { A.lse[(size_t)b * h + head] = lse2 * kLn2; s_lse2[head] = lse2; }
  }
  __syncthreads();
  if (A.accumulate && cnt > 0 && active) {
    const int32_t* idx = A.sel_idx + (size_t)b * A.sel_cap;
    const float* lg = A.logits + (size_t)b * h * A.sel_cap;
    for (int j = tid; j < cnt; j += kCombineThreads) {
      float t = 0.0f;
      for (int head = 0; head < h; ++head) t += fast_exp2(lg[(size_t)head * A.sel_cap + j] - s_lse2[head]);
      const int slot = idx[j];
      if (slot >= 0 && slot < A.cap) sq.score[slot] += t;
    }
  }
  if (A.advance_step && tid == 0 && active) sq.step = sq.step + 1;
}

template <int EB, int D>
hipError_t launch_attend_t(const AttendArgs& A, const AttendPlan& plan, int n_seq, hipStream_t st) {
  constexpr int U = 4;
  constexpr int HPW = kWave / (D / Elems<EB>::N);
  const size_t lds = A.want_logits ? (size_t)HPW * plan.chunk_max * sizeof(float) : 0;
  dim3 grid(plan.n_chunks, plan.n_head_groups, n_seq);
  hipLaunchKernelGGL((k_attend<EB, D, U>), grid, dim3(kAttThreads), lds, st, A);
  return hipGetLastError();
}

}  // namespace

AttendPlan make_attend_plan(const adsa_params& p) {
  AttendPlan a;
  const int epl = 16 / elem_bytes(p);
  a.lanes_per_row = p.head_dim / epl;
  a.heads_per_wave = kWave / a.lanes_per_row;
  a.n_head_groups = (p.n_heads + a.heads_per_wave - 1) / a.heads_per_wave;
  // enough workgroups to put ~3 on each of the 256 CUs, but never chunks shorter than 16 tokens
  const int target_wgs = 768;
  int pairs = p.n_seq * a.n_head_groups;
  int nc = (target_wgs + pairs - 1) / pairs;
  int max_by_len = p.sel_cap / 16;
  if (max_by_len < 1) max_by_len = 1;
  if (nc > max_by_len) nc = max_by_len;
  if (nc > 64) nc = 64;
  if (nc < 1) nc = 1;
  a.n_chunks = nc;
  a.chunk_max = (p.sel_cap + nc - 1) / nc + 1;
  return a;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Workspace make_workspace(const adsa_params& p, const AttendPlan& plan) {
  Workspace w;
  size_t off = 0;
  w.logits_off = off;
  off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.n_heads * p.sel_cap, 256);
  w.partial_off = off;   // ml then acc
  off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.n_heads * plan.n_chunks * 2, 256);
  off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.n_heads * plan.n_chunks * p.head_dim, 256);
  w.plan_off = off;
  off = align_up(off + sizeof(int32_t) * (size_t)p.n_seq * 4, 256);
  w.vcos_off = off;
  w.vcos_u_off = off;
  if (p.score_mode == ADSA_SCORE_VCOS) {
    off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.cap, 256);
    w.vcos_u_off = off;
    off = align_up(off + sizeof(float) * (size_t)p.n_seq * vcos_tiles(p.cap) * p.n_heads * p.head_dim, 256);
  }
  w.total = off;
  return w;
}

static float* part_ml_ptr(char* ws, const Workspace& w) { return reinterpret_cast<float*>(ws + w.partial_off); }
static float* part_acc_ptr(char* ws, const Workspace& w, const adsa_params& p, const AttendPlan& plan) {
  return reinterpret_cast<float*>(
      ws + align_up(w.partial_off + sizeof(float) * (size_t)p.n_seq * p.n_heads * plan.n_chunks * 2, 256));
}

hipError_t launch_attend(const adsa_params& p, const AttendPlan& plan, const adsa_seq* seqs, const void* q,
                         const int32_t* sel_idx, const int32_t* sel_cnt, char* ws, const Workspace& w,
                         bool want_logits, hipStream_t st) {
  AttendArgs A;
  A.seqs = seqs; A.q = (const char*)q; A.sel_idx = sel_idx; A.sel_cnt = sel_cnt;
  A.logits = reinterpret_cast<float*>(ws + w.logits_off);
  A.part_ml = part_ml_ptr(ws, w);
  A.part_acc = part_acc_ptr(ws, w, p, plan);
  A.n_heads = p.n_heads; A.sel_cap = p.sel_cap; A.chunk_max = plan.chunk_max; A.cap = p.cap;
  A.want_logits = want_logits ? 1 : 0;
  const int eb = elem_bytes(p);
  A.slot_stride_b = (long long)p.kv_slot_stride * eb;
  A.head_stride_b = (long long)p.kv_head_stride * eb;
  const float scale = p.softmax_scale != 0.0f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  A.scale_log2 = scale * kLog2e;
  if (eb == 2 && p.head_dim == 64) return launch_attend_t<2, 64>(A, plan, p.n_seq, st);
  if (eb == 2 && p.head_dim == 128) return launch_attend_t<2, 128>(A, plan, p.n_seq, st);
  if (eb == 4 && p.head_dim == 64) return launch_attend_t<4, 64>(A, plan, p.n_seq, st);
  if (eb == 4 && p.head_dim == 128) return launch_attend_t<4, 128>(A, plan, p.n_seq, st);
  return hipErrorInvalidValue;
}

hipError_t launch_combine(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs,
                          const int32_t* sel_idx, const int32_t* sel_cnt, void* out, float* lse,
                          char* ws, const Workspace& w, bool accumulate, bool advance_step, hipStream_t st) {
  CombineArgs A;
  A.seqs = seqs; A.sel_idx = sel_idx; A.sel_cnt = sel_cnt;
  A.logits = reinterpret_cast<const float*>(ws + w.logits_off);
  A.part_ml = part_ml_ptr(ws, w);
  A.part_acc = part_acc_ptr(ws, w, p, plan);
  A.out = (char*)out; A.lse = lse;
  A.n_heads = p.n_heads; A.head_dim = p.head_dim; A.sel_cap = p.sel_cap; A.n_chunks = plan.n_chunks;
  A.cap = p.cap;
  A.elem_bytes = elem_bytes(p); A.accumulate = accumulate ? 1 : 0; A.advance_step = advance_step ? 1 : 0;
  hipLaunchKernelGGL(k_combine, dim3(p.n_seq), dim3(kCombineThreads), 0, st, A);
  return hipGetLastError();
}

}  // namespace adsa
