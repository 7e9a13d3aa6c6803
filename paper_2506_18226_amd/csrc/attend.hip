// Gather flash-decode of the ADSA decode path (gfx950): Eq. 5's gather fused with softmax
// attention over the selected slots, split over the index list, with the cache append
// (Section 4.2), the split merge and the attention-mass update fused into the same launch.
//
//  k_attend : grid (token chunk, head group, sequence).  Every sequence splits ITS OWN attended
//             count evenly over the chunks.  A wave reads one token's rows for `heads_per_wave`
//             heads with a single streaming 16-byte-per-lane load (1 KiB contiguous in
//             [slot][head][D] layout), reduces q.k over the lanes of a row with DPP, and keeps an
//             online-softmax state (m, l, acc) in registers, fp32, log2 domain.  The four waves of
//             a workgroup interleave the chunk's tokens and merge through LDS; one partial per
//             (sequence, head, chunk) and the scaled logits go to the workspace.
//             The LAST workgroup to finish a (sequence, head group) merges its partials into
//             out / lse and sums, per attended token, the probability over its heads; the LAST
//             head group of a sequence adds those sums to score[] in head-group order, finishes the
//             append (pos, n_res) and advances the step.  "Last" is decided by an arrival counter
//             after a device-scope fence, so nothing ever waits on another workgroup.
#include <hip/hip_ext.h>

#include "adsa_internal.h"
#include "adsa_partition.h"

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

// 16-byte streaming load: K/V rows are read once per step, so keep them out of the caches' way
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const char* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
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

// chunk c of a list of cnt tokens split evenly over nc chunks
__device__ __forceinline__ int chunk_begin(int cnt, int c, int nc) { return (int)(((long long)cnt * c) / nc); }

struct AttendArgs {
  adsa_seq* seqs;
  const char* q;
  const char* k_new;
  const char* v_new;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  char* out;
  float* lse;
  float* logits;        // [n_seq][n_heads][lg_stride]   scaled logits, log2 units
  float* part_ml;       // [n_seq][n_heads][n_chunks][2]
  float* part_acc;      // [n_seq][n_heads][n_chunks][D]
  float* psum;          // [n_seq][n_hg][lg_stride]      per head group: sum over its heads of p
  int32_t* counters;    // [n_seq][n_hg + 1]             arrival counters, zero between launches
  int n_heads, n_hg, sel_cap, lg_stride, chunk_max, cap;
  int grid_h, grid_w;
  int accumulate, append, advance;     // advance: step += 1 at the end
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
  __shared__ float s_lse2[HPW];
  __shared__ int s_ticket;

  const int chunk = blockIdx.x, hg = blockIdx.y, b = blockIdx.z, n_chunks = gridDim.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int cnt = min(A.sel_cnt[b], A.sel_cap);
  if (cnt <= 0) {                                   // inactive or rejected sequence: zero-filled row
    if (chunk == 0) {
      for (int o = tid; o < HPW * D; o += kAttThreads) {
        const int head = hg * HPW + o / D;
        if (head < A.n_heads) {
          const size_t oi = ((size_t)b * A.n_heads + head) * D + (o % D);
          if (EB == 4) reinterpret_cast<float*>(A.out)[oi] = 0.0f;
          else reinterpret_cast<uint16_t*>(A.out)[oi] = 0;
          if (o % D == 0) A.lse[(size_t)b * A.n_heads + head] = 0.0f;
        }
      }
    }
    return;
  }
  const int t_begin = chunk_begin(cnt, chunk, n_chunks), t_end = chunk_begin(cnt, chunk + 1, n_chunks);
  if (t_begin >= t_end) return;                     // fewer tokens than chunks
  const int n_nonempty = min(cnt, n_chunks);

  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int sub = lane / LPR, dl = lane - sub * LPR;
  const int head = hg * HPW + sub;
  const bool head_ok = head < A.n_heads;
  const int head_c = head_ok ? head : A.n_heads - 1;

  adsa_seq& sq = A.seqs[b];
  const int step = sq.step, n_res = sq.n_res;
  const int new_slot = (A.append && step >= 1) ? n_res : -1;   // n_res is bumped by the very last workgroup
  float qf[EPL];
  const size_t row_off = ((size_t)b * A.n_heads + head_c) * D * EB + dl * 16;
  {
    const uint4 qr = *reinterpret_cast<const uint4*>(A.q + row_off);
    Elems<EB>::unpack(qr, qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] *= A.scale_log2;
  }
  const long long lane_off = (long long)head_c * A.head_stride_b + dl * 16;
  char* kb = reinterpret_cast<char*>(sq.k) + lane_off;
  char* vb = reinterpret_cast<char*>(sq.v) + lane_off;
  const int32_t* idx = A.sel_idx + (size_t)b * A.sel_cap;

  float m = -INFINITY, l = 0.0f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.0f;

  for (int t = t_begin + wave * U; t < t_end; t += kAttWaves * U) {
    uint4 kr[U], vr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tt = min(t + u, t_end - 1);         // wave-uniform: scalar index load
      const int slot = min(max(idx[tt], 0), A.cap - 1);   // never touch memory outside the cache
      if (slot == new_slot) {                       // the query token itself: take it from k_new / v_new
        kr[u] = *reinterpret_cast<const uint4*>(A.k_new + row_off);
        vr[u] = *reinterpret_cast<const uint4*>(A.v_new + row_off);
        if (head_ok && t + u < t_end) {             // ... and append it to the cache (Section 4.2)
          *reinterpret_cast<uint4*>(kb + (long long)slot * A.slot_stride_b) = kr[u];
          *reinterpret_cast<uint4*>(vb + (long long)slot * A.slot_stride_b) = vr[u];
        }
      } else {
        const long long off = (long long)slot * A.slot_stride_b;
        kr[u] = load_stream16(kb + off);
        vr[u] = load_stream16(vb + off);
      }
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
    if (A.accumulate && dl == 0) {
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

  // ---- merge the four waves through LDS, one partial per (head, chunk) to the workspace
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
  if (A.accumulate) {
    const int len = t_end - t_begin;
    for (int i = tid; i < HPW * len; i += kAttThreads) {
      const int sb = i / len, j = i - sb * len;
      const int hd = hg * HPW + sb;
      if (hd < A.n_heads)
        A.logits[((size_t)b * A.n_heads + hd) * A.lg_stride + t_begin + j] = s_dyn[sb * A.chunk_max + j];
    }
  }

  // ---- arrival: the last workgroup of this (sequence, head group) merges the chunks
  int32_t* ctr = A.counters + (size_t)b * (A.n_hg + 1);
  __threadfence();
  __syncthreads();
  if (tid == 0) s_ticket = atomicAdd(&ctr[hg], 1);
  __syncthreads();
  if (s_ticket != n_nonempty - 1) return;
  __threadfence();                                  // acquire: see every chunk's partials and logits
  if (tid == 0) ctr[hg] = 0;                        // ready for the next launch

  for (int o = tid; o < HPW * D; o += kAttThreads) {
    const int sb = o / D, d = o - sb * D;
    const int hd = hg * HPW + sb;
    if (hd >= A.n_heads) continue;
    const size_t pbase = ((size_t)b * A.n_heads + hd) * n_chunks;
    float M = -INFINITY;
    for (int c = 0; c < n_chunks; ++c)
      if (chunk_begin(cnt, c, n_chunks) < chunk_begin(cnt, c + 1, n_chunks)) M = fmaxf(M, A.part_ml[(pbase + c) * 2]);
    float L = 0.0f, a = 0.0f;
    for (int c = 0; c < n_chunks; ++c) {
      if (chunk_begin(cnt, c, n_chunks) >= chunk_begin(cnt, c + 1, n_chunks)) continue;   // empty chunk
      const float wgt = fast_exp2(A.part_ml[(pbase + c) * 2] - M);
      L = fmaf(A.part_ml[(pbase + c) * 2 + 1], wgt, L);
      a = fmaf(A.part_acc[(pbase + c) * D + d], wgt, a);
    }
    const float val = a / L;
    const size_t oi = ((size_t)b * A.n_heads + hd) * D + d;
    if (EB == 4) reinterpret_cast<float*>(A.out)[oi] = val;
    else reinterpret_cast<uint16_t*>(A.out)[oi] = (uint16_t)f32_to_bf16_rne(val);
    if (d == 0) {
      const float lse2 = M + __log2f(L);
      A.lse[(size_t)b * A.n_heads + hd] = lse2 * kLn2;
      s_lse2[sb] = lse2;
    }
  }
  if (!(A.accumulate || A.append || A.advance)) return;
  __syncthreads();
  if (A.accumulate) {
    // per attended token: probability summed over this group's heads, ascending head order
    const float* lg = A.logits + ((size_t)b * A.n_heads + hg * HPW) * A.lg_stride;
    float* ps = A.psum + ((size_t)b * A.n_hg + hg) * A.lg_stride;
    const int heads_here = min(HPW, A.n_heads - hg * HPW);
    for (int j = tid; j < cnt; j += kAttThreads) {
      float t = 0.0f;
      for (int sb = 0; sb < heads_here; ++sb) t += fast_exp2(lg[(size_t)sb * A.lg_stride + j] - s_lse2[sb]);
      ps[j] = t;
    }
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) s_ticket = atomicAdd(&ctr[A.n_hg], 1);
  __syncthreads();
  if (s_ticket != A.n_hg - 1) return;
  __threadfence();
  if (tid == 0) ctr[A.n_hg] = 0;

  // ---- the last head group of the sequence: score update, end of append, step counter
  if (A.accumulate) {
    const float* ps = A.psum + (size_t)b * A.n_hg * A.lg_stride;
    for (int j = tid; j < cnt; j += kAttThreads) {
      const int slot = idx[j];
      if (slot < 0 || slot >= A.cap) continue;
      float inc = 0.0f;
      for (int g = 0; g < A.n_hg; ++g) inc += ps[(size_t)g * A.lg_stride + j];
      const float base = slot == new_slot ? 0.0f : sq.score[slot];   // a new slot starts at 0
      sq.score[slot] = base + inc;
    }
  } else if (new_slot >= 0 && tid == 0) {
    sq.score[new_slot] = 0.0f;
  }
  if (tid == 0) {
    if (new_slot >= 0) { sq.pos[new_slot] = sq.grid_origin + step - 1; sq.n_res = n_res + 1; }
    if (A.advance) sq.step = step + 1;
  }
}

template <int EB, int D>
hipError_t launch_attend_t(const AttendArgs& A, const AttendPlan& plan, int n_seq, hipStream_t st,
                           hipEvent_t ev_start, hipEvent_t ev_stop) {
  constexpr int U = 4;
  constexpr int HPW = kWave / (D / Elems<EB>::N);
  const size_t lds = A.accumulate ? (size_t)HPW * plan.chunk_max * sizeof(float) : 0;
  dim3 grid(plan.n_chunks, plan.n_head_groups, n_seq);
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL((k_attend<EB, D, U>), grid, dim3(kAttThreads), (uint32_t)lds, st, ev_start, ev_stop, 0, A);
  else
    hipLaunchKernelGGL((k_attend<EB, D, U>), grid, dim3(kAttThreads), lds, st, A);
  return hipGetLastError();
}

__global__ void k_zero_words(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
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
  w.lg_stride = (int)align_up((size_t)p.sel_cap, 4);
  w.counters_off = off;
  off = align_up(off + sizeof(int32_t) * (size_t)p.n_seq * (plan.n_head_groups + 1), 256);
  w.persistent_bytes = off;     // must stay zero between launches
  w.logits_off = off;
  off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.n_heads * w.lg_stride, 256);
  w.psum_off = off;
  off = align_up(off + sizeof(float) * (size_t)p.n_seq * plan.n_head_groups * w.lg_stride, 256);
  w.part_ml_off = off;
  off = align_up(off + sizeof(float) * (size_t)p.n_seq * p.n_heads * plan.n_chunks * 2, 256);
  w.part_acc_off = off;
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

hipError_t launch_workspace_init(char* ws, const Workspace& w, hipStream_t st) {
  const size_t words = w.persistent_bytes / 4;
  hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(ws + w.counters_off), words);
  return hipGetLastError();
}

hipError_t launch_attend(const adsa_params& p, const AttendPlan& plan, adsa_seq* seqs, const void* q,
                         const void* k_new, const void* v_new, const int32_t* sel_idx, const int32_t* sel_cnt,
                         void* out, float* lse, char* ws, const Workspace& w, bool accumulate, bool append,
                         bool advance, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  AttendArgs A;
  A.seqs = seqs; A.q = (const char*)q; A.k_new = (const char*)k_new; A.v_new = (const char*)v_new;
  A.sel_idx = sel_idx; A.sel_cnt = sel_cnt; A.out = (char*)out; A.lse = lse;
  A.logits = reinterpret_cast<float*>(ws + w.logits_off);
  A.part_ml = reinterpret_cast<float*>(ws + w.part_ml_off);
  A.part_acc = reinterpret_cast<float*>(ws + w.part_acc_off);
  A.psum = reinterpret_cast<float*>(ws + w.psum_off);
  A.counters = reinterpret_cast<int32_t*>(ws + w.counters_off);
  A.n_heads = p.n_heads; A.n_hg = plan.n_head_groups; A.sel_cap = p.sel_cap; A.lg_stride = w.lg_stride;
  A.chunk_max = plan.chunk_max; A.cap = p.cap; A.grid_h = p.grid_h; A.grid_w = p.grid_w;
  A.accumulate = accumulate ? 1 : 0; A.append = append ? 1 : 0; A.advance = advance ? 1 : 0;
  const int eb = elem_bytes(p);
  A.slot_stride_b = (long long)p.kv_slot_stride * eb;
  A.head_stride_b = (long long)p.kv_head_stride * eb;
  const float scale = p.softmax_scale != 0.0f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  A.scale_log2 = scale * kLog2e;
  if (eb == 2 && p.head_dim == 64) return launch_attend_t<2, 64>(A, plan, p.n_seq, st, ev_start, ev_stop);
  if (eb == 2 && p.head_dim == 128) return launch_attend_t<2, 128>(A, plan, p.n_seq, st, ev_start, ev_stop);
  if (eb == 4 && p.head_dim == 64) return launch_attend_t<4, 64>(A, plan, p.n_seq, st, ev_start, ev_stop);
  if (eb == 4 && p.head_dim == 128) return launch_attend_t<4, 128>(A, plan, p.n_seq, st, ev_start, ev_stop);
  return hipErrorInvalidValue;
}

}  // namespace adsa
