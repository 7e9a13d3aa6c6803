// TopK-V redundancy score of the ADSA decode path (gfx950): Eq. 2-3, the mean pairwise cosine
// similarity of a candidate's V vector (all heads concatenated) to the other candidates.
//
// The N x N cosine matrix is never formed.  With v^_i = v_i / max(|v_i|, 1e-8) and
// u = sum_j v^_j over the candidates,  S_i = (v^_i . u - v^_i . v^_i) / (N - 1): two streaming
// passes over the candidates' V rows instead of O(N^2 D) work.
//
//  k_vcos_norm_usum : grid (slot tile, sequence).  A wave holds a slot's whole row in registers: inverse
//                     norm by a wave reduction, then the normalised row is added to the wave's column
//                     sums; the waves' sums are added in LDS into a per-tile partial of u
//                     (deterministic order, no atomics, every row read once).
//  k_vcos_score     : grid (slot tile, sequence).  Sums the tile partials of u into LDS, counts the
//                     candidates, then a wave per slot takes the dot product and writes S_i into
//                     score[slot] (non-candidate slots keep their score).
#include "adsa_internal.h"
#include "adsa_partition.h"

namespace adsa {
namespace {

constexpr int kVcThreads = 256;
constexpr int kVcWaves = kVcThreads / kWave;
constexpr int kVcTile = 64;                 // slots per workgroup
constexpr int kVcMaxDim = 8192;             // n_heads * head_dim limit of the LDS copy of u

struct VcosArgs {
  const adsa_seq* seqs_c;
  adsa_seq* seqs;
  float* inv_norm;      // [n_seq][cap]
  float* u_part;        // [n_seq][n_tiles][dim]
  float* s_out;         // [n_seq][cap] where S_i goes when score[] holds the fused form's rows, else NULL
  int n_heads, head_dim, elem_bytes, cap, n_tiles;
  int grid_h, grid_w, R, w, for_compaction, recent_m, evict_policy;
  long long slot_stride_b, head_stride_b;
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
  return x;
}

// candidate test for slot i of sequence sq (false for inactive sequences / non row-end compaction)
__device__ __forceinline__ bool vcos_candidate(const VcosArgs& A, const QueryCell& c, int pos) {
  if (A.for_compaction && A.evict_policy == ADSA_EVICT_ROW_END) return evict_class(c, pos) == 1;
  return select_class(c, pos) == 1;     // also the streaming eviction: the incoming query's partition
}

__device__ __forceinline__ bool vcos_active(const VcosArgs& A, const adsa_seq& sq) {
  if (sq.step < 0 || sq.status != 0 || sq.n_res < 0 || sq.n_res > A.cap) return false;
  if (sq.step > A.grid_h * A.grid_w) return false;
  if (!A.for_compaction) return true;
  if (A.evict_policy == ADSA_EVICT_REUSE_SLOT && sq.hole != 0) return false;     // room was made already
  if (A.s_out && sq.vcos_u && sq.vcos_u[A.n_heads * A.head_dim + 1] == (float)(sq.step + 1))
    return false;                                       // the attention launch left this step's numbers
  if (A.evict_policy != ADSA_EVICT_ROW_END) return sq.step >= 1 && sq.n_res == A.cap;
  return is_row_end(sq.step, A.grid_h, A.grid_w);
}

// load 4 consecutive elements (column group g of the concatenated row) of slot `slot`
__device__ __forceinline__ float4 load4(const VcosArgs& A, const char* vbase, int slot, int g) {
  const int col = g * 4, head = col / A.head_dim, d = col - head * A.head_dim;
  const char* p = vbase + (long long)slot * A.slot_stride_b + (long long)head * A.head_stride_b;
  if (A.elem_bytes == 4) return reinterpret_cast<const float4*>(p)[d / 4];
  const uint2 r = reinterpret_cast<const uint2*>(p)[d / 4];
  return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                     __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}

// GPL = column groups (of 4) per lane: a wave holds a whole concatenated V row in registers, so every
// row is read from HBM once: norm by a wave reduction, then the normalised row goes into the wave's
// running column sums.  The four waves' sums meet in LDS in wave order (deterministic).
template <int GPL>
__global__ __launch_bounds__(kVcThreads) void k_vcos_norm_usum(VcosArgs A) {
  extern __shared__ float s_acc[];                     // [kVcWaves][groups*4]
  const int tile = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const adsa_seq& sq = A.seqs_c[b];
  if (!vcos_active(A, sq)) return;
  const int n = sq.n_res, s0 = tile * kVcTile;
  if (s0 >= n) return;
  const int s1 = min(n, s0 + kVcTile);
  const QueryCell cell = make_query_cell(sq, sq.step, A.grid_w, A.R, A.w, A.recent_m);
  const char* vbase = reinterpret_cast<const char*>(sq.v);
  const int groups = A.n_heads * A.head_dim / 4;
  float4 acc[GPL];
#pragma unroll
  for (int k = 0; k < GPL; ++k) acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i = s0 + wave; i < s1; i += kVcWaves) {       // ascending slots per wave: fixed summation order
    float inv = 0.0f;                                     // 0 marks "not a candidate"
    if (vcos_candidate(A, cell, sq.pos[i])) {             // wave-uniform
      float4 x[GPL];
      float ss = 0.0f;
#pragma unroll
      for (int k = 0; k < GPL; ++k) {
        const int g = lane + k * kWave;
        x[k] = g < groups ? load4(A, vbase, i, g) : make_float4(0.f, 0.f, 0.f, 0.f);
        ss = fmaf(x[k].x, x[k].x, ss); ss = fmaf(x[k].y, x[k].y, ss);
        ss = fmaf(x[k].z, x[k].z, ss); ss = fmaf(x[k].w, x[k].w, ss);
      }
      ss = wave_sum(ss);
      inv = 1.0f / fmaxf(sqrtf(ss), 1e-8f);
#pragma unroll
      for (int k = 0; k < GPL; ++k) {
        acc[k].x = fmaf(x[k].x, inv, acc[k].x); acc[k].y = fmaf(x[k].y, inv, acc[k].y);
        acc[k].z = fmaf(x[k].z, inv, acc[k].z); acc[k].w = fmaf(x[k].w, inv, acc[k].w);
      }
    }
    if (lane == 0) A.inv_norm[(size_t)b * A.cap + i] = inv;
  }
#pragma unroll
  for (int k = 0; k < GPL; ++k) {
    const int g = lane + k * kWave;
    if (g < groups) reinterpret_cast<float4*>(s_acc + (size_t)wave * groups * 4)[g] = acc[k];
  }
  __syncthreads();
  float* up = A.u_part + ((size_t)b * A.n_tiles + tile) * (size_t)(groups * 4);
  for (int g = tid; g < groups; g += kVcThreads) {
    float4 t = reinterpret_cast<const float4*>(s_acc)[g];
#pragma unroll
    for (int w = 1; w < kVcWaves; ++w) {
      const float4 o = reinterpret_cast<const float4*>(s_acc + (size_t)w * groups * 4)[g];
      t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w;
    }
    reinterpret_cast<float4*>(up)[g] = t;
  }
}

__global__ __launch_bounds__(kVcThreads) void k_vcos_score(VcosArgs A) {
  extern __shared__ float s_u[];                       // [dim]
  __shared__ int s_cnt[kVcWaves];
  const int tile = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  adsa_seq& sq = A.seqs[b];
  if (!vcos_active(A, sq)) return;
  const int n = sq.n_res, s0 = tile * kVcTile;
  if (s0 >= n) return;
  const int s1 = min(n, s0 + kVcTile);
  const int groups = A.n_heads * A.head_dim / 4;
  const int tiles_used = (n + kVcTile - 1) / kVcTile;
  const float* up = A.u_part + (size_t)b * A.n_tiles * (size_t)(groups * 4);
  for (int g = tid; g < groups; g += kVcThreads) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = 0; t < tiles_used; ++t) {             // ascending tile order: deterministic
      const float4 x = reinterpret_cast<const float4*>(up + (size_t)t * groups * 4)[g];
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    reinterpret_cast<float4*>(s_u)[g] = acc;
  }
  int my = 0;
  const float* invs = A.inv_norm + (size_t)b * A.cap;
  for (int i = tid; i < n; i += kVcThreads) my += invs[i] != 0.0f;
  for (int d = 32; d >= 1; d >>= 1) my += __shfl_xor(my, d, kWave);
  if (lane == 0) s_cnt[wave] = my;
  __syncthreads();
  int N = 0;
  for (int w = 0; w < kVcWaves; ++w) N += s_cnt[w];
  const char* vbase = reinterpret_cast<const char*>(sq.v);
  for (int i = s0 + wave; i < s1; i += kVcWaves) {
    const float inv = invs[i];
    if (inv == 0.0f) continue;                          // wave-uniform
    float dot = 0.0f, ss = 0.0f;
    for (int g = lane; g < groups; g += kWave) {
      const float4 x = load4(A, vbase, i, g);
      const float4 uu = reinterpret_cast<const float4*>(s_u)[g];
      dot = fmaf(x.x, uu.x, dot); dot = fmaf(x.y, uu.y, dot); dot = fmaf(x.z, uu.z, dot); dot = fmaf(x.w, uu.w, dot);
      ss = fmaf(x.x, x.x, ss); ss = fmaf(x.y, x.y, ss); ss = fmaf(x.z, x.z, ss); ss = fmaf(x.w, x.w, ss);
    }
    dot = wave_sum(dot);
    ss = wave_sum(ss);
    // remove the i == j term (1 for a normal row, 0 for a zero row) and average over the others
    const float self = ss * inv * inv;
    const float S = N > 1 ? (dot * inv - self) / (float)(N - 1) : 0.0f;
    if (lane == 0) {
      if (A.s_out) A.s_out[(size_t)b * A.cap + i] = S;
      else sq.score[i] = S;
    }
  }
}

// ADSA_SCORE_VCOS_FUSED: bring u to the candidate set of the NEXT step, after this step's eviction plan and
// before its attention launch (which takes every row's dot product with u).  One workgroup per sequence.
// If u belongs to this step: subtract the evicted row, add the rows that turn from local to candidate
// (normally the one token that leaves the 1-D window).  Otherwise: a fresh sum over the next step's
// candidates.  Wave w handles slots w, w+4, ... in ascending order into its own LDS copy of u; the copies
// are added in wave order, so the result does not depend on timing.
struct AdvArgs {
  adsa_seq* seqs;
  int n_heads, head_dim, elem_bytes, cap, grid_h, grid_w, R, w, recent_m;
  long long slot_stride_b, head_stride_b;
};

__global__ __launch_bounds__(kVcThreads) void k_vcos_advance(AdvArgs A) {
  extern __shared__ float s_u[];                        // [kVcWaves][dim]
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  adsa_seq& sq = A.seqs[b];
  float* U = sq.vcos_u;
  if (sq.step < 0 || sq.status != 0 || U == nullptr) return;
  const int s = sq.step, n = sq.n_res, dim = A.n_heads * A.head_dim, groups = dim / 4;
  if (n < 0 || n > A.cap) return;
  float* tags = U + dim;
  if (s + 1 > A.grid_h * A.grid_w) {                    // no later step evicts
    if (tid == 0) tags[0] = 0.0f;
    return;
  }
  const bool incremental = tags[0] == (float)(s + 1);   // u is the sum over THIS step's candidates
  const int victim = sq.hole - 1;                       // slot freed by this step's eviction, or -1
  const QueryCell now = make_query_cell(sq, s, A.grid_w, A.R, A.w, A.recent_m);
  const QueryCell next = make_query_cell(sq, s + 1, A.grid_w, A.R, A.w, A.recent_m);
  for (int c = tid; c < dim; c += kVcThreads) {
    s_u[c] = incremental ? U[c] : 0.0f;
#pragma unroll
    for (int w = 1; w < kVcWaves; ++w) s_u[(size_t)w * dim + c] = 0.0f;
  }
  __syncthreads();
  // what happens to each slot: +1 joins u, -1 leaves it, 0 nothing (classified by all threads at once)
  signed char* s_sign = reinterpret_cast<signed char*>(s_u + (size_t)kVcWaves * dim);   // [cap]
  for (int i = tid; i < n; i += kVcThreads) {
    const int pos = sq.pos[i];
    const bool cand_next = select_class(next, pos) == 1;
    int sign = 0;
    if (incremental) {
      const bool cand_now = select_class(now, pos) == 1;
      if (i == victim) sign = cand_now ? -1 : 0;
      else if (cand_next && !cand_now) sign = 1;
    } else if (cand_next && i != victim) sign = 1;
    s_sign[i] = (signed char)sign;
  }
  __syncthreads();
  VcosArgs L;                                           // for load4()
  L.head_dim = A.head_dim; L.elem_bytes = A.elem_bytes; L.slot_stride_b = A.slot_stride_b; L.head_stride_b = A.head_stride_b;
  const char* vbase = reinterpret_cast<const char*>(sq.v);
  float* mine = s_u + (size_t)wave * dim;
  for (int base = 0; base < n; base += kWave) {         // wave w owns slots w, w+4, ...: ascending, fixed order
    const int my = base + lane;
    const int sg = (my < n && (my % kVcWaves) == wave) ? (int)s_sign[my] : 0;
    unsigned long long todo = __ballot(sg != 0);
    while (todo) {
      const int src = __ffsll((long long)todo) - 1;
      todo &= todo - 1;
      const int i = base + src;
      const float sign = (float)__shfl(sg, src, kWave);
      float ss = 0.0f;
      for (int g = lane; g < groups; g += kWave) {
        const float4 x = load4(L, vbase, i, g);
        ss = fmaf(x.x, x.x, ss); ss = fmaf(x.y, x.y, ss); ss = fmaf(x.z, x.z, ss); ss = fmaf(x.w, x.w, ss);
      }
      ss = wave_sum(ss);
      const float f = sign / fmaxf(sqrtf(ss), 1e-8f);
      for (int g = lane; g < groups; g += kWave) {
        const float4 x = load4(L, vbase, i, g);
        float4 t = reinterpret_cast<float4*>(mine)[g];
        t.x = fmaf(x.x, f, t.x); t.y = fmaf(x.y, f, t.y); t.z = fmaf(x.z, f, t.z); t.w = fmaf(x.w, f, t.w);
        reinterpret_cast<float4*>(mine)[g] = t;
      }
    }
  }
  __syncthreads();
  for (int c = tid; c < dim; c += kVcThreads) {
    float t = s_u[c];
#pragma unroll
    for (int w = 1; w < kVcWaves; ++w) t += s_u[(size_t)w * dim + c];
    U[c] = t;
  }
  if (tid == 0) tags[0] = (float)(s + 2);               // u now belongs to step s + 1
}

}  // namespace

// four copies of u and one byte per slot
size_t vcos_advance_lds_bytes(const adsa_params& p) {
  return sizeof(float) * (size_t)p.n_heads * p.head_dim * kVcWaves + (((size_t)p.cap + 15) / 16) * 16;
}

hipError_t launch_vcos_advance(const adsa_params& p, adsa_seq* seqs, hipStream_t st) {
  const size_t lds = vcos_advance_lds_bytes(p);
  if (lds > 64 * 1024) return hipErrorInvalidValue;
  AdvArgs A;
  A.seqs = seqs; A.n_heads = p.n_heads; A.head_dim = p.head_dim; A.elem_bytes = elem_bytes(p); A.cap = p.cap;
  A.grid_h = p.grid_h; A.grid_w = p.grid_w; A.R = p.win_rows_back; A.w = p.win_col_radius; A.recent_m = p.win_recent_m;
  A.slot_stride_b = (long long)p.kv_slot_stride * A.elem_bytes;
  A.head_stride_b = (long long)p.kv_head_stride * A.elem_bytes;
  hipLaunchKernelGGL(k_vcos_advance, dim3(p.n_seq), dim3(kVcThreads), lds, st, A);
  return hipGetLastError();
}

hipError_t launch_vcos(const adsa_params& p, adsa_seq* seqs, bool for_compaction, char* ws,
                       const Workspace& w, hipStream_t st) {
  const int dim = p.n_heads * p.head_dim;
  if (dim > kVcMaxDim) return hipErrorInvalidValue;
  VcosArgs A;
  A.seqs_c = seqs; A.seqs = seqs;
  A.inv_norm = reinterpret_cast<float*>(ws + w.vcos_off);
  A.u_part = reinterpret_cast<float*>(ws + w.vcos_u_off);
  A.s_out = p.score_mode == ADSA_SCORE_VCOS_FUSED ? reinterpret_cast<float*>(ws + w.vcos_s_off) : nullptr;
  A.n_heads = p.n_heads; A.head_dim = p.head_dim; A.elem_bytes = elem_bytes(p); A.cap = p.cap;
  A.n_tiles = (p.cap + kVcTile - 1) / kVcTile;
  A.grid_h = p.grid_h; A.grid_w = p.grid_w; A.R = p.win_rows_back; A.w = p.win_col_radius;
  A.for_compaction = for_compaction ? 1 : 0; A.recent_m = p.win_recent_m; A.evict_policy = p.evict_policy;
  A.slot_stride_b = (long long)p.kv_slot_stride * A.elem_bytes;
  A.head_stride_b = (long long)p.kv_head_stride * A.elem_bytes;
  dim3 grid(A.n_tiles, p.n_seq);
  const int gpl = (dim / 4 + kWave - 1) / kWave;          // column groups per lane: 1..32
  const size_t lds1 = sizeof(float) * (size_t)dim * kVcWaves;
  if (gpl <= 4) hipLaunchKernelGGL(k_vcos_norm_usum<4>, grid, dim3(kVcThreads), lds1, st, A);
  else if (gpl <= 6) hipLaunchKernelGGL(k_vcos_norm_usum<6>, grid, dim3(kVcThreads), lds1, st, A);
  else if (gpl <= 8) hipLaunchKernelGGL(k_vcos_norm_usum<8>, grid, dim3(kVcThreads), lds1, st, A);
  else if (gpl <= 16) hipLaunchKernelGGL(k_vcos_norm_usum<16>, grid, dim3(kVcThreads), lds1, st, A);
  else {
    // (64..128 KB of LDS, above the default per-launch limit: allowed once per device by vcos_prepare_kernels)
    hipLaunchKernelGGL(k_vcos_norm_usum<32>, grid, dim3(kVcThreads), lds1, st, A);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_vcos_score, grid, dim3(kVcThreads), sizeof(float) * (size_t)dim, st, A);
  return hipGetLastError();
}

int vcos_tiles(int cap) { return (cap + kVcTile - 1) / kVcTile; }

// The widest first-pass kernel may need up to 128 KB of dynamic LDS (n_heads * head_dim = 8192 floats x 4 waves):
// allowed here, once per device, at the library's first use of that device.
hipError_t vcos_prepare_kernels() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_vcos_norm_usum<32>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
}

}  // namespace adsa
