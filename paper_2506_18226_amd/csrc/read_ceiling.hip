// Measurement aid (not part of the library): what a kernel that ONLY reads the attention kernel's bytes achieves on
// this GPU, in the attention kernel's launch shape and access pattern -- the ceiling its HBM roofline fraction is
// read against.  768 workgroups x 4 waves (one per (sequence, head) of the XXL-shaped layer); a workgroup reads
// `rows` consecutive 128-byte rows of its head's K region and of its V region with 16-byte nontemporal loads, U row
// pairs per lane in flight, and does nothing with them.  48 distinct layers are cycled so that nothing is served
// from a cache.  Prints the kernel-only duration (HIP events on the dispatch) and the back-to-back time per launch.
// Two variants answer "would more bytes in flight, or bytes in flight that do not cost registers, help?": the same
// read as a rolling ring of U row pairs per lane (the oldest pair is consumed, its registers refilled), and the
// same ring with the rows sent global -> LDS directly (128-bit LDS-direct loads, no register staging; a first
// launch checks every lane's LDS contents against a plain load).
//   read_ceiling [rows ...]        default rows: 673 524 256
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
#define GLOBAL_AS __attribute__((address_space(1)))
#define LDS_AS __attribute__((address_space(3)))
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kUnits = 768, kCap = 696, kLayers = 48, kU = 4;

__global__ __launch_bounds__(256) void k_plain_read(const char* Kp, const char* Vp, unsigned unit_stride, int n_rows, float* out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane >> 3, dl = lane & 7;          // 8 lanes x 16 bytes cover a row; a wave-load covers 8 rows
  const GLOBAL_AS char* K = (const GLOBAL_AS char*)Kp + (size_t)blockIdx.x * unit_stride + dl * 16;
  const GLOBAL_AS char* V = (const GLOBAL_AS char*)Vp + (size_t)blockIdx.x * unit_stride + dl * 16;
  unsigned acc = 0;
  for (int g0 = wave * 8 * kU; g0 < n_rows; g0 += 32 * kU) {
    u32x4 a[kU], b[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      int r = g0 + u * 8 + sub;
      if (r >= n_rows) r = n_rows - 1;
      a[u] = __builtin_nontemporal_load((const GLOBAL_AS u32x4*)(K + r * 128u));
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      int r = g0 + u * 8 + sub;
      if (r >= n_rows) r = n_rows - 1;
      b[u] = __builtin_nontemporal_load((const GLOBAL_AS u32x4*)(V + r * 128u));
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) acc += a[u].x ^ a[u].y ^ a[u].z ^ a[u].w ^ b[u].x ^ b[u].y ^ b[u].z ^ b[u].w;
  }
  if (acc == 0x12345678u) out[blockIdx.x] = 1.0f;     // keeps the loads alive; never true for the fill values
}


// the same bytes as a rolling ring: unit k of a wave = rows (wave + 4k) * 8 + sub; U units in flight
template <int kRing>
__global__ __launch_bounds__(256) void k_ring_read(const char* Kp, const char* Vp, unsigned unit_stride, int n_rows, float* out) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane >> 3, dl = lane & 7;
  const GLOBAL_AS char* K = (const GLOBAL_AS char*)Kp + (size_t)blockIdx.x * unit_stride + dl * 16;
  const GLOBAL_AS char* V = (const GLOBAL_AS char*)Vp + (size_t)blockIdx.x * unit_stride + dl * 16;
  const int n_units = (n_rows + 7) / 8;
  const int n_mine = n_units > wave ? (n_units - wave + 3) / 4 : 0;
  const int n_trips = (n_mine + kRing - 1) / kRing;
  u32x4 a[kRing], b[kRing];
  unsigned acc = 0;
  auto issue = [&](int u, int k) {
    int r = (wave + 4 * k) * 8 + sub;
    if (r >= n_rows) r = n_rows - 1;
    a[u] = __builtin_nontemporal_load((const GLOBAL_AS u32x4*)(K + r * 128u));
    b[u] = __builtin_nontemporal_load((const GLOBAL_AS u32x4*)(V + r * 128u));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
#pragma unroll
  for (int u = 0; u < kRing; ++u) issue(u, u);
  int kn = kRing;
  for (int t = 1; t < n_trips; ++t) {
#pragma unroll
    for (int u = 0; u < kRing; ++u) {
      acc += a[u].x ^ a[u].y ^ a[u].z ^ a[u].w ^ b[u].x ^ b[u].y ^ b[u].z ^ b[u].w;
      asm volatile("" : "+v"(acc) : : "memory");
      issue(u, kn + u);
    }
    kn += kRing;
  }
#pragma unroll
  for (int u = 0; u < kRing; ++u) acc += a[u].x ^ a[u].y ^ a[u].z ^ a[u].w ^ b[u].x ^ b[u].y ^ b[u].z ^ b[u].w;
  if (acc == 0x12345678u) out[blockIdx.x] = 1.0f;
}

// the same ring with LDS-direct loads: lane i's 16 bytes land at (wave-uniform LDS address) + 16 i; 2 KB of LDS per unit
template <int kRing, bool CHECK>
__global__ __launch_bounds__(256) void k_ring_read_lds(const char* Kp, const char* Vp, unsigned unit_stride, int n_rows, float* out,
                                                     unsigned* bad) {
  extern __shared__ __attribute__((aligned(16))) char lds[];     // 4 waves x kRing units x 2 KB
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane >> 3, dl = lane & 7;
  const GLOBAL_AS char* K = (const GLOBAL_AS char*)Kp + (size_t)blockIdx.x * unit_stride + dl * 16;
  const GLOBAL_AS char* V = (const GLOBAL_AS char*)Vp + (size_t)blockIdx.x * unit_stride + dl * 16;
  char* my = lds + wave * (kRing * 2048);
  const int n_units = (n_rows + 7) / 8;
  const int n_mine = n_units > wave ? (n_units - wave + 3) / 4 : 0;
  const int n_trips = (n_mine + kRing - 1) / kRing;
  unsigned acc = 0;
  auto issue = [&](int u, int k) {
    int r = (wave + 4 * k) * 8 + sub;
    if (r >= n_rows) r = n_rows - 1;
    __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(K + r * 128u), (LDS_AS void*)(my + u * 2048), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(V + r * 128u), (LDS_AS void*)(my + u * 2048 + 1024), 16, 0, 0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  auto consume = [&](int u, int k) {
    const u32x4 a = *(const u32x4*)(my + u * 2048 + lane * 16);
    const u32x4 b = *(const u32x4*)(my + u * 2048 + 1024 + lane * 16);
    acc += a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w;
    if (CHECK && k < n_mine) {
      int r = (wave + 4 * k) * 8 + sub;
      if (r >= n_rows) r = n_rows - 1;
      const u32x4 ea = *(const GLOBAL_AS u32x4*)(K + r * 128u);
      const u32x4 eb = *(const GLOBAL_AS u32x4*)(V + r * 128u);
      if (ea.x != a.x || ea.y != a.y || ea.z != a.z || ea.w != a.w || eb.x != b.x || eb.y != b.y || eb.z != b.z || eb.w != b.w)
        atomicAdd(bad, 1u);
    }
    asm volatile("" : "+v"(acc) : : "memory");
  };
#pragma unroll
  for (int u = 0; u < kRing; ++u) issue(u, u);
  int kn = kRing;
  for (int t = 1; t < n_trips; ++t) {
#pragma unroll
    for (int u = 0; u < kRing; ++u) {
      asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 * (kRing - 1)) : "memory");      // the oldest unit has landed in LDS
      consume(u, kn - kRing + u);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                            // read out before the unit is overwritten
      issue(u, kn + u);
    }
    kn += kRing;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int u = 0; u < kRing; ++u) consume(u, kn - kRing + u);
  if (acc == 0x12345678u) out[blockIdx.x] = 1.0f;
}

template <int kRing, bool LDS>
void time_ring(int n_rows, std::vector<char*>& K, std::vector<char*>& V, float* out, unsigned* bad, std::vector<hipEvent_t>& ev) {
  const size_t lds = (size_t)4 * kRing * 2048;
  unsigned mism = 0;
  if (LDS) {
    CK(hipMemset(bad, 0, 4));
    hipLaunchKernelGGL((k_ring_read_lds<kRing, true>), dim3(kUnits), dim3(256), lds, 0, K[0], V[0], kCap * 128u, n_rows, out, bad);
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(&mism, bad, 4, hipMemcpyDeviceToHost));
  }
  int k = 0;
  for (int it = 0; it < 3; ++it)                      // the first round is a warm-up
    for (int l = 0; l < kLayers; ++l) {
      hipEvent_t e0 = it ? ev[k] : nullptr, e1 = it ? ev[k + 1] : nullptr;
      if (LDS) hipExtLaunchKernelGGL((k_ring_read_lds<kRing, false>), dim3(kUnits), dim3(256), lds, 0, e0, e1, 0, K[l], V[l], kCap * 128u, n_rows, out, bad);
      else hipExtLaunchKernelGGL((k_ring_read<kRing>), dim3(kUnits), dim3(256), 0, 0, e0, e1, 0, K[l], V[l], kCap * 128u, n_rows, out);
      if (it) k += 2;
    }
  CK(hipDeviceSynchronize());
  double kern = 0;
  for (int i = 0; i < k; i += 2) { float ms; CK(hipEventElapsedTime(&ms, ev[i], ev[i + 1])); kern += ms; }
  const double us = 1e3 * kern / (k / 2), bytes = (double)kUnits * n_rows * 128 * 2;
  if (LDS) printf("  ring of %d pairs, global -> LDS direct: kernel only %.2f us = %.1f%% of 8 TB/s (lanes whose LDS contents differ from a plain load: %u)\n", kRing, us, bytes / us / 1e3 / 80.0, mism);
  else printf("  ring of %d pairs in registers: kernel only %.2f us = %.1f%% of 8 TB/s\n", kRing, us, bytes / us / 1e3 / 80.0);
}

int main(int argc, char** argv) {
  std::vector<int> rows;
  for (int i = 1; i < argc; ++i) rows.push_back(atoi(argv[i]));
  if (rows.empty()) rows = {673, 524, 256};
  const size_t layer_bytes = (size_t)kUnits * kCap * 128;
  std::vector<char*> K(kLayers), V(kLayers);
  std::vector<unsigned> pattern(layer_bytes / 4 + 1);
  for (size_t i = 0; i < pattern.size(); ++i) pattern[i] = (unsigned)i * 2654435761u;
  for (int l = 0; l < kLayers; ++l) {
    CK(hipMalloc(&K[l], layer_bytes)); CK(hipMalloc(&V[l], layer_bytes));
    CK(hipMemcpy(K[l], pattern.data(), layer_bytes, hipMemcpyHostToDevice));
    CK(hipMemcpy(V[l], pattern.data() + 1, layer_bytes, hipMemcpyHostToDevice));
  }
  float* out; CK(hipMalloc(&out, 1 << 16));
  unsigned* bad; CK(hipMalloc(&bad, 4));
  const int reps = 2;
  std::vector<hipEvent_t> ev(2 * kLayers * reps);
  for (auto& e : ev) CK(hipEventCreate(&e));
  hipEvent_t w0, w1; CK(hipEventCreate(&w0)); CK(hipEventCreate(&w1));
  for (int n_rows : rows) {
    if (n_rows < 1 || n_rows > kCap) { printf("rows must be in 1..%d\n", kCap); return 1; }
    const double bytes = (double)kUnits * n_rows * 128 * 2;
    float wall = 0;
    for (int pass = 0; pass < 3; ++pass) {             // back to back, no events (the last pass counts)
      CK(hipEventRecord(w0, 0));
      for (int it = 0; it < reps; ++it)
        for (int l = 0; l < kLayers; ++l)
          hipLaunchKernelGGL(k_plain_read, dim3(kUnits), dim3(256), 0, 0, K[l], V[l], kCap * 128u, n_rows, out);
      CK(hipEventRecord(w1, 0)); CK(hipDeviceSynchronize()); CK(hipEventElapsedTime(&wall, w0, w1));
    }
    int k = 0;
    for (int it = 0; it < reps; ++it)
      for (int l = 0; l < kLayers; ++l, k += 2)
        hipExtLaunchKernelGGL(k_plain_read, dim3(kUnits), dim3(256), 0, 0, ev[k], ev[k + 1], 0, K[l], V[l], kCap * 128u, n_rows, out);
    CK(hipDeviceSynchronize());
    double kern = 0;
    for (int i = 0; i < k; i += 2) { float ms; CK(hipEventElapsedTime(&ms, ev[i], ev[i + 1])); kern += ms; }
    const double us = 1e3 * kern / (k / 2);
    printf("plain read, %d rows per (sequence, head), %.1f MB per launch: kernel only %.2f us -> %.0f GB/s = %.1f%% of 8 TB/s; "
           "back to back %.2f us per launch\n", n_rows, bytes / 1e6, us, bytes / us / 1e3, bytes / us / 1e3 / 80.0,
           1e3 * wall / (reps * kLayers));
    if (n_rows == rows[0]) {                          // the in-flight variants, on the first size only
      time_ring<2, false>(n_rows, K, V, out, bad, ev); time_ring<4, false>(n_rows, K, V, out, bad, ev);
      time_ring<8, false>(n_rows, K, V, out, bad, ev);
      time_ring<4, true>(n_rows, K, V, out, bad, ev); time_ring<8, true>(n_rows, K, V, out, bad, ev);
    }
  }
  return 0;
}
