// Measurement aid (not part of the library): what a kernel that ONLY reads the attention kernel's bytes achieves on
// this GPU, in the attention kernel's launch shape and access pattern -- the ceiling its HBM roofline fraction is
// read against.  768 workgroups x 4 waves (one per (sequence, head) of the XXL-shaped layer); a workgroup reads
// `rows` consecutive 128-byte rows of its head's K region and of its V region with 16-byte nontemporal loads, U row
// pairs per lane in flight, and does nothing with them.  48 distinct layers are cycled so that nothing is served
// from a cache.  Prints the kernel-only duration (HIP events on the dispatch) and the back-to-back time per launch.
//   read_ceiling [rows ...]        default rows: 673 524 256
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
#define GLOBAL_AS __attribute__((address_space(1)))
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

int main(int argc, char** argv) {
  std::vector<int> rows;
  for (int i = 1; i < argc; ++i) rows.push_back(atoi(argv[i]));
  if (rows.empty()) rows = {673, 524, 256};
  const size_t layer_bytes = (size_t)kUnits * kCap * 128;
  std::vector<char*> K(kLayers), V(kLayers);
  for (int l = 0; l < kLayers; ++l) {
    CK(hipMalloc(&K[l], layer_bytes)); CK(hipMalloc(&V[l], layer_bytes));
    CK(hipMemset(K[l], 1, layer_bytes)); CK(hipMemset(V[l], 2, layer_bytes));
  }
  float* out; CK(hipMalloc(&out, 1 << 16));
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
  }
  return 0;
}
