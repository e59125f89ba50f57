// Reference timings for the dense row passes: kernels that do nothing but read what a pool
// pass has to read.  The dense configuration (n = 1,000,000 rows of d = 1024 fp32, pools of
// 16,384 rows = 64 MiB drawn through a random permutation) is rebuilt with zero-filled rows
// (only addresses matter).  Every figure is the time per launch of 60 launches recorded in one
// HIP graph and replayed (the way the library's steps are launched), best of five replays.
//
//   bare_read_probe            prints the table
//
// Measurement tool only: nothing in the library links or calls it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

typedef float f4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                       \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);         \
      exit(1);                                                                      \
    }                                                                               \
  } while (0)

constexpr int kD = 1024;  // floats per row

// One wave per contiguous chunk of pool positions (the split the row passes use), RIF rows
// requested before any is used, non-temporal 128-bit loads, rows found through `idx`.
template <int RIF>
__global__ __launch_bounds__(1024) void k_read_rows(const float *x, const int *idx, int P, float *out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nwaves = gridDim.x * nw, gw = blockIdx.x * nw + wave;
  const int per = P / nwaves, rem = P % nwaves;
  const int lo = gw * per + min(gw, rem), hi = lo + per + (gw < rem ? 1 : 0);
  float acc = 0.f;
  for (int j = lo; j < hi; j += RIF) {
    f4 v[RIF][4];
#pragma unroll
    for (int r = 0; r < RIF; ++r) {
      const int row = idx[min(j + r, hi - 1)];
      const f4 *p = reinterpret_cast<const f4 *>(x + (size_t)row * kD);
#pragma unroll
      for (int q = 0; q < 4; ++q) v[r][q] = __builtin_nontemporal_load(p + q * 64 + lane);
    }
#pragma unroll
    for (int r = 0; r < RIF; ++r)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc += v[r][q].x + v[r][q].y + v[r][q].z + v[r][q].w;
  }
  if (acc == 12345.678f) out[0] = acc;  // never true for zero rows: keeps the loads alive
}

// Plain grid-stride read of n4 128-bit pieces.
__global__ __launch_bounds__(256) void k_read_stream(const f4 *x, size_t n4, float *out) {
  float acc = 0.f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    const f4 v = __builtin_nontemporal_load(x + i);
    acc += v.x + v.y + v.z + v.w;
  }
  if (acc == 12345.678f) out[0] = acc;
}

__global__ void k_nothing(float *out) {
  if (threadIdx.x == 9999) out[1] = 1.f;
}

int main() {
  const size_t n = 1000000;
  const int P = 16384, NPOOL = 60;
  float *x, *out;
  CK(hipMalloc(&x, n * kD * sizeof(float)));
  CK(hipMemset(x, 0, n * kD * sizeof(float)));
  CK(hipMalloc(&out, 1024));
  std::mt19937 gen(1);
  std::vector<int> perm(n);
  for (size_t i = 0; i < n; ++i) perm[i] = (int)i;
  std::shuffle(perm.begin(), perm.end(), gen);
  int *dperm;
  CK(hipMalloc(&dperm, n * sizeof(int)));
  CK(hipMemcpy(dperm, perm.data(), n * sizeof(int), hipMemcpyHostToDevice));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  hipStream_t st;
  CK(hipStreamCreate(&st));

  auto time_graph = [&](const char *name, auto enqueue, int reps, double bytes) {
    hipGraph_t gr;
    hipGraphExec_t ge;
    CK(hipStreamBeginCapture(st, hipStreamCaptureModeGlobal));
    for (int r = 0; r < reps; ++r) enqueue(r);
    CK(hipStreamEndCapture(st, &gr));
    CK(hipGraphInstantiate(&ge, gr, nullptr, nullptr, 0));
    CK(hipGraphLaunch(ge, st));
    CK(hipStreamSynchronize(st));
    float best = 1e9f;
    for (int k = 0; k < 5; ++k) {
      CK(hipEventRecord(e0, st));
      CK(hipGraphLaunch(ge, st));
      CK(hipEventRecord(e1, st));
      CK(hipStreamSynchronize(st));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      best = std::min(best, ms);
    }
    const double us = best * 1e3 / reps;
    if (bytes > 0)
      printf("%-58s %7.2f us per launch  %6.0f GB/s (%4.1f %% of 8 TB/s)\n", name, us, bytes / us / 1e3,
             bytes / us / 1e3 / 80.0);
    else
      printf("%-58s %7.2f us per launch\n", name, us);
    CK(hipGraphExecDestroy(ge));
    CK(hipGraphDestroy(gr));
  };

  const double pool_bytes = (double)P * kD * 4;
  printf("bare reads of one pool (16,384 rows of 4 KiB = 64 MiB) per launch, 60 launches per graph\n");
  time_graph("nothing (64 blocks x 256): launch cadence", [&](int) {
    hipLaunchKernelGGL(k_nothing, dim3(64), dim3(256), 0, st, out); }, NPOOL, 0);
  time_graph("random rows, 256 blocks x 16 waves, 1 row in flight", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<1>, dim3(256), dim3(1024), 0, st, x, dperm + (size_t)r * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 256 blocks x 16 waves, 2 rows in flight", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(1024), 0, st, x, dperm + (size_t)r * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 256 blocks x 16 waves, 4 rows in flight", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<4>, dim3(256), dim3(1024), 0, st, x, dperm + (size_t)r * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 256 blocks x 8 waves, 2 rows in flight", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)r * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 256 blocks x 8 waves, 4 rows in flight", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<4>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)r * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 1024 blocks x 4 waves, 4 rows in flight", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<4>, dim3(1024), dim3(256), 0, st, x, dperm + (size_t)r * P, P, out); }, NPOOL, pool_bytes);
  time_graph("consecutive 64 MiB, 2048 blocks x 4 waves", [&](int r) {
    hipLaunchKernelGGL(k_read_stream, dim3(2048), dim3(256), 0, st,
                       reinterpret_cast<const f4 *>(x + (size_t)r * P * kD), (size_t)P * kD / 4, out); }, NPOOL, pool_bytes);
  // re-reads: does a pool that was read one, two or four launches ago come back faster (from the
  // 256 MB memory-side cache) than one read for the first time?
  time_graph("random rows, 8 waves x 2, the same pool every launch", [&](int) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 8 waves x 2, two pools in turn (128 MiB)", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)(r % 2) * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 8 waves x 2, three pools in turn (192 MiB)", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)(r % 3) * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 8 waves x 2, four pools in turn (256 MiB)", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)(r % 4) * P, P, out); }, NPOOL, pool_bytes);
  time_graph("random rows, 8 waves x 2, six pools in turn (384 MiB)", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)(r % 6) * P, P, out); }, NPOOL, pool_bytes);
  time_graph("4 pools (256 MiB) of random rows in one launch, 8 waves x 2", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)(r % 15) * 4 * P, 4 * P, out); }, NPOOL, 4 * pool_bytes);
  time_graph("16 pools (1 GiB) of random rows in one launch, 8 waves x 2", [&](int r) {
    hipLaunchKernelGGL(k_read_rows<2>, dim3(256), dim3(512), 0, st, x, dperm + (size_t)(r % 3) * 16 * P, 16 * P, out); }, 12, 16 * pool_bytes);
  time_graph("the whole matrix (4.1 GB) consecutively, one launch", [&](int) {
    hipLaunchKernelGGL(k_read_stream, dim3(2048), dim3(256), 0, st, reinterpret_cast<const f4 *>(x), n * kD / 4, out); }, 3, (double)n * kD * 4);
  return 0;
}
