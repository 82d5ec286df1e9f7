// Sustained rate of back-to-back bf16 matrix instructions on this machine: the practical ceiling under the
// published matrix peak (the shader clock under matrix load sits below the nominal one).  Built by
// paper_2503_03588_amd/build.py; bench.py runs it and reports the best line as `measured_peaks.mfma_bf16_tflops`.
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <int NACC>
__global__ __launch_bounds__(512) void k32(float* out, int iters) {
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x + e); b[e] = (__bf16)(float)(threadIdx.x * 3 + e); }
  f32x16 c[NACC];
  for (int i = 0; i < NACC; ++i) for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i], 0, 0, 0);
  }
  float s = 0; for (int i = 0; i < NACC; ++i) for (int r = 0; r < 16; ++r) s += c[i][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
template <int NACC>
__global__ __launch_bounds__(512) void k16(float* out, int iters) {
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x + e); b[e] = (__bf16)(float)(threadIdx.x * 3 + e); }
  f32x4 c[NACC];
  for (int i = 0; i < NACC; ++i) for (int r = 0; r < 4; ++r) c[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[i], 0, 0, 0);
  }
  float s = 0; for (int i = 0; i < NACC; ++i) for (int r = 0; r < 4; ++r) s += c[i][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
int main() {
  float* out; hipMalloc(&out, 256 * 8 * 1024 * 4);
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  double best = 0.0;
  auto run = [&](const char* name, auto kern, int threads, int nacc, double flop_per_mfma, int grid) {
    int iters = 20000;
    hipLaunchKernelGGL(kern, grid, threads, 0, 0, out, 100); hipDeviceSynchronize();
    hipEventRecord(e0); hipLaunchKernelGGL(kern, grid, threads, 0, 0, out, iters); hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    double fl = (double)grid * (threads / 64) * iters * nacc * flop_per_mfma;
    printf("%-34s %8.3f ms  %8.1f TFLOP/s\n", name, ms, fl / ms / 1e9);
    if (fl / ms / 1e9 > best) best = fl / ms / 1e9;
  };
  run("32x32x16 4acc 8w/CU x256", k32<4>, 512, 4, 32768.0, 256);
  run("32x32x16 2acc 8w/CU x256", k32<2>, 512, 2, 32768.0, 256);
  run("32x32x16 4acc 4w/CU x256", k32<4>, 256, 4, 32768.0, 256);
  run("32x32x16 4acc 8w/CU x512 WG", k32<4>, 512, 4, 32768.0, 512);
  run("16x16x32 4acc 8w/CU x256", k16<4>, 512, 4, 16384.0, 256);
  run("16x16x32 8acc 8w/CU x256", k16<8>, 512, 8, 16384.0, 256);
  run("32x32x16 4acc 8w/CU x256 (again)", k32<4>, 512, 4, 32768.0, 256);
  printf("RESULT mfma_bf16_tflops=%.1f\n", best);
  return 0;
}
