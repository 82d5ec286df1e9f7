#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// mode 0: all 8 waves MFMA only. mode 1: waves 0-3 MFMA, waves 4-7 VALU only. mode 2: all waves VALU only.
// mode 3: every wave interleaves 1 MFMA + NV independent VALU (same stream). mode 4: waves 0-3 MFMA, 4-7 exp only
template <int MODE, int NV>
__global__ __launch_bounds__(512) void k(float* out, int iters) {
  int wave = threadIdx.x >> 6;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x + e); b[e] = (__bf16)(float)(threadIdx.x * 3 + e); }
  f32x16 c[4];
  for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
  float v[8]; for (int i = 0; i < 8; ++i) v[i] = threadIdx.x * 0.001f + i;
  bool do_mfma = MODE == 0 || MODE == 3 || ((MODE == 1 || MODE == 4) && wave < 4);
  bool do_valu = MODE == 2 || ((MODE == 1 || MODE == 4) && wave >= 4);
  if (MODE == 3) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < NV; ++j) v[j % 8] = __builtin_fmaf(v[j % 8], 1.0001f, 0.5f);
      }
    }
  } else if (do_mfma) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i], 0, 0, 0);
    }
  } else if (do_valu) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        if (MODE == 4) v[j % 8] = __builtin_amdgcn_exp2f(v[j % 8]);
        else v[j % 8] = __builtin_fmaf(v[j % 8], 1.0001f, 0.5f);
      }
    }
  }
  float s = 0; for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) s += c[i][r];
  for (int i = 0; i < 8; ++i) s += v[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
int main() {
  float* out; hipMalloc(&out, 256 * 512 * 4);
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  auto run = [&](const char* name, auto kern, double mfma_waves, double valu_waves, int valu_per_iter) {
    int iters = 20000;
    hipLaunchKernelGGL(kern, 256, 512, 0, 0, out, 100); hipDeviceSynchronize();
    hipEventRecord(e0); hipLaunchKernelGGL(kern, 256, 512, 0, 0, out, iters); hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    double fl = 256.0 * mfma_waves * iters * 4 * 32768.0;
    double vops = 256.0 * valu_waves * iters * (double)valu_per_iter;
    printf("%-46s %8.3f ms  MFMA %7.1f TFLOP/s   VALU %6.2f Gwave-inst/s (%.2f clk/inst/SIMD @2.0GHz)\n", name, ms, fl / ms / 1e9, vops / ms / 1e6,
           vops > 0 ? (ms * 1e-3 * 2.0e9 * 1024) / vops : 0.0);
  };
  run("mode0: 8 waves MFMA", k<0, 0>, 8, 0, 0);
  run("mode2: 8 waves VALU fma", k<2, 0>, 0, 8, 32);
  run("mode1: 4 waves MFMA + 4 waves VALU fma", k<1, 0>, 4, 4, 32);
  run("mode4: 4 waves MFMA + 4 waves exp", k<4, 0>, 4, 4, 32);
  run("mode3: 8 waves, 1 MFMA + 2 VALU interleaved", k<3, 2>, 8, 8, 8);
  run("mode3: 8 waves, 1 MFMA + 4 VALU interleaved", k<3, 4>, 8, 8, 16);
  run("mode3: 8 waves, 1 MFMA + 6 VALU interleaved", k<3, 6>, 8, 8, 24);
  run("mode3: 8 waves, 1 MFMA + 8 VALU interleaved", k<3, 8>, 8, 8, 32);
  return 0;
}
