// Streaming micro-benchmark: how fast the bytes of one decode step (batch 16, 8 KV heads, 65536-token caches,
// 13 attended blocks of 64 tokens: 54.5 MB in 16 KB pieces) can merely be loaded, for several work splits, with
// addresses known at launch, rotating over six caches so that the reads are cold.  Built by
// paper_2503_03588_amd/build.py; bench.py runs it and reports the best cold line and the empty-launch time as
// `measured_peaks.decode_shaped_read_*`.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
constexpr int NBLK = 13;
__constant__ int c_blocks[NBLK];
constexpr size_t SLAB = 65536ull * 256;  // bytes per (b,kvh) for K (same for V)

// variant A: one WG (256 thr) per (slab, block): 16KB K + 16KB V
__global__ __launch_bounds__(256) void kA(const char* K, const char* V, float* out) {
  int blk = blockIdx.x, slab = blockIdx.y;
  const char* kp = K + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
  const char* vp = V + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
  uint4 acc = make_uint4(0,0,0,0);
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    uint4 a = *(const uint4*)(kp + (threadIdx.x + 256 * x) * 16);
    uint4 b = *(const uint4*)(vp + (threadIdx.x + 256 * x) * 16);
    acc.x ^= a.x ^ b.x; acc.y ^= a.y ^ b.y; acc.z ^= a.z ^ b.z; acc.w ^= a.w ^ b.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1.f;
}
// variant B: one WG (1024 thr) per slab, all 13 blocks; PER = WGs per slab (1 or 2)
template <int PER>
__global__ __launch_bounds__(1024) void kB(const char* K, const char* V, float* out) {
  int slab = blockIdx.x / PER, part = blockIdx.x % PER;
  uint4 acc = make_uint4(0,0,0,0);
  for (int blk = part; blk < NBLK; blk += PER) {
    const char* kp = K + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
    const char* vp = V + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
    uint4 a = *(const uint4*)(kp + threadIdx.x * 16);
    uint4 b = *(const uint4*)(vp + threadIdx.x * 16);
    acc.x ^= a.x ^ b.x; acc.y ^= a.y ^ b.y; acc.z ^= a.z ^ b.z; acc.w ^= a.w ^ b.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1.f;
}
// variant C: single-wave WGs, one per (slab, block)
__global__ __launch_bounds__(64) void kC(const char* K, const char* V, float* out) {
  int blk = blockIdx.x, slab = blockIdx.y;
  const char* kp = K + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
  const char* vp = V + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
  uint4 acc = make_uint4(0,0,0,0);
#pragma unroll
  for (int x = 0; x < 16; ++x) {
    uint4 a = *(const uint4*)(kp + (threadIdx.x + 64 * x) * 16);
    uint4 b = *(const uint4*)(vp + (threadIdx.x + 64 * x) * 16);
    acc.x ^= a.x ^ b.x; acc.y ^= a.y ^ b.y; acc.z ^= a.z ^ b.z; acc.w ^= a.w ^ b.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1.f;
}
template <int KSTRIDED>
__global__ __launch_bounds__(512) void kD(const char* K, const char* V, float* out) {
  int slab = blockIdx.x; int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int g = lane & 15, q4 = lane >> 4;
  uint4 acc = make_uint4(0,0,0,0);
  for (int blk = wave; blk < NBLK; blk += 8) {
    const char* kp = K + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
    const char* vp = V + slab * SLAB + (size_t)c_blocks[blk] * 64 * 256;
    uint4 kr[16], vr[16];
#pragma unroll
    for (int tau = 0; tau < 4; ++tau) {
      int tk = 32 * (tau >> 1) + 8 * (g >> 2) + 4 * (tau & 1) + (g & 3);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (KSTRIDED) kr[tau * 4 + c] = *(const uint4*)(kp + tk * 256 + 64 * c + 16 * q4);
        else kr[tau * 4 + c] = *(const uint4*)(kp + (lane + 64 * (tau * 4 + c)) * 16);
      }
    }
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 8; ++r) vr[x * 8 + r] = *(const uint4*)(vp + (32 * x + 8 * q4 + r) * 256 + 16 * g);
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc.x ^= kr[i].x ^ vr[i].x; acc.y ^= kr[i].y ^ vr[i].y; acc.z ^= kr[i].z ^ vr[i].z; acc.w ^= kr[i].w ^ vr[i].w; }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1.f;
}
__global__ void kEmpty(float* out) { if (threadIdx.x == 9999) out[0] = 0; }
__global__ void kTiny(float* out) { out[blockIdx.x * 64 + threadIdx.x] = 1.f; }

int main() {
  const int NSLAB = 128, NC = 6;
  int blocks[NBLK] = {0,511,767,895,959,991,1007,1015,1019,1020,1021,1022,1023};
  CK(hipMemcpyToSymbol(HIP_SYMBOL(c_blocks), blocks, sizeof(blocks)));
  std::vector<char*> Ks(NC), Vs(NC);
  for (int i = 0; i < NC; ++i) { CK(hipMalloc(&Ks[i], NSLAB * SLAB)); CK(hipMalloc(&Vs[i], NSLAB * SLAB)); CK(hipMemset(Ks[i], 1 + i, NSLAB * SLAB)); CK(hipMemset(Vs[i], 7 + i, NSLAB * SLAB)); }
  float* out; CK(hipMalloc(&out, 1 << 20));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  double best_cold = 1e30, empty_us = 0.0;
  auto timeit = [&](const char* name, auto launch, int iters) {
    for (int i = 0; i < 12; ++i) launch(i);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < iters; ++i) launch(i);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    double us = ms * 1e3 / iters;
    printf("%-40s %8.2f us/launch  %6.2f TB/s (54.5MB)\n", name, us, 54.5e6 / us / 1e6);
    const bool cold = strstr(name, "cold") != nullptr && strstr(name, "2 dependent") == nullptr;
    if (cold && us < best_cold) best_cold = us;
    if (strstr(name, "empty")) empty_us = us;
  };
  timeit("empty kernel", [&](int i) { hipLaunchKernelGGL(kEmpty, 1, 64, 0, 0, out); }, 200);
  timeit("tiny kernel 1664x64", [&](int i) { hipLaunchKernelGGL(kTiny, 1664, 64, 0, 0, out); }, 200);
  timeit("A 1664 WG x256thr cold", [&](int i) { hipLaunchKernelGGL(kA, dim3(NBLK, NSLAB), 256, 0, 0, Ks[i % NC], Vs[i % NC], out); }, 120);
  timeit("A 1664 WG x256thr warm", [&](int i) { hipLaunchKernelGGL(kA, dim3(NBLK, NSLAB), 256, 0, 0, Ks[0], Vs[0], out); }, 120);
  timeit("B 128 WG x1024thr cold", [&](int i) { hipLaunchKernelGGL(kB<1>, 128, 1024, 0, 0, Ks[i % NC], Vs[i % NC], out); }, 120);
  timeit("B 128 WG x1024thr warm", [&](int i) { hipLaunchKernelGGL(kB<1>, 128, 1024, 0, 0, Ks[0], Vs[0], out); }, 120);
  timeit("B2 256 WG x1024thr cold", [&](int i) { hipLaunchKernelGGL(kB<2>, 256, 1024, 0, 0, Ks[i % NC], Vs[i % NC], out); }, 120);
  timeit("C 1664 WG x64thr cold", [&](int i) { hipLaunchKernelGGL(kC, dim3(NBLK, NSLAB), 64, 0, 0, Ks[i % NC], Vs[i % NC], out); }, 120);
  timeit("C 1664 WG x64thr warm", [&](int i) { hipLaunchKernelGGL(kC, dim3(NBLK, NSLAB), 64, 0, 0, Ks[0], Vs[0], out); }, 120);
  timeit("D 128 WG x512 K strided cold", [&](int i) { hipLaunchKernelGGL(kD<1>, 128, 512, 0, 0, Ks[i % NC], Vs[i % NC], out); }, 120);
  timeit("D 128 WG x512 K strided warm", [&](int i) { hipLaunchKernelGGL(kD<1>, 128, 512, 0, 0, Ks[0], Vs[0], out); }, 120);
  timeit("D 128 WG x512 K coalesced cold", [&](int i) { hipLaunchKernelGGL(kD<0>, 128, 512, 0, 0, Ks[i % NC], Vs[i % NC], out); }, 120);
  timeit("D 128 WG x512 K coalesced warm", [&](int i) { hipLaunchKernelGGL(kD<0>, 128, 512, 0, 0, Ks[0], Vs[0], out); }, 120);
  timeit("A + tiny (2 dependent kernels) cold", [&](int i) { hipLaunchKernelGGL(kA, dim3(NBLK, NSLAB), 256, 0, 0, Ks[i % NC], Vs[i % NC], out); hipLaunchKernelGGL(kTiny, 128, 256, 0, 0, out); }, 120);
  printf("RESULT decode_shaped_read_cold_us=%.2f empty_launch_us=%.2f bytes=54525952\n", best_cold, empty_us);
  return 0;
}
