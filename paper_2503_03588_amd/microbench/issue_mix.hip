// Probe: sustained MFMA rate of an in-stream mix  MFMA + NV fma + NE exp + ND LDS reads  per slot, 8 waves per CU.
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define FMA(v) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(v) : "v"(ka), "v"(kb))
#define EXP(v) asm volatile("v_exp_f32 %0, %0" : "+v"(v))
#define MFMA(c, a) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b))
#define LDS128(d, addr, off) asm volatile("ds_read_b128 %0, %1 offset:" #off : "=v"(d) : "v"(addr))
#define LDSTR(d, addr, off) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #off : "=v"(d) : "v"(addr))
#define WAIT(n) asm volatile("s_waitcnt lgkmcnt(" #n ")")

// DSK: 0 none, 1 = one b128 per slot, 2 = two tr_b64 per slot, 3 = alternate (QK-like half, PV-like half)
// The fragment read in slot s is consumed by the MFMA of slot s+3 (registers rotate over 4 buffers).
template <int NV, int NE, int DSK, int USEFRAG>
__global__ __launch_bounds__(512) void k(float* out, long long* cyc, int iters) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[65536];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) ((float*)lds)[i] = (i & 7) * 0.5f;
  __syncthreads();
  bf16x8 b;
  for (int e = 0; e < 8; ++e) b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 3);
  f32x16 c0, c1, c2, c3;
  for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; c2[r] = 0.f; c3[r] = 0.f; }
  float v0 = threadIdx.x * 0.001f, v1 = v0 + 1, v2 = v0 + 2, v3 = v0 + 3, v4 = v0 + 4, v5 = v0 + 5, v6 = v0 + 6;
  float ka = 0.999f, kb = 0.0001f;
  uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds + (wave & 3) * 8192 + lane * 16;
  uint32_t addr8 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds + (wave & 3) * 8192 + lane * 8;
  bf16x8 f0 = b, f1 = b, f2 = b, f3 = b;   // fragment ring
  f32x2 h0, h1;
#define VAL() { if (NV > 0) FMA(v0); if (NV > 1) FMA(v1); if (NV > 2) FMA(v2); if (NV > 3) FMA(v3); if (NV > 4) FMA(v4); if (NE > 0) EXP(v5); if (NE > 1) EXP(v6); }
#define RD128(f, off) { if (DSK == 1 || DSK == 3) LDS128(f, addr, off); }
#define RDTR(f, off) { if (DSK == 2 || DSK == 4) { LDSTR(h0, addr8, off); LDSTR(h1, addr8, off + 512); f = __builtin_bit_cast(bf16x8, __builtin_shufflevector(h0, h1, 0, 1, 2, 3)); } }
  long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    // 8 slots; reads for slot s+3; waits allow the 3 newest reads (b128) or 6 newest (tr pairs) to be outstanding
    if (DSK == 1) {
      WAIT(2); MFMA(c0, f0); RD128(f3, 0);    VAL();
      WAIT(2); MFMA(c1, f1); RD128(f0, 1024); VAL();
      WAIT(2); MFMA(c2, f2); RD128(f1, 2048); VAL();
      WAIT(2); MFMA(c3, f3); RD128(f2, 3072); VAL();
      WAIT(2); MFMA(c0, f0); RD128(f3, 4096); VAL();
      WAIT(2); MFMA(c1, f1); RD128(f0, 5120); VAL();
      WAIT(2); MFMA(c2, f2); RD128(f1, 6144); VAL();
      WAIT(2); MFMA(c3, f3); RD128(f2, 7168); VAL();
    } else if (DSK == 2) {
      WAIT(4); MFMA(c0, f0); RDTR(f3, 0);    VAL();
      WAIT(4); MFMA(c1, f1); RDTR(f0, 1024); VAL();
      WAIT(4); MFMA(c2, f2); RDTR(f1, 2048); VAL();
      WAIT(4); MFMA(c3, f3); RDTR(f2, 3072); VAL();
      WAIT(4); MFMA(c0, f0); RDTR(f3, 4096); VAL();
      WAIT(4); MFMA(c1, f1); RDTR(f0, 5120); VAL();
      WAIT(4); MFMA(c2, f2); RDTR(f1, 6144); VAL();
      WAIT(4); MFMA(c3, f3); RDTR(f2, 7168); VAL();
    } else {
      MFMA(c0, f0); VAL(); MFMA(c1, f1); VAL(); MFMA(c2, f2); VAL(); MFMA(c3, f3); VAL();
      MFMA(c0, f0); VAL(); MFMA(c1, f1); VAL(); MFMA(c2, f2); VAL(); MFMA(c3, f3); VAL();
    }
  }
  long long t1 = clock64();
  float s = v0 + v1 + v2 + v3 + v4 + v5 + v6;
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && lane == 0) cyc[wave] = t1 - t0;
}

int main() {
  float* out; hipMalloc(&out, 256 * 512 * 4);
  long long* cyc; hipMalloc(&cyc, 64); long long hc[8];
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  auto run = [&](const char* name, auto kern, int threads) {
    int iters = 10000;
    hipLaunchKernelGGL(kern, 256, threads, 0, 0, out, cyc, 100); hipDeviceSynchronize();
    hipEventRecord(e0); hipLaunchKernelGGL(kern, 256, threads, 0, 0, out, cyc, iters); hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    hipMemcpy(hc, cyc, 64, hipMemcpyDeviceToHost);
    int nw = threads / 64;
    double mx = 0; for (int w = 0; w < nw; ++w) mx = hc[w] > mx ? hc[w] : mx;
    // SIMD cycles per MFMA: waves per SIMD = nw/4; each wave does 8 MFMAs per iter
    double per = mx / iters / (8.0 * nw / 4);
    printf("%-44s %8.3f ms  clk/iter(max wave) %7.1f  SIMD clk per MFMA %5.1f  (MFMA util %4.0f%%)\n", name, ms, mx / iters, per, 3200.0 / per);
  };
  run("8w MFMA only", k<0, 0, 0, 0>, 512);
  run("8w MFMA + 3 fma + 1 exp", k<3, 1, 0, 0>, 512);
  run("8w MFMA + 4 fma + 1 exp", k<4, 1, 0, 0>, 512);
  run("8w MFMA + 5 fma + 1 exp", k<5, 1, 0, 0>, 512);
  run("8w MFMA + 1 b128", k<0, 0, 1, 0>, 512);
  run("8w MFMA + 1 b128 + 3 fma + 1 exp", k<3, 1, 1, 0>, 512);
  run("8w MFMA + 1 b128 + 4 fma + 1 exp", k<4, 1, 1, 0>, 512);
  run("8w MFMA + 2 tr64", k<0, 0, 2, 0>, 512);
  run("8w MFMA + 2 tr64 + 3 fma + 1 exp", k<3, 1, 2, 0>, 512);
  run("8w MFMA + 2 tr64 + 4 fma + 1 exp", k<4, 1, 2, 0>, 512);
  run("8w MFMA + 2 tr64 + 5 fma + 1 exp", k<5, 1, 2, 0>, 512);
  run("4w MFMA + 1 b128 + 4 fma + 1 exp", k<4, 1, 1, 0>, 256);
  run("4w MFMA + 2 tr64 + 4 fma + 1 exp", k<4, 1, 2, 0>, 256);
  return 0;
}
