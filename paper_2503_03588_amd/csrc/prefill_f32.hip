// fp32 prefill (Equation 1 over the listed key blocks) with plain FMA arithmetic.
// This is the full-precision path: fp32 inputs, fp32 products and sums.
//
// One workgroup owns KT consecutive query rows of one head (KT = min(B, 64)):
// four lanes share a row, each holding an interleaved quarter of the head
// dimension.  Key/value tiles of KT tokens are staged in LDS; for each tile the
// four lanes form partial dot products, add them with two lane exchanges, take
// the tile's row maximum, and accumulate exp2-weighted values (online softmax).
#include <math.h>
#include "common.h"

namespace {

struct f32_params {
  const float* q; const float* k; const float* v; float* o; float* lse;
  const int32_t* kv_cnt; const int32_t* kv_idx;
  int32_t max_k, nb, B, hq, hkv, dense;
  int64_t N;
  float c2;   // softmax scale * log2(e)
};

template <int D, int KT>
__global__ __launch_bounds__(4 * KT) void pa_prefill_f32_kernel(f32_params p) {
  constexpr int DQ = D / 4;        // floats of the head dimension per lane
  constexpr int NCH = DQ / 4;      // float4 chunks per lane; chunk m covers d = 16m + 4c .. +3
  __shared__ float4 Ks[KT * D / 4];
  __shared__ float4 Vs[KT * D / 4];

  const int tiles_per_block = p.B / KT;
  const int qb = blockIdx.x / tiles_per_block;
  const int qt = blockIdx.x % tiles_per_block;
  const int h = blockIdx.y, b = blockIdx.z;
  const int kvh = h / (p.hq / p.hkv);
  const int r = threadIdx.x >> 2, c = threadIdx.x & 3;
  const int64_t qrow = (int64_t)qb * p.B + (int64_t)qt * KT + r;
  const bool row_ok = qrow < p.N;

  const float4* q4 = reinterpret_cast<const float4*>(p.q + (((int64_t)b * p.hq + h) * p.N + (row_ok ? qrow : 0)) * D);
  const float4* kbase = reinterpret_cast<const float4*>(p.k + ((int64_t)b * p.hkv + kvh) * p.N * D);
  const float4* vbase = reinterpret_cast<const float4*>(p.v + ((int64_t)b * p.hkv + kvh) * p.N * D);

  float4 qreg[NCH];
#pragma unroll
  for (int m = 0; m < NCH; ++m) qreg[m] = row_ok ? q4[4 * m + c] : make_float4(0.f, 0.f, 0.f, 0.f);
  float4 acc[NCH];
#pragma unroll
  for (int m = 0; m < NCH; ++m) acc[m] = make_float4(0.f, 0.f, 0.f, 0.f);
  float m_run = -INFINITY, l_run = 0.f;

  int n_list = p.dense ? qb + 1 : p.kv_cnt[qb];
  if (!p.dense && n_list > p.max_k) n_list = p.max_k;

  for (int t = 0; t < n_list; ++t) {
    int j = p.dense ? t : p.kv_idx[(int64_t)qb * p.max_k + t];
    if (j < 0 || j > qb) continue;                     // uniform over the workgroup
    const int n_kt = (j == qb) ? qt + 1 : tiles_per_block;   // key tiles past the query tile are fully masked
    for (int kt = 0; kt < n_kt; ++kt) {
      const int64_t key0 = (int64_t)j * p.B + (int64_t)kt * KT;
      __syncthreads();
      for (int e = threadIdx.x; e < KT * D / 4; e += 4 * KT) {
        int64_t krow = key0 + e / (D / 4);
        bool ok = krow < p.N;
        Ks[e] = ok ? kbase[key0 * (D / 4) + e] : make_float4(0.f, 0.f, 0.f, 0.f);
        Vs[e] = ok ? vbase[key0 * (D / 4) + e] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      __syncthreads();

      float s[KT];
#pragma unroll
      for (int jj = 0; jj < KT; ++jj) {
        float part = 0.f;
#pragma unroll
        for (int m = 0; m < NCH; ++m) {
          float4 kk = Ks[jj * (D / 4) + 4 * m + c];
          part = fmaf(qreg[m].x, kk.x, part);
          part = fmaf(qreg[m].y, kk.y, part);
          part = fmaf(qreg[m].z, kk.z, part);
          part = fmaf(qreg[m].w, kk.w, part);
        }
        part += __shfl_xor(part, 1);
        part += __shfl_xor(part, 2);
        s[jj] = part * p.c2;
      }
      if (j == qb && kt == qt) {     // diagonal tile: token-level causality
#pragma unroll
        for (int jj = 0; jj < KT; ++jj) if (jj > r) s[jj] = -INFINITY;
      }
      float tmax = s[0];
#pragma unroll
      for (int jj = 1; jj < KT; ++jj) tmax = fmaxf(tmax, s[jj]);
      const float m_new = fmaxf(m_run, tmax);          // finite: key 0 of the first tile is always visible
      const float alpha = exp2f(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int m = 0; m < NCH; ++m) { acc[m].x *= alpha; acc[m].y *= alpha; acc[m].z *= alpha; acc[m].w *= alpha; }
#pragma unroll
      for (int jj = 0; jj < KT; ++jj) {
        const float pj = exp2f(s[jj] - m_new);
        l_run += pj;
#pragma unroll
        for (int m = 0; m < NCH; ++m) {
          float4 vv = Vs[jj * (D / 4) + 4 * m + c];
          acc[m].x = fmaf(pj, vv.x, acc[m].x);
          acc[m].y = fmaf(pj, vv.y, acc[m].y);
          acc[m].z = fmaf(pj, vv.z, acc[m].z);
          acc[m].w = fmaf(pj, vv.w, acc[m].w);
        }
      }
      m_run = m_new;
    }
  }

  if (row_ok) {
    const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;    // a row whose list is empty: o = 0, lse = -inf
    float4* o4 = reinterpret_cast<float4*>(p.o + (((int64_t)b * p.hq + h) * p.N + qrow) * D);
#pragma unroll
    for (int m = 0; m < NCH; ++m)
      o4[4 * m + c] = make_float4(acc[m].x * inv, acc[m].y * inv, acc[m].z * inv, acc[m].w * inv);
    if (p.lse && c == 0)
      p.lse[((int64_t)b * p.hq + h) * p.N + qrow] = (m_run + log2f(l_run)) * 0.69314718055994530942f;
  }
}

template <int D, int KT>
int launch(const f32_params& p, int32_t batch, hipStream_t stream) {
  dim3 grid((uint32_t)p.nb * (uint32_t)(p.B / KT), (uint32_t)p.hq, (uint32_t)batch);
  hipLaunchKernelGGL((pa_prefill_f32_kernel<D, KT>), grid, dim3(4 * KT), 0, stream, p);
  return pa_note_hip(hipGetLastError());
}

}  // namespace

int pa_launch_prefill_f32(const pa_prefill_args& a) {
  f32_params p;
  p.q = (const float*)a.q; p.k = (const float*)a.k; p.v = (const float*)a.v; p.o = (float*)a.o; p.lse = a.lse;
  p.kv_cnt = a.kv_cnt; p.kv_idx = a.kv_idx; p.max_k = a.max_k; p.nb = a.nb; p.B = a.pat.block;
  p.hq = a.hq; p.hkv = a.hkv; p.dense = (a.pat.flags & POWATTN_DENSE) ? 1 : 0;
  p.N = a.seq_len;
  p.c2 = a.scale * 1.44269504088896340736f;
  if (a.hq > 65535 || a.batch > 65535) return POWATTN_UNSUPPORTED;
  const int B = a.pat.block;
  const int kt = (B % 64 == 0) ? 64 : (B % 32 == 0 ? 32 : 16);
  if (a.head_dim == 64) {
    if (kt == 64) return launch<64, 64>(p, a.batch, a.stream);
    if (kt == 32) return launch<64, 32>(p, a.batch, a.stream);
    return launch<64, 16>(p, a.batch, a.stream);
  }
  if (kt == 64) return launch<128, 64>(p, a.batch, a.stream);
  if (kt == 32) return launch<128, 32>(p, a.batch, a.stream);
  return launch<128, 16>(p, a.batch, a.stream);
}
