// bf16 prefill on the gfx950 matrix cores: Equation 1 (Section 3.1) over the
// key blocks listed for each query block (Algorithm 1 lifted to blocks), as a
// flash-style online softmax with fp32 accumulation.
//
// Decomposition.  A workgroup owns one (batch, KV head, query block) and up to
// NW "tasks"; a task is one query head of the GQA group x one slice of 32*CT
// consecutive query tokens, and belongs to one wavefront.  All wavefronts of
// the workgroup share the K/V tiles staged in LDS, which is what lifts the
// arithmetic intensity: a 64-key tile is read from HBM/L2 once per workgroup
// and used by every head of the group.
//
// Per 64-key tile a wavefront computes, with v_mfma_f32_32x32x16_bf16,
//   S^T = K Q^T   (A = K rows from LDS, B = Q^T held in registers)
//   O^T += V^T P^T (A = V^T through transposing LDS reads, B = P^T)
// In the transposed form every lane owns one query column: the 32 scores a
// lane holds per tile belong to the same query, so row max / row sum need a
// single exchange between lane l and lane l+32, and the accumulator layout of
// S^T is already the B-operand layout of the second product (the key order
// inside a 16-key step is permuted identically for P^T and V^T, which a
// contraction does not care about).
#include <math.h>
#include <stdlib.h>
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int KT = 64;  // keys per staged tile

struct bf16_params {
  const __bf16* q; const __bf16* k; const __bf16* v; __bf16* o; float* lse;
  const int32_t* kv_cnt; const int32_t* kv_idx;
  int32_t max_k, nb, B, hq, hkv, G, dense;
  int32_t subs;      // 64-key tiles per block
  int32_t tasks;     // G * B / (32*CT)
  int32_t chunks;    // workgroups per (batch, kv head, query block)
  int32_t per_xcd;   // workgroups per XCD partition
  int64_t total_wg;
  int64_t N;
  float c2;          // softmax scale * log2(e)
};

// Position inside the flattened sequence of 64-key tiles of one query block.
struct tile_pos {
  int t;   // list position
  int j;   // key block
  int u;   // 64-key tile inside the block
  bool valid;
};

__device__ __forceinline__ int list_len(const bf16_params& p, int i) {
  if (p.dense) return i + 1;
  int n = p.kv_cnt[i];
  return n < p.max_k ? n : p.max_k;
}

// first list position >= t whose entry is a causal block, or n
__device__ __forceinline__ tile_pos seek(const bf16_params& p, int i, int n, int t) {
  tile_pos r;
  r.u = 0;
  for (; t < n; ++t) {
    int j = p.dense ? t : p.kv_idx[(int64_t)i * p.max_k + t];
    if (j >= 0 && j <= i) { r.t = t; r.j = j; r.valid = true; return r; }
  }
  r.t = n; r.j = 0; r.valid = false;
  return r;
}

__device__ __forceinline__ tile_pos advance(const bf16_params& p, int i, int n, tile_pos c, int subs_diag) {
  const int lim = (c.j == i) ? subs_diag : p.subs;
  if (c.u + 1 < lim) { c.u += 1; return c; }
  return seek(p, i, n, c.t + 1);
}

template <int D, int CT, int NW>
__global__ __launch_bounds__(64 * NW) void pa_prefill_bf16_kernel(bf16_params p) {
  constexpr int QW = 32 * CT;        // query tokens per wavefront
  constexpr int NT = 64 * NW;
  constexpr int KSTR = D + 8;        // LDS row pitch of K in elements: 16-lane groups of a b128 read hit distinct banks
  constexpr int VSTR = D + 32;       // LDS row pitch of V: the 4 rows x 64 B of a transposing read hit distinct banks
  constexpr int CPR = D / 8;         // 16-byte chunks per K/V row
  constexpr int CHUNKS = KT * CPR;   // chunks per tile
  constexpr int CPT = (CHUNKS + NT - 1) / NT;  // chunks per thread
  constexpr int NC = D / 16;         // 16-wide steps of the head dimension
  constexpr int ND = D / 32;         // 32-row tiles of O^T

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __bf16* Ks = reinterpret_cast<__bf16*>(smem);   // [2][KT][KSTR]
  __bf16* Vs = Ks + 2 * KT * KSTR;                // [2][KT][VSTR]

  // ---- which work item: consecutive items stay on one XCD (one L2) ----
  const int pid = blockIdx.x;
  const int slot = pid >> 3;
  int64_t L = (int64_t)(pid & 7) * p.per_xcd + slot;
  if (slot >= p.per_xcd || L >= p.total_wg) return;
  const int chunk = (int)(L % p.chunks); L /= p.chunks;
  const int i = p.nb - 1 - (int)(L % p.nb); L /= p.nb;   // longest rows first (matters for the dense list)
  const int kvh = (int)(L % p.hkv);
  const int b = (int)(L / p.hkv);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int ln = lane & 31, hh = lane >> 5;
  const int slices = p.B / QW;
  const int task = chunk * NW + wave;
  const bool active = task < p.tasks;
  const int g = active ? task / slices : 0;
  const int sl = active ? task % slices : 0;
  const int h = kvh * p.G + g;
  const int q_in_blk = sl * QW;                       // first query of this wavefront inside the block
  const int64_t q0 = (int64_t)i * p.B + q_in_blk;

  // tiles of the diagonal block needed by any wavefront of this workgroup
  int last_task = chunk * NW + NW - 1;
  if (last_task > p.tasks - 1) last_task = p.tasks - 1;
  int max_sl = (last_task / slices > (chunk * NW) / slices) ? slices - 1 : last_task % slices;
  const int subs_diag = (max_sl * QW + QW - 1) / KT + 1;

  // ---- Q^T fragments: lane = query column, 8 consecutive d per 16-wide step ----
  bf16x8 qf[CT][NC];
  const __bf16* qbase = p.q + (((int64_t)b * p.hq + h) * p.N) * D;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int64_t tok = q0 + 32 * ct + ln;
    const bool ok = active && tok < p.N;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[ct][c] = ok ? *reinterpret_cast<const bf16x8*>(qbase + tok * D + 16 * c + 8 * hh) : z;
    }
  }

  f32x16 O[ND][CT];
#pragma unroll
  for (int dt = 0; dt < ND; ++dt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[dt][ct][r] = 0.f;
  float m_run[CT], l_run[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) { m_run[ct] = -INFINITY; l_run[ct] = 0.f; }

  const __bf16* kbase = p.k + (((int64_t)b * p.hkv + kvh) * p.N) * D;
  const __bf16* vbase = p.v + (((int64_t)b * p.hkv + kvh) * p.N) * D;

  uint4 kreg[CPT], vreg[CPT];
  auto load_tile = [&](const tile_pos& tp) {
    const int64_t key0 = (int64_t)tp.j * p.B + (int64_t)tp.u * KT;
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const int c = tid + x * NT;
      const int row = c / CPR;
      const bool ok = (CHUNKS % NT == 0 || c < CHUNKS) && (key0 + row) < p.N;
      const int64_t off = key0 * D + (int64_t)c * 8;
      kreg[x] = ok ? *reinterpret_cast<const uint4*>(kbase + off) : make_uint4(0, 0, 0, 0);
      vreg[x] = ok ? *reinterpret_cast<const uint4*>(vbase + off) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const int c = tid + x * NT;
      if (CHUNKS % NT == 0 || c < CHUNKS) {
        const int row = c / CPR, col = c % CPR;
        *reinterpret_cast<uint4*>(Ks + (buf * KT + row) * KSTR + col * 8) = kreg[x];
        *reinterpret_cast<uint4*>(Vs + (buf * KT + row) * VSTR + col * 8) = vreg[x];
      }
    }
  };

  const int n_list = list_len(p, i);
  tile_pos cur = seek(p, i, n_list, 0);
  if (cur.valid) {
    load_tile(cur);
    store_tile(0);
  }
  __syncthreads();
  int buf = 0;

  while (cur.valid) {
    const tile_pos nxt = advance(p, i, n_list, cur, subs_diag);
    if (nxt.valid) load_tile(nxt);

    const bool diag = (cur.j == i);
    const int key_in_blk = cur.u * KT;
    // tiles of the diagonal block that start after this wavefront's last query are fully masked
    if (active && !(diag && key_in_blk > q_in_blk + QW - 1)) {
      const __bf16* Kb = Ks + buf * KT * KSTR;
      const __bf16* Vb = Vs + buf * KT * VSTR;

      // ---- S^T = K Q^T ----
      f32x16 S[2][CT];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int r = 0; r < 16; ++r) S[rt][ct][r] = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Kb + (32 * rt + ln) * KSTR + 16 * c + 8 * hh);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
            S[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ct][c], S[rt][ct], 0, 0, 0);
        }
      }

      // ---- online softmax; register r of tile rt is key 32rt + 8(r/4) + 4hh + r%4 ----
      const bool need_mask = diag && (key_in_blk + KT - 1 > q_in_blk);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        if (need_mask) {
          const int qpos = q_in_blk + 32 * ct + ln;
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int kpos = key_in_blk + 32 * rt + 8 * (r >> 2) + 4 * hh + (r & 3);
              if (kpos > qpos) S[rt][ct][r] = -INFINITY;
            }
        }
        float mx = S[0][ct][0];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[rt][ct][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run[ct], mx * p.c2);
        const float alpha = __builtin_amdgcn_exp2f(m_run[ct] - m_new);
        m_run[ct] = m_new;
        float rowsum = 0.f;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float pv = __builtin_amdgcn_exp2f(fmaf(S[rt][ct][r], p.c2, -m_new));
            rowsum += pv;
            S[rt][ct][r] = pv;
          }
        l_run[ct] = l_run[ct] * alpha + rowsum;
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[dt][ct][r] *= alpha;
      }

      // ---- O^T += V^T P^T, 16 keys per step ----
      const int vrow = 4 * hh + ((lane & 15) >> 2);
      const int vcol = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int rt = kk >> 1, r0 = 8 * (kk & 1);
        bf16x8 pf[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int e = 0; e < 8; ++e) pf[ct][e] = (__bf16)S[rt][ct][r0 + e];
#pragma unroll
        for (int dt = 0; dt < ND; ++dt) {
          const __bf16* vp = Vb + (16 * kk + vrow) * VSTR + 32 * dt + vcol;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 8 * VSTR));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
            O[dt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ct], O[dt][ct], 0, 0, 0);
        }
      }
    }

    if (!nxt.valid) break;
    store_tile(buf ^ 1);
    __syncthreads();
    buf ^= 1;
    cur = nxt;
  }

  // ---- epilogue: register r of tile dt is d = 32dt + 8(r/4) + 4hh + r%4 ----
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const float ltot = l_run[ct] + __shfl_xor(l_run[ct], 32);
    const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
    const int64_t tok = q0 + 32 * ct + ln;
    if (active && tok < p.N) {
      __bf16* orow = p.o + (((int64_t)b * p.hq + h) * p.N + tok) * D;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(O[dt][ct][4 * g4 + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g4 + 4 * hh) = w;
        }
      if (p.lse && hh == 0)
        p.lse[((int64_t)b * p.hq + h) * p.N + tok] = (m_run[ct] + log2f(ltot)) * 0.69314718055994530942f;
    }
  }
}

template <int D, int CT, int NW>
int launch(const bf16_params& p, hipStream_t stream) {
  constexpr size_t lds = (size_t)2 * KT * ((D + 8) + (D + 32)) * sizeof(__bf16);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pa_prefill_bf16_kernel<D, CT, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return pa_note_hip(e);
    attr_done = true;
  }
  const int64_t grid = (int64_t)p.per_xcd * 8;
  hipLaunchKernelGGL((pa_prefill_bf16_kernel<D, CT, NW>), dim3((uint32_t)grid), dim3(64 * NW), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}

template <int D, int CT>
int launch_nw(const bf16_params& p, int nw, hipStream_t stream) {
  if constexpr (CT == 1) {
    if (nw == 8) return launch<D, 1, 8>(p, stream);
  }
  return launch<D, CT, 4>(p, stream);
}

}  // namespace

int pa_launch_prefill_bf16(const pa_prefill_args& a) {
  static const int env_ct = [] { const char* s = getenv("POWATTN_PREFILL_CT"); return s ? atoi(s) : 0; }();
  const int ct = (env_ct == 1 || env_ct == 2) ? env_ct : 1;

  bf16_params p;
  p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.o = (__bf16*)a.o; p.lse = a.lse;
  p.kv_cnt = a.kv_cnt; p.kv_idx = a.kv_idx; p.max_k = a.max_k; p.nb = a.nb; p.B = a.pat.block;
  p.hq = a.hq; p.hkv = a.hkv; p.G = a.hq / a.hkv; p.dense = (a.pat.flags & POWATTN_DENSE) ? 1 : 0;
  p.subs = p.B / KT;
  p.N = a.seq_len;
  p.c2 = a.scale * 1.44269504088896340736f;
  const int64_t tasks = (int64_t)p.G * p.B / (32 * ct);
  if (tasks > (1 << 20)) return POWATTN_UNSUPPORTED;
  p.tasks = (int32_t)tasks;
  // 64-query wavefronts need the whole register file of a SIMD (one wavefront per SIMD, 4 per
  // workgroup); 32-query wavefronts fit two per SIMD (8 per workgroup)
  const int nw = (ct == 1 && p.tasks > 4) ? 8 : 4;
  p.chunks = (p.tasks + nw - 1) / nw;
  p.total_wg = (int64_t)a.batch * a.hkv * a.nb * p.chunks;
  const int64_t per_xcd = (p.total_wg + 7) / 8;
  if (per_xcd * 8 > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  p.per_xcd = (int32_t)per_xcd;

  if (a.head_dim == 128) return ct == 2 ? launch_nw<128, 2>(p, nw, a.stream) : launch_nw<128, 1>(p, nw, a.stream);
  return ct == 2 ? launch_nw<64, 2>(p, nw, a.stream) : launch_nw<64, 1>(p, nw, a.stream);
}
