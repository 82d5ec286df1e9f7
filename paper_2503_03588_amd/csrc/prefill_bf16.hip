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
//
// Memory pipeline.  A query block attends only a dozen key blocks, so a tile's
// compute (about a microsecond) is shorter than a trip to HBM: one tile of
// prefetch leaves the matrix cores waiting.  K/V tiles therefore travel
// global -> LDS asynchronously (global_load_lds_dwordx4, no registers in
// between) into a ring of NS stages, NS-1 tiles ahead of the compute; a
// wavefront waits on its own loads with s_waitcnt vmcnt(n) and one barrier per
// tile makes the stage visible and frees the oldest one.  The asynchronous
// copy cannot pad rows, so bank conflicts are avoided by a XOR swizzle of the
// 16-byte chunk index with the row index, applied on the global-address side.
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
typedef __attribute__((address_space(3))) char lds_char;

constexpr int KT = 64;          // keys per staged tile
constexpr float RESCALE_TAU = 8.0f;   // running max is only raised when exceeded by 2^8 (see softmax below)

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

// The block list of one query block is copied into LDS once; a lookup is then an LDS read made
// wavefront-uniform with v_readfirstlane.  Going through LDS matters: a lookup from global memory
// inside the tile loop would be a vector load, and waiting for it would also wait for every
// asynchronous tile copy in flight.
constexpr int LIST_CAP = 1024;   // longest block list the kernel accepts (the dense list is implicit)

struct list_view {
  const int* lds;   // the row in LDS
  int n;            // entries
  bool dense;
};

__device__ __forceinline__ int list_at(const list_view& L, int t) {
  return L.dense ? t : __builtin_amdgcn_readfirstlane(L.lds[t]);
}

// first list position >= t whose entry is a causal block, or n
__device__ __forceinline__ tile_pos seek(const list_view& L, int i, int t) {
  tile_pos r;
  r.u = 0;
  for (; t < L.n; ++t) {
    const int j = list_at(L, t);
    if (j >= 0 && j <= i) { r.t = t; r.j = j; r.valid = true; return r; }
  }
  r.t = L.n; r.j = 0; r.valid = false;
  return r;
}

// Positions are the same in every lane; saying so keeps the loop control on the scalar unit.
__device__ __forceinline__ tile_pos uniform(tile_pos r) {
  r.t = __builtin_amdgcn_readfirstlane(r.t);
  r.j = __builtin_amdgcn_readfirstlane(r.j);
  r.u = __builtin_amdgcn_readfirstlane(r.u);
  r.valid = __builtin_amdgcn_readfirstlane((int)r.valid) != 0;
  return r;
}

__device__ __forceinline__ tile_pos advance(const list_view& L, int i, tile_pos c, int subs, int subs_diag) {
  const int lim = (c.j == i) ? subs_diag : subs;
  if (c.u + 1 < lim) { c.u += 1; return uniform(c); }
  return uniform(seek(L, i, c.t + 1));
}

// Asynchronous 16-byte-per-lane copy global -> LDS: lane l's data lands at lds_off + 16*l.
// Written as inline assembly on purpose: the compiler then does not pair every later LDS read
// with a full vmcnt(0) wait, and the waits are placed by hand (wait_vmcnt below).  M0 carries
// the LDS offset; nothing else in this kernel uses M0.
__device__ __forceinline__ void async_copy16(const void* gptr, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_off) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // s_waitcnt vmcnt(N) only
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// XOR swizzle of the 16-byte chunk index inside a row, as a function of the row's low bits.
// D = 128 (16 chunks per row): any 16 consecutive rows map one chunk column onto 16 different
// bank groups (K fragment reads), and 4 consecutive rows x 4 consecutive chunks map onto 16
// different bank groups (transposing V reads).  D = 64 (8 chunks per row, two rows per 256 B).
template <int D>
__device__ __forceinline__ int swz(int row) {
  if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  return (row >> 1) & 7;
}

template <int D, int CT, int NW, int NS>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(CT == 1 ? 2 : 1, CT == 1 ? 2 : 1)))
void pa_prefill_bf16_kernel(bf16_params p) {
  constexpr int QW = 32 * CT;        // query tokens per wavefront
  constexpr int ROWB = 2 * D;        // bytes per K/V row
  constexpr int CPR = D / 8;         // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;      // rows covered by one wavefront-wide copy instruction
  constexpr int IPT = KT / RPI;      // copy instructions per K (or V) tile
  constexpr int IPW = IPT / NW;      // ... per wavefront
  constexpr int LPT = 2 * IPW;       // copies per wavefront per tile (K and V)
  constexpr int TILEB = KT * ROWB;   // bytes of a K (or V) tile
  constexpr int STAGEB = 2 * TILEB;  // K then V
  constexpr int NC = D / 16;         // 16-wide steps of the head dimension
  constexpr int ND = D / 32;         // 32-row tiles of O^T
  static_assert(IPT % NW == 0, "tile copies must divide over the wavefronts");
  static_assert((NS - 1) * LPT < 64, "outstanding copies must fit the vmcnt counter");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

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
  const int max_sl = (last_task / slices > (chunk * NW) / slices) ? slices - 1 : last_task % slices;
  const int subs_diag = (max_sl * QW + QW - 1) / KT + 1;

  const __bf16* kbase = p.k + (((int64_t)b * p.hkv + kvh) * p.N) * D;
  const __bf16* vbase = p.v + (((int64_t)b * p.hkv + kvh) * p.N) * D;

  // ---- asynchronous tile copy: this wavefront's share of tile `tp` into ring stage `stage` ----
  const int cp_row = lane / CPR, cp_chunk = lane % CPR;
  auto issue_tile = [&](const tile_pos& tp, int stage) {
    const int64_t key0 = (int64_t)tp.j * p.B + (int64_t)tp.u * KT;
#pragma unroll
    for (int x = 0; x < IPW; ++x) {
      const int inst = wave * IPW + x;                 // rows RPI*inst .. +RPI-1 of the tile
      const int row = RPI * inst + cp_row;
      int64_t grow = key0 + row;
      if (grow > p.N - 1) grow = p.N - 1;              // ragged tail: repeat the last row (it is masked, but must be finite)
      const int64_t off = grow * D + ((cp_chunk ^ swz<D>(row)) << 3);
      const uint32_t dst = lds0 + stage * STAGEB + inst * 1024;
      async_copy16(kbase + off, __builtin_amdgcn_readfirstlane(dst));
      async_copy16(vbase + off, __builtin_amdgcn_readfirstlane(dst + TILEB));
    }
  };

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

  // ---- fill the ring ----
  __shared__ int s_list[LIST_CAP];
  list_view Ls;
  Ls.dense = p.dense != 0;
  Ls.lds = s_list;
  {
    int n = p.dense ? i + 1 : p.kv_cnt[i];
    if (!p.dense && n > p.max_k) n = p.max_k;
    if (!p.dense && n > LIST_CAP) n = LIST_CAP;          // the host refuses longer rows
    Ls.n = __builtin_amdgcn_readfirstlane(n);
  }
  if (!p.dense) {
    for (int e = tid; e < Ls.n; e += 64 * NW) s_list[e] = p.kv_idx[(int64_t)i * p.max_k + e];
    __syncthreads();
  }
  tile_pos cur = uniform(seek(Ls, i, 0));
  tile_pos pre = cur;                 // the prefetch position runs NS-1 tiles ahead of the compute position
  int issued = 0;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) {
    if (pre.valid) {
      issue_tile(pre, s);
      pre = advance(Ls, i, pre, p.subs, subs_diag);
      ++issued;
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

  // per-lane pieces of the swizzled LDS addresses
  const int k_sw = swz<D>(ln);                               // rows 32rt + ln share their low bits with ln
  const int v_r4 = 4 * hh + ((lane & 15) >> 2);              // row of the first transposing read inside a 16-key step
  const int v_x = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1); // chunk inside the 32-wide d tile
  const int v_sw0 = swz<D>(v_r4), v_sw1 = swz<D>(v_r4 + 8);

  // Q fragments and the first tiles must have arrived before the loop; waiting here, once, also tells
  // the compiler that none of its own loads is outstanding inside the loop, so that it does not add
  // full vmcnt(0) waits there (they would drain the asynchronous copies as well).
  wait_vmcnt<0>();

  int t = 0;
  while (cur.valid) {
    // tile t has landed once at most the younger tiles' copies are outstanding
    const int pending = issued - (t + 1);
    if (pending >= NS - 1) wait_vmcnt<(NS - 1) * LPT>();
    else if (pending == 2 && NS > 3) wait_vmcnt<(NS > 3 ? 2 : 0) * LPT>();
    else if (pending == 1 && NS > 2) wait_vmcnt<(NS > 2 ? 1 : 0) * LPT>();
    else wait_vmcnt<0>();
    __syncthreads();   // every wavefront's share is in LDS; everybody is done with the stage refilled below
    if (pre.valid) {
      issue_tile(pre, (t + NS - 1) % NS);
      pre = advance(Ls, i, pre, p.subs, subs_diag);
      ++issued;
    }

    const bool diag = (cur.j == i);
    const int key_in_blk = cur.u * KT;
    // tiles of the diagonal block that start after this wavefront's last query are fully masked
    if (active && !(diag && key_in_blk > q_in_blk + QW - 1)) {
      const unsigned char* Kb = smem + (t % NS) * STAGEB;
      const unsigned char* Vb = Kb + TILEB;

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
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Kb + (32 * rt + ln) * ROWB + (((2 * c + hh) ^ k_sw) << 4));
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
        mx = fmaxf(mx, __shfl_xor(mx, 32)) * p.c2;
        // The reference point m of the exponentials need not be the exact running maximum: any m
        // gives the same o and lse as long as exp2(s - m) stays in range.  It is raised only when a
        // score exceeds it by more than RESCALE_TAU (p <= 2^tau), which makes the rescaling of O
        // (64 multiplies per lane) a rare, wavefront-uniform branch instead of a per-tile cost.
        const bool raise = mx > m_run[ct] + RESCALE_TAU;     // also true for the first tile (m = -inf)
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
          const float m_new = raise ? mx : m_run[ct];
          const float alpha = __builtin_amdgcn_exp2f(m_run[ct] - m_new);   // exp2(-inf) = 0 on the first tile
          m_run[ct] = m_new;
          l_run[ct] *= alpha;
#pragma unroll
          for (int dt = 0; dt < ND; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[dt][ct][r] *= alpha;
        }
        const float m_ref = m_run[ct];
        float rowsum = 0.f;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float pv = __builtin_amdgcn_exp2f(fmaf(S[rt][ct][r], p.c2, -m_ref));
            rowsum += pv;
            S[rt][ct][r] = pv;
          }
        l_run[ct] += rowsum;
      }

      // ---- O^T += V^T P^T, 16 keys per step ----
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
          const int cl = 4 * dt + v_x;
          const unsigned char* vp0 = Vb + (16 * kk + v_r4) * ROWB + ((cl ^ v_sw0) << 4) + 8 * (lane & 1);
          const unsigned char* vp1 = Vb + (16 * kk + v_r4 + 8) * ROWB + ((cl ^ v_sw1) << 4) + 8 * (lane & 1);
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp0));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp1));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
            O[dt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ct], O[dt][ct], 0, 0, 0);
        }
      }
    }

    cur = advance(Ls, i, cur, p.subs, subs_diag);
    ++t;
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

template <int D, int CT, int NW, int NS>
int launch(const bf16_params& p, hipStream_t stream) {
  constexpr size_t lds = (size_t)NS * 2 * KT * 2 * D;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pa_prefill_bf16_kernel<D, CT, NW, NS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return pa_note_hip(e);
    attr_done = true;
  }
  const int64_t grid = (int64_t)p.per_xcd * 8;
  hipLaunchKernelGGL((pa_prefill_bf16_kernel<D, CT, NW, NS>), dim3((uint32_t)grid), dim3(64 * NW), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}

}  // namespace

int pa_launch_prefill_bf16(const pa_prefill_args& a) {
  constexpr int ct = 1;   // 32-query wavefronts, two per SIMD (64-query wavefronts measured slower)

  bf16_params p;
  p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.o = (__bf16*)a.o; p.lse = a.lse;
  p.kv_cnt = a.kv_cnt; p.kv_idx = a.kv_idx; p.max_k = a.max_k; p.nb = a.nb; p.B = a.pat.block;
  p.hq = a.hq; p.hkv = a.hkv; p.G = a.hq / a.hkv; p.dense = (a.pat.flags & POWATTN_DENSE) ? 1 : 0;
  p.subs = p.B / KT;
  if (!p.dense && a.max_k > LIST_CAP) return POWATTN_UNSUPPORTED;
  p.N = a.seq_len;
  p.c2 = a.scale * 1.44269504088896340736f;
  const int64_t tasks = (int64_t)p.G * p.B / (32 * ct);
  if (tasks > (1 << 20)) return POWATTN_UNSUPPORTED;
  p.tasks = (int32_t)tasks;
  const int nw = p.tasks > 4 ? 8 : 4;
  p.chunks = (p.tasks + nw - 1) / nw;
  p.total_wg = (int64_t)a.batch * a.hkv * a.nb * p.chunks;
  const int64_t per_xcd = (p.total_wg + 7) / 8;
  if (per_xcd * 8 > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  p.per_xcd = (int32_t)per_xcd;

  // ring of 4 stages: 128 KB of LDS at head_dim 128, 64 KB at head_dim 64
  if (a.head_dim == 128) return nw == 8 ? launch<128, 1, 8, 4>(p, a.stream) : launch<128, 1, 4, 4>(p, a.stream);
  return nw == 8 ? launch<64, 1, 8, 4>(p, a.stream) : launch<64, 1, 4, 4>(p, a.stream);
}
