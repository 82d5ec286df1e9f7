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

// The work of one query block is a sequence of 64-key tiles.  For a block list it is written once,
// as the first key of every tile, into a table in LDS (a lookup is then an LDS read made wavefront-
// uniform with v_readfirstlane); for the dense list it is implicit.  Keeping memory out of the tile
// loop matters: a vector load there would have to be waited for together with every asynchronous
// tile copy in flight.
constexpr int TILE_CAP = 4096;   // tiles per query block with an explicit list (16 KB of LDS)

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
  static_assert(NS >= 3 && NS <= 4 && (NS - 1) * LPT < 64, "outstanding copies must fit the vmcnt counter");

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
  auto issue_tile = [&](int64_t key0, int stage) {
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
  __shared__ int s_tile[TILE_CAP];     // first key of tile t (explicit lists only)
  __shared__ int s_ntiles;
  const int64_t blk0 = (int64_t)i * p.B;   // first key of the diagonal block
  int n_tiles;
  if (p.dense) {
    n_tiles = i * p.subs + subs_diag;      // blocks 0..i-1 in full, then the needed part of block i
  } else {
    if (tid == 0) {
      int n = p.kv_cnt[i];
      if (n > p.max_k) n = p.max_k;
      int w = 0;
      for (int e = 0; e < n; ++e) {
        const int j = p.kv_idx[(int64_t)i * p.max_k + e];
        if (j < 0 || j > i) continue;                       // padding, or not causal: skipped
        const int lim = (j == i) ? subs_diag : p.subs;
        for (int u = 0; u < lim && w < TILE_CAP; ++u) s_tile[w++] = j * p.B + u * KT;
      }
      s_ntiles = w;
    }
    __syncthreads();
    n_tiles = s_ntiles;
  }
  n_tiles = __builtin_amdgcn_readfirstlane(n_tiles);
  auto tile_key0 = [&](int t) -> int {       // wavefront-uniform
    return p.dense ? t * KT : __builtin_amdgcn_readfirstlane(s_tile[t]);
  };

  // ---- fill the ring: the copies run NS-1 tiles ahead of the compute ----
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < n_tiles) issue_tile(tile_key0(s), s);

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

  // Per-lane byte offsets of the swizzled LDS reads inside a stage, computed once: the XOR cannot
  // be folded into an instruction's immediate offset, the row steps (32 rows of K, 16 and 8 rows of V)
  // can.
  uint32_t k_off[NC];                 // K fragment of d-step c, row ln
  {
    const int sw = swz<D>(ln);        // rows 32rt + ln share their low bits with ln
#pragma unroll
    for (int c = 0; c < NC; ++c) k_off[c] = ln * ROWB + (((2 * c + hh) ^ sw) << 4);
  }
  uint32_t v_off0[ND], v_off1[ND];    // the two transposing reads of d tile dt, 16-key step 0
  {
    const int r4 = 4 * hh + ((lane & 15) >> 2);              // row of the first read inside a 16-key step
    const int x = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1); // chunk inside the 32-wide d tile
#pragma unroll
    for (int dt = 0; dt < ND; ++dt) {
      v_off0[dt] = TILEB + r4 * ROWB + (((4 * dt + x) ^ swz<D>(r4)) << 4) + 8 * (lane & 1);
      v_off1[dt] = TILEB + (r4 + 8) * ROWB + (((4 * dt + x) ^ swz<D>(r4 + 8)) << 4) + 8 * (lane & 1);
    }
  }

  // Q fragments and the first tiles must have arrived before the loop; waiting here, once, also tells
  // the compiler that none of its own loads is outstanding inside the loop, so that it does not add
  // full vmcnt(0) waits there (they would drain the asynchronous copies as well).
  wait_vmcnt<0>();

  for (int t = 0; t < n_tiles; ++t) {
    // tile t has landed once at most the younger tiles' copies are outstanding
    const int younger = n_tiles - 1 - t < NS - 2 ? n_tiles - 1 - t : NS - 2;
    if (younger >= 2 && NS > 3) wait_vmcnt<(NS > 3 ? 2 : 0) * LPT>();
    else if (younger == 1 && NS > 2) wait_vmcnt<(NS > 2 ? 1 : 0) * LPT>();
    else wait_vmcnt<0>();
    __syncthreads();   // every wavefront's share is in LDS; everybody is done with the stage refilled below
    if (t + NS - 1 < n_tiles) issue_tile(tile_key0(t + NS - 1), (t + NS - 1) % NS);

    const int key0 = tile_key0(t);
    const bool diag = key0 >= blk0;
    const int key_in_blk = key0 - (int)blk0;
    // tiles of the diagonal block that start after this wavefront's last query are fully masked
    if (active && !(diag && key_in_blk > q_in_blk + QW - 1)) {
      const unsigned char* Sb = smem + (t % NS) * STAGEB;

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
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Sb + k_off[c] + rt * (32 * ROWB));
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
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Sb + v_off0[dt] + kk * (16 * ROWB)));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Sb + v_off1[dt] + kk * (16 * ROWB)));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
            O[dt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ct], O[dt][ct], 0, 0, 0);
        }
      }
    }

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
  if (!p.dense && (int64_t)a.max_k * p.subs > TILE_CAP) return POWATTN_UNSUPPORTED;
  if (a.seq_len > 0x7fffffffLL - 1024) return POWATTN_UNSUPPORTED;   // key positions are kept in 32 bits
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
