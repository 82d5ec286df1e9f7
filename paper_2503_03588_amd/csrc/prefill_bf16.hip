// bf16 prefill on the gfx950 matrix cores: Equation 1 (Section 3.1) over the
// key blocks listed for each query block (Algorithm 1 lifted to blocks), as a
// flash-style online softmax with fp32 accumulation.
//
// Decomposition.  A workgroup owns one (batch, KV head, query block) and up to
// NW "tasks"; a task is one query head of the GQA group x 32 consecutive query
// tokens, and belongs to one wavefront.  All wavefronts of the workgroup share
// the K/V tiles staged in LDS, which is what lifts the arithmetic intensity: a
// 64-key tile is read from HBM/L2 once per workgroup and used by every head of
// the group.
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
// Software pipeline.  On this chip matrix and vector instructions overlap well
// only when they are interleaved in one wavefront's instruction stream; two
// wavefronts of a SIMD that alternate between a matrix phase and a vector phase
// mostly wait for each other.  The tile loop is therefore skewed: iteration t
// issues the 16 matrix instructions of S(t+1) next to the exponentials of the
// second half of S(t), and the 16 matrix instructions of O += P(t) V(t) next to
// the row maximum of S(t+1) and the exponentials of its first half.  The whole
// iteration is one basic block (the causal mask is a template variant, the
// rescaling of O a rare branch at its end) and scheduling groups spell out the
// interleaving.
//
// Memory pipeline.  K/V tiles travel global -> LDS asynchronously
// (global_load_lds_dwordx4, no registers in between) into a ring of NS stages;
// a wavefront waits on its own loads with s_waitcnt vmcnt(n) and one barrier
// per tile makes the stage visible and frees the oldest one.  The asynchronous
// copy cannot pad rows, so bank conflicts are avoided by a XOR swizzle of the
// 16-byte chunk index with the row index, applied on the global-address side.
#include <math.h>
#include <stdlib.h>
#include <type_traits>
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64;          // keys per staged tile
constexpr int QW = 32;          // query tokens per wavefront
constexpr float RESCALE_TAU = 8.0f;   // running max is only raised when exceeded by 2^8 (see softmax below)

struct bf16_params {
  const __bf16* q; const __bf16* k; const __bf16* v; __bf16* o; float* lse;
  const int32_t* kv_cnt; const int32_t* kv_idx;
  int32_t max_k, nb, B, hq, hkv, G, dense;
  int32_t subs;      // 64-key tiles per block
  int32_t tasks;     // G * B / 32
  int32_t chunks;    // workgroups per (batch, kv head, query block)
  int32_t per_xcd;   // workgroups per XCD partition
  int64_t total_wg;
  int64_t N;
  float c2;          // softmax scale * log2(e)
};

// The work of one query block is a sequence of 64-key tiles: the tiles of the listed blocks before
// the diagonal one in list order, then the tiles of the diagonal block (the order of a sum is free,
// and with the causally masked tiles last a wavefront simply stops after the last tile it needs).
// For a block list the sequence is written once, as the first key of every tile, into a table in
// LDS (a lookup is then an LDS read made wavefront-uniform with v_readfirstlane); for the dense list
// it is implicit.  Keeping global memory out of the tile loop matters: a vector load there would
// have to be waited for together with every asynchronous tile copy in flight.
constexpr int TILE_CAP = 4096;   // tiles per query block with an explicit list (16 KB of LDS)

// Asynchronous 16-byte-per-lane copy global -> LDS: lane l's data lands at lds_off + 16*l.
// Written as inline assembly on purpose: the compiler then does not pair every later LDS read
// with a full vmcnt(0) wait, and the waits are placed by hand (wait_vmcnt below).  M0 carries
// the LDS offset; nothing else in this kernel uses M0.
__device__ __forceinline__ void async_copy16(const void* sbase, uint32_t voff, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_off) : "memory");
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

template <int D, int NW, int NS>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void pa_prefill_bf16_kernel(bf16_params p) {
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
  static_assert(NS == 4 && (NS - 1) * LPT < 64, "outstanding copies must fit the vmcnt counter");

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

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, and the compiler knows it
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

  // ---- asynchronous tile copy: this wavefront's share of the tile starting at key0 into a ring stage ----
  // The tile's base address is scalar; a lane adds the byte offset of its row and (swizzled) chunk.
  const int cp_row = lane / CPR, cp_chunk = lane % CPR;
  uint32_t cp_cb[IPW];                                 // swizzled chunk, in bytes, of copy instruction x
#pragma unroll
  for (int x = 0; x < IPW; ++x) cp_cb[x] = (uint32_t)((cp_chunk ^ swz<D>(RPI * (wave * IPW + x) + cp_row)) << 4);
  auto issue_tile = [&](int key0, int stage) {
    // ragged tail: rows beyond the sequence repeat its last row (they are masked, but must be finite)
    const int last = (int)p.N - 1;
    const int k0 = key0 < last ? key0 : last;
    const int lim = last - k0;
    const __bf16* kt = kbase + (int64_t)k0 * D;
    const __bf16* vt = vbase + (int64_t)k0 * D;
#pragma unroll
    for (int x = 0; x < IPW; ++x) {
      const int inst = wave * IPW + x;                 // rows RPI*inst .. +RPI-1 of the tile
      int row = RPI * inst + cp_row;
      row = row < lim ? row : lim;
      const uint32_t voff = (uint32_t)row * ROWB + cp_cb[x];
      const uint32_t dst = lds0 + stage * STAGEB + inst * 1024;
      async_copy16(kt, voff, __builtin_amdgcn_readfirstlane(dst));
      async_copy16(vt, voff, __builtin_amdgcn_readfirstlane(dst + TILEB));
    }
  };

  // ---- Q^T fragments: lane = query column, 8 consecutive d per 16-wide step ----
  bf16x8 qf[NC];
  {
    const __bf16* qbase = p.q + (((int64_t)b * p.hq + h) * p.N) * D;
    const int64_t tok = q0 + ln;
    const bool ok = active && tok < p.N;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[c] = ok ? *reinterpret_cast<const bf16x8*>(qbase + tok * D + 16 * c + 8 * hh) : z;
    }
  }

  // ---- the tile sequence ----
  __shared__ int s_tile[TILE_CAP];     // first key of tile t (explicit lists only)
  __shared__ int s_cnt[2];             // tiles in total, tiles before the diagonal block
  int n_tiles, n_before;
  if (p.dense) {
    n_before = i * p.subs;                 // blocks 0..i-1 in full, then the needed part of block i
    n_tiles = n_before + subs_diag;
  } else {
    if (wave == 0) {
      // the first wavefront reads the row of the list, 64 entries at a time, and writes the tiles of the
      // blocks before the diagonal one in list order (ranks by a prefix count over the lanes)
      int n = p.kv_cnt[i];
      if (n > p.max_k) n = p.max_k;
      n = __builtin_amdgcn_readfirstlane(n);
      int blocks = 0;
      bool has_diag = false;
      for (int base = 0; base < n; base += 64) {
        const int e = base + lane;
        const int j = e < n ? p.kv_idx[(int64_t)i * p.max_k + e] : -1;
        const bool valid = j >= 0 && j < i;                  // not padding, causal, not the diagonal block (below)
        const uint64_t vm = __builtin_amdgcn_ballot_w64(valid);
        has_diag = has_diag || __builtin_amdgcn_ballot_w64(j == i) != 0;
        const int rank = blocks + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vm, 0));
        if (valid)
          for (int u = 0; u < p.subs; ++u) s_tile[rank * p.subs + u] = j * p.B + u * KT;
        blocks += __builtin_popcountll(vm);
      }
      int w = blocks * p.subs;
      if (lane == 0) s_cnt[1] = w;
      if (has_diag) {
        if (lane < subs_diag) s_tile[w + lane] = i * p.B + lane * KT;
        w += subs_diag;
      }
      if (lane == 0) s_cnt[0] = w;
    }
    __syncthreads();
    n_tiles = s_cnt[0];
    n_before = s_cnt[1];
  }
  n_tiles = __builtin_amdgcn_readfirstlane(n_tiles);
  n_before = __builtin_amdgcn_readfirstlane(n_before);
  auto tile_key0 = [&](int t) -> int {       // wavefront-uniform
    return p.dense ? t * KT : __builtin_amdgcn_readfirstlane(s_tile[t]);
  };
  // tiles this wavefront computes: everything before the diagonal block, then the diagonal tiles
  // that start at or before its last query (later ones are fully masked for it)
  int n_my = 0;
  if (active) {
    int dg = n_tiles - n_before;
    const int need = (q_in_blk + QW - 1) / KT + 1;
    if (dg > need) dg = need;
    n_my = n_before + dg;
  }
  n_my = __builtin_amdgcn_readfirstlane(n_my);

  // ---- fill the ring: the copies run NS-1 tiles ahead ----
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < n_tiles) issue_tile(tile_key0(s), s);

  f32x16 O[ND];
#pragma unroll
  for (int dt = 0; dt < ND; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;

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

  // ---- pieces of the pipeline ----
  constexpr int NSLOT = 2 * NC + 4 * ND;   // matrix instructions per tile: 32 at head_dim 128, 16 at 64
  constexpr int VPS = 32 / NSLOT;          // the vector work of a tile is cut into 32 portions: portions per matrix instruction
  constexpr int PF = 3;                    // LDS reads run this many matrix instructions ahead of their use
  const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  // causal mask inside the diagonal block; element rg (0..31) of a tile is key 32(rg/16) + 8((rg%16)/4) + 4hh + rg%4
  auto mask = [&](f32x16 (&S)[2], int key_in_blk) {
    const int qpos = q_in_blk + ln;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kpos = key_in_blk + 32 * rt + 8 * (r >> 2) + 4 * hh + (r & 3);
        if (kpos > qpos) S[rt][r] = -INFINITY;
      }
  };
  // maximum over both halves of the wavefront (lane l and lane l+32 hold the same query column)
  auto both_halves_max = [](float x) -> float {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, r[0]), __builtin_bit_cast(float, r[1]));
  };
  // p = exp2(s*c2 - m) of element rg
  auto pexp = [&](const f32x16 (&S)[2], int rg, float m_ref) -> float {
    return __builtin_amdgcn_exp2f(fmaf(S[rg >> 4][rg & 15], p.c2, -m_ref));
  };
  auto pack2 = [](float x, float y) -> uint32_t {   // two fp32 -> two bf16 (round to nearest even) in one register
    const f32x2 v = {x, y};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  };
  // A operand of matrix instruction `slot` of a tile step: K rows (slots 0..2NC-1: d-step c = slot/2, key half
  // rt = slot%2), then V^T (16-key step kk, d tile dt) through two transposing reads
  auto load_frag = [&](int slot, const uint32_t (&ka)[NC], const uint32_t (&va0)[ND], const uint32_t (&va1)[ND]) -> bf16x8 {
    if (slot < 2 * NC)
      return *reinterpret_cast<const lds_bf16x8*>((uintptr_t)(ka[slot >> 1] + (slot & 1) * (32 * ROWB)));
    const int kk = (slot - 2 * NC) / ND, dt = (slot - 2 * NC) % ND;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(va0[dt] + kk * (16 * ROWB)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(va1[dt] + kk * (16 * ROWB)));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto stage_addresses = [&](int kstage, int vstage, uint32_t (&ka)[NC], uint32_t (&va0)[ND], uint32_t (&va1)[ND]) {
#pragma unroll
    for (int c = 0; c < NC; ++c) ka[c] = lds0 + kstage * STAGEB + k_off[c];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt) {
      va0[dt] = lds0 + vstage * STAGEB + v_off0[dt];
      va1[dt] = lds0 + vstage * STAGEB + v_off1[dt];
    }
  };

  // Q fragments and the first tiles must have arrived before the loop; waiting here, once, also tells
  // the compiler that none of its own loads is outstanding inside the loop, so that it does not add
  // full vmcnt(0) waits there (they would drain the asynchronous copies as well).
  wait_vmcnt<0>();
  __syncthreads();

  // ---- pipeline state: scores of the current tile, the probabilities of its first 16-key step, running (m, l) ----
  // The reference point m of the exponentials need not be the exact running maximum: any m gives the
  // same o and lse as long as exp2(s - m) stays in range.  It is raised only when a score exceeds it by
  // more than RESCALE_TAU (p <= 2^tau), which makes the rescaling of O (64 multiplies per lane) a
  // rare, wavefront-uniform branch instead of a per-tile cost.
  f32x16 Sc[2];
  u32x4 P0;
  float m_run = -INFINITY, l_run = 0.f;
  if (n_my > 0) {
    uint32_t ka[NC], va0[ND], va1[ND];
    stage_addresses(0, 0, ka, va0, va1);
#pragma unroll
    for (int sl2 = 0; sl2 < 2 * NC; ++sl2)
      Sc[sl2 & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_frag(sl2, ka, va0, va1), qf[sl2 >> 1],
                                                            sl2 < 2 ? zero16 : Sc[sl2 & 1], 0, 0, 0);
    if (n_before == 0) mask(Sc, 0);        // the first tile is already a diagonal one
    float mx = Sc[0][0];
#pragma unroll
    for (int rg = 1; rg < 32; ++rg) mx = fmaxf(mx, Sc[rg >> 4][rg & 15]);
    m_run = both_halves_max(mx) * p.c2;
    float pe[8];
#pragma unroll
    for (int rg = 0; rg < 8; ++rg) { pe[rg] = pexp(Sc, rg, m_run); l_run += pe[rg]; }
#pragma unroll
    for (int j = 0; j < 4; ++j) P0[j] = pack2(pe[2 * j], pe[2 * j + 1]);
  }

  // Start of every iteration: tile t+1 has landed once at most tile t+2's copies are outstanding
  // (tiles 0..NS-2 landed above); the barrier makes every wavefront's share of it visible and tells
  // that everybody is done with tile t-1, whose stage is refilled.
  auto top = [&](int t) {
    if (t + 2 < n_tiles) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
    __syncthreads();
    if (t + NS - 1 < n_tiles) issue_tile(tile_key0(t + NS - 1), (t + NS - 1) % NS);
  };

  // One step of the skewed loop.  Matrix instructions: the 2NC of S(t+1) = K(t+1) Q^T, then the 4ND of
  // O += V(t)^T P(t)^T.  Vector work, cut into 32 portions that are spread evenly over them: the
  // exponentials of elements 8..31 of S(t) (element rg feeds 16-key step rg/8 of the second product, so
  // each is ready before its step), then the column maximum of S(t+1) and the new reference point, then the
  // exponentials of elements 0..7 of S(t+1).  The source order IS the schedule: a scheduling barrier after
  // every matrix instruction keeps the compiler from regrouping the stream into a matrix phase and a
  // vector phase.  `masked` selects the variant that applies the causal mask to S(t+1).
  auto step = [&](int t, auto masked) {
    constexpr bool MASKED = decltype(masked)::value;
    uint32_t ka[NC], va0[ND], va1[ND];
    stage_addresses((t + 1) % NS, t % NS, ka, va0, va1);
    top(t);
    bf16x8 fr[NSLOT];
    f32x16 Sn[2];
    u32x4 Pk[4], Pn;
    Pk[0] = P0;
    float pe[32], pn[8];
    float rs = 0.f, rs_n = 0.f, mx = 0.f, m_new = 0.f, alpha = 1.f;
    bool raise = false;
#pragma unroll
    for (int s0 = 0; s0 < PF; ++s0) fr[s0] = load_frag(s0, ka, va0, va1);
#pragma unroll
    for (int sl2 = 0; sl2 < NSLOT; ++sl2) {
      if (sl2 + PF < NSLOT) fr[sl2 + PF] = load_frag(sl2 + PF, ka, va0, va1);
      // ---- vector portions of this slot ----
#pragma unroll
      for (int vs = sl2 * VPS; vs < (sl2 + 1) * VPS; ++vs) {
        if (vs < 18) {
#pragma unroll
          for (int e = (4 * vs) / 3; e < (4 * (vs + 1)) / 3; ++e) {
            const int rg = 8 + e;
            pe[rg] = pexp(Sc, rg, m_run);
            rs += pe[rg];
            if (rg & 1) Pk[rg >> 3][(rg & 7) >> 1] = pack2(pe[rg - 1], pe[rg]);
          }
          if (MASKED && vs == 17) mask(Sn, (t + 1 - n_before) * KT);
        } else if (vs < 21) {
          constexpr int lo[3] = {0, 11, 22}, hi[3] = {11, 22, 32};
          if (vs == 18) mx = Sn[0][0];
#pragma unroll
          for (int rg = lo[vs - 18]; rg < hi[vs - 18]; ++rg) mx = fmaxf(mx, Sn[rg >> 4][rg & 15]);
        } else if (vs == 21) {
          mx = both_halves_max(mx) * p.c2;
          raise = mx > m_run + RESCALE_TAU;
        } else if (vs == 22) {
          m_new = raise ? mx : m_run;
          alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        } else if (vs < 29) {
#pragma unroll
          for (int rg = (4 * (vs - 23)) / 3; rg < (4 * (vs - 22)) / 3; ++rg) {
            pn[rg] = pexp(Sn, rg, m_new);
            rs_n += pn[rg];
            if (rg & 1) Pn[rg >> 1] = pack2(pn[rg - 1], pn[rg]);
          }
          // results that are only used by the next step: keep their computation here, in the shadow of
          // the matrix instructions, instead of letting it sink to the end of the iteration
          if (vs == 28) asm volatile("" ::"v"(Pn), "v"(rs_n));
        }
      }
      // ---- the matrix instruction ----
      if (sl2 < 2 * NC) {
        Sn[sl2 & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[sl2], qf[sl2 >> 1], sl2 < 2 ? zero16 : Sn[sl2 & 1], 0, 0, 0);
      } else {
        const int kk = (sl2 - 2 * NC) / ND, dt = (sl2 - 2 * NC) % ND;
        O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[sl2], __builtin_bit_cast(bf16x8, Pk[kk]), O[dt], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += rs;
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
    }
    l_run += rs_n;
    m_run = m_new;
    Sc[0] = Sn[0]; Sc[1] = Sn[1];
    P0 = Pn;
  };
  // Only the last tile a wavefront computes needs the mask: the diagonal tiles before it lie entirely
  // below its first query.  Every wavefront runs n_tiles iterations (the barriers are shared): plain
  // steps, masked steps, its last tile, then idle iterations that only copy.
  int t_mask = n_before + q_in_blk / KT;
  if (t_mask > n_my) t_mask = n_my;
  const int T1 = t_mask > 1 ? t_mask - 1 : 0, T2 = n_my > 1 ? n_my - 1 : 0;
  int t = 0;
  for (; t < T1; ++t) step(t, std::false_type{});
  for (; t < T2; ++t) step(t, std::true_type{});
  for (; t < n_my; ++t) {
    // ---- last tile of this wavefront: the rest of P(t), O += P(t) V(t) ----
    uint32_t ka[NC], va0[ND], va1[ND];
    stage_addresses(t % NS, t % NS, ka, va0, va1);
    top(t);
    u32x4 Pk[4];
    Pk[0] = P0;
    float pe[32];
#pragma unroll
    for (int rg = 8; rg < 32; ++rg) {
      pe[rg] = pexp(Sc, rg, m_run);
      l_run += pe[rg];
      if (rg & 1) Pk[rg >> 3][(rg & 7) >> 1] = pack2(pe[rg - 1], pe[rg]);
    }
#pragma unroll
    for (int sl2 = 2 * NC; sl2 < NSLOT; ++sl2) {
      const int kk = (sl2 - 2 * NC) / ND, dt = (sl2 - 2 * NC) % ND;
      O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_frag(sl2, ka, va0, va1), __builtin_bit_cast(bf16x8, Pk[kk]), O[dt], 0, 0, 0);
    }
  }
  for (; t < n_tiles; ++t) top(t);

  // ---- epilogue: register r of tile dt is d = 32dt + 8(r/4) + 4hh + r%4 ----
  {
    const float ltot = l_run + __shfl_xor(l_run, 32);
    const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
    const int64_t tok = q0 + ln;
    if (active && tok < p.N) {
      __bf16* orow = p.o + (((int64_t)b * p.hq + h) * p.N + tok) * D;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(O[dt][4 * g4 + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g4 + 4 * hh) = w;
        }
      if (p.lse && hh == 0)
        p.lse[((int64_t)b * p.hq + h) * p.N + tok] = (m_run + log2f(ltot)) * 0.69314718055994530942f;
    }
  }
}

template <int D, int NW, int NS>
int launch(const bf16_params& p, hipStream_t stream) {
  constexpr size_t lds = (size_t)NS * 2 * KT * 2 * D;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pa_prefill_bf16_kernel<D, NW, NS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return pa_note_hip(e);
    attr_done = true;
  }
  const int64_t grid = (int64_t)p.per_xcd * 8;
  hipLaunchKernelGGL((pa_prefill_bf16_kernel<D, NW, NS>), dim3((uint32_t)grid), dim3(64 * NW), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}

}  // namespace

int pa_launch_prefill_bf16(const pa_prefill_args& a) {
  bf16_params p;
  p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.o = (__bf16*)a.o; p.lse = a.lse;
  p.kv_cnt = a.kv_cnt; p.kv_idx = a.kv_idx; p.max_k = a.max_k; p.nb = a.nb; p.B = a.pat.block;
  p.hq = a.hq; p.hkv = a.hkv; p.G = a.hq / a.hkv; p.dense = (a.pat.flags & POWATTN_DENSE) ? 1 : 0;
  p.subs = p.B / KT;
  if (!p.dense && (int64_t)a.max_k * p.subs > TILE_CAP) return POWATTN_UNSUPPORTED;
  if (a.seq_len > 0x7fffffffLL - 1024) return POWATTN_UNSUPPORTED;   // key positions are kept in 32 bits
  p.N = a.seq_len;
  p.c2 = a.scale * 1.44269504088896340736f;
  const int64_t tasks = (int64_t)p.G * p.B / QW;
  if (tasks > (1 << 20)) return POWATTN_UNSUPPORTED;
  p.tasks = (int32_t)tasks;
  const int nw = p.tasks > 4 ? 8 : 4;
  p.chunks = (p.tasks + nw - 1) / nw;
  p.total_wg = (int64_t)a.batch * a.hkv * a.nb * p.chunks;
  const int64_t per_xcd = (p.total_wg + 7) / 8;
  if (per_xcd * 8 > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  p.per_xcd = (int32_t)per_xcd;

  // ring of 4 stages: 128 KB of LDS at head_dim 128, 64 KB at head_dim 64
  if (a.head_dim == 128) return nw == 8 ? launch<128, 8, 4>(p, a.stream) : launch<128, 4, 4>(p, a.stream);
  return nw == 8 ? launch<64, 8, 4>(p, a.stream) : launch<64, 4, 4>(p, a.stream);
}

