// Gradients of Equation 1 (Section 3.1) under the block pattern of Algorithm 1, bf16 inputs, fp32 accumulation.
// The paper trains with the sparse pattern in place (Section 4.1), which needs dQ, dK and dV of
//   O = softmax(mask(scale Q K^T)) V.
// With P the softmax (recomputed from the saved log-sum-exp), dP = dO V^T, Delta_i = sum_d dO_id O_id and
// dS = P * (dP - Delta):   dQ = scale dS K,   dK = scale dS^T Q,   dV = P^T dO.
//
// Two kernels:
//   dq    : a workgroup per (batch, KV head, query block, group of query-head slices) walks the row's key blocks
//           (the lists powattn_mask_build writes), as the forward pass does; wavefront = 32 queries of one head,
//           lane = one query.  S^T = K Q^T and dP^T = V dO^T share the K/V tiles in LDS; dQ^T += K^T dS^T.
//           It also forms Delta = rowsum(dO * O) of its rows (dO is in its registers anyway) and leaves it, with
//           the log-sum-exp in base-2 units, in the workspace for the kernel below.
//   dkv   : a workgroup per (batch, KV head, key block) walks the COLUMN of the block mask: the query blocks
//           j .. j+W-1 and j + 2^k (closed form), all of them for a sink block; wavefront = 32 keys, lane = one key.
//           Q and dO tiles of 64 queries go through LDS; dV^T += dO^T P, dK^T += Q^T dS.  A sink block's column is
//           as long as the sequence: it is cut into parts that add into an fp32 buffer, converted at the end.
//           At 128 keys per block the two halves of this work sit on different wavefronts (dkv_split below).
// Both products of a pair reuse the forward kernel's operand trick: in the transposed form the accumulator layout
// of the first product is the B-operand layout of the second (the permutation of the contraction index inside a
// 16-step is applied to both operands).  Tiles use the forward kernel's LDS layout (chunk-major kilobytes, padded),
// copied asynchronously global -> LDS, two stages, one barrier per tile.  Not yet scheduled by hand.
#include <math.h>
#include <type_traits>
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;

constexpr int KT = 64;            // rows per staged tile
constexpr int TILE_CAP = 2048;    // tiles per query block in the dq kernel
constexpr int PART = 16;          // query blocks per part of a sink block's column
constexpr int PFD = 2;            // matrix instructions per group of LDS fragment reads
constexpr int NSTG = 2;           // LDS stages of the tile stream: copies run NSTG-1 tiles ahead of the products (3 was
                                  // slower: the extra LDS halves the workgroups per compute unit at block 64)
constexpr float LOG2E = 1.44269504088896340736f;
constexpr int dq_stages(int) { return 2; }   // LDS stages of the dQ kernel's tile stream (see there)

struct bwd_params {
  const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* o; const __bf16* dout; const float* lse;
  __bf16* dq; __bf16* dk; __bf16* dv;
  float* delta;          // [batch, hq, N]
  float* lse2;           // [batch, hq, N]: the log-sum-exp in base-2 units (lse * log2 e)
  float* dk_sink;        // [batch, hkv, sink_rows, D] fp32 sums of the sink blocks' parts
  float* dv_sink;
  const int32_t* kv_cnt; const int32_t* kv_idx;
  int32_t max_k, nb, B, W, S; uint32_t flags;
  int32_t hq, hkv, G, subs, tasks, chunks;
  int32_t sink_blocks;   // min(S, nb) (0 when the column of no block is cut)
  int32_t max_parts;     // parts of the longest column
  int64_t N;
  float scale, c2;
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void async_copy16(const void* sbase, uint32_t voff, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_off) : "memory", "m0");
}
// the same with the LDS offset given as a scalar base plus a constant
template <int OFF>
__device__ __forceinline__ void async_copy16_at(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base), "n"(OFF) : "memory", "scc", "m0");
}
// one dword per lane: lane l's value lands at lds_off + 4*l
__device__ __forceinline__ void async_copy4(const void* addr, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(addr), "s"(lds_off) : "memory", "m0");
}
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* ptr) {
  const uint64_t u = (uint64_t)(uintptr_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return (const T*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t pack2(float x, float y) {
  const f32x2 v = {x, y};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Geometry of a staged tile of 64 rows x D bf16 (the forward kernel's layout).
template <int D>
struct tile_geo {
  static constexpr int ROWB = 2 * D;
  static constexpr int CPR = D / 8;
  static constexpr int RPI = 64 / CPR;          // rows per wavefront-wide copy instruction
  static constexpr int IPT = KT / RPI;          // copy instructions per tile
  static constexpr int SRB = 1024 + 16 * RPI;   // LDS distance between consecutive copy instructions' kilobytes
  static constexpr int TILEB = IPT * SRB;
  static constexpr int NC = D / 16;             // 16-wide steps of the head dimension
  static constexpr int ND = D / 32;             // 32-row tiles of a transposed accumulator
  static constexpr int K_C = 32 * RPI, K_RT = (32 / RPI) * SRB;
  static constexpr int V_KK = (16 / RPI) * SRB, V_DT = 4 * RPI * 16, V_HI = (8 / RPI) * SRB;
};

// copy instruction X of a wavefront's share of a tile, and the ones after it (instruction number wave + X * NWV)
template <int D, int NWV, int X>
__device__ __forceinline__ void copy_tile_unrolled(const __bf16* sb, int row0w, int lim, uint32_t chunk_off, uint32_t wdst) {
  using G = tile_geo<D>;
  if constexpr (X < G::IPT / NWV) {
    int row = row0w + G::RPI * NWV * X;
    row = row < lim ? row : lim;
    async_copy16_at<X * NWV * G::SRB>(sb, (uint32_t)row * G::ROWB + chunk_off, wdst);
    copy_tile_unrolled<D, NWV, X + 1>(sb, row0w, lim, chunk_off, wdst);
  }
}
// Copies rows row0 .. row0+63 of a row-major [rows, D] array (rows beyond `last_row` repeat it) into the LDS tile
// at `dst`; the NWV wavefronts of the workgroup share the tile's copy instructions.
template <int D, int NWV>
__device__ __forceinline__ void copy_tile(const __bf16* base, int64_t row0, int64_t last_row, uint32_t dst, int wave, int lane) {
  using G = tile_geo<D>;
  const int cp_row = lane % G::RPI, cp_chunk = lane / G::RPI;
  int64_t r0 = row0 < last_row ? row0 : last_row;
  const int lim = (int)(last_row - r0);
  const __bf16* sb = uniform_ptr(base + r0 * D);
  if constexpr (G::IPT % NWV == 0) {
    // a known number of copy instructions per wavefront: straight-line code, LDS offsets as constants
    const uint32_t wdst = __builtin_amdgcn_readfirstlane(dst + wave * G::SRB);
    const int row0w = G::RPI * wave + cp_row;
    copy_tile_unrolled<D, NWV, 0>(sb, row0w, lim, (uint32_t)(cp_chunk << 4), wdst);
  } else {
    for (int inst = wave; inst < G::IPT; inst += NWV) {
      int row = G::RPI * inst + cp_row;
      row = row < lim ? row : lim;
      const uint32_t voff = (uint32_t)row * G::ROWB + (cp_chunk << 4);
      async_copy16(sb, voff, __builtin_amdgcn_readfirstlane(dst + inst * G::SRB));
    }
  }
}
// A operand "rows of the tile": rows 32rt + (lane%32), elements 16c + 8(lane/32) .. +7
template <int D>
__device__ __forceinline__ bf16x8 row_frag(uint32_t tile, int c, int rt, int lane) {
  using G = tile_geo<D>;
  const int ln = lane & 31, hh = lane >> 5;
  const uint32_t a = tile + (ln / G::RPI) * G::SRB + ((hh * G::RPI + ln % G::RPI) << 4) + c * G::K_C + rt * G::K_RT;
  return *reinterpret_cast<const lds_bf16x8*>((uintptr_t)a);
}
// A operand "transposed tile": row = element 32dt + lane%32 of the head dimension, contraction over the tile's rows
// 16kk .. 16kk+15 in the order {0..3, 8..11} + 4(lane/32), {4..7, 12..15} for the other half-wave
template <int D>
__device__ __forceinline__ bf16x8 tr_frag(uint32_t tile, int kk, int dt, int lane) {
  using G = tile_geo<D>;
  const int hh = lane >> 5;
  const int r4 = 4 * hh + ((lane & 15) >> 2);
  const int x = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
  const uint32_t a = tile + (r4 / G::RPI) * G::SRB + ((x * G::RPI + r4 % G::RPI) << 4) + 8 * (lane & 1) + kk * G::V_KK + dt * G::V_DT;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)a);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(a + G::V_HI));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// B operand "rows held in registers": lane = row (lane%32), elements 16c + 8(lane/32) .. +7; zero when !ok
template <int D>
__device__ __forceinline__ void reg_rows(const __bf16* row, bool ok, int lane, bf16x8 (&f)[D / 16]) {
  const int hh = lane >> 5;
#pragma unroll
  for (int c = 0; c < D / 16; ++c) {
    const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    f[c] = ok ? *reinterpret_cast<const bf16x8*>(row + 16 * c + 8 * hh) : z;
  }
}
// N matrix instructions whose A operands come from LDS, software-pipelined with scheduling barriers (left alone,
// the compiler reads each fragment right before its use into the same registers, and a wavefront that is alone on
// its SIMD waits out every LDS latency).
template <int N, int GRP, class LoadF, class MmaF>
__device__ __forceinline__ void pipelined_mfma(LoadF load, MmaF mma) {
  // groups of GRP instructions: the reads of the next group go out together before the current group's matrix
  // instructions, so that one wait serves a whole group
  static_assert(N % GRP == 0, "instructions must come in whole groups");
  bf16x8 fr[N];
#pragma unroll
  for (int m = 0; m < GRP; ++m) fr[m] = load(m);
#pragma unroll
  for (int g = 0; g < N / GRP; ++g) {
    if (g + 1 < N / GRP) {
#pragma unroll
      for (int j = 0; j < GRP; ++j) fr[(g + 1) * GRP + j] = load((g + 1) * GRP + j);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < GRP; ++j) mma(g * GRP + j, fr[g * GRP + j]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Element rg (0..15) of a 32x32 accumulator is row 8(rg/4) + 4(lane/32) + rg%4, column lane%32.
__device__ __forceinline__ int acc_row(int rg, int hh) { return 8 * (rg >> 2) + 4 * hh + (rg & 3); }

__global__ __launch_bounds__(256) void pa_bwd_zero_kernel(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// ---------------------------------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------------------------------
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void pa_bwd_dq_kernel(bwd_params p) {
  using G = tile_geo<D>;
  constexpr int NC = G::NC, ND = G::ND;
  constexpr int STAGEB = 2 * G::TILEB;           // K tile then V tile
  // LDS stages of the tile stream: the copies run NST-1 tiles ahead of the products.  Two: four stages for the
  // workgroups of eight wavefronts (which have their compute unit to themselves anyway) were measured 5 % slower
  // at the 128K workload, three halve the workgroups per compute unit at blocks of 64 keys.
  constexpr int NST = dq_stages(NW);
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  __shared__ int s_tile[TILE_CAP];
  __shared__ int s_ntiles;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, hh = lane >> 5;
  const int slices = p.B / 32;

  // item: ((b*hkv + kvh)*nb + i)*chunks + chunk
  int64_t L = blockIdx.x;
  const int chunk = (int)(L % p.chunks); L /= p.chunks;
  const int i = (int)(L % p.nb); L /= p.nb;
  const int kvh = (int)(L % p.hkv);
  const int b = (int)(L / p.hkv);

  // ---- the row's tiles: every 64-key tile of every listed block up to the diagonal one ----
  // The first wavefront reads 64 list entries at a time, one per lane (a single thread walking the list pays a
  // trip to memory per entry, at the start of every workgroup); the rank of a valid entry is a prefix count.
  if (wave == 0) {
    int n = p.kv_cnt[i];
    if (n > p.max_k) n = p.max_k;
    n = __builtin_amdgcn_readfirstlane(n);
    int blocks = 0;
    for (int base = 0; base < n; base += 64) {
      const int e = base + lane;
      const int j = e < n ? p.kv_idx[(int64_t)i * p.max_k + e] : -1;
      const bool valid = j >= 0 && j <= i;
      const uint64_t vm = __builtin_amdgcn_ballot_w64(valid);
      const int rank = blocks + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vm, 0));
      if (valid)
        for (int u = 0; u < p.subs; ++u)
          if (rank * p.subs + u < TILE_CAP) s_tile[rank * p.subs + u] = j * p.B + u * KT;
      blocks += __builtin_popcountll(vm);
    }
    if (lane == 0) s_ntiles = blocks * p.subs < TILE_CAP ? blocks * p.subs : TILE_CAP;
  }
  __syncthreads();
  const int n_tiles = s_ntiles;

  const int task = chunk * NW + wave;
  const bool active = task < p.tasks;
  const int g = active ? task / slices : 0, sl = active ? task % slices : 0;
  const int h = kvh * p.G + g;
  const int64_t tok = (int64_t)i * p.B + sl * 32 + ln;          // this lane's query
  const bool ok = active && tok < p.N;
  const int64_t qrow = ((int64_t)b * p.hq + h) * p.N + (ok ? tok : 0);

  const __bf16* kslab = p.k + ((int64_t)b * p.hkv + kvh) * p.N * D;
  const __bf16* vslab = p.v + ((int64_t)b * p.hkv + kvh) * p.N * D;
  static_assert(G::IPT % NW == 0, "tile copies must divide over the wavefronts");
  constexpr int CPF = 2 * G::IPT / NW;     // copies per wavefront and fill (K and V)
  auto fill = [&](int t) {
    const int key0 = s_tile[t];
    const uint32_t dst = lds0 + (t % NST) * STAGEB;
    copy_tile<D, NW>(kslab, key0, p.N - 1, dst, wave, lane);
    copy_tile<D, NW>(vslab, key0, p.N - 1, dst + G::TILEB, wave, lane);
  };
  // the first tiles are requested before this wavefront's own rows: their copies would queue behind those loads
  for (int s0 = 0; s0 < NST - 1; ++s0)
    if (s0 < n_tiles) fill(s0);

  bf16x8 qf[NC], dof[NC];
  reg_rows<D>(p.q + qrow * D, ok, lane, qf);
  reg_rows<D>(p.dout + qrow * D, ok, lane, dof);
  // Delta = rowsum(dO * O) of this lane's row and its log-sum-exp in base-2 units: formed here, where the row of dO
  // is in registers anyway (the two halves of the wavefront hold the two halves of the row), and left in the
  // workspace for the dK/dV kernel, which follows on the stream.  Every row belongs to exactly one task.
  float lse2 = INFINITY, dl = 0.f;                               // exp2(s - inf) = 0: idle lanes contribute nothing
  {
    bf16x8 of[NC];
    reg_rows<D>(p.o + qrow * D, ok, lane, of);
    float part = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 8; ++e) part = fmaf((float)of[c][e], (float)dof[c][e], part);
    part += __shfl_xor(part, 32);
    if (ok) {
      dl = part;
      lse2 = p.lse[qrow] * LOG2E;
      if (hh == 0) { p.delta[qrow] = dl; p.lse2[qrow] = lse2; }
    }
  }
  const int tok32 = (int)tok, n32 = (int)p.N;                    // positions fit 32 bits (checked by the host)

  f32x16 acc[ND];
#pragma unroll
  for (int dt = 0; dt < ND; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;
  // Tile t has landed when only the fills of tiles t+1 .. t+NST-2 are outstanding (the counter retires in
  // order).  Near the end, where fewer fills follow, wait for all.  (The loads of Q and dO above are younger than
  // the first fills; the compiler waits for them before their first use, which covers everything older.)
  for (int t = 0; t < n_tiles; ++t) {
    if (t + NST - 1 <= n_tiles) wait_vmcnt<(NST - 2) * CPF>(); else wait_vmcnt<0>();
    __syncthreads();                       // tile t has landed for everybody; everybody is done with tile t-1
    if (t + NST - 1 < n_tiles) fill(t + NST - 1);        // into the stage tile t-1 has just left
    const int key0 = s_tile[t];
    // tiles that start beyond this wavefront's last query are masked out entirely for it
    if (!active || (int64_t)key0 > (int64_t)i * p.B + sl * 32 + 31) continue;
    const uint32_t kt = lds0 + (t % NST) * STAGEB, vt = kt + G::TILEB;
    f32x16 S[2], dP[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) { S[rt][r] = 0.f; dP[rt][r] = 0.f; }
    // instruction m: d-step c = m/4, key half rt = (m/2)%2, S (K tile) or dP (V tile) = m%2: four independent chains
    pipelined_mfma<4 * NC, PFD>(
        [&](int m) { return row_frag<D>((m & 1) ? vt : kt, m >> 2, (m >> 1) & 1, lane); },
        [&](int m, bf16x8 a) {
          const int c = m >> 2, rt = (m >> 1) & 1;
          if (m & 1) dP[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dof[c], dP[rt], 0, 0, 0);
          else S[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[c], S[rt], 0, 0, 0);
        });
    // dS^T = P^T * (dP^T - Delta), packed to bf16 in the B-operand order of the next product
    u32x4 ds[4];
    // Only tiles that reach the diagonal or the end of the sequence need the mask (wavefront-uniform test); the
    // others skip the compares and selects.  Idle lanes (query beyond the sequence) carry lse = inf: P = 0.
    auto elements = [&](auto masked) {
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          float x[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            // computed for every element and selected afterwards: a conditional exponential becomes a branch
            const float pr = __builtin_amdgcn_exp2f(fmaf(S[rt][r + e], p.c2, -lse2));
            x[e] = pr * (dP[rt][r + e] - dl);
            if (decltype(masked)::value) {
              const int key = key0 + 32 * rt + acc_row(r + e, hh);
              x[e] = (key <= tok32 && key < n32) ? x[e] : 0.f;
            }
          }
          const int rg = 16 * rt + r;
          ds[rg >> 3][(rg & 7) >> 1] = pack2(x[0], x[1]);
        }
    };
    if ((int64_t)key0 + KT - 1 > (int64_t)i * p.B + sl * 32 || (int64_t)key0 + KT > p.N) elements(std::true_type{});
    else elements(std::false_type{});
    pipelined_mfma<4 * ND, PFD>(
        [&](int m) { return tr_frag<D>(kt, m / ND, m % ND, lane); },
        [&](int m, bf16x8 a) {
          acc[m % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, ds[m / ND]), acc[m % ND], 0, 0, 0);
        });
  }
  wait_vmcnt<0>();

  // element r of tile dt is d = 32dt + 8(r/4) + 4hh + r%4 of this lane's query row: 8-byte pieces
  if (ok) {
    __bf16* out = p.dq + qrow * D;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const u32x2 w = {pack2(acc[dt][4 * r4] * p.scale, acc[dt][4 * r4 + 1] * p.scale),
                         pack2(acc[dt][4 * r4 + 2] * p.scale, acc[dt][4 * r4 + 3] * p.scale)};
        *reinterpret_cast<u32x2*>(out + 32 * dt + 8 * r4 + 4 * hh) = w;
      }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------------------------------------------
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void pa_bwd_dkv_kernel(bwd_params p) {
  using G = tile_geo<D>;
  constexpr int NC = G::NC, ND = G::ND;
  constexpr int STAGEB = 2 * G::TILEB + 512;     // Q tile, dO tile, 64 log-sum-exps, 64 Deltas
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, hh = lane >> 5;
  const int kvh = blockIdx.y, b = blockIdx.z;

  // ---- which key block, which part of its column ----
  int j, part;
  // the parts of the sink blocks' columns come first in the launch: they are the longest workgroups (PART query
  // blocks each against a dozen for an ordinary column), and the last ones to start should be the shortest
  const int n_extra = p.sink_blocks * (p.max_parts - 1);
  if ((int)blockIdx.x >= n_extra) { j = (int)blockIdx.x - n_extra; part = 0; }
  else {
    const int e = (int)blockIdx.x;
    j = e / (p.max_parts - 1);
    part = 1 + e % (p.max_parts - 1);
  }
  const bool whole_column = j < p.sink_blocks;                    // a sink block: every later query block
  const int parts = whole_column ? (p.nb - j + PART - 1) / PART : 1;
  if (part >= parts) return;                                      // uniform over the workgroup
  // entries of the column: query blocks j .. j+n_win-1, then j + 2^k for 2^k >= the window
  const int weff = (p.flags & POWATTN_POWER) ? (p.W > 1 ? p.W : 1) : p.W;
  int n_win, n_ent, first_pow = 1;
  if (whole_column) {
    n_win = p.nb - j - part * PART;
    if (n_win > PART) n_win = PART;
    n_ent = n_win;
  } else {
    n_win = weff < p.nb - j ? weff : p.nb - j;
    n_ent = n_win;
    if (p.flags & POWATTN_POWER) {
      while (first_pow < weff) first_pow <<= 1;
      for (int64_t pw = first_pow; j + pw < p.nb; pw <<= 1) ++n_ent;
    }
  }
  auto entry = [&](int e) -> int {
    if (whole_column) return j + part * PART + e;
    if (e < n_win) return j + e;
    return j + (first_pow << (e - n_win));
  };

  // ---- this lane's key: its K and V rows stay in registers as B operands ----
  const int64_t key = (int64_t)j * p.B + 32 * wave + ln;
  const bool kok = key < p.N;
  const int key32 = (int)key, n32 = (int)p.N;          // positions fit 32 bits (checked by the host)
  const int64_t krow = ((int64_t)b * p.hkv + kvh) * p.N + (kok ? key : 0);
  bf16x8 kf[NC], vf[NC];
  reg_rows<D>(p.k + krow * D, kok, lane, kf);
  reg_rows<D>(p.v + krow * D, kok, lane, vf);

  f32x16 dkt[ND], dvt[ND];
#pragma unroll
  for (int dt = 0; dt < ND; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkt[dt][r] = 0.f; dvt[dt][r] = 0.f; }

  // tile sequence: entry e, query head g of the group, 64-query piece u of the block
  const int n_tiles = n_ent * p.G * p.subs;
  // Two cursors walk it, one for the copies (ahead) and one for the products; they advance digit by digit, so
  // that the loop has no divisions.
  struct cursor_t { int u, gg, e; };
  auto advance = [&](cursor_t& c) {
    if (++c.u == p.subs) { c.u = 0; if (++c.gg == p.G) { c.gg = 0; ++c.e; } }
  };
  auto locate = [&](const cursor_t& c, int& i, int& h, int64_t& q0) {
    i = entry(c.e);
    h = kvh * p.G + c.gg;
    q0 = (int64_t)i * p.B + c.u * KT;
  };
  cursor_t cf = {0, 0, 0}, cc = {0, 0, 0};
  auto fill = [&](int t) {
    int i, h; int64_t q0;
    locate(cf, i, h, q0);
    advance(cf);
    const uint32_t dst = lds0 + (t % NSTG) * STAGEB;
    const int64_t head_rows = ((int64_t)b * p.hq + h) * p.N;
    copy_tile<D, NW>(p.q + head_rows * D, q0, p.N - 1, dst, wave, lane);
    copy_tile<D, NW>(p.dout + head_rows * D, q0, p.N - 1, dst + G::TILEB, wave, lane);
    if (wave == 0) {
      // the tile's 64 log-sum-exps and Deltas, copied asynchronously like the tiles (a load through registers
      // would make this wavefront wait for memory in every iteration); rows beyond the sequence repeat the last
      // one and are masked where they are used
      int64_t qi = q0 + lane;
      qi = qi < p.N ? qi : p.N - 1;
      const uint32_t vdst = __builtin_amdgcn_readfirstlane(dst + 2 * G::TILEB);
      async_copy4(p.lse2 + head_rows + qi, vdst);
      async_copy4(p.delta + head_rows + qi, vdst + 256);
    }
  };
  static_assert(G::IPT % NW == 0, "tile copies must divide over the wavefronts");
  constexpr int CPF = 2 * G::IPT / NW;     // copies per wavefront and fill (Q and dO); the first wavefront adds two
  for (int s0 = 0; s0 < NSTG - 1; ++s0)
    if (s0 < n_tiles) fill(s0);
  for (int t = 0; t < n_tiles; ++t) {
    if (t + NSTG - 1 <= n_tiles) {
      if (wave == 0) wait_vmcnt<(NSTG - 2) * (CPF + 2)>(); else wait_vmcnt<(NSTG - 2) * CPF>();
    } else {
      wait_vmcnt<0>();
    }
    __syncthreads();
    if (t + NSTG - 1 < n_tiles) fill(t + NSTG - 1);
    int i, h; int64_t q0;
    locate(cc, i, h, q0);
    advance(cc);
    const uint32_t qt = lds0 + (t % NSTG) * STAGEB, dot = qt + G::TILEB;
    const float* vec = reinterpret_cast<const float*>(smem + (t % NSTG) * STAGEB + 2 * G::TILEB);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // (no shortcut for halves that the causal mask or the end of the sequence empties: the mask below zeroes
      // them, and a branch around the products makes the compiler copy the 128 accumulator registers)
      f32x16 S, dP;
#pragma unroll
      for (int r = 0; r < 16; ++r) { S[r] = 0.f; dP[r] = 0.f; }
      pipelined_mfma<2 * NC, PFD>(
          [&](int m) { return row_frag<D>((m & 1) ? dot : qt, m >> 1, half, lane); },
          [&](int m, bf16x8 a) {
            if (m & 1) dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vf[m >> 1], dP, 0, 0, 0);
            else S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[m >> 1], S, 0, 0, 0);
          });
      u32x4 pp[2], dsp[2];
      auto elements = [&](auto masked) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int lr0 = 32 * half + 8 * r4 + 4 * hh;                // rows lr0 .. lr0+3 of the tile
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(vec + lr0);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(vec + 64 + lr0);
          float x[4], y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // computed for every element and selected afterwards: a conditional exponential becomes a branch
            const float pr = __builtin_amdgcn_exp2f(fmaf(S[4 * r4 + e], p.c2, -l4[e]));
            x[e] = pr;
            y[e] = pr * (dP[4 * r4 + e] - d4[e]);
            if (decltype(masked)::value) {
              const int qi = (int)q0 + lr0 + e;
              const bool att = kok && qi >= key32 && qi < n32;
              x[e] = att ? x[e] : 0.f;
              y[e] = att ? y[e] : 0.f;
            }
          }
          const int r = 4 * r4;
          pp[r >> 3][(r & 7) >> 1] = pack2(x[0], x[1]);
          pp[r >> 3][((r & 7) >> 1) + 1] = pack2(x[2], x[3]);
          dsp[r >> 3][(r & 7) >> 1] = pack2(y[0], y[1]);
          dsp[r >> 3][((r & 7) >> 1) + 1] = pack2(y[2], y[3]);
        }
      };
      // the mask matters on the diagonal block and where queries or keys run past the sequence (uniform test)
      if (i == j || q0 + KT > p.N || ((int64_t)j + 1) * p.B > p.N) elements(std::true_type{});
      else elements(std::false_type{});
      // instruction m: 16-query step k2 = m / (2 ND), d tile dt = (m/2) % ND, dV (dO tile) or dK (Q tile) = m%2
      pipelined_mfma<4 * ND, PFD>(
          [&](int m) { return tr_frag<D>((m & 1) ? qt : dot, 2 * half + m / (2 * ND), (m >> 1) % ND, lane); },
          [&](int m, bf16x8 a) {
            const int k2 = m / (2 * ND), dt = (m >> 1) % ND;
            if (m & 1) dkt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, dsp[k2]), dkt[dt], 0, 0, 0);
            else dvt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pp[k2]), dvt[dt], 0, 0, 0);
          });
    }
  }
  wait_vmcnt<0>();

  if (!kok) return;
  if (!whole_column) {
    __bf16* ok_ = p.dk + krow * D;
    __bf16* ov_ = p.dv + krow * D;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const u32x2 wk = {pack2(dkt[dt][4 * r4] * p.scale, dkt[dt][4 * r4 + 1] * p.scale),
                          pack2(dkt[dt][4 * r4 + 2] * p.scale, dkt[dt][4 * r4 + 3] * p.scale)};
        const u32x2 wv = {pack2(dvt[dt][4 * r4], dvt[dt][4 * r4 + 1]), pack2(dvt[dt][4 * r4 + 2], dvt[dt][4 * r4 + 3])};
        *reinterpret_cast<u32x2*>(ok_ + 32 * dt + 8 * r4 + 4 * hh) = wk;
        *reinterpret_cast<u32x2*>(ov_ + 32 * dt + 8 * r4 + 4 * hh) = wv;
      }
  } else {
    const int64_t srow = ((int64_t)b * p.hkv + kvh) * ((int64_t)p.sink_blocks * p.B) + key;   // key < sink_blocks * B
    float* sk = p.dk_sink + srow * D;
    float* sv = p.dv_sink + srow * D;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int d = 32 * dt + acc_row(r, hh);
        atomicAdd(sk + d, dkt[dt][r] * p.scale);
        atomicAdd(sv + d, dvt[dt][r]);
      }
  }
}

// dK, dV with the two halves of the work on different wavefronts (blocks of 64 or 128 keys).  The kernel above keeps
// both transposed accumulators plus the K and V rows of its keys in one wavefront: more than 256 registers, one
// wavefront per SIMD, nothing to overlap with.  Here every 32-key slice has a wavefront that forms S and P and
// accumulates dV^T, and one that forms dP and dS and accumulates dK^T.  P travels through LDS, lane to same lane
// (both hold the same element layout), and the second wavefront runs one tile behind the first, so that the step's
// one barrier orders the exchange.  Each needs about 170 registers: two per SIMD, one of each kind.
template <int D, int NSL>
__global__ __launch_bounds__(128 * NSL) __attribute__((amdgpu_waves_per_eu(2, 2)))
void pa_bwd_dkv_split_kernel(bwd_params p) {
  using G = tile_geo<D>;
  constexpr int NW = 2 * NSL;
  constexpr int NC = G::NC, ND = G::ND;
  constexpr int STAGEB = 2 * G::TILEB + 512;     // Q tile, dO tile, 64 log-sum-exps, 64 Deltas
  constexpr int NST = 3;                         // tile t+1 arriving, tile t (P side), tile t-1 (dS side)
  constexpr int PBUF = NSL * 4096;               // P of one tile: per slice 2 halves x 2 KB
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, hh = lane >> 5;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int slice = wave % NSL;
  const bool krole = wave >= NSL;                // false: S, P, dV^T; true: dP, dS, dK^T

  int j, part;
  // the parts of the sink blocks' columns come first in the launch: they are the longest workgroups (PART query
  // blocks each against a dozen for an ordinary column), and the last ones to start should be the shortest
  const int n_extra = p.sink_blocks * (p.max_parts - 1);
  if ((int)blockIdx.x >= n_extra) { j = (int)blockIdx.x - n_extra; part = 0; }
  else {
    const int e = (int)blockIdx.x;
    j = e / (p.max_parts - 1);
    part = 1 + e % (p.max_parts - 1);
  }
  const bool whole_column = j < p.sink_blocks;
  const int parts = whole_column ? (p.nb - j + PART - 1) / PART : 1;
  if (part >= parts) return;
  const int weff = (p.flags & POWATTN_POWER) ? (p.W > 1 ? p.W : 1) : p.W;
  int n_win, n_ent, first_pow = 1;
  if (whole_column) {
    n_win = p.nb - j - part * PART;
    if (n_win > PART) n_win = PART;
    n_ent = n_win;
  } else {
    n_win = weff < p.nb - j ? weff : p.nb - j;
    n_ent = n_win;
    if (p.flags & POWATTN_POWER) {
      while (first_pow < weff) first_pow <<= 1;
      for (int64_t pw = first_pow; j + pw < p.nb; pw <<= 1) ++n_ent;
    }
  }
  auto entry = [&](int e) -> int {
    if (whole_column) return j + part * PART + e;
    if (e < n_win) return j + e;
    return j + (first_pow << (e - n_win));
  };

  // this lane's key; its K row (P side) or V row (dS side) as B operand
  const int64_t key = (int64_t)j * p.B + 32 * slice + ln;
  const bool kok = key < p.N;
  const int key32 = (int)key, n32 = (int)p.N;
  const int64_t krow = ((int64_t)b * p.hkv + kvh) * p.N + (kok ? key : 0);
  bf16x8 xf[NC];

  f32x16 acc[ND];
#pragma unroll
  for (int dt = 0; dt < ND; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;

  const int n_tiles = n_ent * p.G * p.subs;
  // The tiles of the column in order: the 64-query tiles of a query block, for each head of the group, for each
  // entry of the column.  A cursor carries what a tile needs (query block, first query, first row of the head's
  // slab, LDS stage) and moves on by additions: one runs ahead with the copies, one goes with the products.
  struct cursor_t { int u, gg, e, i; int64_t q0, head_rows; uint32_t stage; };
  auto advance = [&](cursor_t& c) {
    c.stage = c.stage == (NST - 1) * STAGEB ? 0u : c.stage + STAGEB;
    if (++c.u < p.subs) { c.q0 += KT; return; }
    c.u = 0;
    if (++c.gg < p.G) { c.head_rows += p.N; }
    else {
      c.gg = 0;
      c.head_rows -= (int64_t)(p.G - 1) * p.N;
      if (++c.e < n_ent) c.i = entry(c.e);
    }
    c.q0 = (int64_t)c.i * p.B;
  };
  cursor_t cf;                                   // the copies' cursor
  cf.u = 0; cf.gg = 0; cf.e = 0; cf.i = entry(0); cf.q0 = (int64_t)cf.i * p.B;
  cf.head_rows = ((int64_t)b * p.hq + (int64_t)kvh * p.G) * p.N; cf.stage = 0;
  cursor_t cc = cf;                              // this wavefront's products
  auto fill = [&]() {
    const int64_t q0 = cf.q0, head_rows = cf.head_rows;
    const uint32_t dst = lds0 + cf.stage;
    advance(cf);
    copy_tile<D, NW>(p.q + head_rows * D, q0, p.N - 1, dst, wave, lane);
    copy_tile<D, NW>(p.dout + head_rows * D, q0, p.N - 1, dst + G::TILEB, wave, lane);
    if (wave == 0) {
      int64_t qi = q0 + lane;
      qi = qi < p.N ? qi : p.N - 1;
      const uint32_t vdst = __builtin_amdgcn_readfirstlane(dst + 2 * G::TILEB);
      async_copy4(p.lse2 + head_rows + qi, vdst);
      async_copy4(p.delta + head_rows + qi, vdst + 256);
    }
  };
  static_assert(G::IPT % NW == 0, "tile copies must divide over the wavefronts");
  fill();
  // (after the first tile's copies: they would queue behind these row-per-lane loads)
  reg_rows<D>((krole ? p.v : p.k) + krow * D, kok, lane, xf);
  // iteration it: the P side works on tile it, the dS side on tile it-1
  for (int it = 0; it <= n_tiles; ++it) {
    wait_vmcnt<0>();
    __syncthreads();      // tile it has landed; P of tile it-1 is in LDS; everybody is done with tile it-2
    if (it + 1 < n_tiles) fill();                 // tile it+1
    const int t = krole ? it - 1 : it;
    if (t < 0 || t >= n_tiles) continue;          // uniform per wavefront; the barriers stay matched
    const int i = cc.i;
    const int64_t q0 = cc.q0;
    const uint32_t qt = lds0 + cc.stage, dot = qt + G::TILEB;
    const float* vec = reinterpret_cast<const float*>(smem + cc.stage + 2 * G::TILEB);
    advance(cc);
    const bool need_mask = i == j || q0 + KT > p.N || ((int64_t)j + 1) * p.B > p.N;
    unsigned char* pb = smem + NST * STAGEB + (t & 1) * PBUF + slice * 4096 + lane * 16;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      f32x16 X;           // S on the P side, dP on the dS side
#pragma unroll
      for (int r = 0; r < 16; ++r) X[r] = 0.f;
      const uint32_t rows_from = krole ? dot : qt;
      pipelined_mfma<NC, PFD>(
          [&](int m) { return row_frag<D>(rows_from, m, half, lane); },
          [&](int m, bf16x8 a) { X = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xf[m], X, 0, 0, 0); });
      u32x4 w[2];         // packed P (P side) or dS (dS side): the B operand of the second product
      u32x4* slot = reinterpret_cast<u32x4*>(pb + half * 2048);
      if (!krole) {
        auto elements = [&](auto masked) {
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const int lr0 = 32 * half + 8 * r4 + 4 * hh;
            const f32x4 l4 = *reinterpret_cast<const f32x4*>(vec + lr0);
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              x[e] = __builtin_amdgcn_exp2f(fmaf(X[4 * r4 + e], p.c2, -l4[e]));
              if (decltype(masked)::value) {
                const int qi = (int)q0 + lr0 + e;
                x[e] = (kok && qi >= key32 && qi < n32) ? x[e] : 0.f;
              }
            }
            const int r = 4 * r4;
            w[r >> 3][(r & 7) >> 1] = pack2(x[0], x[1]);
            w[r >> 3][((r & 7) >> 1) + 1] = pack2(x[2], x[3]);
          }
        };
        if (need_mask) elements(std::true_type{}); else elements(std::false_type{});
        slot[0] = w[0];                            // lane l's two 16-byte pieces at l*16 and 1024 + l*16
        slot[64] = w[1];
      } else {
        const u32x4 p0 = slot[0], p1 = slot[64];   // bf16 P of the same elements, masked by its producer
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int lr0 = 32 * half + 8 * r4 + 4 * hh;
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(vec + 64 + lr0);
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * r4 + e;
            const uint32_t pk = (r < 8 ? p0 : p1)[(r & 7) >> 1];
            const float pr = __builtin_bit_cast(float, (r & 1) ? (pk & 0xffff0000u) : (pk << 16));
            y[e] = pr * (X[r] - d4[e]);
          }
          const int r = 4 * r4;
          w[r >> 3][(r & 7) >> 1] = pack2(y[0], y[1]);
          w[r >> 3][((r & 7) >> 1) + 1] = pack2(y[2], y[3]);
        }
      }
      const uint32_t cols_from = krole ? qt : dot;
      pipelined_mfma<2 * ND, PFD>(
          [&](int m) { return tr_frag<D>(cols_from, 2 * half + m / ND, m % ND, lane); },
          [&](int m, bf16x8 a) {
            acc[m % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, w[m / ND]), acc[m % ND], 0, 0, 0);
          });
    }
  }
  wait_vmcnt<0>();

  if (!kok) return;
  const float f = krole ? p.scale : 1.0f;
  if (!whole_column) {
    __bf16* out = (krole ? p.dk : p.dv) + krow * D;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const u32x2 wv = {pack2(acc[dt][4 * r4] * f, acc[dt][4 * r4 + 1] * f), pack2(acc[dt][4 * r4 + 2] * f, acc[dt][4 * r4 + 3] * f)};
        *reinterpret_cast<u32x2*>(out + 32 * dt + 8 * r4 + 4 * hh) = wv;
      }
  } else {
    const int64_t srow = ((int64_t)b * p.hkv + kvh) * ((int64_t)p.sink_blocks * p.B) + key;
    float* sums = (krole ? p.dk_sink : p.dv_sink) + srow * D;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) atomicAdd(sums + 32 * dt + acc_row(r, hh), acc[dt][r] * f);
  }
}

// the sink blocks' fp32 sums -> bf16 rows of dK and dV
template <int D>
__global__ __launch_bounds__(256) void pa_bwd_sink_store_kernel(bwd_params p, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;      // over [batch*hkv, sink_rows, D]
  if (e >= total) return;
  const int64_t sink_rows = (int64_t)p.sink_blocks * p.B;
  const int d = (int)(e % D);
  const int64_t key = (e / D) % sink_rows, bh = e / (D * sink_rows);
  if (key >= p.N) return;
  p.dk[(bh * p.N + key) * D + d] = (__bf16)p.dk_sink[e];
  p.dv[(bh * p.N + key) * D + d] = (__bf16)p.dv_sink[e];
}

template <int D, int NW>
int launch_dq(const bwd_params& p, int64_t items, hipStream_t stream) {
  constexpr size_t lds = dq_stages(NW) * 2 * (size_t)tile_geo<D>::TILEB;
  static std::atomic<unsigned long long> done{0};
  if (int st = pa_allow_dynamic_lds(reinterpret_cast<const void*>(&pa_bwd_dq_kernel<D, NW>), lds, done)) return st;
  hipLaunchKernelGGL((pa_bwd_dq_kernel<D, NW>), dim3((uint32_t)items), dim3(64 * NW), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}
template <int D, int NW>
int launch_dkv(const bwd_params& p, dim3 grid, hipStream_t stream) {
  constexpr size_t lds = NSTG * (2 * (size_t)tile_geo<D>::TILEB + 512);
  static std::atomic<unsigned long long> done{0};
  if (int st = pa_allow_dynamic_lds(reinterpret_cast<const void*>(&pa_bwd_dkv_kernel<D, NW>), lds, done)) return st;
  hipLaunchKernelGGL((pa_bwd_dkv_kernel<D, NW>), grid, dim3(64 * NW), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}

template <int D, int NSL>
int launch_dkv_split(const bwd_params& p, dim3 grid, hipStream_t stream) {
  constexpr size_t lds = 3 * (2 * (size_t)tile_geo<D>::TILEB + 512) + 2 * (size_t)NSL * 4096;
  static std::atomic<unsigned long long> done{0};
  if (int st = pa_allow_dynamic_lds(reinterpret_cast<const void*>(&pa_bwd_dkv_split_kernel<D, NSL>), lds, done)) return st;
  hipLaunchKernelGGL((pa_bwd_dkv_split_kernel<D, NSL>), grid, dim3(128 * NSL), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t pa_backward_workspace_bytes(const powattn_pattern& pat, int32_t batch, int32_t hq, int32_t hkv, int64_t seq_len, int32_t head_dim) {
  const int64_t nb = (seq_len + pat.block - 1) / pat.block;
  const int64_t sink_rows = (pat.sink < nb ? pat.sink : nb) * (int64_t)pat.block;
  return 2 * align256((size_t)batch * hq * seq_len * sizeof(float)) +
         2 * align256((size_t)batch * hkv * sink_rows * head_dim * sizeof(float));
}

int pa_launch_backward_bf16(const pa_backward_args& a) {
  bwd_params p;
  p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.o = (const __bf16*)a.o;
  p.dout = (const __bf16*)a.dout; p.lse = a.lse;
  p.dq = (__bf16*)a.dq; p.dk = (__bf16*)a.dk; p.dv = (__bf16*)a.dv;
  p.kv_cnt = a.kv_cnt; p.kv_idx = a.kv_idx; p.max_k = a.max_k; p.nb = a.nb;
  p.B = a.pat.block; p.W = a.pat.window; p.S = a.pat.sink; p.flags = a.pat.flags;
  p.hq = a.hq; p.hkv = a.hkv; p.G = a.hq / a.hkv; p.subs = p.B / KT;
  p.N = a.seq_len; p.scale = a.scale; p.c2 = a.scale * LOG2E;
  if ((int64_t)a.max_k * p.subs > TILE_CAP) return POWATTN_UNSUPPORTED;
  if (a.seq_len > 0x7fffffffLL - 1024) return POWATTN_UNSUPPORTED;
  if (p.B > 256) return POWATTN_UNSUPPORTED;                       // a wavefront per 32 keys of the block, at most 8
  if (a.batch > 65535 || a.hkv > 65535) return POWATTN_UNSUPPORTED;
  const int64_t tasks = (int64_t)p.G * p.B / 32;
  if (tasks > (1 << 20)) return POWATTN_UNSUPPORTED;
  p.tasks = (int32_t)tasks;
  // eight wavefronts per workgroup when a query block has that many tasks and blocks of 128 keys or more; at
  // blocks of 64 keys four (two workgroups per compute unit that are not in step with each other: 4-7 % faster
  // at configuration 2's shape than one workgroup of eight)
  const int nwq = (p.tasks > 4 && p.B >= 128) ? 8 : 4;
  p.chunks = (p.tasks + nwq - 1) / nwq;
  p.sink_blocks = a.pat.sink < a.nb ? a.pat.sink : a.nb;
  p.max_parts = p.sink_blocks > 0 ? (a.nb + PART - 1) / PART : 1;
  if (p.max_parts < 2) p.max_parts = 2;                            // keeps the part arithmetic of the kernel defined

  // workspace: Delta, the log-sum-exp in base 2, then the sink blocks' sums
  unsigned char* ws = (unsigned char*)a.workspace;
  p.delta = (float*)ws;
  ws += align256((size_t)a.batch * a.hq * a.seq_len * sizeof(float));
  p.lse2 = (float*)ws;
  ws += align256((size_t)a.batch * a.hq * a.seq_len * sizeof(float));
  const int64_t sink_elems = (int64_t)a.batch * a.hkv * p.sink_blocks * p.B * a.head_dim;
  p.dk_sink = (float*)ws;
  ws += align256((size_t)sink_elems * sizeof(float));
  p.dv_sink = (float*)ws;

  int st = POWATTN_OK;
  if (sink_elems > 0) {
    const int64_t zb = (2 * (int64_t)(align256((size_t)sink_elems * sizeof(float)) / sizeof(float)) + 255) / 256;
    hipLaunchKernelGGL(pa_bwd_zero_kernel, dim3((uint32_t)zb), dim3(256), 0, a.stream, p.dk_sink,
                       2 * (int64_t)(align256((size_t)sink_elems * sizeof(float)) / sizeof(float)));
    st = pa_note_hip(hipGetLastError());
    if (st != POWATTN_OK) return st;
  }

  const int64_t items = (int64_t)a.batch * a.hkv * a.nb * p.chunks;
  if (items > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  if (a.head_dim == 128) st = nwq == 8 ? launch_dq<128, 8>(p, items, a.stream) : launch_dq<128, 4>(p, items, a.stream);
  else st = nwq == 8 ? launch_dq<64, 8>(p, items, a.stream) : launch_dq<64, 4>(p, items, a.stream);
  if (st != POWATTN_OK) return st;

  const int64_t gx = (int64_t)a.nb + (int64_t)p.sink_blocks * (p.max_parts - 1);
  if (gx > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  const dim3 grid((uint32_t)gx, (uint32_t)a.hkv, (uint32_t)a.batch);
  const int nwk = p.B / 32;
  // blocks of 128 keys: the kernel with the work of a key slice split over two wavefronts (measured 10 % faster
  // at the 128K workload; at 64 keys a workgroup of that kind has only four wavefronts and is slightly slower)
  if (a.head_dim == 128)
    st = nwk == 2 ? launch_dkv<128, 2>(p, grid, a.stream) : nwk == 4 ? launch_dkv_split<128, 4>(p, grid, a.stream) : launch_dkv<128, 8>(p, grid, a.stream);
  else
    st = nwk == 2 ? launch_dkv<64, 2>(p, grid, a.stream) : nwk == 4 ? launch_dkv_split<64, 4>(p, grid, a.stream) : launch_dkv<64, 8>(p, grid, a.stream);
  if (st != POWATTN_OK) return st;

  if (sink_elems > 0) {
    const int64_t sb = (sink_elems + 255) / 256;
    if (a.head_dim == 128)
      hipLaunchKernelGGL((pa_bwd_sink_store_kernel<128>), dim3((uint32_t)sb), dim3(256), 0, a.stream, p, sink_elems);
    else
      hipLaunchKernelGGL((pa_bwd_sink_store_kernel<64>), dim3((uint32_t)sb), dim3(256), 0, a.stream, p, sink_elems);
    st = pa_note_hip(hipGetLastError());
  }
  return st;
}
