// Split-K decode: one query token per sequence attends its KV cache under the
// prefill pattern (Section 4.1: the same pattern in both phases).  The query
// sits at t = kv_len-1; the attended block list of row floor(t/B) comes from
// the closed form of Algorithm 1, inside the kernel.
//
// The step reads 2*D*2 bytes per attended token and does a handful of flops
// with them: it is bound by HBM bandwidth and latency, so the kernel is built
// around having every byte in flight at once and keeping the dependent chain
// after the loads short.
//
//  * A workgroup of 8 wavefronts owns one (sequence, KV head[, split]).  The
//    attended tokens are cut into 64-token chunks, dealt round-robin to the
//    splits and their wavefronts; a wavefront issues all K and V loads of a
//    chunk before touching any.
//  * Everything stays in registers.  K rows are loaded straight into the
//    A-operand layout of v_mfma_f32_16x16x32_bf16 (S^T = K q^T, the G query
//    heads of the group are the 16 columns, unused ones zero).  V is loaded
//    fully coalesced as 8 tokens x 8 d per lane and transposed inside the lane
//    (32 byte-permutes per 8x8 block) into the A operand of O^T += V^T P^T.
//    The K rows are fetched in a permuted token order chosen so that the
//    accumulator layout of S^T is the B-operand layout of the second product.
//  * Each wavefront keeps a running (max, sum, O) over its chunks; the eight
//    partials meet in LDS.  With one workgroup per (sequence, KV head) that is
//    the result; with several, every workgroup leaves its unnormalised partial
//    in the workspace as tagged 8-byte packets, waits until memory has taken
//    them, and then reads the packets of the other workgroups: the one whose
//    packets landed last finds all of them in place and writes the output (a
//    second launch would cost more than the whole merge).  There are no
//    counters and nothing in the workspace has to be initialised: a packet
//    is valid when its tag matches the generation number that the (sequence,
//    KV head) keeps in the workspace and that the finishing workgroup advances.
//    Packet stores and loads act at device scope by themselves; no fence is
//    used, because a device-scope fence writes back and invalidates a whole L2
//    on this chip.
//  * With several work items per compute unit (large batches) persistent
//    workgroups take over (pa_decode_stream_kernel): the loads of the next item
//    are in flight while the current one is merged.
#include <math.h>
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int CH = 64;         // tokens per chunk
constexpr int NW = 8;          // wavefronts per workgroup
constexpr int MAXG = 16;       // query heads per KV head (columns of the MFMA tile)

struct dec_params {
  const __bf16* q; const __bf16* k; const __bf16* v; const int32_t* kv_len;
  __bf16* o; float* lse;
  float* partials;      // [batch, hq, splits, D + 2] floats when splits > 1 and a merge kernel follows
  uint64_t* packets;    // the same shape as (value, tag) packets when the workgroups merge among themselves
  uint32_t* gen;        // [batch, hkv] generation numbers of the packets (any initial value)
  int64_t capacity;
  int32_t B, W, S; uint32_t flags;
  int32_t hq, hkv, G, splits, subs;
  uint32_t subs_magic;  // ceil(2^32 / subs) for subs > 1: slot / subs = umulhi(slot, subs_magic) for every slot of a row
  int32_t fused;        // 1: the workgroups of a (sequence, KV head) merge their partials among themselves
  float c2;
  const int32_t* block_table;   // paged cache: page of block j of sequence b at [b * table_stride + j]; else null
  int32_t table_stride;
  int64_t n_pages;
};

// ---- merging the workgroups of a (sequence, KV head) without a second kernel ----
// Every value of a partial result travels as one 8-byte packet (value, tag), written and read with single 8-byte
// device-scope accesses, so a reader sees a value together with its tag or not at all.  The tag is derived from the
// generation number g that the (sequence, KV head) keeps in the workspace, read at the start of the kernel, and from
// the split.  Protocol of a workgroup: store its packets; wait until memory has acknowledged every one of them
// (s_waitcnt, then the workgroup's barrier); load the packets of the other splits; if every tag is the expected one,
// combine all partials in split order, write the output and store g + 1 as the new generation.
//  * Some workgroup finishes: order the workgroups by the time at which the last of their stores was acknowledged;
//    the latest one loads after that, when every other workgroup's packets are in memory.
//  * Several may finish: they combine the same values in the same order and write the same bits.
//  * Nothing stale is taken for valid: what the workspace holds from the call before carries generation g - 1 (the
//    finisher advanced it only after every workgroup of the pair had stored, hence had read g), and the very first
//    call on a workspace meets whatever the memory held: a word there passes for a tag only if it equals
//    ~g ^ ((split + 1) << 24) for the word g found in the same memory (never for a memory filled with one byte
//    value, zeros included).
//  * No workgroup waits for another one: whoever finds a packet missing simply leaves.
// Calls that may run at the same time must not share a workspace (they would share generation numbers).
constexpr int MAX_FUSED_SPLITS = 16;
__device__ __forceinline__ uint32_t dec_tag(uint32_t gen, int split) { return ~gen ^ ((uint32_t)(split + 1) << 24); }
__device__ __forceinline__ void dec_put(uint64_t* slot, float x, uint32_t tag) {
  __hip_atomic_store(slot, ((uint64_t)tag << 32) | __builtin_bit_cast(uint32_t, x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t dec_get(const uint64_t* slot) {
  return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// LDS layout of the wavefronts' partial outputs: the 32 values a lane holds (d = 32*q4 + x) form a row of 36 floats,
// so that the 16 lanes of a store (4 heads x 4 groups) start 36 floats apart and cover all banks between them.
constexpr int OROW = 36;
template <int D>
__device__ __forceinline__ int dec_o_at(int wave, int G, int g, int d) { return (((wave * G + g) * (D / 32) + (d >> 5)) * OROW) + (d & 31); }
template <int D>
constexpr size_t dec_o_bytes(int G) { return (size_t)NW * G * (D / 32) * OROW * sizeof(float); }

// The query's row of the pattern in closed form: [0, sink_end) ++ {i - 2^k inside [pow_lo, win_start), k
// descending} ++ [win_start, i].  Uniform over a workgroup, so all of it runs on the scalar unit.
struct dec_row {
  pa_row_shape rs;
  int64_t t, i;          // position of the query, its block
  int n_pow, k_max;      // isolated blocks i - 2^k for k = k_max, k_max-1, ...: n_pow of them
  int n_slots;           // 64-token chunks of the attended blocks
};
__device__ __forceinline__ dec_row dec_row_of(const dec_params& p, int64_t len) {
  dec_row r;
  if (len < 1) len = 1;
  if (len > p.capacity) len = p.capacity;
  r.t = len - 1;
  // t / B = (t / 64) / subs, through the same multiply-high as the slots while the quotient is exact
  static_assert(CH == 64, "the block index is formed from 64-token chunks");
  const int64_t chunk_of_t = r.t >> 6;
  r.i = p.subs == 1 ? chunk_of_t
      : chunk_of_t < (1 << 25) ? (int64_t)__umulhi((unsigned)chunk_of_t, p.subs_magic) : chunk_of_t / p.subs;
  r.rs = pa_shape_of_row(p.W, p.S, p.flags, r.i);
  // The isolated blocks i - 2^k lie inside [pow_lo, win_start) exactly for i - win_start < 2^k <= i - pow_lo:
  // a contiguous range of exponents, found with two leading-zero counts instead of a loop over the powers.
  r.n_pow = 0; r.k_max = 0;
  if (p.flags & POWATTN_POWER) {
    const int64_t below = r.i - r.rs.win_start, upto = r.i - r.rs.pow_lo;
    if (upto >= 1) {
      const int k_min = below > 0 ? 64 - __builtin_clzll((unsigned long long)below) : 0;
      r.k_max = 63 - __builtin_clzll((unsigned long long)upto);
      r.n_pow = r.k_max >= k_min ? r.k_max - k_min + 1 : 0;
    }
  }
  const int n_blocks = (int)r.rs.sink_end + r.n_pow + (int)(r.i - r.rs.win_start + 1);
  r.n_slots = n_blocks * p.subs;
  return r;
}
__device__ __forceinline__ int64_t dec_block_at(const dec_row& r, int lp) {   // lp-th attended block, ascending
  if (lp < r.rs.sink_end) return lp;
  lp -= (int)r.rs.sink_end;
  if (lp >= r.n_pow) return r.rs.win_start + (lp - r.n_pow);
  return r.i - ((int64_t)1 << (r.k_max - lp));
}
// Chunk `slot` of the row: its block, the chunk inside the block, the tokens of it the query attends (<= 0: none)
struct dec_place { int64_t blk; int sub; int n_tok; };
__device__ __forceinline__ dec_place dec_place_of(const dec_params& p, const dec_row& r, int slot) {
  // (no division in the kernel: a 64-bit one costs more than the rest of the address arithmetic)
  dec_place c;
  const int lp = p.subs == 1 ? slot : (int)__umulhi((unsigned)slot, p.subs_magic);
  c.sub = slot - lp * p.subs;
  c.blk = dec_block_at(r, lp);
  const int64_t left = r.t + 1 - (c.blk * p.B + (int64_t)c.sub * CH);      // causal: tokens tok0..t are attended
  c.n_tok = left >= CH ? CH : (int)left;
  return c;
}
// First K and V row of a chunk: in the contiguous cache, or in its page (page numbers outside the pool are clamped
// into it: a bad table gives wrong numbers, never an access outside the pool)
__device__ __forceinline__ int64_t dec_chunk_offset(const dec_params& p, int b, int kvh, const dec_place& c, int64_t page, int D) {
  if (!p.block_table) return (((int64_t)b * p.hkv + kvh) * p.capacity + c.blk * p.B + (int64_t)c.sub * CH) * D;
  page = page < 0 ? 0 : (page >= p.n_pages ? p.n_pages - 1 : page);
  return ((page * p.hkv + kvh) * p.B + (int64_t)c.sub * CH) * D;
}

// The registers of one 64-token chunk: every load of it is issued before any is used.
template <int D>
struct dec_chunk {
  u32x4 kraw[4][D / 32];
  u32x4 vraw[2][8];
};
// K tile 2x+y, row rho = lane%16 holds token 32x + 8(rho/4) + 4y + rho%4: with this order the S^T
// accumulator of lane (g, q4) holds tokens 32x + 8*q4 + (0..7), which is what P^T must supply below.
// V: lane (dg = lane%16, tg = lane/16) takes tokens 32x + 8tg + (0..7), d = 8dg .. 8dg+7.
template <int D>
__device__ __forceinline__ void dec_issue(dec_chunk<D>& c, const __bf16* kb, const __bf16* vb, int n_tok, int g, int q4) {
  constexpr int NC = D / 32, CPR = D / 8;
#pragma unroll
  for (int tau = 0; tau < 4; ++tau) {
    const int tk = 32 * (tau >> 1) + 8 * (g >> 2) + 4 * (tau & 1) + (g & 3);
#pragma unroll
    for (int cc = 0; cc < NC; ++cc)
      c.kraw[tau][cc] = tk < n_tok ? *reinterpret_cast<const u32x4*>(kb + tk * D + 32 * cc + 8 * q4) : u32x4{0, 0, 0, 0};
  }
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int tk = 32 * x + 8 * q4 + r;
      c.vraw[x][r] = (g < CPR && tk < n_tok) ? *reinterpret_cast<const u32x4*>(vb + tk * D + 8 * g) : u32x4{0, 0, 0, 0};
    }
}
// One online-softmax update with the chunk: S^T = K q^T, then O^T += V^T P^T.
template <int D>
__device__ __forceinline__ void dec_consume(const dec_chunk<D>& c, const bf16x8 (&qf)[D / 32], int n_tok, float c2, int q4,
                                            float& m_run, float& l_run, f32x4 (&O)[8]) {
  constexpr int NC = D / 32;
  f32x4 S[4];
#pragma unroll
  for (int tau = 0; tau < 4; ++tau) {
    S[tau] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cc = 0; cc < NC; ++cc)
      S[tau] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, c.kraw[tau][cc]), qf[cc], S[tau], 0, 0, 0);
  }
  // ---- online softmax; S[2x+y][r] is token 32x + 8*q4 + 4y + r of head g ----
  float mx = -INFINITY;
#pragma unroll
  for (int tau = 0; tau < 4; ++tau)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int tk = 32 * (tau >> 1) + 8 * q4 + 4 * (tau & 1) + r;
      S[tau][r] = tk < n_tok ? S[tau][r] * c2 : -INFINITY;
      mx = fmaxf(mx, S[tau][r]);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));                // finite: token 0 of the chunk is attended
  const float m_new = fmaxf(m_run, mx);
  const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
  m_run = m_new;
  float rowsum = 0.f;
#pragma unroll
  for (int tau = 0; tau < 4; ++tau)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      S[tau][r] = __builtin_amdgcn_exp2f(S[tau][r] - m_new);
      rowsum += S[tau][r];
    }
  l_run = l_run * alpha + rowsum;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) O[j][r] *= alpha;

  // ---- O^T += V^T P^T: 32 tokens per step; MFMA j covers d = 8*row + j ----
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    bf16x8 pf;
#pragma unroll
    for (int e = 0; e < 8; ++e) pf[e] = (__bf16)S[2 * x + (e >> 2)][e & 3];
    // transpose the lane's 8 tokens x 8 d block: pairs of tokens share a dword
    uint32_t tr[4][8];                                // tr[a][d]: tokens 2a, 2a+1 at d
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int kd = 0; kd < 4; ++kd) {
        const uint32_t r0 = c.vraw[x][2 * a][kd], r1 = c.vraw[x][2 * a + 1][kd];
        tr[a][2 * kd] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);       // low halves: d = 2kd
        tr[a][2 * kd + 1] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);   // high halves: d = 2kd+1
      }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32x4 vf = {tr[0][j], tr[1][j], tr[2][j], tr[3][j]};
      O[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), pf, O[j], 0, 0, 0);
    }
  }
}
// q^T fragments: column g, 8 consecutive d per 32-wide step
template <int D>
__device__ __forceinline__ void dec_load_q(bf16x8 (&qf)[D / 32], const dec_params& p, int b, int kvh, int g, int q4) {
  const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  const __bf16* qp = p.q + ((int64_t)b * p.hq + (int64_t)kvh * p.G + (g < p.G ? g : 0)) * D;
#pragma unroll
  for (int c = 0; c < D / 32; ++c)
    qf[c] = g < p.G ? *reinterpret_cast<const bf16x8*>(qp + 32 * c + 8 * q4) : z;
}

// The lane number, computed afresh wherever it is called: the compiler cannot carry the value of an earlier call
// over, so nothing derived from it has to stay in (or be spilled from) a register across the chunk loads and the
// matrix products, where every register counts.  (A spilled register in the persistent kernel is reloaded behind
// the next chunk's loads and has to wait for all of them.)
__device__ __forceinline__ int dec_lane_now() {
  int l;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
  return l;
}

// The wavefront's partial output into LDS: lane (g, q4) holds O[j][r] = o[g][d = 32*q4 + 8r + j], eight
// consecutive d per r, written as two 16-byte stores into the lane's padded row.
template <int D>
__device__ __forceinline__ void dec_stash(float* s_o, int wave, int G, int g, int q4, const f32x4 (&O)[8]) {
  if (32 * q4 >= D) return;
  f32x4* row = reinterpret_cast<f32x4*>(s_o + dec_o_at<D>(wave, G, g, 32 * q4));
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    row[2 * r] = f32x4{O[0][r], O[1][r], O[2][r], O[3][r]};
    row[2 * r + 1] = f32x4{O[4][r], O[5][r], O[6][r], O[7][r]};
  }
}

template <int D>
__global__ __launch_bounds__(64 * NW) void pa_decode_kernel(dec_params p) {
  __shared__ float s_m[NW][MAXG], s_l[NW][MAXG];
  extern __shared__ __attribute__((aligned(16))) float s_o_dyn[];   // [NW][G][D/32][OROW] partial outputs of the wavefronts

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  // the wavefront's number as a scalar and the lane from the hardware's lane count: the thread index itself need
  // not stay in a vector register through the chunk loop, where every register counts
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int g = lane & 15, q4 = lane >> 4;    // column (query head) and k-group of this lane

  // The sequence length and the generation of this (sequence, KV head)'s packets (needed only at the end) are
  // both uniform: two scalar loads, one wait.  Written as assembly so that the generation number lives in a
  // scalar register from the start (a vector register held across the chunk loop costs a spill to scratch
  // memory, and a kernel that uses scratch memory starts later).  Both words were written before this kernel
  // started, so the scalar cache, which is empty at the start of a kernel, returns what memory holds.
  uint32_t gen;
  int len_b;
  asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %3, 0x0\n\ts_waitcnt lgkmcnt(0)"
               : "=&s"(gen), "=&s"(len_b)
               : "s"(p.gen + (int64_t)b * p.hkv + kvh), "s"(p.kv_len + b)
               : "memory");

  const dec_row row = dec_row_of(p, len_b);
  bf16x8 qf[D / 32];
  dec_load_q<D>(qf, p, b, kvh, g, q4);

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 O[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) O[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // chunks are dealt round-robin to the splits (slot = wave * splits + split), so that the workgroups of a
  // (sequence, KV head) stream nearly equal amounts (13 chunks over 2 workgroups: 7 + 6 instead of 8 + 5)
  for (int slot = wave * p.splits + split; slot < row.n_slots; slot += p.splits * NW) {
    const dec_place pl = dec_place_of(p, row, slot);
    if (pl.n_tok <= 0) continue;                         // chunk of the diagonal block beyond the query
    // paged cache: the block's page comes from the table (one more dependent look-up; blk < table_stride,
    // because len <= table_stride * B); a page holds the block's tokens of every KV head
    const int64_t page = p.block_table ? p.block_table[(int64_t)b * p.table_stride + pl.blk] : 0;
    const int64_t off = dec_chunk_offset(p, b, kvh, pl, page, D);
    dec_chunk<D> c;
    dec_issue<D>(c, p.k + off, p.v + off, pl.n_tok, g, q4);
    dec_consume<D>(c, qf, pl.n_tok, p.c2, q4, m_run, l_run, O);
  }

  // ---- merge the wavefronts through LDS ----
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (g < p.G) {
    if (q4 == 0) { s_m[wave][g] = m_run; s_l[wave][g] = l_run; }
    dec_stash<D>(s_o_dyn, wave, p.G, g, q4, O);
  }
  __syncthreads();

  // thread e owns output (head gg, component d); with up to 16 heads per KV head a thread owns several
  const int tid = wave * 64 + (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  constexpr int EPT = MAXG * D / (64 * NW);            // at most this many outputs per thread
  float accs[EPT], Ms[EPT], Ls[EPT];
#pragma unroll
  for (int x = 0; x < EPT; ++x) {
    const int e = tid + x * 64 * NW;
    accs[x] = 0.f; Ms[x] = -INFINITY; Ls[x] = 0.f;
    if (e >= p.G * D) continue;
    const int gg = e / D, d = e % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, s_m[w][gg]);
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wt = s_l[w][gg] > 0.f ? __builtin_amdgcn_exp2f(s_m[w][gg] - M) : 0.f;
      L = fmaf(wt, s_l[w][gg], L);
      acc = fmaf(wt, s_o_dyn[dec_o_at<D>(w, p.G, gg, d)], acc);
    }
    accs[x] = acc; Ms[x] = M; Ls[x] = L;
    const int h = kvh * p.G + gg;
    if (p.splits == 1) {
      p.o[((int64_t)b * p.hq + h) * D + d] = (__bf16)(acc / L);      // L > 0: chunk 0 of the row is never empty
      if (p.lse && d == 0) p.lse[(int64_t)b * p.hq + h] = (M + log2f(L)) * 0.69314718055994530942f;
    } else if (!p.fused) {
      // a merge kernel follows: plain stores
      float* part = p.partials + (((int64_t)b * p.hq + h) * p.splits + split) * (D + 2);
      part[d] = acc;
      if (d == 0) { part[D] = M; part[D + 1] = L; }                  // an idle split leaves M = -inf, L = 0
    } else {
      uint64_t* pk = p.packets + (((int64_t)b * p.hq + h) * p.splits + split) * (D + 2);
      const uint32_t tag = dec_tag(gen, split);
      dec_put(pk + d, acc, tag);
      if (d == 0) { dec_put(pk + D, M, tag); dec_put(pk + D + 1, L, tag); }
    }
  }
  if (p.splits == 1 || !p.fused) return;

  // ---- the workgroups of this (sequence, KV head) merge among themselves (protocol above) ----
  __builtin_amdgcn_s_waitcnt(0);                       // vmcnt(0): memory has acknowledged this thread's packets
  __syncthreads();                                     // ... and every other thread's of this workgroup
  bool valid = true;
  float o_out[EPT], lse_out[EPT];
#pragma unroll
  for (int x = 0; x < EPT; ++x) {
    const int e = tid + x * 64 * NW;
    o_out[x] = 0.f; lse_out[x] = 0.f;
    if (e >= p.G * D) continue;
    const int gg = e / D, d = e % D;
    const int h = kvh * p.G + gg;
    const uint64_t* pk = p.packets + ((int64_t)b * p.hq + h) * p.splits * (D + 2);
    float M = -INFINITY, L = 0.f, acc = 0.f;
    for (int s0 = 0; s0 < p.splits; s0 += 8) {
      uint64_t pm[8], pl[8], po[8];
#pragma unroll
      for (int y = 0; y < 8; ++y) {                    // all loads of (up to) eight splits before any is looked at
        pm[y] = pl[y] = po[y] = 0;
        if (s0 + y < p.splits && s0 + y != split) {    // uniform over the workgroup; its own partial is in registers
          const uint64_t* ps = pk + (int64_t)(s0 + y) * (D + 2);
          pm[y] = dec_get(ps + D); pl[y] = dec_get(ps + D + 1); po[y] = dec_get(ps + d);
        }
      }
#pragma unroll
      for (int y = 0; y < 8; ++y) {
        const int s1 = s0 + y;
        if (s1 >= p.splits) break;
        float ms, ls, os;
        if (s1 == split) { ms = Ms[x]; ls = Ls[x]; os = accs[x]; }   // this workgroup's own partial: the same bits
        else {
          const uint32_t want = dec_tag(gen, s1);
          valid = valid && (uint32_t)(pm[y] >> 32) == want && (uint32_t)(pl[y] >> 32) == want && (uint32_t)(po[y] >> 32) == want;
          ms = __builtin_bit_cast(float, (uint32_t)pm[y]); ls = __builtin_bit_cast(float, (uint32_t)pl[y]);
          os = __builtin_bit_cast(float, (uint32_t)po[y]);
        }
        if (ls > 0.f) {                                              // idle splits hold no outputs
          const float Mn = fmaxf(M, ms);
          const float r0 = L > 0.f ? __builtin_amdgcn_exp2f(M - Mn) : 0.f, r1 = __builtin_amdgcn_exp2f(ms - Mn);
          L = L * r0 + ls * r1;
          acc = acc * r0 + os * r1;
          M = Mn;
        }
      }
    }
    o_out[x] = acc / L;
    lse_out[x] = (M + log2f(L)) * 0.69314718055994530942f;
  }
  if (!__syncthreads_and(valid ? 1 : 0)) return;       // some packet has not landed: its workgroup will finish
#pragma unroll
  for (int x = 0; x < EPT; ++x) {
    const int e = tid + x * 64 * NW;
    if (e >= p.G * D) continue;
    const int gg = e / D, d = e % D;
    const int h = kvh * p.G + gg;
    p.o[((int64_t)b * p.hq + h) * D + d] = (__bf16)o_out[x];
    if (p.lse && d == 0) p.lse[(int64_t)b * p.hq + h] = lse_out[x];
  }
  if (tid == 0) __hip_atomic_store(p.gen + (int64_t)b * p.hkv + kvh, gen + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Large batches: persistent workgroups.  With many more (sequence, KV head, split) items than compute units the
// kernel above leaves every compute unit without a byte in flight while a workgroup looks its sequence length up and
// while it merges (one workgroup fits at a time: its wavefronts hold a whole chunk in registers).  Here a workgroup
// walks through items, and through an item in passes of NW chunks (wavefront w takes chunk w + NW * pass of the
// item's share of the row, keeping its running (max, sum, O) over the passes); a wavefront requests its chunk of the
// next pass (of this item or the next one) as soon as the registers of the current one are free, before the workgroup
// merges a finished item through LDS, and the sequence length and the page of a chunk are read two passes and one
// pass ahead.  With one split per (sequence, KV head), which is how the library launches it once there is at least
// one (sequence, KV head) pair per compute unit, the outputs are written here and no merge follows; with several
// splits the partials go to the workspace with plain stores for the merge kernel below.
template <int D>
__global__ __launch_bounds__(64 * NW) void pa_decode_stream_kernel(dec_params p, int n_items, int n_pass) {
  __shared__ float s_m[2][NW][MAXG], s_l[2][NW][MAXG];
  extern __shared__ __attribute__((aligned(16))) float s_o_dyn[];   // [2][NW][G][D/32][OROW] partial outputs of the wavefronts, two items
  // (wavefront number as a scalar; the lane number is taken afresh in every phase of a step: dec_lane_now)
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int stride = (int)gridDim.x;
  const int per_b = p.hkv * p.splits;

  struct item_t { int b, kvh, split; };
  auto item_of = [&](int w) -> item_t {
    item_t it;
    const int w2 = w < n_items ? w : n_items - 1;          // beyond the end: any valid item (its loads are not issued)
    it.b = w2 / per_b;
    const int r = w2 - it.b * per_b;
    it.kvh = r / p.splits;
    it.split = r - it.kvh * p.splits;
    return it;
  };
  // The workgroup's steps: all passes of its first item (number blockIdx.x of the launch), then of the item
  // `stride` further on, and so on; a step is kept as (item number, pass) and advanced without a division.
  struct step_t { int w, pass; };
  auto after = [&](const step_t& st) -> step_t {
    return st.pass + 1 < n_pass ? step_t{st.w, st.pass + 1} : step_t{st.w + stride, 0};
  };
  // Where this wavefront's chunk of a step lies, given the sequence length:
  struct plan_t { item_t it; dec_place pl; bool has; };
  auto plan_of = [&](const step_t& st, int len) -> plan_t {
    plan_t pn;
    const int w = st.w, pass = st.pass;
    pn.it = item_of(w);
    const dec_row row = dec_row_of(p, len);
    const int slot = (wave + NW * pass) * p.splits + pn.it.split;
    pn.pl = dec_place_of(p, row, slot < row.n_slots ? slot : 0);
    pn.has = w < n_items && slot < row.n_slots && pn.pl.n_tok > 0;
    return pn;
  };
  auto page_ptr = [&](const plan_t& pn) -> const int32_t* {
    return p.block_table ? p.block_table + (int64_t)pn.it.b * p.table_stride + pn.pl.blk : p.kv_len;
  };

  // the scalar pipeline: plan and page of the step after this one, length of the one after that
  step_t st0{(int)blockIdx.x, 0};                         // the current step, and the three after it
  step_t st1 = after(st0), st2 = after(st1), st3 = after(st2);
  plan_t cur = plan_of(st0, p.kv_len[item_of(st0.w).b]);
  int cur_page = *page_ptr(cur);
  plan_t nxt = plan_of(st1, p.kv_len[item_of(st1.w).b]);
  int nxt_page = *page_ptr(nxt);
  int len2 = p.kv_len[item_of(st2.w).b];

  dec_chunk<D> c;
  bf16x8 qf[D / 32];
  auto request = [&](const plan_t& pn, int page) {
    const int lane = dec_lane_now(), g = lane & 15, q4 = lane >> 4;
    dec_load_q<D>(qf, p, pn.it.b, pn.it.kvh, g, q4);
    const int64_t off = dec_chunk_offset(p, pn.it.b, pn.it.kvh, pn.pl, page, D);
    dec_issue<D>(c, p.k + off, p.v + off, pn.has ? pn.pl.n_tok : 0, g, q4);   // no tokens: no loads
  };
  request(cur, cur_page);

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 O[8];
  int n = 0;                                              // items finished so far: selects the LDS buffer
  for (; st0.w < n_items; st0 = st1, st1 = st2, st2 = st3, st3 = after(st3)) {
    const int pass = st0.pass;
    // ---- this wavefront's chunk of the step ----
    if (pass == 0) {
      m_run = -INFINITY; l_run = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) O[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    {
      const int q4 = dec_lane_now() >> 4;
      if (cur.has) dec_consume<D>(c, qf, cur.pl.n_tok, p.c2, q4, m_run, l_run, O);
    }
    const bool last_pass = pass == n_pass - 1;
    const int buf = n & 1;
    float* s_o = s_o_dyn + (size_t)buf * (dec_o_bytes<D>(p.G) / sizeof(float));
    if (last_pass) {
      const int lane = dec_lane_now(), g = lane & 15, q4 = lane >> 4;
      float l_all = l_run + __shfl_xor(l_run, 16);
      l_all += __shfl_xor(l_all, 32);
      if (g < p.G) {
        if (q4 == 0) { s_m[buf][wave][g] = m_run; s_l[buf][wave][g] = l_all; }
        dec_stash<D>(s_o, wave, p.G, g, q4, O);
      }
    }
    // ---- the next step's bytes are requested before this item is merged ----
    const item_t done = cur.it;
    cur = nxt; cur_page = nxt_page;
    request(cur, cur_page);
    nxt = plan_of(st2, len2);
    nxt_page = *page_ptr(nxt);
    len2 = p.kv_len[item_of(st3.w).b];
    if (!last_pass) continue;
    __syncthreads();     // the item's partials are in LDS; the other buffer is free again (its readers passed here)
    ++n;

    for (int e = wave * 64 + dec_lane_now(); e < p.G * D; e += 64 * NW) {
      const int gg = e / D, d = e % D;
      float M = -INFINITY;
#pragma unroll
      for (int wv = 0; wv < NW; ++wv) M = fmaxf(M, s_m[buf][wv][gg]);
      float L = 0.f, acc = 0.f;
#pragma unroll
      for (int wv = 0; wv < NW; ++wv) {
        const float wt = s_l[buf][wv][gg] > 0.f ? __builtin_amdgcn_exp2f(s_m[buf][wv][gg] - M) : 0.f;
        L = fmaf(wt, s_l[buf][wv][gg], L);
        acc = fmaf(wt, s_o[dec_o_at<D>(wv, p.G, gg, d)], acc);
      }
      const int h = done.kvh * p.G + gg;
      if (p.splits == 1) {
        p.o[((int64_t)done.b * p.hq + h) * D + d] = (__bf16)(acc / L);      // L > 0: chunk 0 of the row is never empty
        if (p.lse && d == 0) p.lse[(int64_t)done.b * p.hq + h] = (M + log2f(L)) * 0.69314718055994530942f;
      } else {
        float* part = p.partials + (((int64_t)done.b * p.hq + h) * p.splits + done.split) * (D + 2);
        part[d] = acc;
        if (d == 0) { part[D] = M; part[D + 1] = L; }                        // an idle split leaves M = -inf, L = 0
      }
    }
  }
}

// Merges the partials of the splits: one wavefront per (sequence, query head).  The loads of
// eight splits are issued together so that their latencies overlap.
template <int D>
__global__ __launch_bounds__(64) void pa_decode_merge_kernel(dec_params p) {
  constexpr int DPL = D / 64;
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const float* part = p.partials + ((int64_t)b * p.hq + h) * p.splits * (D + 2);
  float M = -INFINITY, L = 0.f;
  float acc[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) acc[e] = 0.f;
  for (int s0 = 0; s0 < p.splits; s0 += 8) {
    float m8[8], l8[8], o8[8][DPL];
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const int s = s0 + x < p.splits ? s0 + x : p.splits - 1;    // clamp: stay inside the row of partials
      const float* ps = part + (int64_t)s * (D + 2);
      m8[x] = ps[D];
      l8[x] = s0 + x < p.splits ? ps[D + 1] : 0.f;
#pragma unroll
      for (int e = 0; e < DPL; ++e) o8[x][e] = ps[lane + 64 * e];
    }
    float Mn = M;
#pragma unroll
    for (int x = 0; x < 8; ++x) if (l8[x] > 0.f) Mn = fmaxf(Mn, m8[x]);
    const float resc = L > 0.f ? __builtin_amdgcn_exp2f(M - Mn) : 0.f;
    L *= resc;
#pragma unroll
    for (int e = 0; e < DPL; ++e) acc[e] *= resc;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      if (l8[x] > 0.f) {                                          // idle splits wrote no outputs
        const float wt = __builtin_amdgcn_exp2f(m8[x] - Mn);
        L = fmaf(wt, l8[x], L);
#pragma unroll
        for (int e = 0; e < DPL; ++e) acc[e] = fmaf(wt, o8[x][e], acc[e]);
      }
    }
    M = Mn;
  }
#pragma unroll
  for (int e = 0; e < DPL; ++e) p.o[((int64_t)b * p.hq + h) * D + lane + 64 * e] = (__bf16)(acc[e] / L);
  if (p.lse && lane == 0) p.lse[(int64_t)b * p.hq + h] = (M + log2f(L)) * 0.69314718055994530942f;
}

}  // namespace

// Workgroups per (sequence, KV head).  A workgroup has all loads of eight 64-token chunks in
// flight at once; a second pass over further chunks would pay the memory latency again, so a row
// with more chunks is cut into several workgroups whose partials a small second kernel merges.
// Small batches are cut further so that more of the 256 compute units pull on the memory system.
int32_t pa_decode_splits(const powattn_pattern* pat, int32_t batch, int32_t hkv, int64_t capacity) {
  const int32_t mk = powattn_max_k(pat, capacity);
  if (mk < 1) return 0;
  const int64_t slots = (int64_t)mk * (pat->block / CH);
  const int64_t base = (int64_t)batch * hkv;
  int64_t s = (slots + NW - 1) / NW;                 // one pass per workgroup
  if (s > 8) s = 8;
  if (base * s < 256) {                              // not enough workgroups to cover the chip
    int64_t want = (256 + base - 1) / base;
    const int64_t cap = slots / 2 > 1 ? slots / 2 : 1;
    if (want > cap) want = cap;
    if (want > s) s = want;
  }
  if (s > 1024) s = 1024;
  return (int32_t)s;
}

// Workspace of a decode call: the generation numbers of the (sequence, KV head) pairs (one 32-bit word each,
// padded to 256 bytes), then room for the partial results as 8-byte packets (the float form of the two-kernel
// merge uses the first half of it).
size_t pa_decode_workspace_layout(int32_t batch, int32_t hq, int32_t hkv, int32_t head_dim, int32_t n_split, size_t* header_bytes) {
  const size_t hdr = ((size_t)batch * hkv * sizeof(uint32_t) + 255) & ~(size_t)255;
  if (header_bytes) *header_bytes = hdr;
  const size_t partials = (size_t)batch * hq * n_split * (size_t)(head_dim + 2) * sizeof(uint64_t);
  return hdr + ((partials + 255) & ~(size_t)255);
}

// ---- the library's own scratch buffer, for callers that cannot allocate a workspace ----
// One array per GPU, held until the process ends; its address on a device is looked up once, with that device
// current, and kept.  The array's name is a host-side handle only: device code and HIP calls get the looked-up
// pointer.  Zero when the module is loaded, which the merge protocol above does not even need.
static __device__ __align__(256) unsigned char scratch[POWATTN_STATIC_SCRATCH_BYTES];

int pa_decode_scratch(void** ptr_out, size_t* bytes_out) {
  static std::atomic<void*> dev_ptr[64];           // per device; null = not looked up yet
  int dev = 0;
  pa_current_device(&dev, nullptr);
  void* ptr = dev_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return pa_note_hip(e);
    if (!ptr) return pa_note_hip(hipErrorInvalidSymbol);
    dev_ptr[dev].store(ptr, std::memory_order_release);   // threads that race here store the same address
  }
  *ptr_out = ptr;
  *bytes_out = sizeof(scratch);
  return POWATTN_OK;
}

int pa_launch_decode_bf16(const pa_decode_args& a) {
  if (a.n_split < 1) return POWATTN_UNSUPPORTED;
  if (a.hkv > 65535 || a.batch > 65535 || a.hq > 65535 * 16) return POWATTN_UNSUPPORTED;
  dec_params p;
  p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.kv_len = a.kv_len;
  p.o = (__bf16*)a.o; p.lse = a.lse;
  size_t hdr = 0;
  pa_decode_workspace_layout(a.batch, a.hq, a.hkv, a.head_dim, a.n_split, &hdr);
  p.gen = (uint32_t*)a.workspace;
  p.packets = (uint64_t*)((char*)a.workspace + hdr);
  p.partials = (float*)((char*)a.workspace + hdr);
  p.capacity = a.capacity;
  p.B = a.pat.block; p.W = a.pat.window; p.S = a.pat.sink; p.flags = a.pat.flags;
  p.hq = a.hq; p.hkv = a.hkv; p.G = a.hq / a.hkv; p.splits = a.n_split; p.subs = a.pat.block / CH;
  p.subs_magic = p.subs > 1 ? (uint32_t)(((1ull << 32) + p.subs - 1) / p.subs) : 0u;
  p.c2 = a.scale * 1.44269504088896340736f;
  p.block_table = a.block_table; p.table_stride = a.table_stride; p.n_pages = a.n_pages;
  // few enough splits that every workgroup can afford to read all the others' partials: they merge among
  // themselves; otherwise the merge kernel follows
  p.fused = (a.n_split > 1 && a.n_split <= MAX_FUSED_SPLITS) ? 1 : 0;
  int n_cu = 1;
  pa_current_device(nullptr, &n_cu);
  // As many work items as compute units, or more: persistent workgroups that keep bytes in flight across items.
  // With at least one (sequence, KV head) pair per compute unit a pair is one item, walked in passes of NW chunks, and the
  // outputs are written by the same kernel; with fewer pairs but still four (sequence, KV head, split) items per
  // compute unit the splits stay (one pass each, more items to balance) and the merge kernel follows.
  {
    const int64_t pairs = (int64_t)a.batch * a.hkv;
    const int64_t max_slots = (int64_t)powattn_max_k(&a.pat, a.capacity) * p.subs;
    int stream_splits = 0;
    if (pairs >= (int64_t)n_cu) stream_splits = 1;
    else if (pairs * a.n_split >= 4 * (int64_t)n_cu && max_slots <= (int64_t)a.n_split * NW) stream_splits = a.n_split;
    const int64_t items = pairs * stream_splits;
    if (stream_splits > 0 && items <= 0x7fffffff / 4 && max_slots <= 0x7fffffff / 4) {
      p.fused = 0;
      p.splits = stream_splits;
      const int n_pass = (int)((max_slots + (int64_t)stream_splits * NW - 1) / ((int64_t)stream_splits * NW));
      const size_t lds2 = 2 * (a.head_dim == 128 ? dec_o_bytes<128>(p.G) : dec_o_bytes<64>(p.G));   // at most 144 KB
      static std::atomic<unsigned long long> attr_done[2];
      const int which = a.head_dim == 128 ? 0 : 1;
      const void* fn = which == 0 ? reinterpret_cast<const void*>(&pa_decode_stream_kernel<128>)
                                  : reinterpret_cast<const void*>(&pa_decode_stream_kernel<64>);
      if (int st = pa_allow_dynamic_lds(fn, 2 * (which == 0 ? dec_o_bytes<128>(MAXG) : dec_o_bytes<64>(MAXG)), attr_done[which])) return st;
      const dim3 pgrid((uint32_t)n_cu);
      if (a.head_dim == 128)
        hipLaunchKernelGGL((pa_decode_stream_kernel<128>), pgrid, dim3(64 * NW), lds2, a.stream, p, (int)items, n_pass);
      else
        hipLaunchKernelGGL((pa_decode_stream_kernel<64>), pgrid, dim3(64 * NW), lds2, a.stream, p, (int)items, n_pass);
      int st = pa_note_hip(hipGetLastError());
      if (st != POWATTN_OK || stream_splits == 1) return st;
      dim3 mgrid((uint32_t)a.hq, (uint32_t)a.batch);
      if (a.head_dim == 128)
        hipLaunchKernelGGL((pa_decode_merge_kernel<128>), mgrid, dim3(64), 0, a.stream, p);
      else
        hipLaunchKernelGGL((pa_decode_merge_kernel<64>), mgrid, dim3(64), 0, a.stream, p);
      return pa_note_hip(hipGetLastError());
    }
  }
  dim3 grid((uint32_t)a.n_split, (uint32_t)a.hkv, (uint32_t)a.batch);
  const size_t lds = a.head_dim == 128 ? dec_o_bytes<128>(p.G) : dec_o_bytes<64>(p.G);   // at most 72 KB (G <= 16)
  {
    static std::atomic<unsigned long long> attr_done[2];
    const int which = a.head_dim == 128 ? 0 : 1;
    const void* fn = which == 0 ? reinterpret_cast<const void*>(&pa_decode_kernel<128>)
                                : reinterpret_cast<const void*>(&pa_decode_kernel<64>);
    if (int st = pa_allow_dynamic_lds(fn, which == 0 ? dec_o_bytes<128>(MAXG) : dec_o_bytes<64>(MAXG), attr_done[which])) return st;
  }
  if (a.head_dim == 128)
    hipLaunchKernelGGL((pa_decode_kernel<128>), grid, dim3(64 * NW), lds, a.stream, p);
  else
    hipLaunchKernelGGL((pa_decode_kernel<64>), grid, dim3(64 * NW), lds, a.stream, p);
  int st = pa_note_hip(hipGetLastError());
  if (st != POWATTN_OK || a.n_split == 1 || p.fused) return st;
  dim3 mgrid((uint32_t)a.hq, (uint32_t)a.batch);
  if (a.head_dim == 128)
    hipLaunchKernelGGL((pa_decode_merge_kernel<128>), mgrid, dim3(64), 0, a.stream, p);
  else
    hipLaunchKernelGGL((pa_decode_merge_kernel<64>), mgrid, dim3(64), 0, a.stream, p);
  return pa_note_hip(hipGetLastError());
}
