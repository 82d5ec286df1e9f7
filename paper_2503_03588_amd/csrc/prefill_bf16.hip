// bf16 prefill on the gfx950 matrix cores: Equation 1 (Section 3.1) over the
// key blocks listed for each query block (Algorithm 1 lifted to blocks), as a
// flash-style online softmax with fp32 accumulation.
//
// Decomposition.  A work item is one (batch, KV head, query block) and up to NW
// "tasks"; a task is one query head of the GQA group x 32 consecutive query
// tokens, and belongs to one wavefront.  A workgroup is persistent: it walks
// through its share of the work items, and the K/V tile stream, the block list
// and the Q rows of the next item are fetched while the current one computes
// (a query block attends only a dozen key blocks, so an item lasts some tens of
// microseconds and three dependent trips to memory at its start would cost a
// sixth of it).  All wavefronts of the workgroup share the K/V tiles staged in
// LDS, which is what lifts the arithmetic intensity: a 64-key tile is read from
// HBM/L2 once per workgroup and used by every head of the group.
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
// rescaling of O a rare branch at its end), written in the order it is to be
// issued, with a scheduling barrier after every matrix instruction.  A SIMD
// issues about one instruction of any kind every 4 to 5 cycles, whichever of its
// wavefronts it comes from, and a matrix instruction keeps the matrix core busy
// for 32: the step is bound by its instruction count (about ten per matrix
// instruction), so waits are shared by pairs of matrix instructions, addresses
// are immediates and the tile copies ride along in the same stream.
//
// Memory pipeline.  K/V tiles travel global -> LDS asynchronously
// (global_load_lds_dwordx4, no registers in between) into a ring of NS stages;
// a wavefront waits on its own loads with s_waitcnt vmcnt(n) and one barrier
// per tile makes the stage visible and frees the oldest one.  One copy
// instruction moves 1 KB (RPI consecutive rows); inside that kilobyte the lanes
// are permuted so that it lands chunk-major (16-byte chunk c of row a at slot
// c*RPI + a), and consecutive kilobytes are 16*RPI bytes apart.  Fragment reads
// are then free of bank conflicts and every fragment address is one per-lane
// base plus an immediate offset.
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
  int32_t max_k, nb, B, hq, hkv, G, dense, batch;
  int32_t subs;      // 64-key tiles per block
  int32_t tasks;     // G * B / 32
  int32_t chunks;    // workgroups per (batch, kv head, query block)
  int32_t per_xcd;   // work items per XCD partition
  int32_t xcd_split; // sequences of different lengths, one or two KV heads: XCDs that share a KV head's items (else 0)
  int64_t per_kvh;   // ... and the items of one KV head
  int32_t chain;     // items may be chained in persistent workgroups
  int64_t total_wg;
  int64_t N;         // keys in the context: query q_start + r attends keys <= q_start + r, all of them < N
  int64_t q_start;   // position of the first query row of Q/O (anywhere inside block i0); 0 for a whole-sequence prefill
  int64_t q_rows;    // rows of Q/O per head (N - q_start)
  int64_t kv_rows;   // rows per (batch, KV head) slab of K/V (N, or the capacity of a cache)
  int32_t i0;        // first query block: q_start / B
  float c2;          // softmax scale * log2(e)
  const int32_t* seq_len;   // padded batch of sequences of different lengths: device array [batch]; N is then the padded length
  const int32_t* q_start_dev;   // with seq_len: every sequence's own first query position, device array [batch] (seq_len[b]
                                // is then the number of its query rows); null: all sequences start at 0
  const int32_t* block_table;   // paged cache: device [batch, table_stride], page of every block; k, v are the page pools
  int32_t table_stride, n_pages;
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
// the LDS offset and is declared as clobbered.
__device__ __forceinline__ void async_copy16(const void* sbase, uint32_t voff, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_off) : "memory", "m0");
}
// the same with the LDS offset given as a scalar base plus a constant
template <int OFF>
__device__ __forceinline__ void async_copy16_at(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base), "n"(OFF) : "memory", "scc", "m0");
}

// a wavefront-uniform pointer, forced into scalar registers
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* ptr) {
  const uint64_t u = (uint64_t)(uintptr_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return (const T*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // s_waitcnt vmcnt(N) only
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// DENSE: the implicit list {0..i} instead of a block list.  CHAIN: the launch chains work items in persistent
// workgroups (two half-size tile tables, list rows prefetched); otherwise one workgroup per item.  VARLEN: every
// sequence of the batch has its own length, read from device memory; the work items are numbered as if all had the
// padded length, and a workgroup passes over the items of query blocks that a sequence does not have.  PAGED: K and V
// are pools of pages of one block each; the tile table then also holds every tile's first row in the pool, looked up
// in the sequence's block table when the table is written (explicit lists, chained items only).
template <int D, int NW, int NS, bool DENSE, bool CHAIN, bool VARLEN, bool PAGED>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void pa_prefill_bf16_kernel(bf16_params p) {
  constexpr int ROWB = 2 * D;        // bytes per K/V row
  constexpr int CPR = D / 8;         // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;      // rows covered by one wavefront-wide copy instruction
  constexpr int IPT = KT / RPI;      // copy instructions per K (or V) tile
  constexpr int IPW = IPT / NW;      // ... per wavefront
  constexpr int LPT = 2 * IPW;       // copies per wavefront per tile (K and V)
  constexpr int SRB = 1024 + 16 * RPI;       // LDS distance between the kilobytes of consecutive copy instructions
  constexpr int TILEB = IPT * SRB;   // LDS bytes of a K (or V) tile
  constexpr int STAGEB = 2 * TILEB;  // K then V
  constexpr int NC = D / 16;         // 16-wide steps of the head dimension
  constexpr int ND = D / 32;         // 32-row tiles of O^T
  constexpr int MIN_STEPS = NS - 1;  // an item that is followed by another one lasts at least this many steps
  static_assert(IPT % NW == 0, "tile copies must divide over the wavefronts");
  static_assert(NS == 4 && (NS - 1) * LPT + NC + 1 < 64, "outstanding copies must fit the vmcnt counter");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;
  __shared__ int s_tile[TILE_CAP];     // first key of every tile of an item; two halves when items are chained
  __shared__ int s_cnt[2][2];          // per table: tiles in total, tiles before the diagonal block
  __shared__ int s_raw[NW][64];        // per wavefront: the raw list row of the item after next (entry 63 = its length)

  const int pid = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, and the compiler knows it
  const int ln = lane & 31, hh = lane >> 5;
  const int slices = p.B / QW;
  // Which task of a work item this wavefront takes.  Wavefronts w and w+4 share a SIMD; the tasks of the lower
  // half of a query block stop one diagonal tile before those of the upper half.  With four 32-query slices per
  // head (blocks of 128 keys) tasks w and w+4 are the same slice of two heads, and whole SIMDs would idle in the
  // item's last step while the others carry two wavefronts; the tasks are dealt so that every SIMD gets one
  // wavefront of either kind (wavefront w: head (w>>1)&1, slice (w&1) + 2(w>>2)).
  const int wtask = (NW == 8 && slices == 4) ? ((wave & 1) | (((wave >> 2) & 1) << 1) | (((wave >> 1) & 1) << 2)) : wave;

  // ---- this workgroup's work items: item k is number xcd*per_xcd + cuslot + nslots*k of the launch, so that
  // the workgroups of one XCD (one L2) work on neighbouring query blocks at any time ----
  const int xcd = pid & 7, cuslot = pid >> 3, nslots = (int)(gridDim.x >> 3);
  int n_raw = 0;                       // item numbers that fall to this workgroup
  int64_t first_item = (int64_t)xcd * p.per_xcd + cuslot;
  int item_step = nslots;
  if (VARLEN && p.xcd_split > 1) {
    // Sequences of different lengths and 1 or 2 KV heads: the XCDs that share a KV head take its item numbers
    // in turn (number m goes to XCD m mod split of the head's group) instead of a contiguous part each, which would
    // be some of the sequences and as much work as those happen to have.
    const int sub = xcd % p.xcd_split;
    const int64_t m0 = sub + (int64_t)p.xcd_split * cuslot;
    item_step = p.xcd_split * nslots;
    if (m0 < p.per_kvh) n_raw = (int)((p.per_kvh - m0 + item_step - 1) / item_step);
    first_item = (int64_t)(xcd / p.xcd_split) * p.per_kvh + m0;
  } else {
    int64_t lim = p.total_wg - (int64_t)xcd * p.per_xcd;
    if (lim > p.per_xcd) lim = p.per_xcd;
    if (lim > cuslot) n_raw = (int)((lim - cuslot + nslots - 1) / nslots);
  }
  if (n_raw == 0) return;
  constexpr bool chained = CHAIN;      // tables in halves, list rows prefetched
  constexpr int tab_half = CHAIN ? (PAGED ? TILE_CAP / 4 : TILE_CAP / 2) : 0;
  constexpr int PHYS = TILE_CAP / 2;   // paged: entry e's first pool row sits at s_tile[PHYS + e]
  static_assert(!PAGED || (CHAIN && !DENSE), "paged caches: explicit lists, chained items");

  // Items are numbered L = ((b*hkv + kvh)*nb + r)*chunks + chunk with r counting query blocks from the last one
  // down (longest rows first, which matters for the dense list); with sequences of different lengths
  // L = ((kvh*batch + b)*nb + r)*chunks + chunk, so that the contiguous share of an XCD spans all sequences (one KV
  // head each when there are eight) and the XCDs finish together whatever the mix of lengths.  The first item is decoded by division, the
  // following ones by adding the stride nslots digit by digit with carries: all scalar, no division in the loop.
  struct item_t { int chunk, r, kvh, b, i, subs_diag, n, qs; };   // n: keys (= tokens) of the item's sequence; qs: its first query
  auto finish_item = [&](item_t& it) {
    it.i = p.i0 + p.nb - 1 - it.r;
    if (VARLEN) {                      // uniform over the workgroup: scalar loads; values outside [0, N] are clamped
      int qs = 0;
      if (p.q_start_dev) {
        qs = p.q_start_dev[it.b];
        qs = qs < 0 ? 0 : (qs > (int)p.N ? (int)p.N : qs);
        it.i += qs / p.B;              // the launch numbers a sequence's query blocks from its own first one
      }
      const int n = p.seq_len[it.b];
      it.qs = qs;
      int room = (int)p.N - qs;        // rows that fit the context, and the slab of Q/O
      if ((int64_t)room > p.q_rows) room = (int)p.q_rows;
      it.n = qs + (n < 0 ? 0 : (n > room ? room : n));
    }
    // tiles of the diagonal block needed by any wavefront of the item
    int last_task = it.chunk * NW + NW - 1;
    if (last_task > p.tasks - 1) last_task = p.tasks - 1;
    const int max_sl = (last_task / slices > (it.chunk * NW) / slices) ? slices - 1 : last_task % slices;
    it.subs_diag = (max_sl * QW + QW - 1) / KT + 1;
  };
  auto digits = [&](uint32_t L) -> item_t {
    item_t it;
    it.chunk = (int)(L % (uint32_t)p.chunks); L /= (uint32_t)p.chunks;
    it.r = (int)(L % (uint32_t)p.nb); L /= (uint32_t)p.nb;
    if (VARLEN) {                      // the KV head is the slowest digit: an XCD's share then holds every sequence
      it.b = (int)(L % (uint32_t)p.batch);
      it.kvh = (int)(L / (uint32_t)p.batch);
    } else {
      it.kvh = (int)(L % (uint32_t)p.hkv);
      it.b = (int)(L / (uint32_t)p.hkv);
    }
    it.i = 0; it.subs_diag = 0; it.n = 0; it.qs = 0;
    return it;
  };
  const item_t stride = digits((uint32_t)item_step);
  auto next_item = [&](const item_t& cur) -> item_t {
    item_t it = cur;
    it.chunk += stride.chunk; if (it.chunk >= p.chunks) { it.chunk -= p.chunks; ++it.r; }
    if (VARLEN) {
      it.r += stride.r;       if (it.r >= p.nb) { it.r -= p.nb; ++it.b; }
      it.b += stride.b;       if (it.b >= p.batch) { it.b -= p.batch; ++it.kvh; }
      it.kvh += stride.kvh;
    } else {
      it.r += stride.r;       if (it.r >= p.nb) { it.r -= p.nb; ++it.kvh; }
      it.kvh += stride.kvh;   if (it.kvh >= p.hkv) { it.kvh -= p.hkv; ++it.b; }
      it.b += stride.b;
    }
    finish_item(it);
    return it;
  };
  item_t it = stride, it1 = stride, it2 = stride;   // the current item, the next one, the one after (set below)
  // Sequences of different lengths: an item exists when its query block starts inside its sequence.  raw2 is the
  // position of it2 among this workgroup's item numbers; next_valid steps to the next existing item (finish_item
  // is only ever called for item numbers of the launch, so the length look-up stays inside the array).
  int n_items = n_raw, raw2 = 0;
  // keys of an item's sequence (one value for the whole launch unless the sequences have lengths of their own)
  auto keys_of = [&](const item_t& x) -> int { return VARLEN ? x.n : (int)p.N; };
  auto exists = [&](const item_t& x) -> bool { return !VARLEN || (x.n > x.qs && (int64_t)x.i * p.B < x.n); };
  // position of the first row of Q/O
  auto qs_of = [&](const item_t& x) -> int64_t { return VARLEN ? (int64_t)x.qs : p.q_start; };
  auto next_valid = [&](const item_t& cur, int& raw) -> item_t {
    item_t x = cur;
    while (raw + 1 < n_raw) {
      ++raw;
      x = next_item(x);
      if (exists(x)) return x;
    }
    raw = n_raw;
    return cur;                        // none left: never used as an item (the loop below counts the existing ones)
  };

  // ---- tile tables (explicit lists only) ----
  // Writes the table of an item from its list row: lane e holds entry e (j), n entries in all; the tiles of the
  // blocks before the diagonal one in list order (ranks by a prefix count over the lanes), then the diagonal ones.
  // Called by the first wavefront, once per 64 entries.
  // (paged: `page` is the page of the lane's block j, `page_i` that of the diagonal block)
  auto pool_row = [&](const item_t& it, int page) -> int {   // first row of a page's slab for the item's KV head
    page = page < 0 ? 0 : (page >= p.n_pages ? p.n_pages - 1 : page);
    return (page * p.hkv + it.kvh) * p.B;
  };
  auto table_rows = [&](int tab, const item_t& it, int j, int page, int& blocks, bool& has_diag) {
    const bool valid = j >= 0 && j < it.i;                  // not padding, causal, not the diagonal block
    const uint64_t vm = __builtin_amdgcn_ballot_w64(valid);
    has_diag = has_diag || __builtin_amdgcn_ballot_w64(j == it.i) != 0;
    const int rank = blocks + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(vm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vm, 0));
    if (valid)
      for (int u = 0; u < p.subs; ++u) {
        s_tile[tab * tab_half + rank * p.subs + u] = j * p.B + u * KT;
        if (PAGED) s_tile[PHYS + tab * tab_half + rank * p.subs + u] = pool_row(it, page) + u * KT;
      }
    blocks += __builtin_popcountll(vm);
  };
  auto table_finish = [&](int tab, const item_t& it, int page_i, int blocks, bool has_diag) {
    int w = blocks * p.subs;
    if (lane == 0) s_cnt[tab][1] = w;
    if (has_diag) {
      if (lane < it.subs_diag) {
        s_tile[tab * tab_half + w + lane] = it.i * p.B + lane * KT;
        if (PAGED) s_tile[PHYS + tab * tab_half + w + lane] = pool_row(it, page_i) + lane * KT;
      }
      w += it.subs_diag;
    }
    if (lane == 0) s_cnt[tab][0] = w;
    if (w == 0 && lane == 0) {                              // an empty row still has an entry to look up
      s_tile[tab * tab_half] = 0;
      if (PAGED) s_tile[PHYS + tab * tab_half] = 0;
    }
  };
  // the page of block j of the item's sequence (any j: the index is clamped into the table)
  auto page_of = [&](const item_t& it, int j) -> int {
    if (!PAGED) return 0;
    j = j < 0 ? 0 : (j >= p.table_stride ? p.table_stride - 1 : j);
    return p.block_table[(int64_t)it.b * p.table_stride + j];
  };
  auto table_from_memory = [&](int tab, const item_t& it) {          // first wavefront
    int n = p.kv_cnt[it.i];
    if (n > p.max_k) n = p.max_k;
    n = __builtin_amdgcn_readfirstlane(n);
    int blocks = 0;
    bool has_diag = false;
    for (int base = 0; base < n; base += 64) {
      const int e = base + lane;
      const int j = e < n ? p.kv_idx[(int64_t)it.i * p.max_k + e] : -1;
      table_rows(tab, it, j, page_of(it, j), blocks, has_diag);
    }
    table_finish(tab, it, page_of(it, it.i), blocks, has_diag);
  };
  // first wavefront; the row was copied earlier into s_raw[0].  Paged: the pages of the row's blocks are requested by
  // row_pages at the start of an item and used here, after the Q fragments have been arranged.
  auto row_entry = [&]() -> int {
    int n = __builtin_amdgcn_readfirstlane(s_raw[0][63]);
    if (n > p.max_k) n = p.max_k;
    const int raw = s_raw[0][lane];
    return lane < n ? raw : -1;
  };
  auto table_from_row = [&](int tab, const item_t& it, int page, int page_i) {
    const int j = row_entry();
    int blocks = 0;
    bool has_diag = false;
    table_rows(tab, it, j, page, blocks, has_diag);
    table_finish(tab, it, page_i, blocks, has_diag);
  };
  // Asynchronous copy of the list row of item k into this wavefront's s_raw (every wavefront issues it, so
  // that all of them count the same number of outstanding copies; only the first one's copy is read).
  auto copy_row = [&](const item_t& it) {
    const int32_t* src = reinterpret_cast<const int32_t*>(p.k);      // dense: a dummy 4-byte read
    if (!DENSE) {
      const int e = lane < p.max_k ? lane : p.max_k - 1;
      src = lane == 63 ? p.kv_cnt + it.i : p.kv_idx + (int64_t)it.i * p.max_k + e;
    }
    const uint32_t dst = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)&s_raw[0][0] + wave * 256;
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(__builtin_amdgcn_readfirstlane(dst)) : "memory", "m0");
  };

  // ---- asynchronous tile copy: this wavefront's share of the tile starting at key0 into a ring stage ----
  // The tile's base address is scalar; a lane adds the byte offset of its row and chunk.
  const int cp_row = lane % RPI, cp_chunk = lane / RPI;   // lane l carries chunk l/RPI of row l%RPI of its kilobyte
  // A fill is prepared once (scalar part) and issued as LPT separate copies, so that a step can spread them
  // over its matrix instructions instead of queueing all wavefronts' copies behind one another after the barrier.
  const __bf16* f_kt = p.k;
  const __bf16* f_vt = p.v;
  int f_lim = 0;
  int c_n = 1;                         // keys of the sequence whose tiles the cursor (below) is copying
  uint32_t f_dst = 0;
  const uint32_t w_dst = __builtin_amdgcn_readfirstlane(lds0 + wave * IPW * SRB);   // this wavefront's share of stage 0
  int f_row[IPW];                                      // this lane's row in each of the wavefront's copy instructions
#pragma unroll
  for (int x = 0; x < IPW; ++x) f_row[x] = RPI * (wave * IPW + x) + cp_row;
  const uint32_t f_chunk = (uint32_t)cp_chunk << 4;
  auto fill_prep = [&](const __bf16* kbase, const __bf16* vbase, int key0, int phys0, uint32_t dst) {
    // ragged tail: rows beyond the sequence repeat its last row (they are masked, but must be finite)
    const int last = (VARLEN ? c_n : (int)p.N) - 1;   // of the sequence whose tiles the cursor is copying
    const int k0 = key0 < last ? key0 : last;
    f_lim = last - k0;
    // paged: the tile's rows in the pool (a tile that starts beyond the sequence lies in the page of its last key)
    const int64_t row0 = PAGED ? (int64_t)phys0 + (k0 - key0) : (int64_t)k0;
    // (scalar values may live in vector registers when scalar registers are short: pin the bases down)
    f_kt = uniform_ptr(kbase + row0 * D);
    f_vt = uniform_ptr(vbase + row0 * D);
    f_dst = dst;
  };
  auto fill_copy = [&](auto jc) {                      // copy j of LPT: instruction x = j/2 of this wavefront, K then V
    constexpr int j = decltype(jc)::value;
    int row = f_row[j >> 1];                           // rows RPI*inst .. +RPI-1 of the tile, inst = wave*IPW + j/2
    row = row < f_lim ? row : f_lim;
    const uint32_t voff = (uint32_t)row * ROWB | f_chunk;
    if (j & 1) async_copy16_at<(j >> 1) * SRB + TILEB>(f_vt, voff, f_dst);
    else async_copy16_at<(j >> 1) * SRB>(f_kt, voff, f_dst);
  };
  static_assert(LPT <= 8, "fill_part lists the copies");
  auto fill_part = [&](int j) {                        // j is a constant wherever this is called (unrolled loops)
    switch (j) {
      case 0: fill_copy(std::integral_constant<int, 0>{}); break;
      case 1: fill_copy(std::integral_constant<int, 1 % LPT>{}); break;
      case 2: fill_copy(std::integral_constant<int, 2 % LPT>{}); break;
      case 3: fill_copy(std::integral_constant<int, 3 % LPT>{}); break;
      case 4: fill_copy(std::integral_constant<int, 4 % LPT>{}); break;
      case 5: fill_copy(std::integral_constant<int, 5 % LPT>{}); break;
      case 6: fill_copy(std::integral_constant<int, 6 % LPT>{}); break;
      default: fill_copy(std::integral_constant<int, 7 % LPT>{}); break;
    }
  };

  // ---- the tile stream: a cursor runs NS-1 fills ahead of the compute, across item boundaries ----
  // An item that has a successor lasts at least MIN_STEPS steps (short rows are padded with fills that nobody
  // reads), so the cursor is never more than one item ahead and two tables are enough.
  int c_k = 0, c_pos = 0, c_ntiles = 0, c_steps = 0, c_last = 0;
  uint32_t c_dst = w_dst;       // this wavefront's share of the stage the next fill goes to
  uint32_t c_tab = 0;           // LDS address of the table the cursor reads
  int pref_key = 0;             // table entry of the cursor's position, read from LDS one fill ahead of its use
  int pref_phys = 0;            // paged: the same entry's first pool row
  const __bf16* c_kb = p.k;
  const __bf16* c_vb = p.v;
  auto cursor_enter = [&](int k, const item_t& it) {
    c_k = k; c_pos = 0;
    if (VARLEN) c_n = it.n;
    c_ntiles = DENSE ? it.i * p.subs + it.subs_diag : __builtin_amdgcn_readfirstlane(s_cnt[k & 1][0]);
    c_last = c_ntiles > 0 ? c_ntiles - 1 : 0;
    if (!DENSE) {
      c_tab = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)&s_tile[(k & 1) * tab_half]);
      pref_key = s_tile[(k & 1) * tab_half];
      if (PAGED) pref_phys = s_tile[PHYS + (k & 1) * tab_half];
    }
    c_steps = (k + 1 < n_items && c_ntiles < MIN_STEPS) ? MIN_STEPS : c_ntiles;
    if (!PAGED) {                // (paged: the pools' bases, set once)
      c_kb = p.k + (((int64_t)it.b * p.hkv + it.kvh) * p.kv_rows) * D;
      c_vb = p.v + (((int64_t)it.b * p.hkv + it.kvh) * p.kv_rows) * D;
    }
  };
  // Prepares the next fill of the stream.  After the end of the stream the fills go on, re-reading the last
  // tile of the last item into stages nobody reads: every step then issues the same number of copies, and
  // the waits can count them.  The table entry of a fill is read from LDS during the previous fill, so that
  // its latency is not exposed right after the step's barrier.
  auto next_fill = [&]() {
    if (c_pos >= c_steps && c_k + 1 < n_items)
      cursor_enter(c_k + 1, it1);      // the cursor is never more than one item ahead of the compute
    // Beyond the tiles of the row (padding steps, and after the end of the stream) the last tile is copied again.
    int key0;
    if (DENSE) key0 = (c_pos < c_last ? c_pos : c_last) * KT;
    else key0 = __builtin_amdgcn_readfirstlane(pref_key);
    fill_prep(c_kb, c_vb, key0, PAGED ? __builtin_amdgcn_readfirstlane(pref_phys) : 0, c_dst);
    c_dst = c_dst == w_dst + (NS - 1) * STAGEB ? w_dst : c_dst + STAGEB;
    ++c_pos;
    if (!DENSE) {
      const uint32_t at = c_tab + 4 * (uint32_t)(c_pos < c_last ? c_pos : c_last);
      pref_key = *reinterpret_cast<const __attribute__((address_space(3))) int*>((uintptr_t)at);
      if (PAGED) pref_phys = *reinterpret_cast<const __attribute__((address_space(3))) int*>((uintptr_t)(at + 4 * PHYS));
    }
  };
  auto fill_all = [&]() {
#pragma unroll
    for (int j = 0; j < LPT; ++j) fill_part(j);
  };

  // ---- Q^T fragments: lane = query column.  The contraction index of S^T = K Q^T may be permuted freely as long
  // as K and Q agree, and here 16-wide step c of lane half hh takes the d values 8(c + NC*hh) .. +7, so that a
  // lane's fragments are the D contiguous bytes at D*hh of its row.  They are loaded quad-wise: in load m the four
  // lanes of a quad read 64 contiguous bytes of ONE of the quad's four rows, and a 4x4 transpose inside the quad
  // (q_arrange) then hands every lane the pieces of its own row.  Loading row-per-lane (every lane 16 bytes of
  // its own row) costs the compute unit's address unit a cache-line look-up per lane: ~4 k cycles for the 64
  // loads of a workgroup, queued at every item boundary in front of the tile copies and the output stores.
  constexpr int QE = NC / 4;                 // 64-byte pieces per lane half of a row
  u32x4 qraw[NC];
  bf16x8 qf[NC];
  auto load_q = [&](const item_t& it) {
    const int task = it.chunk * NW + wtask;
    const bool act = task < p.tasks;
    const int g = act ? task / slices : 0, sl = act ? task % slices : 0;
    const int64_t tok0 = (int64_t)it.i * p.B + sl * QW + (ln & ~3);          // first row of this lane's quad
    const __bf16* qbase = p.q + (((int64_t)it.b * p.hq + it.kvh * p.G + g) * p.q_rows + (tok0 - qs_of(it))) * D
                          + (D / 2) * hh + 8 * (lane & 3);
#pragma unroll
    for (int m = 0; m < NC; ++m) {
      const int rho = m / QE, e = m % QE;
      const bool ok = act && tok0 + rho < keys_of(it) && tok0 + rho >= qs_of(it);   // (a chunk may start inside a block)
      qraw[m] = ok ? *reinterpret_cast<const u32x4*>(qbase + (int64_t)rho * D + 32 * e) : u32x4{0, 0, 0, 0};
    }
  };
  // qraw[rho*QE + e] of lane j (of its quad) is piece 4e + j of row rho; qf[4e + j'] of lane rho is that piece
  auto q_arrange = [&]() {
    const bool odd = lane & 1, upper = lane & 2;
    auto quad_xor1 = [](uint32_t x) -> uint32_t { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true); };
    auto quad_xor2 = [](uint32_t x) -> uint32_t { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true); };
#pragma unroll
    for (int e = 0; e < QE; ++e) {
      uint32_t c[4][4];
#pragma unroll
      for (int rho = 0; rho < 4; ++rho)
#pragma unroll
        for (int w = 0; w < 4; ++w) c[rho][w] = qraw[rho * QE + e][w];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        // stage 1: lanes i and i^1 trade c[k^1]; stage 2: lanes i and i^2 trade c[k^2] (all permutes evaluated
        // before any select: a lane can only be read while it is active)
        const uint32_t x0 = quad_xor1(c[0][w]), x1 = quad_xor1(c[1][w]), x2 = quad_xor1(c[2][w]), x3 = quad_xor1(c[3][w]);
        const uint32_t a0 = odd ? x1 : c[0][w], a1 = odd ? c[1][w] : x0;
        const uint32_t a2 = odd ? x3 : c[2][w], a3 = odd ? c[3][w] : x2;
        const uint32_t y0 = quad_xor2(a0), y1 = quad_xor2(a1), y2 = quad_xor2(a2), y3 = quad_xor2(a3);
        c[0][w] = upper ? y2 : a0; c[2][w] = upper ? a2 : y0;
        c[1][w] = upper ? y3 : a1; c[3][w] = upper ? a3 : y1;
      }
#pragma unroll
      for (int k2 = 0; k2 < 4; ++k2) {
        const u32x4 v4 = {c[k2][0], c[k2][1], c[k2][2], c[k2][3]};
        qf[4 * e + k2] = __builtin_bit_cast(bf16x8, v4);
      }
    }
  };

  // ---- start of the stream: tables of the first two items, fills 0..NS-2, Q of the first item ----
  it = digits((uint32_t)first_item);
  finish_item(it);
  if (VARLEN) {
    // count this workgroup's existing items, then set out on the first three
    n_items = exists(it) ? 1 : 0;
    {
      item_t x = it;
      for (int raw = 1; raw < n_raw; ++raw) { x = next_item(x); n_items += exists(x) ? 1 : 0; }
    }
    if (n_items == 0) return;
    if (!exists(it)) it = next_valid(it, raw2);
    it1 = next_valid(it, raw2);
    it2 = next_valid(it1, raw2);
  } else {
    it1 = next_item(it);
    it2 = next_item(it1);
  }
  if (!DENSE) {
    if (wave == 0) {
      table_from_memory(0, it);
      if (chained && n_items > 1) table_from_memory(1, it1);
    }
    __syncthreads();
  }
  cursor_enter(0, it);
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) { next_fill(); fill_all(); }
  load_q(it);

  // Per-lane LDS base addresses of the fragment reads: ka inside the stage whose K tile is multiplied next,
  // va inside the stage whose V tile is multiplied next; they are advanced in place from stage to stage.
  // K fragment (d-step c, key half rt) of lane (ln, hh): row 32rt + ln, chunk c + NC*hh (as the Q fragments).
  constexpr int K_C = 16 * RPI, K_RT = (32 / RPI) * SRB;                 // offsets per d-step and per key half
  const uint32_t ka0 = lds0 + (ln / RPI) * SRB + ((hh * NC * RPI + ln % RPI) << 4);
  // V^T fragment (16-key step kk, d tile dt): two transposing reads, rows 16kk + r4 and 16kk + r4 + 8,
  // chunk 4dt + x, 8-byte half lane&1
  constexpr int V_KK = (16 / RPI) * SRB, V_DT = 4 * RPI * 16, V_HI = (8 / RPI) * SRB;
  uint32_t va0;
  {
    const int r4 = 4 * hh + ((lane & 15) >> 2);              // row of the first read inside a 16-key step
    const int x = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1); // chunk inside the 32-wide d tile
    va0 = lds0 + TILEB + (r4 / RPI) * SRB + ((x * RPI + r4 % RPI) << 4) + 8 * (lane & 1);
  }
  // One scalar ring offset serves both: K(t+1) sits one stage after V(t), so ka moves on at the start of a step
  // and va catches up with it at the end.
  uint32_t ka = ka0, va = va0, ring_off = 0;
  auto advance_k = [&]() {
    ring_off = ring_off == (NS - 1) * STAGEB ? 0u : ring_off + STAGEB;
    ka = ka0 + ring_off;
  };
  auto advance_v = [&]() { va = va0 + ring_off; };

  // ---- pieces of the pipeline ----
  constexpr int NSLOT = 2 * NC + 4 * ND;   // matrix instructions per tile: 32 at head_dim 128, 16 at 64
  constexpr int VPS = 32 / NSLOT;          // the vector work of a tile is cut into 32 portions: portions per matrix instruction
  constexpr int PF = 2;                    // LDS reads are issued for a pair of matrix instructions at a time, one pair ahead
  const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  int q_in_blk = 0;                        // first query of this wavefront inside the block (per item)

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
  auto load_frag = [&](int slot) -> bf16x8 {
    if (slot < 2 * NC)
      return *reinterpret_cast<const lds_bf16x8*>((uintptr_t)(ka + (slot >> 1) * K_C + (slot & 1) * K_RT));
    const int kk = (slot - 2 * NC) / ND, dt = (slot - 2 * NC) % ND;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(va + kk * V_KK + dt * V_DT));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(va + kk * V_KK + dt * V_DT + V_HI));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // Q fragments and the first tiles must have arrived before the first item; waiting here, once, also tells
  // the compiler that none of its own loads is outstanding inside the loops, so that it does not add
  // full vmcnt(0) waits there (they would drain the asynchronous copies as well).
  wait_vmcnt<0>();
  __syncthreads();

  for (int k = 0; k < n_items; ++k) {
    const bool more = k + 1 < n_items;
    // ---- per-item geometry ----
    const int task = it.chunk * NW + wtask;
    const bool active = task < p.tasks;
    const int g = active ? task / slices : 0;
    const int sl = active ? task % slices : 0;
    const int h = it.kvh * p.G + g;
    q_in_blk = sl * QW;
    const int64_t q0 = (int64_t)it.i * p.B + q_in_blk;
    int n_tiles, n_before;
    if (DENSE) {
      n_before = it.i * p.subs;               // blocks 0..i-1 in full, then the needed part of block i
      n_tiles = n_before + it.subs_diag;
    } else {
      n_tiles = __builtin_amdgcn_readfirstlane(s_cnt[k & 1][0]);
      n_before = __builtin_amdgcn_readfirstlane(s_cnt[k & 1][1]);
    }
    const int n_steps = (more && n_tiles < MIN_STEPS) ? MIN_STEPS : n_tiles;
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

    // The Q rows requested during the previous item are needed from here on.  Touching them on every path
    // makes the compiler wait for them here, once, instead of guarding each later use inside the loops
    // with a wait that would also drain the asynchronous copies.
#pragma unroll
    for (int c = 0; c < NC; ++c) asm volatile("" : "+v"(qraw[c]));
    // paged: the pages of the next item's blocks are requested here and used below, behind the arranging of Q
    int nx_page = 0, nx_page_i = 0;
    if (PAGED && wave == 0 && k >= 1 && more) {
      nx_page = page_of(it1, row_entry());
      nx_page_i = page_of(it1, it1.i);
    }
    q_arrange();

    // ---- look-ahead: the table of the next item from its prefetched list row (the first two tables were
    // built above), and the copy of the row of the item after it ----
    if (chained) {
      if (!DENSE && wave == 0 && k >= 1 && more) table_from_row((k + 1) & 1, it1, nx_page, nx_page_i);
      copy_row(k + 2 < n_items ? it2 : it);
    }

    f32x16 O[ND];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;

    // ---- pipeline state: scores of the current tile, the probabilities of its first 16-key step, running (m, l) ----
    // The reference point m of the exponentials need not be the exact running maximum: any m gives the
    // same o and lse as long as exp2(s - m) stays in range.  It is raised only when a score exceeds it by
    // more than RESCALE_TAU (p <= 2^tau), which makes the rescaling of O (64 multiplies per lane) a
    // rare, wavefront-uniform branch instead of a per-tile cost.
    f32x16 Sc[2], Sd[2];     // scores of the current tile; the steps alternate between the two
    u32x4 P0;
    float m_run = -INFINITY, l_run = 0.f;
    if (n_my > 0) {
#pragma unroll
      for (int sl2 = 0; sl2 < 2 * NC; ++sl2)
        Sc[sl2 & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_frag(sl2), qf[sl2 >> 1],
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

    // Start of every step: the fill after this step's (it carries K of the next tile) has landed once at most
    // the one younger fill's copies are outstanding, plus, in the first two steps of an item, the list-row copy
    // issued at its start.  The barrier makes every wavefront's share visible and tells that everybody is done
    // with the stage of the previous step, which the fill prepared here overwrites.
    auto top = [&](int t) {
      if (chained && t < 2) wait_vmcnt<LPT + 1>(); else wait_vmcnt<LPT>();
      __syncthreads();
      next_fill();
    };

    // One step of the skewed loop.  Matrix instructions: the 2NC of S(t+1) = K(t+1) Q^T, then the 4ND of
    // O += V(t)^T P(t)^T.  Vector work, cut into 32 portions that are spread evenly over them: the
    // exponentials of elements 8..31 of S(t) (element rg feeds 16-key step rg/8 of the second product, so
    // each is ready before its step), then the column maximum of S(t+1) and the new reference point, then the
    // exponentials of elements 0..7 of S(t+1).  The source order IS the schedule: a scheduling barrier after
    // every matrix instruction keeps the compiler from regrouping the stream into a matrix phase and a
    // vector phase.  `masked` selects the variant that applies the causal mask to S(t+1).
    auto step = [&](int t, auto masked, f32x16 (&Sc)[2], f32x16 (&Sn)[2]) {
      constexpr bool MASKED = decltype(masked)::value;
      advance_k();               // K(t+1) sits one stage after V(t)
      top(t);
      bf16x8 fr[NSLOT];
      u32x4 Pk[4], Pn;
      Pk[0] = P0;
      float pe[32], pn[8];
      float rs = 0.f, rs_n = 0.f, mx = 0.f, m_new = 0.f, alpha = 1.f;
      bool raise = false;
#pragma unroll
      for (int s0 = 0; s0 < PF; ++s0) fr[s0] = load_frag(s0);
#pragma unroll
      for (int sl2 = 0; sl2 < NSLOT; ++sl2) {
        if (sl2 % 2 == 0 && sl2 + PF < NSLOT) { fr[sl2 + PF] = load_frag(sl2 + PF); fr[sl2 + PF + 1] = load_frag(sl2 + PF + 1); }
        // ---- one of the LPT copies of the fill, evenly spread ----
        if ((sl2 % (NSLOT / LPT)) == NSLOT / LPT / 2) fill_part(sl2 / (NSLOT / LPT));
        // ---- vector portions of this slot ----
#pragma unroll
        for (int vs = sl2 * VPS; vs < (sl2 + 1) * VPS; ++vs) {
          if (vs < 18) {
            // An exponential's result may not be read by the instruction right after it, so the sum and the
            // packing of an element trail its exponential by one element: the exponential ends the portion.
#pragma unroll
            for (int e = (4 * vs) / 3; e < (4 * (vs + 1)) / 3; ++e) {
              const int rg = 8 + e;
              if (rg > 8) {
                rs += pe[rg - 1];
                if (!(rg & 1)) Pk[(rg - 1) >> 3][((rg - 1) & 7) >> 1] = pack2(pe[rg - 2], pe[rg - 1]);
              }
              pe[rg] = pexp(Sc, rg, m_run);
            }
            if (MASKED && vs == 17) mask(Sn, (t + 1 - n_before) * KT);
          } else if (vs < 21) {
            constexpr int lo[3] = {0, 11, 22}, hi[3] = {11, 22, 32};
            if (vs == 18) {
              rs += pe[31];
              Pk[3][3] = pack2(pe[30], pe[31]);
              mx = Sn[0][0];
            }
#pragma unroll
            for (int rg = lo[vs - 18]; rg < hi[vs - 18]; ++rg) mx = fmaxf(mx, Sn[rg >> 4][rg & 15]);
          } else if (vs == 21) {
            mx = both_halves_max(mx) * p.c2;
            raise = mx > m_run + RESCALE_TAU;
          } else if (vs == 22) {
            m_new = raise ? mx : m_run;
          } else if (vs < 29) {
#pragma unroll
            for (int rg = (4 * (vs - 23)) / 3; rg < (4 * (vs - 22)) / 3; ++rg) {
              if (rg > 0) {
                rs_n += pn[rg - 1];
                if (!(rg & 1)) Pn[(rg - 1) >> 1] = pack2(pn[rg - 2], pn[rg - 1]);
              }
              pn[rg] = pexp(Sn, rg, m_new);
            }
          } else if (vs == 29) {
            rs_n += pn[7];
            Pn[3] = pack2(pn[6], pn[7]);
            // results that are only used by the next step: keep their computation here, in the shadow of
            // the matrix instructions, instead of letting it sink to the end of the iteration
            asm volatile("" ::"v"(Pn), "v"(rs_n));
          }
        }
        // ---- the matrix instruction: within a pair the second one goes first, because it waits for the pair's
        // last read and so covers the other one's as well (one wait per pair instead of two) ----
        {
          const int ms = sl2 ^ 1;
          if (ms < 2 * NC) {
            Sn[ms & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ms], qf[ms >> 1], ms < 2 ? zero16 : Sn[ms & 1], 0, 0, 0);
          } else {
            const int kk = (ms - 2 * NC) / ND, dt = (ms - 2 * NC) % ND;
            O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ms], __builtin_bit_cast(bf16x8, Pk[kk]), O[dt], 0, 0, 0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      l_run += rs;
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        alpha = __builtin_amdgcn_exp2f(m_run - m_new);     // 1 in the lanes that keep their reference point
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
      }
      l_run += rs_n;
      m_run = m_new;
      P0 = Pn;
      advance_v();
    };
    // Only the last tile a wavefront computes needs the mask: the diagonal tiles before it lie entirely
    // below its first query.  Every wavefront runs n_steps iterations (the barriers are shared): plain
    // steps, masked steps, its last tile, then idle iterations that only copy.  In the last iteration of the
    // item the Q rows of the next item are requested: no product with Q is left by then.
    int t_mask = n_before + q_in_blk / KT;
    if (t_mask > n_my) t_mask = n_my;
    const int T1 = t_mask > 1 ? t_mask - 1 : 0, T2 = n_my > 1 ? n_my - 1 : 0;
    int t = 0;
    // two steps per trip, the second with the roles of the score registers exchanged: no copies
    for (; t + 1 < T1; t += 2) { step(t, std::false_type{}, Sc, Sd); step(t + 1, std::false_type{}, Sd, Sc); }
    for (; t < T1; ++t) { step(t, std::false_type{}, Sc, Sd); Sc[0] = Sd[0]; Sc[1] = Sd[1]; }
    for (; t < T2; ++t) { step(t, std::true_type{}, Sc, Sd); Sc[0] = Sd[0]; Sc[1] = Sd[1]; }
    // The rest of the item: this wavefront's last tile (t == n_my - 1), then idle iterations that only copy, up to
    // n_steps in all.  The Q rows of the next item are requested in the item's last iteration, after its barrier,
    // at ONE place in straight-line code: inside a loop, or at a second place, the compiler has to assume that
    // earlier loads into the same registers are still under way and drains the whole memory queue first, the
    // tile copies issued just before included (a trip to memory at every item boundary).
    auto last_tile = [&]() {      // the rest of P(t), O += P(t) V(t)
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
        O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_frag(sl2), __builtin_bit_cast(bf16x8, Pk[kk]), O[dt], 0, 0, 0);
      }
    };
    if (t < n_my && t + 1 < n_steps) {          // the last tile, with idle iterations to follow
      advance_k();
      top(t);
      fill_all();
      last_tile();
      advance_v();
      ++t;
    }
    for (; t + 1 < n_steps; ++t) {
      advance_k();
      top(t);
      fill_all();
      advance_v();
    }
    if (t < n_steps) {                          // the item's last iteration: the last tile or an idle one
      advance_k();
      top(t);
      fill_all();
      if (more) load_q(it1);
      if (t < n_my) last_tile();
      advance_v();
      ++t;
    }

    // ---- epilogue ----
    // Register r of tile dt is d = 32dt + 8(r/4) + 4hh + r%4: a lane holds every other 8-byte piece of its
    // output row and lane+32 the pieces in between.  The two lanes first trade pieces (the upper half of the
    // wavefront's copy of one register against the lower half's copy of another) so that lane (q, 0) ends up
    // with the first half of the row and lane (q, 1) with the second, in 16-byte chunks; the row then leaves in
    // half as many, twice as wide stores, which matters because the stores of a whole workgroup queue up in
    // the compute unit's one address unit at the end of every work item.
    {
      const float ltot = l_run + __shfl_xor(l_run, 32);
      const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
      const int64_t tok = q0 + ln;
      constexpr int NP = 4 * ND;                       // 8-byte pieces per lane; piece pc sits at byte 16pc + 8hh of the row
      uint32_t pw[NP][2];
#pragma unroll
      for (int pc = 0; pc < NP; ++pc) {
        const int dt = pc >> 2, r0 = 4 * (pc & 3);
        pw[pc][0] = pack2(O[dt][r0] * inv, O[dt][r0 + 1] * inv);
        pw[pc][1] = pack2(O[dt][r0 + 2] * inv, O[dt][r0 + 3] * inv);
      }
#pragma unroll
      for (int m = 0; m < NP / 2; ++m)
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const auto r = __builtin_amdgcn_permlane32_swap(pw[m][x], pw[m + NP / 2][x], false, false);
          pw[m][x] = r[0];
          pw[m + NP / 2][x] = r[1];
        }
      // Now lane (q, hh) holds NP/2 chunks of 16 bytes, chunk m at byte D*hh + 16m of row q.  Four consecutive
      // lanes hold four consecutive rows; a 4x4 transpose inside every such quad (two butterfly stages of
      // quad permutes) hands lane i chunk 4u+i of all four rows, so that store k of group u writes row k of the
      // quad with its four lanes covering 64 contiguous bytes instead of four different rows.
      const bool odd = lane & 1, upper = lane & 2;
      auto quad_xor1 = [](uint32_t x) -> uint32_t { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true); };
      auto quad_xor2 = [](uint32_t x) -> uint32_t { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true); };
      // The next item's Q rows are waited for here, before the output stores go out: after them the same wait
      // would also wait for the stores to be acknowledged (loads and stores share one counter).
#pragma unroll
      for (int c = 0; c < NC; ++c) asm volatile("" : "+v"(qraw[c]));
      const int li = lane & 3;
      const int64_t tok0 = tok - li;                   // first row of the quad
      __bf16* obase = p.o + (((int64_t)it.b * p.hq + h) * p.q_rows + (tok0 - qs_of(it))) * D + hh * (D / 2) + 8 * li;
#pragma unroll
      for (int u = 0; u < NP / 8; ++u) {
        uint32_t c[4][4];                              // c[m][word]: chunk 4u+m of this lane's row
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int mm = 4 * u + m;
          c[m][0] = pw[mm][0]; c[m][1] = pw[mm][1]; c[m][2] = pw[mm + NP / 2][0]; c[m][3] = pw[mm + NP / 2][1];
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // stage 1: lanes i and i^1 trade c[k^1]; stage 2: lanes i and i^2 trade c[k^2].  The permutes are
          // evaluated by all lanes before anything is selected: a lane can only be read while it is active.
          const uint32_t x0 = quad_xor1(c[0][w]), x1 = quad_xor1(c[1][w]), x2 = quad_xor1(c[2][w]), x3 = quad_xor1(c[3][w]);
          const uint32_t a0 = odd ? x1 : c[0][w], a1 = odd ? c[1][w] : x0;
          const uint32_t a2 = odd ? x3 : c[2][w], a3 = odd ? c[3][w] : x2;
          const uint32_t y0 = quad_xor2(a0), y1 = quad_xor2(a1), y2 = quad_xor2(a2), y3 = quad_xor2(a3);
          c[0][w] = upper ? y2 : a0; c[2][w] = upper ? a2 : y0;
          c[1][w] = upper ? y3 : a1; c[3][w] = upper ? a3 : y1;
        }
        // c[k] is now chunk 4u + li of row tok0 + k
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
          const u32x4 wv = {c[k2][0], c[k2][1], c[k2][2], c[k2][3]};
          if (active && tok0 + k2 < keys_of(it) && tok0 + k2 >= qs_of(it))
            *reinterpret_cast<u32x4*>(obase + (int64_t)k2 * D + 32 * u) = wv;
        }
      }
      if (active && tok < keys_of(it) && tok >= qs_of(it) && p.lse && hh == 0)
        p.lse[((int64_t)it.b * p.hq + h) * p.q_rows + (tok - qs_of(it))] = (m_run + log2f(ltot)) * 0.69314718055994530942f;
    }
    it = it1; it1 = it2; it2 = VARLEN ? next_valid(it2, raw2) : next_item(it2);
  }
  // asynchronous copies must not outlive the workgroup's claim on its LDS
  wait_vmcnt<0>();
}

template <int D, int NW, int NS, bool DENSE, bool CHAIN, bool VARLEN, bool PAGED = false>
int launch_as(const bf16_params& p, hipStream_t stream) {
  constexpr size_t lds = (size_t)NS * 2 * (KT / (512 / D)) * (1024 + 16 * (512 / D));
  static std::atomic<unsigned long long> attr_done{0};
  if (int st = pa_allow_dynamic_lds(reinterpret_cast<const void*>(&pa_prefill_bf16_kernel<D, NW, NS, DENSE, CHAIN, VARLEN, PAGED>), lds, attr_done))
    return st;
  // One workgroup per work item, or, when the items can be chained (the block lists are short enough for the
  // look-ahead tables and registers), one persistent workgroup per compute unit that walks through its share.
  int64_t grid = (int64_t)p.per_xcd * 8;
  if (CHAIN) {
    int n_cu = 0;
    pa_current_device(nullptr, &n_cu);
    if (n_cu < 8) n_cu = 8;
    const int64_t persistent = (int64_t)(n_cu / 8) * 8;
    if (grid > persistent) grid = persistent;
  }
  hipLaunchKernelGGL((pa_prefill_bf16_kernel<D, NW, NS, DENSE, CHAIN, VARLEN, PAGED>), dim3((uint32_t)grid), dim3(64 * NW), lds, stream, p);
  return pa_note_hip(hipGetLastError());
}

template <int D, int NW, int NS>
int launch(const bf16_params& p, hipStream_t stream) {
  if (p.block_table) return p.seq_len ? launch_as<D, NW, NS, false, true, true, true>(p, stream) : launch_as<D, NW, NS, false, true, false, true>(p, stream);
  if (p.seq_len) {
    if (p.dense) return launch_as<D, NW, NS, true, true, true>(p, stream);
    return p.chain ? launch_as<D, NW, NS, false, true, true>(p, stream) : launch_as<D, NW, NS, false, false, true>(p, stream);
  }
  if (p.dense) return launch_as<D, NW, NS, true, true, false>(p, stream);     // the implicit list is always chained
  return p.chain ? launch_as<D, NW, NS, false, true, false>(p, stream) : launch_as<D, NW, NS, false, false, false>(p, stream);
}

}  // namespace


int pa_launch_prefill_bf16(const pa_prefill_args& a) {
  bf16_params p;
  p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.o = (__bf16*)a.o; p.lse = a.lse;
  p.kv_cnt = a.kv_cnt; p.kv_idx = a.kv_idx; p.max_k = a.max_k; p.nb = a.nb; p.B = a.pat.block;
  p.hq = a.hq; p.hkv = a.hkv; p.batch = a.batch; p.G = a.hq / a.hkv; p.dense = (a.pat.flags & POWATTN_DENSE) ? 1 : 0;
  p.subs = p.B / KT;
  if (!p.dense && (int64_t)a.max_k * p.subs > TILE_CAP) return POWATTN_UNSUPPORTED;
  if (a.seq_len > 0x7fffffffLL - 1024) return POWATTN_UNSUPPORTED;   // key positions are kept in 32 bits
  p.N = a.seq_len;
  p.q_start = a.q_start; p.q_rows = a.q_rows > 0 ? a.q_rows : a.seq_len - a.q_start; p.kv_rows = a.kv_rows; p.i0 = (int32_t)(a.q_start / a.pat.block);
  p.c2 = a.scale * 1.44269504088896340736f;
  p.seq_len = a.seq_len_dev; p.q_start_dev = a.q_start_dev;
  p.block_table = a.block_table; p.table_stride = a.table_stride; p.n_pages = (int32_t)a.n_pages;
  const int64_t tasks = (int64_t)p.G * p.B / QW;
  if (tasks > (1 << 20)) return POWATTN_UNSUPPORTED;
  p.tasks = (int32_t)tasks;
  const int nw = p.tasks > 4 ? 8 : 4;
  p.chunks = (p.tasks + nw - 1) / nw;
  // Sequences of different lengths: an odd count of block numbers per sequence (the extra one lies behind every
  // sequence and is passed over), so that the power-of-two stride of a workgroup's item numbers walks through all
  // block positions instead of returning to the same few, whose rows exist for different shares of the batch.
  if (a.seq_len_dev && (p.nb & 1) == 0) ++p.nb;
  p.total_wg = (int64_t)a.batch * a.hkv * p.nb * p.chunks;
  int64_t per_xcd = (p.total_wg + 7) / 8;
  p.xcd_split = 0; p.per_kvh = 0;
  if (a.seq_len_dev && a.hkv <= 2) {   // (with four KV heads the contiguous halves measure the same or 1-2 % better)
    p.xcd_split = 8 / a.hkv;
    p.per_kvh = (int64_t)a.batch * p.nb * p.chunks;
    per_xcd = (p.per_kvh + p.xcd_split - 1) / p.xcd_split;
  }
  if (per_xcd * 8 > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  p.per_xcd = (int32_t)per_xcd;
  // chaining keeps the list row of the item after next in 63 lanes and two tile tables in LDS
  p.chain = (p.dense || (a.max_k <= 63 && (int64_t)a.max_k * p.subs <= TILE_CAP / 2)) ? 1 : 0;
  if (a.block_table) {
    // paged: explicit lists whose tile table fits twice over (key positions and pool rows), pool rows in 32 bits
    if (p.dense || a.max_k > 63 || (int64_t)a.max_k * p.subs > TILE_CAP / 4) return POWATTN_UNSUPPORTED;
    if (a.n_pages < 1 || a.table_stride < 1 || a.n_pages * (int64_t)a.hkv * p.B > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  }

  // ring of 4 stages: 128 KB of LDS at head_dim 128, 64 KB at head_dim 64
  if (a.head_dim == 128) return nw == 8 ? launch<128, 8, 4>(p, a.stream) : launch<128, 4, 4>(p, a.stream);
  return nw == 8 ? launch<64, 8, 4>(p, a.stream) : launch<64, 4, 4>(p, a.stream);
}

