// Host side of the C ABI: argument checks, host-only queries, dispatch.
#include <math.h>
#include <stdio.h>
#include <string.h>
#include "common.h"

static thread_local char g_hip_msg[256] = "";
static thread_local char g_msg_buf[384];

int pa_note_hip(hipError_t e) {
  if (e == hipSuccess) return POWATTN_OK;
  snprintf(g_hip_msg, sizeof(g_hip_msg), "%s", hipGetErrorString(e));
  return POWATTN_HIP_ERROR;
}

void pa_current_device(int* dev_out, int* n_cu_out) {
  static std::atomic<int> n_cu[64];     // zero-initialised; 0 = not looked up yet
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  int v = n_cu[dev].load(std::memory_order_relaxed);
  if (v == 0) {                         // two threads may both look it up: they store the same value
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 1;
    n_cu[dev].store(v, std::memory_order_relaxed);
  }
  if (dev_out) *dev_out = dev;
  if (n_cu_out) *n_cu_out = v;
}

int pa_allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  pa_current_device(&dev, nullptr);
  const unsigned long long bit = 1ull << dev;
  if (done.load(std::memory_order_acquire) & bit) return POWATTN_OK;
  // setting the limit twice is harmless, so threads that race here simply both set it
  hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return pa_note_hip(e);
  done.fetch_or(bit, std::memory_order_release);
  return POWATTN_OK;
}

int pa_check_pattern(const powattn_pattern* p) {
  if (!p) return POWATTN_INVALID_ARG;
  if (p->block < 1 || p->window < 0 || p->sink < 0) return POWATTN_INVALID_ARG;
  if (p->flags & ~(POWATTN_POWER | POWATTN_DENSE)) return POWATTN_INVALID_ARG;
  // without the power term nothing guarantees the diagonal block: need a window
  if (!(p->flags & (POWATTN_POWER | POWATTN_DENSE)) && p->window < 1) return POWATTN_INVALID_ARG;
  return POWATTN_OK;
}

extern "C" int powattn_version(void) { return POWATTN_VERSION_NUMBER; }

extern "C" const char* powattn_strerror(int status) {
  switch (status) {
    case POWATTN_OK: return "ok";
    case POWATTN_INVALID_ARG: return "invalid argument";
    case POWATTN_UNSUPPORTED: return "unsupported head_dim, block size or dtype";
    case POWATTN_WORKSPACE_TOO_SMALL: return "workspace or max_k too small";
    case POWATTN_HIP_ERROR:
      snprintf(g_msg_buf, sizeof(g_msg_buf), "HIP error: %s", g_hip_msg[0] ? g_hip_msg : "(none recorded)");
      return g_msg_buf;
    default: return "unknown status";
  }
}

extern "C" int64_t powattn_num_blocks(const powattn_pattern* p, int64_t seq_len) {
  if (pa_check_pattern(p) != POWATTN_OK || seq_len <= 0) return -POWATTN_INVALID_ARG;
  int64_t nb = (seq_len + p->block - 1) / p->block;
  if (nb > INT32_MAX) return -POWATTN_INVALID_ARG;
  return nb;
}

extern "C" int32_t powattn_row_host(const powattn_pattern* p, int64_t q_block, int32_t* out, int32_t capacity) {
  if (pa_check_pattern(p) != POWATTN_OK || q_block < 0 || q_block > INT32_MAX || capacity < 0) return -POWATTN_INVALID_ARG;
  if (!out && capacity != 0) return -POWATTN_INVALID_ARG;
  int64_t n = pa_for_each_block(p->window, p->sink, p->flags, q_block, [](int64_t) {});
  if (!out) return (int32_t)n;
  if (n > capacity) return -POWATTN_WORKSPACE_TOO_SMALL;
  int32_t w = 0;
  pa_for_each_block(p->window, p->sink, p->flags, q_block, [&](int64_t j) { out[w++] = (int32_t)j; });
  return w;
}

extern "C" int32_t powattn_max_k(const powattn_pattern* p, int64_t seq_len) {
  int64_t nb = powattn_num_blocks(p, seq_len);
  if (nb < 0) return (int32_t)nb;
  if (p->flags & POWATTN_DENSE) return (int32_t)nb;
  // Rows up to W+S-1 attend every earlier block (i+1 of them); beyond that the count is
  // W + S + #{k : W <= 2^k <= i-S}, which only grows with i.  The last row is the longest.
  return (int32_t)pa_for_each_block(p->window, p->sink, p->flags, nb - 1, [](int64_t) {});
}

static bool supported_head_dim(int32_t d) { return d == 64 || d == 128; }

extern "C" int powattn_prefill(const powattn_pattern* pattern,
                               const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                               const void* q, const void* k, const void* v, void* o, float* lse,
                               int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                               int64_t seq_len, int32_t head_dim, int32_t dtype,
                               float softmax_scale, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k || !v || !o) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || seq_len < 1 || head_dim < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  const bool dense = (pattern->flags & POWATTN_DENSE) != 0;
  if (!dense && (!d_kv_cnt || !d_kv_idx || max_k < 1)) return POWATTN_INVALID_ARG;
  int64_t nb = powattn_num_blocks(pattern, seq_len);
  if (nb < 0) return POWATTN_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;  // NaN
  if (dtype != POWATTN_BF16 && dtype != POWATTN_F32) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if ((int64_t)batch * n_q_heads > 65535 * 16) return POWATTN_UNSUPPORTED;

  pa_prefill_args a;
  a.pat = *pattern;
  a.kv_cnt = d_kv_cnt; a.kv_idx = d_kv_idx; a.max_k = max_k;
  a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads;
  a.seq_len = seq_len; a.q_start = 0; a.kv_rows = seq_len; a.q_rows = 0; a.nb = (int32_t)nb; a.head_dim = head_dim;
  a.seq_len_dev = nullptr;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.stream = (hipStream_t)hip_stream;
  if (dtype == POWATTN_F32) {
    const int32_t B = pattern->block;
    if (B < 16 || B > 256 || B % 16 != 0) return POWATTN_UNSUPPORTED;
    return pa_launch_prefill_f32(a);
  }
  if (pattern->block % 64 != 0 || pattern->block > 1024) return POWATTN_UNSUPPORTED;
  return pa_launch_prefill_bf16(a);
}

extern "C" int powattn_prefill_chunk(const powattn_pattern* pattern,
                                     const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                     const void* q, const void* k_cache, const void* v_cache, void* o, float* lse,
                                     int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                     int64_t q_start, int64_t q_len, int64_t cache_capacity,
                                     int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k_cache || !v_cache || !o) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1) return POWATTN_INVALID_ARG;
  if (q_start < 0 || q_len < 1 || cache_capacity < 1 || q_start > INT64_MAX - q_len) return POWATTN_INVALID_ARG;
  if (q_start + q_len > cache_capacity) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  const bool dense = (pattern->flags & POWATTN_DENSE) != 0;
  if (!dense && (!d_kv_cnt || !d_kv_idx || max_k < 1)) return POWATTN_INVALID_ARG;
  const int64_t seq_len = q_start + q_len;
  if (powattn_num_blocks(pattern, seq_len) < 0) return POWATTN_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;  // NaN
  if (dtype != POWATTN_BF16) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if ((int64_t)batch * n_q_heads > 65535 * 16) return POWATTN_UNSUPPORTED;
  if (pattern->block % 64 != 0 || pattern->block > 1024) return POWATTN_UNSUPPORTED;

  pa_prefill_args a;
  a.pat = *pattern;
  a.kv_cnt = d_kv_cnt; a.kv_idx = d_kv_idx; a.max_k = max_k;
  a.q = q; a.k = k_cache; a.v = v_cache; a.o = o; a.lse = lse;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads;
  a.seq_len = seq_len; a.q_start = q_start; a.kv_rows = cache_capacity; a.q_rows = 0; a.seq_len_dev = nullptr;
  // query blocks are the pattern's blocks: the first one is partial when the chunk starts inside a block
  a.nb = (int32_t)((seq_len + pattern->block - 1) / pattern->block - q_start / pattern->block);
  a.head_dim = head_dim;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.stream = (hipStream_t)hip_stream;
  return pa_launch_prefill_bf16(a);
}

extern "C" int powattn_prefill_chunk_paged(const powattn_pattern* pattern,
                                           const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                           const void* q, const void* k_pages, const void* v_pages,
                                           const int32_t* d_block_table, int32_t table_stride, int64_t n_pages,
                                           void* o, float* lse,
                                           int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                           int64_t q_start, int64_t q_len,
                                           int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k_pages || !v_pages || !o || !d_block_table) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1) return POWATTN_INVALID_ARG;
  if (table_stride < 1 || n_pages < 1) return POWATTN_INVALID_ARG;
  if (q_start < 0 || q_len < 1 || q_start > INT64_MAX - q_len) return POWATTN_INVALID_ARG;
  if (q_start + q_len > (int64_t)table_stride * pattern->block) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  if (!d_kv_cnt || !d_kv_idx || max_k < 1) return POWATTN_INVALID_ARG;
  const int64_t seq_len = q_start + q_len;
  if (powattn_num_blocks(pattern, seq_len) < 0) return POWATTN_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;  // NaN
  if (pattern->flags & POWATTN_DENSE) return POWATTN_UNSUPPORTED;     // the implicit list has no table to hold pool rows
  if (dtype != POWATTN_BF16) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if ((int64_t)batch * n_q_heads > 65535 * 16) return POWATTN_UNSUPPORTED;
  if (pattern->block % 64 != 0 || pattern->block > 1024) return POWATTN_UNSUPPORTED;

  pa_prefill_args a;
  a.pat = *pattern;
  a.kv_cnt = d_kv_cnt; a.kv_idx = d_kv_idx; a.max_k = max_k;
  a.q = q; a.k = k_pages; a.v = v_pages; a.o = o; a.lse = lse;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads;
  a.seq_len = seq_len; a.q_start = q_start; a.kv_rows = 0; a.q_rows = 0; a.seq_len_dev = nullptr;
  a.block_table = d_block_table; a.table_stride = table_stride; a.n_pages = n_pages;
  a.nb = (int32_t)((seq_len + pattern->block - 1) / pattern->block - q_start / pattern->block);
  a.head_dim = head_dim;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.stream = (hipStream_t)hip_stream;
  return pa_launch_prefill_bf16(a);
}

extern "C" int powattn_prefill_batch_paged(const powattn_pattern* pattern,
                                           const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                           const void* q, const void* k_pages, const void* v_pages,
                                           const int32_t* d_block_table, int32_t table_stride, int64_t n_pages,
                                           const int32_t* d_q_start, const int32_t* d_q_len, int64_t q_rows,
                                           void* o, float* lse,
                                           int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                           int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k_pages || !v_pages || !o || !d_block_table || !d_q_start || !d_q_len) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1) return POWATTN_INVALID_ARG;
  if (table_stride < 1 || n_pages < 1 || q_rows < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  if (!d_kv_cnt || !d_kv_idx || max_k < 1) return POWATTN_INVALID_ARG;
  const int64_t max_ctx = (int64_t)table_stride * pattern->block;      // the longest context the tables can describe
  if (q_rows > max_ctx) return POWATTN_INVALID_ARG;
  if (powattn_num_blocks(pattern, max_ctx) < 0) return POWATTN_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;  // NaN
  if (pattern->flags & POWATTN_DENSE) return POWATTN_UNSUPPORTED;
  if (dtype != POWATTN_BF16) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if ((int64_t)batch * n_q_heads > 65535 * 16) return POWATTN_UNSUPPORTED;
  if (pattern->block % 64 != 0 || pattern->block > 1024) return POWATTN_UNSUPPORTED;

  pa_prefill_args a;
  a.pat = *pattern;
  a.kv_cnt = d_kv_cnt; a.kv_idx = d_kv_idx; a.max_k = max_k;
  a.q = q; a.k = k_pages; a.v = v_pages; a.o = o; a.lse = lse;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads;
  a.seq_len = max_ctx; a.q_start = 0; a.kv_rows = 0; a.q_rows = q_rows;
  a.seq_len_dev = d_q_len; a.q_start_dev = d_q_start;
  a.block_table = d_block_table; a.table_stride = table_stride; a.n_pages = n_pages;
  // query blocks a piece of q_rows rows can touch when it starts anywhere inside a block
  a.nb = (int32_t)((q_rows + pattern->block - 2) / pattern->block + 1);
  a.head_dim = head_dim;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.stream = (hipStream_t)hip_stream;
  return pa_launch_prefill_bf16(a);
}

extern "C" int powattn_prefill_varlen(const powattn_pattern* pattern,
                                      const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                      const void* q, const void* k, const void* v, void* o, float* lse,
                                      int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                      const int32_t* d_seq_len, int64_t padded_len,
                                      int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k || !v || !o || !d_seq_len) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || padded_len < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  const bool dense = (pattern->flags & POWATTN_DENSE) != 0;
  if (!dense && (!d_kv_cnt || !d_kv_idx || max_k < 1)) return POWATTN_INVALID_ARG;
  const int64_t nb = powattn_num_blocks(pattern, padded_len);
  if (nb < 0) return POWATTN_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;
  if (dtype != POWATTN_BF16) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if (pattern->block % 64 != 0 || pattern->block > 1024) return POWATTN_UNSUPPORTED;
  if ((int64_t)batch * n_q_heads > 65535 * 16) return POWATTN_UNSUPPORTED;

  // One launch for the whole batch: the work items are numbered as if every sequence had padded_len tokens, and
  // the kernel, which reads the lengths from device memory, passes over the query blocks a sequence does not have
  // (the rows of the lists do not depend on the sequence length, so all sequences walk the same lists).
  pa_prefill_args a;
  a.pat = *pattern;
  a.kv_cnt = d_kv_cnt; a.kv_idx = d_kv_idx; a.max_k = max_k;
  a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads;
  a.seq_len = padded_len; a.q_start = 0; a.kv_rows = padded_len; a.q_rows = padded_len;
  a.nb = (int32_t)nb;
  a.head_dim = head_dim;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.stream = (hipStream_t)hip_stream;
  a.seq_len_dev = d_seq_len;
  return pa_launch_prefill_bf16(a);
}

extern "C" size_t powattn_decode_workspace_bytes(const powattn_pattern* pattern, int32_t batch,
                                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                                 int64_t cache_capacity) {
  if (pa_check_pattern(pattern) != POWATTN_OK) return 0;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || cache_capacity < 1) return 0;
  if (n_q_heads % n_kv_heads != 0) return 0;
  int32_t ns = pa_decode_splits(pattern, batch, n_kv_heads, cache_capacity);
  if (ns < 1) return 0;
  // a generation number per (batch, KV head); per (batch, q head, split): head_dim unnormalised outputs +
  // running max + running sum, as 8-byte packets.  With a single split the kernel writes the result directly.
  return pa_decode_workspace_layout(batch, n_q_heads, n_kv_heads, head_dim, ns, nullptr);
}

// The three decode entry points share everything but where the cache and the workspace come from.
// use_scratch: the library's static buffer instead of a caller's workspace.
static int decode_common(const powattn_pattern* pattern, const void* q, const void* k, const void* v,
                         const int32_t* d_kv_len, int64_t capacity, void* o, float* lse,
                         int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         int32_t dtype, float softmax_scale, void* workspace, size_t workspace_bytes, bool use_scratch,
                         const int32_t* block_table, int32_t table_stride, int64_t n_pages, void* hip_stream) {
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;
  if (dtype != POWATTN_BF16) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if (pattern->block % 64 != 0 || pattern->block > 1024) return POWATTN_UNSUPPORTED;
  if (pattern->flags & POWATTN_DENSE) return POWATTN_UNSUPPORTED;
  if (n_q_heads / n_kv_heads > 16) return POWATTN_UNSUPPORTED;
  if (powattn_num_blocks(pattern, capacity) < 0) return POWATTN_INVALID_ARG;
  size_t need = powattn_decode_workspace_bytes(pattern, batch, n_q_heads, n_kv_heads, head_dim, capacity);
  if (need == 0) return POWATTN_INVALID_ARG;
  if (use_scratch) {
    // sizes are checked against the stated maximum before the device is touched
    if (need > (size_t)POWATTN_STATIC_SCRATCH_BYTES) return POWATTN_WORKSPACE_TOO_SMALL;
    int st = pa_decode_scratch(&workspace, &workspace_bytes);
    if (st != POWATTN_OK) return st;
  }
  if (!workspace || workspace_bytes < need) return POWATTN_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)workspace & 255u) != 0) return POWATTN_INVALID_ARG;

  pa_decode_args a;
  a.pat = *pattern;
  a.q = q; a.k = k; a.v = v; a.kv_len = d_kv_len; a.capacity = capacity;
  a.o = o; a.lse = lse;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads; a.head_dim = head_dim;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.workspace = workspace;
  a.n_split = pa_decode_splits(pattern, batch, n_kv_heads, capacity);
  a.stream = (hipStream_t)hip_stream;
  a.block_table = block_table; a.table_stride = table_stride; a.n_pages = n_pages;
  return pa_launch_decode_bf16(a);
}

extern "C" int powattn_decode(const powattn_pattern* pattern,
                              const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* d_kv_len, int64_t cache_capacity,
                              void* o, float* lse,
                              int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                              int32_t dtype, float softmax_scale,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k_cache || !v_cache || !d_kv_len || !o) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || cache_capacity < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  return decode_common(pattern, q, k_cache, v_cache, d_kv_len, cache_capacity, o, lse, batch, n_q_heads, n_kv_heads,
                       head_dim, dtype, softmax_scale, workspace, workspace_bytes, false, nullptr, 0, 0, hip_stream);
}

extern "C" int powattn_decode_static(const powattn_pattern* pattern,
                                     const void* q, const void* k_cache, const void* v_cache,
                                     const int32_t* d_kv_len, int64_t cache_capacity,
                                     void* o, float* lse,
                                     int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                     int32_t dtype, float softmax_scale, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k_cache || !v_cache || !d_kv_len || !o) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || cache_capacity < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  return decode_common(pattern, q, k_cache, v_cache, d_kv_len, cache_capacity, o, lse, batch, n_q_heads, n_kv_heads,
                       head_dim, dtype, softmax_scale, nullptr, 0, true, nullptr, 0, 0, hip_stream);
}

extern "C" int powattn_decode_paged(const powattn_pattern* pattern,
                                    const void* q, const void* k_pages, const void* v_pages, int64_t n_pages,
                                    const int32_t* d_block_table, int32_t table_stride,
                                    const int32_t* d_kv_len,
                                    void* o, float* lse,
                                    int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                    int32_t dtype, float softmax_scale,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k_pages || !v_pages || !d_block_table || !d_kv_len || !o) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || n_pages < 1 || table_stride < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  const int64_t capacity = (int64_t)table_stride * pattern->block;      // tokens a sequence's table can hold
  return decode_common(pattern, q, k_pages, v_pages, d_kv_len, capacity, o, lse, batch, n_q_heads, n_kv_heads,
                       head_dim, dtype, softmax_scale, workspace, workspace_bytes, false,
                       d_block_table, table_stride, n_pages, hip_stream);
}

extern "C" size_t powattn_backward_workspace_bytes(const powattn_pattern* pattern, int32_t batch, int32_t n_q_heads,
                                                   int32_t n_kv_heads, int64_t seq_len, int32_t head_dim) {
  if (pa_check_pattern(pattern) != POWATTN_OK) return 0;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || seq_len < 1) return 0;
  if (n_q_heads % n_kv_heads != 0) return 0;
  return pa_backward_workspace_bytes(*pattern, batch, n_q_heads, n_kv_heads, seq_len, head_dim);
}

extern "C" int powattn_backward(const powattn_pattern* pattern,
                                const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                const void* q, const void* k, const void* v, const void* o, const float* lse,
                                const void* d_o, void* dq, void* dk, void* dv,
                                int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int64_t seq_len,
                                int32_t head_dim, int32_t dtype, float softmax_scale,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !d_kv_cnt || !d_kv_idx) return POWATTN_INVALID_ARG;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || seq_len < 1 || max_k < 1) return POWATTN_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return POWATTN_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return POWATTN_INVALID_ARG;
  if (dtype != POWATTN_BF16) return POWATTN_UNSUPPORTED;
  if (!supported_head_dim(head_dim)) return POWATTN_UNSUPPORTED;
  if (pattern->block != 64 && pattern->block != 128 && pattern->block != 256) return POWATTN_UNSUPPORTED;
  if (pattern->flags & POWATTN_DENSE) return POWATTN_UNSUPPORTED;
  const int64_t nb = powattn_num_blocks(pattern, seq_len);
  if (nb < 0) return POWATTN_INVALID_ARG;
  if (nb > 0x7fffffffLL) return POWATTN_UNSUPPORTED;
  const int32_t need_k = powattn_max_k(pattern, seq_len);
  if (need_k < 0) return POWATTN_INVALID_ARG;
  if (max_k < need_k) return POWATTN_WORKSPACE_TOO_SMALL;      // the lists must be the pattern's own rows
  const size_t need = pa_backward_workspace_bytes(*pattern, batch, n_q_heads, n_kv_heads, seq_len, head_dim);
  if (!workspace || workspace_bytes < need) return POWATTN_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)workspace & 255u) != 0) return POWATTN_INVALID_ARG;

  pa_backward_args a;
  a.pat = *pattern;
  a.kv_cnt = d_kv_cnt; a.kv_idx = d_kv_idx; a.max_k = max_k;
  a.q = q; a.k = k; a.v = v; a.o = o; a.dout = d_o; a.lse = lse;
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.batch = batch; a.hq = n_q_heads; a.hkv = n_kv_heads; a.nb = (int32_t)nb; a.head_dim = head_dim;
  a.seq_len = seq_len;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
  a.workspace = workspace;
  a.stream = (hipStream_t)hip_stream;
  return pa_launch_backward_bf16(a);
}
