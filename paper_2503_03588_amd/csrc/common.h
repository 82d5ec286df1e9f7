// Shared host-side declarations of the library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/powattn.h"
#include "pattern.h"

#define POWATTN_VERSION_NUMBER 108  // 0.1.8; moves with every change to a kernel (bench.py ties its profiled traffic figures to it)

// Records a HIP error for powattn_strerror and maps it to a status.
int pa_note_hip(hipError_t e);
int pa_check_pattern(const powattn_pattern* p);

// One-time, per-device launch set-up shared by the launchers; safe to call from several host threads.
// pa_current_device: the current device (clamped to [0, 64)) and its number of compute units (cached).
// pa_allow_dynamic_lds: raises a kernel's dynamic shared memory limit to `bytes` once per device; `done` is the
// caller's file-scope mask of the devices on which it has been raised (bit = device).  Returns a status.
#include <atomic>
void pa_current_device(int* dev, int* n_cu);
int pa_allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<unsigned long long>& done);

struct pa_prefill_args {
  powattn_pattern pat;
  const int32_t* kv_cnt;
  const int32_t* kv_idx;
  int32_t max_k;
  const void* q; const void* k; const void* v; void* o; float* lse;
  int32_t batch, hq, hkv;
  int64_t seq_len;   // keys in the context (q_start + rows of Q)
  int64_t q_start;   // position of the first query row; 0 for a whole-sequence prefill
  int64_t kv_rows;   // rows per (batch, KV head) slab of K/V: seq_len, or the capacity of a cache
  int64_t q_rows;    // rows per (batch, query head) slab of Q/O/LSE; 0: seq_len - q_start
  int32_t nb;      // query blocks: ceil((seq_len - q_start) / block)
  const int32_t* seq_len_dev;   // device [batch]: every sequence's own length, seq_len then being the padded one; or null
  // paged KV cache (k, v are then page pools [n_pages, hkv, block, head_dim]); null: contiguous slabs of kv_rows rows
  const int32_t* q_start_dev = nullptr;   // with seq_len_dev: device [batch], every sequence's first query position
                                          // (seq_len_dev[b] then counts its query rows); null: 0 for all
  const int32_t* block_table = nullptr;   // device [batch, table_stride]: page of every block of every sequence
  int32_t table_stride = 0;
  int64_t n_pages = 0;
  int32_t head_dim;
  float scale;     // softmax scale (natural units)
  hipStream_t stream;
};

int pa_launch_prefill_f32(const pa_prefill_args& a);
int pa_launch_prefill_bf16(const pa_prefill_args& a);

struct pa_decode_args {
  powattn_pattern pat;
  const void* q; const void* k; const void* v;
  const int32_t* kv_len;
  int64_t capacity;
  void* o; float* lse;
  int32_t batch, hq, hkv, head_dim;
  float scale;
  void* workspace;
  int32_t n_split;   // workgroups per (batch, kv head)
  hipStream_t stream;
  // paged cache (block_table != nullptr): k and v are page pools [n_pages, hkv, block, head_dim]; block j of
  // sequence b is page block_table[b * table_stride + j]; capacity is table_stride * block
  const int32_t* block_table;
  int32_t table_stride;
  int64_t n_pages;
};
int pa_launch_decode_bf16(const pa_decode_args& a);
// total workspace bytes of a decode call with n_split workgroups per (sequence, KV head); *header_bytes (may be
// null) receives the size of the generation numbers at its start
size_t pa_decode_workspace_layout(int32_t batch, int32_t hq, int32_t hkv, int32_t head_dim, int32_t n_split, size_t* header_bytes);
// the library's static scratch buffer on the current device: its device address and size
int pa_decode_scratch(void** ptr_out, size_t* bytes_out);

struct pa_backward_args {
  powattn_pattern pat;
  const int32_t* kv_cnt; const int32_t* kv_idx; int32_t max_k;
  const void* q; const void* k; const void* v; const void* o; const void* dout; const float* lse;
  void* dq; void* dk; void* dv;
  int32_t batch, hq, hkv, nb, head_dim;
  int64_t seq_len;
  float scale;
  void* workspace;
  hipStream_t stream;
};
int pa_launch_backward_bf16(const pa_backward_args& a);
size_t pa_backward_workspace_bytes(const powattn_pattern& pat, int32_t batch, int32_t hq, int32_t hkv, int64_t seq_len, int32_t head_dim);
int32_t pa_decode_splits(const powattn_pattern* pat, int32_t batch, int32_t hkv, int64_t capacity);
