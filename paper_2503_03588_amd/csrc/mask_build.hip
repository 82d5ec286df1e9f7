// Block-index generation: one thread per query block emits its ascending list
// of attended key blocks (Algorithm 1 lifted to blocks); a second, optional
// kernel fills the nb x nb byte map.
#include "common.h"

__global__ void pa_mask_rows_kernel(int32_t W, int32_t S, uint32_t flags, int32_t nb,
                                    int32_t* __restrict__ kv_cnt, int32_t* __restrict__ kv_idx, int32_t max_k) {
  int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nb) return;
  int32_t* row = kv_idx + (int64_t)i * max_k;
  int32_t n = 0;
  pa_for_each_block(W, S, flags, (int64_t)i, [&](int64_t j) {
    if (n < max_k) row[n] = (int32_t)j;   // capacity was checked on the host; never write past the row
    ++n;
  });
  kv_cnt[i] = n < max_k ? n : max_k;
  for (int32_t c = n; c < max_k; ++c) row[c] = -1;
}

__global__ void pa_mask_bytes_kernel(int32_t W, int32_t S, uint32_t flags, int32_t nb, uint8_t* __restrict__ bm) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t total = (int64_t)nb * nb;
  if (idx >= total) return;
  int64_t i = idx / nb, j = idx % nb;
  bm[idx] = pa_block_attended(W, S, flags, i, j) ? 1 : 0;
}

extern "C" int powattn_mask_build(const powattn_pattern* pattern, int64_t seq_len,
                                  int32_t* d_kv_cnt, int32_t* d_kv_idx, int32_t max_k,
                                  uint8_t* d_block_mask, void* hip_stream) {
  int st = pa_check_pattern(pattern);
  if (st != POWATTN_OK) return st;
  if (seq_len < 1 || !d_kv_cnt || !d_kv_idx || max_k < 1) return POWATTN_INVALID_ARG;
  int64_t nb64 = powattn_num_blocks(pattern, seq_len);
  if (nb64 < 0) return POWATTN_INVALID_ARG;
  int32_t need = powattn_max_k(pattern, seq_len);
  if (need < 0) return -need;
  if (max_k < need) return POWATTN_WORKSPACE_TOO_SMALL;
  const int32_t nb = (int32_t)nb64;
  hipStream_t stream = (hipStream_t)hip_stream;
  const int threads = 128;
  hipLaunchKernelGGL(pa_mask_rows_kernel, dim3((nb + threads - 1) / threads), dim3(threads), 0, stream,
                     pattern->window, pattern->sink, pattern->flags, nb, d_kv_cnt, d_kv_idx, max_k);
  st = pa_note_hip(hipGetLastError());
  if (st != POWATTN_OK) return st;
  if (d_block_mask) {
    int64_t total = (int64_t)nb * nb;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return POWATTN_UNSUPPORTED;
    hipLaunchKernelGGL(pa_mask_bytes_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream,
                       pattern->window, pattern->sink, pattern->flags, nb, d_block_mask);
    st = pa_note_hip(hipGetLastError());
  }
  return st;
}
