// KV append: the newly generated token's key and value join the request's
// paged KVCache (paper Section 2.1: a generated token is appended to the
// sequence and takes part in all later iterations).
//
// One workgroup per request: the new [H_kv][D] key and value rows are written
// to row kv_len % 16 of block block_table[b][kv_len / 16] (128-bit stores),
// then kv_len is incremented.  The block-table entry must already exist (the
// host allocates a block when kv_len reaches a multiple of 16).  A request
// whose row is full (kv_len == max_blocks_per_seq * 16) is left untouched.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void kv_append_kernel(const char* __restrict__ k_new,
                                                        const char* __restrict__ v_new,
                                                        char* __restrict__ k_blocks, char* __restrict__ v_blocks,
                                                        const int32_t* __restrict__ block_table,
                                                        int32_t* __restrict__ kv_lens, int num_kv_heads,
                                                        int row_bytes, int num_blocks, int max_blocks_per_seq) {
  const int b = blockIdx.x;
  const int pos = kv_lens[b];
  if (pos < 0 || pos >= max_blocks_per_seq * 16) return;
  int blk = block_table[static_cast<size_t>(b) * max_blocks_per_seq + pos / 16];
  blk = min(max(blk, 0), num_blocks - 1);
  const int vec_per_row = row_bytes / 16;
  const int total = num_kv_heads * vec_per_row;
  const size_t slab = static_cast<size_t>(16) * row_bytes;
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    const int h = i / vec_per_row;
    const int c = i - h * vec_per_row;
    const size_t src = (static_cast<size_t>(b) * num_kv_heads + h) * row_bytes + c * 16;
    const size_t dst = (static_cast<size_t>(blk) * num_kv_heads + h) * slab + static_cast<size_t>(pos % 16) * row_bytes + c * 16;
    *reinterpret_cast<u32x4*>(k_blocks + dst) = *reinterpret_cast<const u32x4*>(k_new + src);
    *reinterpret_cast<u32x4*>(v_blocks + dst) = *reinterpret_cast<const u32x4*>(v_new + src);
  }
  __syncthreads();  // every thread has read kv_lens[b] before it changes
  if (threadIdx.x == 0) kv_lens[b] = pos + 1;
}

}  // namespace

extern "C" as_status as_kv_append(const void* k_new, const void* v_new, void* k_blocks, void* v_blocks,
                                  const int32_t* block_table, int32_t* kv_lens, const as_attn_params* p,
                                  void* hip_stream) {
  if (!k_new || !v_new || !k_blocks || !v_blocks || !block_table || !kv_lens || !p)
    return als::fail(AS_EINVAL, "as_kv_append: a required pointer is null");
  if ((reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new) |
       reinterpret_cast<uintptr_t>(k_blocks) | reinterpret_cast<uintptr_t>(v_blocks)) % 16)
    return als::fail(AS_EINVAL, "as_kv_append: k_new, v_new, k_blocks and v_blocks must be 16-byte aligned");
  if (p->batch < 1 || p->num_kv_heads < 1 || p->num_blocks < 1 || p->max_blocks_per_seq < 1)
    return als::fail(AS_EINVAL, "as_kv_append: batch, num_kv_heads, num_blocks, max_blocks_per_seq must be positive");
  if (p->block_size != 16) return als::fail(AS_EUNSUPPORTED, "as_kv_append: block_size %d (only 16 is built)", p->block_size);
  if (p->dtype < AS_DTYPE_F32 || p->dtype > AS_DTYPE_F16)
    return als::fail(AS_EUNSUPPORTED, "as_kv_append: dtype %d", p->dtype);
  const int esz = p->dtype == AS_DTYPE_F32 ? 4 : 2;
  const int row_bytes = p->head_dim * esz;
  if (p->head_dim < 1 || row_bytes % 16)
    return als::fail(AS_EUNSUPPORTED, "as_kv_append: head_dim %d rows are not a multiple of 16 bytes", p->head_dim);
  hipLaunchKernelGGL(kv_append_kernel, dim3(p->batch), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const char*>(k_new), static_cast<const char*>(v_new),
                     static_cast<char*>(k_blocks), static_cast<char*>(v_blocks), block_table, kv_lens,
                     p->num_kv_heads, row_bytes, p->num_blocks, p->max_blocks_per_seq);
  ALS_HIP_CHECK(hipGetLastError());
  return AS_OK;
}
