// KV staging between the pinned host KV pool and the HBM block pool, and the
// copy/compute handshake of the multi-buffered pool.
//
// Paper Section 3.2: the KVCache of in-flight requests lives in a host-memory
// KV pool; a scheduled batch is migrated to the decoding GPU (directly over
// PCIe when no peer GPU buffers it), and the next batch is prefetched
// asynchronously (Fig. 4 step 4) so the transfer overlaps decoding of the
// running batch (Section 4.4).  Section 3.4 case 3 is the reverse move
// (eviction).
//
// Two ways of moving the blocks, chosen per call (as_stage_set_policy):
//  * DMA copies: one hipMemcpyAsync per run of blocks whose host and device
//    ids both advance by one.  The SDMA engines move the data and every
//    compute unit stays with the attention kernel.  Best when runs are long.
//  * Gather kernel: a paged host pool hands out scattered blocks, and one DMA
//    copy per 32-128 KiB block is bound by the per-copy cost, not by the
//    link.  A small persistent grid (64 workgroups) then reads the pinned host
//    blocks directly over the link with 128-bit loads and writes them to their
//    HBM slots (or the reverse); the block ids travel in the kernel arguments,
//    256 per launch, so nothing is allocated and nothing outlives the call.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

std::atomic<int32_t> g_policy{AS_STAGE_AUTO};

// Below this many bytes per run, on average, the gather kernel is used under
// AS_STAGE_AUTO.  Measured on MI355X / PCIe Gen5 (2 GiB per pool, host to
// device): DMA copies reach 2.9 GB/s with 32 KiB runs, 10.7 with 128 KiB, 27.7
// with 512 KiB, 45 with 2 MiB, 53.5 with 8 MiB and 57.6 GB/s as one copy; the
// kernel 55-57 GB/s for every run length.
constexpr size_t kAutoRunBytes = 8u << 20;

constexpr int kGatherIds = 256;        // (host id, device id) pairs per launch
constexpr int kGatherGrid = 64;        // persistent workgroups
constexpr int kPartBytes = 16 * 1024;  // one task: 256 threads x 4 x 16 B
struct GatherIds {
  int64_t host[kGatherIds];
  int32_t dev[kGatherIds];
};

// task = (block i, part, pool): copies up to 16 KiB of one block of one pool.
// All four loads of a thread are issued before its stores, so a workgroup keeps
// 16 KiB in flight over the link.
__global__ __launch_bounds__(256) void gather_kernel(char* host_k, char* host_v, char* dev_k, char* dev_v,
                                                     GatherIds ids, int n, size_t block_bytes,
                                                     int to_device) {
  const int parts = static_cast<int>((block_bytes + kPartBytes - 1) / kPartBytes);
  const int pools = host_v ? 2 : 1;
  const int tasks = n * parts * pools;
  for (int task = blockIdx.x; task < tasks; task += gridDim.x) {
    const int pool = task % pools;
    const int rest = task / pools;
    const int part = rest % parts;
    const int i = rest / parts;
    const size_t in_block = static_cast<size_t>(part) * kPartBytes;
    const size_t hoff = static_cast<size_t>(ids.host[i]) * block_bytes + in_block;
    const size_t doff = static_cast<size_t>(ids.dev[i]) * block_bytes + in_block;
    char* h = (pool ? host_v : host_k) + hoff;
    char* d = (pool ? dev_v : dev_k) + doff;
    const char* src = to_device ? h : d;
    char* dst = to_device ? d : h;
    const size_t bytes = block_bytes - in_block < kPartBytes ? block_bytes - in_block : kPartBytes;
    u32x4 r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const size_t off = static_cast<size_t>(k) * 4096 + threadIdx.x * 16;
      if (off < bytes) r[k] = *reinterpret_cast<const u32x4*>(src + off);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const size_t off = static_cast<size_t>(k) * 4096 + threadIdx.x * 16;
      if (off < bytes) *reinterpret_cast<u32x4*>(dst + off) = r[k];
    }
  }
}

bool is_pinned_host(const void* p) {
  hipPointerAttribute_t attr;
  hipError_t e = hipPointerGetAttributes(&attr, p);
  if (e != hipSuccess) {
    (void)hipGetLastError();  // ordinary pageable memory: clear the sticky error
    return false;
  }
  return attr.type == hipMemoryTypeHost;
}

// Shared by both directions.  `a_ids` index the host pool (int64), `b_ids`
// the device pool (int32).  to_device selects the direction.
as_status move_blocks(const char* what, char* host_k, char* host_v, const int64_t* h_ids,
                      int64_t num_host_blocks, char* dev_k, char* dev_v, const int32_t* d_ids,
                      int32_t num_dev_blocks, int32_t m, size_t block_bytes, void* hip_stream,
                      bool to_device) {
  if (m < 0) return als::fail(AS_EINVAL, "%s: m = %d is negative", what, m);
  if (block_bytes == 0 || block_bytes % 16)
    return als::fail(AS_EINVAL, "%s: block_bytes = %zu must be a positive multiple of 16", what,
                     block_bytes);
  if (!host_k || !dev_k) return als::fail(AS_EINVAL, "%s: K pool pointer is null", what);
  if ((host_v == nullptr) != (dev_v == nullptr))
    return als::fail(AS_EINVAL, "%s: host_v and dev_v must both be given or both be null", what);
  if (m > 0 && (!h_ids || !d_ids)) return als::fail(AS_EINVAL, "%s: id array is null", what);
  if (num_host_blocks <= 0 || num_dev_blocks <= 0)
    return als::fail(AS_EINVAL, "%s: pool sizes must be positive", what);
  for (int32_t i = 0; i < m; ++i) {
    if (h_ids[i] < 0 || h_ids[i] >= num_host_blocks)
      return als::fail(AS_ERANGE, "%s: host block id [%d] = %lld outside [0, %lld)", what, i,
                       static_cast<long long>(h_ids[i]), static_cast<long long>(num_host_blocks));
    if (d_ids[i] < 0 || d_ids[i] >= num_dev_blocks)
      return als::fail(AS_ERANGE, "%s: device block id [%d] = %d outside [0, %d)", what, i,
                       d_ids[i], num_dev_blocks);
  }
  if (m == 0) return AS_OK;
  if (!is_pinned_host(host_k) || (host_v && !is_pinned_host(host_v)))
    return als::fail(AS_EINVAL, "%s: host pool is not pinned (hipHostMalloc) memory", what);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t runs = 1;
  for (int32_t i = 1; i < m; ++i)
    runs += !(h_ids[i] == h_ids[i - 1] + 1 && d_ids[i] == d_ids[i - 1] + 1);
  const int32_t policy = g_policy.load(std::memory_order_relaxed);
  bool use_kernel = policy == AS_STAGE_KERNEL ||
                    (policy == AS_STAGE_AUTO &&
                     static_cast<size_t>(m) * block_bytes < static_cast<size_t>(runs) * kAutoRunBytes);
  char *hk_dev = nullptr, *hv_dev = nullptr;
  if (use_kernel && (reinterpret_cast<uintptr_t>(host_k) | reinterpret_cast<uintptr_t>(host_v) |
                     reinterpret_cast<uintptr_t>(dev_k) | reinterpret_cast<uintptr_t>(dev_v)) % 16) {
    // the kernel moves 128-bit words; pools at odd addresses keep the DMA path
    if (policy == AS_STAGE_KERNEL)
      return als::fail(AS_EINVAL, "%s: pools must be 16-byte aligned for the copy kernel", what);
    use_kernel = false;
  }
  if (use_kernel) {
    // the address the device uses for the pinned host pool; memory that is
    // pinned but not mapped into the device's address space keeps the DMA path
    if (hipHostGetDevicePointer(reinterpret_cast<void**>(&hk_dev), host_k, 0) != hipSuccess ||
        (host_v && hipHostGetDevicePointer(reinterpret_cast<void**>(&hv_dev), host_v, 0) != hipSuccess)) {
      (void)hipGetLastError();
      if (policy == AS_STAGE_KERNEL)
        return als::fail(AS_EINVAL, "%s: host pool is not mapped into the device address space", what);
      use_kernel = false;
    }
  }
  if (use_kernel) {
    const int parts = static_cast<int>((block_bytes + kPartBytes - 1) / kPartBytes);
    for (int32_t i = 0; i < m; i += kGatherIds) {
      GatherIds ids;
      const int n = m - i < kGatherIds ? m - i : kGatherIds;
      for (int j = 0; j < n; ++j) {
        ids.host[j] = h_ids[i + j];
        ids.dev[j] = d_ids[i + j];
      }
      const int64_t tasks = static_cast<int64_t>(n) * parts * (host_v ? 2 : 1);
      const dim3 grid(static_cast<unsigned>(tasks < kGatherGrid ? tasks : kGatherGrid));
      hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, stream, hk_dev, hv_dev, dev_k, dev_v, ids, n,
                         block_bytes, to_device ? 1 : 0);
      ALS_HIP_CHECK(hipGetLastError());
    }
    return AS_OK;
  }
  int32_t i = 0;
  while (i < m) {
    int32_t j = i + 1;
    while (j < m && h_ids[j] == h_ids[j - 1] + 1 && d_ids[j] == d_ids[j - 1] + 1) ++j;
    const size_t bytes = static_cast<size_t>(j - i) * block_bytes;
    const size_t hoff = static_cast<size_t>(h_ids[i]) * block_bytes;
    const size_t doff = static_cast<size_t>(d_ids[i]) * block_bytes;
    if (to_device) {
      ALS_HIP_CHECK(hipMemcpyAsync(dev_k + doff, host_k + hoff, bytes, hipMemcpyHostToDevice, stream));
      if (host_v)
        ALS_HIP_CHECK(hipMemcpyAsync(dev_v + doff, host_v + hoff, bytes, hipMemcpyHostToDevice, stream));
    } else {
      ALS_HIP_CHECK(hipMemcpyAsync(host_k + hoff, dev_k + doff, bytes, hipMemcpyDeviceToHost, stream));
      if (host_v)
        ALS_HIP_CHECK(hipMemcpyAsync(host_v + hoff, dev_v + doff, bytes, hipMemcpyDeviceToHost, stream));
    }
    i = j;
  }
  return AS_OK;
}

}  // namespace

extern "C" as_status as_stage_set_policy(int32_t policy) {
  if (policy != AS_STAGE_AUTO && policy != AS_STAGE_DMA && policy != AS_STAGE_KERNEL)
    return als::fail(AS_EINVAL, "as_stage_set_policy: unknown policy %d", policy);
  g_policy.store(policy, std::memory_order_relaxed);
  return AS_OK;
}

extern "C" as_status as_stage_kv(const void* host_k, const void* host_v, const int64_t* src_ids,
                                 int64_t num_src_blocks, void* dev_k, void* dev_v,
                                 const int32_t* dst_ids, int32_t num_dst_blocks, int32_t m,
                                 size_t block_bytes, void* hip_stream) {
  return move_blocks("as_stage_kv", const_cast<char*>(static_cast<const char*>(host_k)),
                     const_cast<char*>(static_cast<const char*>(host_v)), src_ids, num_src_blocks,
                     static_cast<char*>(dev_k), static_cast<char*>(dev_v), dst_ids,
                     num_dst_blocks, m, block_bytes, hip_stream, true);
}

extern "C" as_status as_unstage_kv(void* host_k, void* host_v, const int64_t* dst_ids,
                                   int64_t num_host_blocks, const void* dev_k, const void* dev_v,
                                   const int32_t* src_ids, int32_t num_dev_blocks, int32_t m,
                                   size_t block_bytes, void* hip_stream) {
  return move_blocks("as_unstage_kv", static_cast<char*>(host_k), static_cast<char*>(host_v),
                     dst_ids, num_host_blocks, const_cast<char*>(static_cast<const char*>(dev_k)),
                     const_cast<char*>(static_cast<const char*>(dev_v)), src_ids, num_dev_blocks,
                     m, block_bytes, hip_stream, false);
}

// ---------------------------------------------------------------------------
// Pipeline handshake
// ---------------------------------------------------------------------------
struct as_pipeline {
  int32_t num_buffers;
  hipStream_t side;
  hipEvent_t ready[8];
  hipEvent_t free_[8];
};

extern "C" as_status as_pipeline_create(as_pipeline** out, int32_t num_buffers) {
  if (!out) return als::fail(AS_EINVAL, "as_pipeline_create: out is null");
  if (num_buffers < 1 || num_buffers > 8)
    return als::fail(AS_EINVAL, "as_pipeline_create: num_buffers = %d outside [1, 8]", num_buffers);
  as_pipeline* p = new (std::nothrow) as_pipeline();
  if (!p) return als::fail(AS_ENOMEM, "as_pipeline_create: out of host memory");
  p->num_buffers = num_buffers;
  p->side = nullptr;
  for (int i = 0; i < 8; ++i) p->ready[i] = p->free_[i] = nullptr;
  hipError_t e = hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking);  // default priority
  for (int i = 0; e == hipSuccess && i < num_buffers; ++i) {
    e = hipEventCreateWithFlags(&p->ready[i], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->free_[i], hipEventDisableTiming);
  }
  if (e != hipSuccess) {
    as_pipeline_destroy(p);
    return als::fail(AS_EHIP, "as_pipeline_create: %s", hipGetErrorString(e));
  }
  *out = p;
  return AS_OK;
}

extern "C" void* as_pipeline_stream(as_pipeline* p) { return p ? p->side : nullptr; }

#define ALS_PIPE_ARGS(name)                                                                  \
  if (!p) return als::fail(AS_EINVAL, name ": pipeline is null");                            \
  if (buf < 0 || buf >= p->num_buffers)                                                      \
    return als::fail(AS_EINVAL, name ": buffer %d outside [0, %d)", buf, p->num_buffers)

extern "C" as_status as_pipeline_begin_stage(as_pipeline* p, int32_t buf) {
  ALS_PIPE_ARGS("as_pipeline_begin_stage");
  // an event that was never recorded is complete: the first use does not wait
  ALS_HIP_CHECK(hipStreamWaitEvent(p->side, p->free_[buf], 0));
  return AS_OK;
}

extern "C" as_status as_pipeline_end_stage(as_pipeline* p, int32_t buf) {
  ALS_PIPE_ARGS("as_pipeline_end_stage");
  ALS_HIP_CHECK(hipEventRecord(p->ready[buf], p->side));
  return AS_OK;
}

extern "C" as_status as_pipeline_acquire(as_pipeline* p, int32_t buf, void* hip_stream) {
  ALS_PIPE_ARGS("as_pipeline_acquire");
  ALS_HIP_CHECK(hipStreamWaitEvent(static_cast<hipStream_t>(hip_stream), p->ready[buf], 0));
  return AS_OK;
}

extern "C" as_status as_pipeline_query(as_pipeline* p, int32_t buf, int32_t* ready) {
  ALS_PIPE_ARGS("as_pipeline_query");
  if (!ready) return als::fail(AS_EINVAL, "as_pipeline_query: ready is null");
  const hipError_t e = hipEventQuery(p->ready[buf]);  // a never-recorded event reads as complete
  if (e != hipSuccess && e != hipErrorNotReady)
    return als::fail(AS_EHIP, "as_pipeline_query: %s", hipGetErrorString(e));
  *ready = e == hipSuccess ? 1 : 0;
  return AS_OK;
}

extern "C" as_status as_pipeline_release(as_pipeline* p, int32_t buf, void* hip_stream) {
  ALS_PIPE_ARGS("as_pipeline_release");
  ALS_HIP_CHECK(hipEventRecord(p->free_[buf], static_cast<hipStream_t>(hip_stream)));
  return AS_OK;
}

extern "C" as_status as_pipeline_destroy(as_pipeline* p) {
  if (!p) return als::fail(AS_EINVAL, "as_pipeline_destroy: pipeline is null");
  hipError_t first = hipSuccess;
  if (p->side) {
    hipError_t e = hipStreamSynchronize(p->side);
    if (e != hipSuccess) first = e;
  }
  for (int i = 0; i < 8; ++i) {
    if (p->ready[i]) (void)hipEventDestroy(p->ready[i]);
    if (p->free_[i]) (void)hipEventDestroy(p->free_[i]);
  }
  if (p->side) (void)hipStreamDestroy(p->side);
  delete p;
  if (first != hipSuccess)
    return als::fail(AS_EHIP, "as_pipeline_destroy: %s", hipGetErrorString(first));
  return AS_OK;
}
