// Batched decode-iteration attention over a paged KV cache, gfx950 (MI355X).
//
// Computes paper Section 2.2 Eq. 2, softmax(q K^T / sqrt(d_k)) V, for one
// query per (request, query head) against that request's kv_len cached keys
// and values.  Per Table 1 the work moves 2*s*h KV elements per token and
// performs as many multiply-adds: it is bound by HBM bandwidth, so the kernel
// is organised around streaming every K/V byte exactly once with fully
// coalesced 128-bit loads and enough of them in flight, not around a GEMM.
//
// Work split.  A request's KV sequence is cut into chunks of `chunk_tokens`
// tokens.  One workgroup (4 wavefronts) handles one (request, chunk, KV head)
// item; items of all requests are flattened into one list so that the time of
// a launch follows the total token count of the batch, not batch * longest
// request.  The list is built on the host and travels in the kernel arguments
// when the host knows the lengths and it is short enough, otherwise a plan
// kernel builds it on the device from kv_lens; either way long items run
// first.  Chunks of one request are merged exactly afterwards (combine
// kernel); a request that fits one chunk is finished by its workgroup directly.
//
// Inside a workgroup.  A tile is one 16-token block of one KV head: a
// contiguous [16][D] slab.  A wavefront owns every 4th tile of the chunk.
// One 128-bit load per lane covers 1 KiB of the slab: LPT = D*sizeof(T)/16
// lanes share a token, so a load instruction brings 64/LPT tokens and the
// wave runs 64/LPT independent online-softmax streams ("token groups").  The
// q.k partial products are summed over the LPT lanes with DPP row operations
// (no LDS traffic); p.v needs no cross-lane step because each lane keeps the
// output dimensions it loaded.  K/V tiles are double-buffered in registers:
// the loads of tile j+1 are issued before tile j is consumed.  With G query
// heads per KV head (grouped-query attention) one K/V tile in registers
// serves all G heads.  At the end the token groups of a wave are merged with
// cross-lane shuffles, the 4 waves through LDS.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <mutex>

#include "common.h"

namespace {

constexpr int kBlock = 16;      // tokens per KV block
constexpr int kWaves = 4;       // wavefronts per workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxChunk = 64 * kWaves * kBlock;  // one block id per lane per wave
constexpr float kNegInf = -__builtin_huge_valf();

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct bf16_t { uint16_t bits; };
struct f16_t { uint16_t bits; };
typedef _Float16 h16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h16x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 h16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int kPerLoad = 4; };
template <> struct Elem<bf16_t> { static constexpr int kPerLoad = 8; };
template <> struct Elem<f16_t> { static constexpr int kPerLoad = 8; };

// ------------------------------------------------------------------ workspace
// [0,256)            PlanHeader
// cu_chunks          int32[batch + 1]   first item of each request
// items              int4[max_items]    (request, chunk index, kv_len, slot of the partial result)
// part_ml            float2[max_items * H_q]   (running max in log2 units, sum)
// part_acc           float[max_items * H_q * D]
struct PlanHeader {
  int32_t total_items;
  int32_t pad[63];
};

struct WorkspaceLayout {
  size_t cu_off, items_off, ml_off, acc_off, total;
  int64_t max_items;
};

inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

WorkspaceLayout layout_for(const as_attn_params& p, int64_t max_items) {
  WorkspaceLayout w;
  w.max_items = max_items;
  w.cu_off = sizeof(PlanHeader);
  w.items_off = align256(w.cu_off + sizeof(int32_t) * (static_cast<size_t>(p.batch) + 1));
  w.ml_off = align256(w.items_off + sizeof(int4) * static_cast<size_t>(w.max_items));
  w.acc_off = align256(w.ml_off + sizeof(float2) * static_cast<size_t>(w.max_items) * p.num_q_heads);
  w.total = align256(w.acc_off + sizeof(float) * static_cast<size_t>(w.max_items) * p.num_q_heads *
                                     p.head_dim);
  return w;
}

// ------------------------------------------------------------------ plan
// Builds the item table on the device (launches too large for the plan that
// travels in the kernel arguments, and calls without host lengths).  A request
// of L tokens has n = ceil(L / chunk) chunks (one when L <= 0: it writes
// zeros).  Order of execution: every full chunk first (request-major), then
// each request's last chunk from long to short (64 length classes, counting
// sort), so that a launch ends on its smallest items.  An item's partial
// result goes to its canonical slot cu_chunks[request] + chunk, cu_chunks =
// exclusive scan of n.
// Every workgroup repeats the two 256-entry scans in LDS (thread t covers
// `per` consecutive requests) and fills its share of the full chunks; the
// requests inside a thread's segment are walked linearly.  Workgroup 0 also
// writes cu_chunks, the header and the last chunks (their order inside a
// length class depends on the run, the results do not: every item owns its
// slot).
__global__ __launch_bounds__(256) void plan_kernel(const int32_t* __restrict__ kv_lens, int batch,
                                                   int chunk, int max_len, PlanHeader* __restrict__ hdr,
                                                   int32_t* __restrict__ cu_chunks,
                                                   int4* __restrict__ items, int64_t max_items) {
  __shared__ int32_t all_incl[256];   // inclusive scan of chunks per thread segment
  __shared__ int32_t full_incl[256];  // inclusive scan of (chunks - 1)
  const int tid = threadIdx.x;
  const int per = (batch + 255) / 256;
  const int lo = min(batch, tid * per);
  const int hi = min(batch, lo + per);
  auto chunks_of = [&](int b) {
    const int32_t L = min(kv_lens[b], max_len);
    return L > 0 ? (L + chunk - 1) / chunk : 1;
  };
  int32_t sum = 0;
  for (int b = lo; b < hi; ++b) sum += chunks_of(b);
  all_incl[tid] = sum;
  full_incl[tid] = sum - (hi - lo);
  __syncthreads();
  // Hillis-Steele inclusive scans over the 256 segment sums
  for (int off = 1; off < 256; off <<= 1) {
    const int32_t va = tid >= off ? all_incl[tid - off] : 0;
    const int32_t vf = tid >= off ? full_incl[tid - off] : 0;
    __syncthreads();
    all_incl[tid] += va;
    full_incl[tid] += vf;
    __syncthreads();
  }
  const int32_t total = all_incl[255];
  const int32_t total_full = full_incl[255];
  if (blockIdx.x == 0) {
    int32_t run = all_incl[tid] - sum;
    for (int b = lo; b < hi; ++b) {
      cu_chunks[b] = run;
      run += chunks_of(b);
    }
    if (tid == 0) {
      cu_chunks[batch] = total;
      hdr->total_items = total;
    }
  }
  const int64_t n = total < max_items ? total : max_items;
  const int64_t n_full = total_full < n ? total_full : n;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + tid; i < n_full;
       i += static_cast<int64_t>(gridDim.x) * 256) {
    // segment with full_excl[seg] <= i < full_incl[seg]
    int a = 0, z = 255;
    while (a < z) {
      const int mid = (a + z) >> 1;
      if (full_incl[mid] > i) z = mid; else a = mid + 1;
    }
    int32_t f = a ? full_incl[a - 1] : 0;   // full chunks before request b
    int32_t s = a ? all_incl[a - 1] : 0;    // all chunks before request b
    int b = a * per;
    for (;; ++b) {                          // ends inside the segment: it holds item i
      const int nch = chunks_of(b);
      if (i < f + nch - 1) break;
      f += nch - 1;
      s += nch;
    }
    const int c = static_cast<int>(i - f);
    // a slot beyond the partial-result arrays can only come from a caller's bound that the lengths
    // exceed: the item is voided (length 0) instead of being allowed to write out of bounds
    items[i] = make_int4(b, c, s + c < max_items ? min(kv_lens[b], max_len) : 0, s + c);
  }
  if (blockIdx.x != 0) return;
  // last chunks: class 0 holds the longest (tokens in the chunk from chunk down
  // to chunk * 63/64 + 1), class 63 the shortest and the empty requests
  __shared__ int32_t cls_count[64];
  __shared__ int32_t cls_next[64];
  auto class_of = [&](int b, int nch) {
    const int32_t L = min(kv_lens[b], max_len);
    const int rem = L > 0 ? L - (nch - 1) * chunk : 1;   // 1 .. chunk
    return 63 - min(63, (rem - 1) * 64 / chunk);
  };
  if (tid < 64) cls_count[tid] = 0;
  __syncthreads();
  for (int b = lo; b < hi; ++b) atomicAdd(&cls_count[class_of(b, chunks_of(b))], 1);
  __syncthreads();
  if (tid == 0) {
    int32_t run = 0;
    for (int k = 0; k < 64; ++k) { cls_next[k] = run; run += cls_count[k]; }
  }
  __syncthreads();
  int32_t s = all_incl[tid] - sum;            // all chunks before this thread's segment
  for (int b = lo; b < hi; ++b) {
    const int nch = chunks_of(b);
    const int64_t i = total_full + atomicAdd(&cls_next[class_of(b, nch)], 1);
    if (i < n) items[i] = make_int4(b, nch - 1, s + nch - 1 < max_items ? min(kv_lens[b], max_len) : 0, s + nch - 1);
    s += nch;
  }
}

// ------------------------------------------------------------------ helpers
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the LPT lanes that share a token; every one of them gets the sum.
template <int LPT>
__device__ __forceinline__ float group_sum(float v) {
  if (LPT >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  if (LPT >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  if (LPT >= 8) v += dpp_move<0x141>(v);   // row_half_mirror
  if (LPT >= 16) v += dpp_move<0x140>(v);  // row_mirror
  if (LPT >= 32) v += __shfl_xor(v, 16);
  return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ uint16_t f32_to_f16_rne(float f) {
  const _Float16 h = static_cast<_Float16>(f);  // v_cvt_f16_f32, round to nearest even
  return __builtin_bit_cast(uint16_t, h);
}

// out_dtype: 0 fp32, 1 bf16, 2 fp16
__device__ __forceinline__ uint16_t f32_to_out16(float f, int out_dtype) {
  return out_dtype == AS_DTYPE_BF16 ? f32_to_bf16_rne(f) : f32_to_f16_rne(f);
}

// Results and split-KV partials leave through non-temporal stores: a workgroup
// writes a few hundred bytes after streaming hundreds of KiB, and ordinary
// (write-back cached) stores of that size were measured to cost far more than
// their share of bytes next to a saturated read stream.
__device__ __forceinline__ void store_out(char* out, size_t idx, float v, int out_dtype) {
  if (out_dtype == AS_DTYPE_F32) __builtin_nontemporal_store(v, reinterpret_cast<float*>(out) + idx);
  else __builtin_nontemporal_store(f32_to_out16(v, out_dtype), reinterpret_cast<uint16_t*>(out) + idx);
}

// dot of the EPL elements a lane holds of one key row with its slice of q
template <typename T> struct Dot;
template <> struct Dot<float> {
  // Reinterpret the whole vector, then index: a bit_cast applied to a single
  // element of the loaded vector makes this compiler read element 0 each time.
  __device__ static __forceinline__ float run(const u32x4& ku, const u32x4& qu) {
    const f32x4 k = __builtin_bit_cast(f32x4, ku);
    const f32x4 q = __builtin_bit_cast(f32x4, qu);
    float s = k.x * q.x;
    s = fmaf(k.y, q.y, s);
    s = fmaf(k.z, q.z, s);
    s = fmaf(k.w, q.w, s);
    return s;
  }
};
template <> struct Dot<bf16_t> {
  // v_dot2c_f32_bf16: two bf16 products accumulated into an fp32 register.
  // The operands are taken as pairs out of a whole <8 x bf16> value: casting
  // single 32-bit lanes of the loaded vector to <2 x bf16> makes this
  // compiler pick lane 0 for every pair.
  __device__ static __forceinline__ float run(const u32x4& ku, const u32x4& qu) {
    const bf16x8_t k = __builtin_bit_cast(bf16x8_t, ku);
    const bf16x8_t q = __builtin_bit_cast(bf16x8_t, qu);
    float s = 0.f;
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k, k, 0, 1), __builtin_shufflevector(q, q, 0, 1), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k, k, 2, 3), __builtin_shufflevector(q, q, 2, 3), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k, k, 4, 5), __builtin_shufflevector(q, q, 4, 5), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k, k, 6, 7), __builtin_shufflevector(q, q, 6, 7), s, false);
    return s;
  }
};

template <> struct Dot<f16_t> {
  // v_dot2c_f32_f16: two fp16 products accumulated into an fp32 register
  __device__ static __forceinline__ float run(const u32x4& ku, const u32x4& qu) {
    const h16x8_t k = __builtin_bit_cast(h16x8_t, ku);
    const h16x8_t q = __builtin_bit_cast(h16x8_t, qu);
    float s = 0.f;
    s = __builtin_amdgcn_fdot2(__builtin_shufflevector(k, k, 0, 1), __builtin_shufflevector(q, q, 0, 1), s, false);
    s = __builtin_amdgcn_fdot2(__builtin_shufflevector(k, k, 2, 3), __builtin_shufflevector(q, q, 2, 3), s, false);
    s = __builtin_amdgcn_fdot2(__builtin_shufflevector(k, k, 4, 5), __builtin_shufflevector(q, q, 4, 5), s, false);
    s = __builtin_amdgcn_fdot2(__builtin_shufflevector(k, k, 6, 7), __builtin_shufflevector(q, q, 6, 7), s, false);
    return s;
  }
};

// widen the EPL elements of one loaded 128-bit word to fp32
template <typename T> struct Widen;
template <> struct Widen<float> {
  __device__ static __forceinline__ void run(const u32x4& vu, float (&o)[4]) {
    const f32x4 v = __builtin_bit_cast(f32x4, vu);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct Widen<bf16_t> {
  __device__ static __forceinline__ void run(const u32x4& v, float (&o)[8]) {
    o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
    o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
  }
};

template <> struct Widen<f16_t> {
  __device__ static __forceinline__ void run(const u32x4& vu, float (&o)[8]) {
    const f32x8 w = __builtin_convertvector(__builtin_bit_cast(h16x8_t, vu), f32x8);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = w[e];
  }
};

__device__ __forceinline__ u32x4 load128(const char* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

struct AttnArgs {
  const char* q;
  const char* k_blocks;
  const char* v_blocks;
  const int32_t* block_table;
  const int32_t* kv_lens;
  char* out;
  const PlanHeader* hdr;
  const int4* items;
  float2* part_ml;
  float* part_acc;
  int32_t num_kv_heads;
  int32_t head_groups;  // workgroups per item: num_q_heads / G
  int32_t kv_div;       // head groups per KV head (1 when G covers the whole GQA group)
  int32_t num_blocks;
  int32_t max_blocks_per_seq;
  int32_t chunk;
  int32_t out_dtype;   // AS_DTYPE_* of out
  int32_t exact_grid;  // grid == total_items * head_groups exactly
  int32_t direct;      // every request is one chunk: item i is request i unless inline_plan reorders
  int32_t inline_plan; // the item table travels in the kernel arguments (InlinePlan)
  float c;             // scale * log2(e)
};

// Small launches carry their work plan in the kernel-argument segment instead
// of having a plan kernel write it to memory first: one 32-bit word per item,
// built on the host from the host copy of the lengths.  4 KiB of kernel
// arguments bound it.  A word holds (request << 20 | chunk << 10 | slot): slot
// is the item's canonical index (request-major), which is where its partial
// result goes, while the position of the word in the table is the order of
// execution -- full chunks first, then the requests' last (shorter) chunks
// from long to short, so that the launch ends on its smallest items.
constexpr int kInlineItems = 960;
static_assert(kInlineItems <= 1024, "chunk index and slot take 10 bits each");
struct InlinePlan {
  uint32_t item[kInlineItems];
};

// Workgroups are handed to the 8 XCDs round-robin by their linear index, and
// every XCD has its own L2 and address-translation cache.  Workgroups with
// neighbouring task indices read neighbouring slabs of the same KV blocks
// (the head index varies fastest), so the task index is derived from the
// workgroup index such that each XCD gets runs of 8 consecutive tasks: within
// every group of 64 workgroups, workgroup 8*k + x (XCD x) takes task 8*x + k.
// Measured on the streaming pattern of this kernel: +1.5 to 2.5 % bandwidth.
constexpr int kXcds = 8;
constexpr int kXcdRun = 8;
__device__ __forceinline__ int task_of_workgroup(int wg, int grid) {
  constexpr int per = kXcds * kXcdRun;
  const int base = wg / per * per;
  if (base + per > grid) return wg;  // ragged last group keeps the plain order
  const int r = wg - base;
  return base + (r % kXcds) * kXcdRun + r / kXcds;
}

// Online-softmax state of one token group for one query head.
template <int EPL>
struct HeadState {
  float m;  // running max of raw q.k (unscaled)
  float l;  // sum of exp2((s - m) * c)
  float acc[EPL];
};

template <typename T, int D, int G, bool MASKED>
__device__ __forceinline__ void consume_tile(const u32x4 (&kr)[kBlock * D * sizeof(T) / 1024],
                                             const u32x4 (&vr)[kBlock * D * sizeof(T) / 1024],
                                             const u32x4 (&qr)[G],
                                             HeadState<Elem<T>::kPerLoad> (&st)[G], float c,
                                             int first_token, int kv_len, int lane) {
  constexpr int EPL = Elem<T>::kPerLoad;
  constexpr int LPT = D / EPL;
  constexpr int TPI = 64 / LPT;
  constexpr int NLD = kBlock / TPI;

  bool valid[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) valid[i] = !MASKED || (first_token + i * TPI + lane / LPT < kv_len);

  float vf[NLD][EPL];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    Widen<T>::run(vr[i], vf[i]);
    if (MASKED) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) vf[i][e] = valid[i] ? vf[i][e] : 0.f;
    }
  }

#pragma unroll
  for (int g = 0; g < G; ++g) {
    float s[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      s[i] = group_sum<LPT>(Dot<T>::run(kr[i], qr[g]));
      if (MASKED) s[i] = valid[i] ? s[i] : kNegInf;
    }
    float mx = s[0];
#pragma unroll
    for (int i = 1; i < NLD; ++i) mx = fmaxf(mx, s[i]);
    const float m_new = fmaxf(st[g].m, mx);
    // a token group that has seen no valid token yet keeps m == -inf; use 0
    // as the reference there so that no inf - inf is formed
    const float ref = (MASKED && m_new == kNegInf) ? 0.f : m_new;
    const float alpha = fast_exp2((st[g].m - ref) * c);
    const float nref = -ref * c;
    float p[NLD];
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      p[i] = fast_exp2(fmaf(s[i], c, nref));
      if (MASKED) p[i] = valid[i] ? p[i] : 0.f;
      psum += p[i];
    }
    st[g].l = fmaf(st[g].l, alpha, psum);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float a = st[g].acc[e] * alpha;
#pragma unroll
      for (int i = 0; i < NLD; ++i) a = fmaf(p[i], vf[i][e], a);
      st[g].acc[e] = a;
    }
    st[g].m = m_new;
  }
}

template <typename T, int D>
__device__ __forceinline__ void load_tile(u32x4 (&r)[kBlock * D * sizeof(T) / 1024], const char* slab,
                                          int lane) {
  constexpr int NLD = kBlock * D * sizeof(T) / 1024;
  const char* p = slab + lane * 16;
#pragma unroll
  for (int i = 0; i < NLD; ++i) r[i] = load128(p + i * 1024);
}

// The same with ordinary loads, which the caches may retain: for launches in which several
// workgroups (slices of one wide group of query heads) read the same KV head's stream side by side.
template <typename T, int D>
__device__ __forceinline__ void load_tile_shared(u32x4 (&r)[kBlock * D * sizeof(T) / 1024], const char* slab,
                                                 int lane) {
  constexpr int NLD = kBlock * D * sizeof(T) / 1024;
  const char* p = slab + lane * 16;
#pragma unroll
  for (int i = 0; i < NLD; ++i) r[i] = *reinterpret_cast<const u32x4*>(p + i * 1024);
}

// merge state `o` (from another token group / wave) into `s`; both in raw-max units
template <int EPL>
__device__ __forceinline__ void merge_state(HeadState<EPL>& s, float om, float ol, const float (&oacc)[EPL],
                                            float c) {
  const float M = fmaxf(s.m, om);
  const float ref = (M == kNegInf) ? 0.f : M;
  const float a = fast_exp2((s.m - ref) * c);
  const float b = fast_exp2((om - ref) * c);
  s.l = s.l * a + ol * b;
#pragma unroll
  for (int e = 0; e < EPL; ++e) s.acc[e] = s.acc[e] * a + oacc[e] * b;
  s.m = M;
}

template <typename T, int D, int G>
__global__ __launch_bounds__(kThreads) void attn_kernel(AttnArgs a, InlinePlan ip) {
  constexpr int EPL = Elem<T>::kPerLoad;
  constexpr int LPT = D / EPL;
  constexpr int NLD = kBlock * D * sizeof(T) / 1024;
  constexpr size_t kSlabBytes = static_cast<size_t>(kBlock) * D * sizeof(T);

  __shared__ float sm_m[kWaves][G];
  __shared__ float sm_l[kWaves][G];
  __shared__ float sm_acc[kWaves][G][D];

  const int Hkv = a.num_kv_heads;
  const int task = task_of_workgroup(blockIdx.x, gridDim.x);
  const int item = task / a.head_groups;
  const int hg = task - item * a.head_groups;  // query heads hg*G .. hg*G+G-1
  const int h = hg / a.kv_div;                       // KV head they read
  if (!a.exact_grid && item >= a.hdr->total_items) return;
  // (request, chunk) of this item.  The block ids of the chunk are requested
  // before the length is known (index clamped into the table row), so that the
  // length and the ids arrive together instead of one after the other.
  int4 it = make_int4(item, 0, 0, 0);
  int slot = item;  // where this item's partial result goes
  if (a.inline_plan) {
    const uint32_t w = ip.item[item];
    it.x = static_cast<int>(w >> 20);
    it.y = static_cast<int>((w >> 10) & 0x3FFu);
    slot = static_cast<int>(w & 0x3FFu);
  } else if (!a.direct) {
    it = a.items[item];
    slot = it.w;
  }
  const int b = it.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int t0 = it.y * a.chunk;
  // lane i holds the id of tile wave + 4*i of the chunk
  int my_id = a.block_table[static_cast<size_t>(b) * a.max_blocks_per_seq +
                            min(t0 / kBlock + wave + kWaves * lane, a.max_blocks_per_seq - 1)];
  my_id = min(max(my_id, 0), a.num_blocks - 1);
  const int kv_len = (a.direct || a.inline_plan) ? min(a.kv_lens[b], a.max_blocks_per_seq * kBlock)
                                                 : it.z;  // cut to the block_table row
  const int Hq = a.head_groups * G;
  const int ntok = min(kv_len - t0, a.chunk);
  if (ntok <= 0) {  // kv_len <= 0: defined result is zeros
    for (int i = tid; i < G * D; i += kThreads) {
      const size_t o = (static_cast<size_t>(b) * Hq + hg * G) * D + i;
      store_out(a.out, o, 0.f, a.out_dtype);
    }
    return;
  }
  const int ntiles = (ntok + kBlock - 1) / kBlock;
  const bool single = kv_len <= a.chunk;

  const int my_tiles = ntiles > wave ? (ntiles - wave + kWaves - 1) / kWaves : 0;

  u32x4 qr[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qr[g] = *reinterpret_cast<const u32x4*>(a.q + ((static_cast<size_t>(b) * Hq + hg * G + g) * D +
                                                  (lane % LPT) * EPL) * sizeof(T));

  HeadState<EPL> st[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    st[g].m = kNegInf;
    st[g].l = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) st[g].acc[e] = 0.f;
  }

  const float c = a.c;
  const size_t head_off = static_cast<size_t>(h) * kSlabBytes;
  const size_t block_stride = static_cast<size_t>(Hkv) * kSlabBytes;

  u32x4 kA[NLD], vA[NLD], kB[NLD], vB[NLD];
  auto tile_off = [&](int i) {
    return static_cast<size_t>(__builtin_amdgcn_readlane(my_id, i)) * block_stride + head_off;
  };
  if (my_tiles > 0) {
    const size_t off = tile_off(0);
    load_tile<T, D>(kA, a.k_blocks + off, lane);
    load_tile<T, D>(vA, a.v_blocks + off, lane);
  }
  // Only the chunk's last tile can be partial.  The hot loop takes pairs of
  // full tiles with the unmasked code; at most two tiles are left for the
  // masked code after it.
  const bool owns_partial = (ntok % kBlock) != 0 && ((ntiles - 1) % kWaves) == wave;
  const int full_tiles = my_tiles - (owns_partial ? 1 : 0);
  int i = 0;
  for (; i + 2 <= full_tiles; i += 2) {
    {
      const size_t off = tile_off(i + 1);
      load_tile<T, D>(kB, a.k_blocks + off, lane);
      load_tile<T, D>(vB, a.v_blocks + off, lane);
    }
    consume_tile<T, D, G, false>(kA, vA, qr, st, c, 0, 0, lane);
    if (i + 2 < my_tiles) {
      const size_t off = tile_off(i + 2);
      load_tile<T, D>(kA, a.k_blocks + off, lane);
      load_tile<T, D>(vA, a.v_blocks + off, lane);
    }
    consume_tile<T, D, G, false>(kB, vB, qr, st, c, 0, 0, lane);
  }
  if (i < my_tiles) {
    const bool haveB = i + 1 < my_tiles;
    if (haveB) {
      const size_t off = tile_off(i + 1);
      load_tile<T, D>(kB, a.k_blocks + off, lane);
      load_tile<T, D>(vB, a.v_blocks + off, lane);
    }
    consume_tile<T, D, G, true>(kA, vA, qr, st, c, t0 + (wave + kWaves * i) * kBlock, kv_len, lane);
    if (haveB)
      consume_tile<T, D, G, true>(kB, vB, qr, st, c, t0 + (wave + kWaves * (i + 1)) * kBlock, kv_len, lane);
  }

  // merge the 64/LPT token groups of the wave (lanes that hold the same dims)
#pragma unroll
  for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float om = __shfl_xor(st[g].m, off);
      const float ol = __shfl_xor(st[g].l, off);
      float oacc[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) oacc[e] = __shfl_xor(st[g].acc[e], off);
      merge_state<EPL>(st[g], om, ol, oacc, c);
    }
  }
  if (lane < LPT) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (lane == 0) { sm_m[wave][g] = st[g].m; sm_l[wave][g] = st[g].l; }
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_acc[wave][g][lane * EPL + e] = st[g].acc[e];
    }
  }
  __syncthreads();

  // final merge over the waves: one thread per (head, output dimension)
  for (int idx = tid; idx < G * D; idx += kThreads) {
    const int g = idx / D;
    const int d = idx - g * D;
    float M = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][g]);
    float l = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float f = fast_exp2((sm_m[w][g] - M) * c);  // M is finite: the chunk has >= 1 token
      l = fmaf(sm_l[w][g], f, l);
      acc = fmaf(sm_acc[w][g][d], f, acc);
    }
    const int hq = hg * G + g;
    if (single) {
      const float o = acc / l;
      const size_t oi = (static_cast<size_t>(b) * Hq + hq) * D + d;
      store_out(a.out, oi, o, a.out_dtype);
    } else {
      const size_t pi = static_cast<size_t>(slot) * Hq + hq;
      __builtin_nontemporal_store(acc, a.part_acc + pi * D + d);
      if (d == 0) {
        __builtin_nontemporal_store(M * c, &a.part_ml[pi].x);
        __builtin_nontemporal_store(l, &a.part_ml[pi].y);
      }
    }
  }
}

// ------------------------------------------------------------------ MFMA path
// Grouped-query attention (G query heads share one KV head), bf16 or fp16,
// D = 128.
// With G >= 4 the vector-ALU kernel above is bound by its own arithmetic (each
// K/V element is used G times), so the two contractions move to the matrix
// cores; the K/V stream, the work split and the merge stay as they are.
//
//   S^T[token][head] = K_tile[16 x 128] . Q^T[128 x 16]      4 x mfma 16x16x32
//   O^T[dim][head]  += V_tile^T[128 x 16] . P^T[16 x 16]     2 x 8 x mfma 16x16x16
//
// Operand layouts (lane l, c = l % 16, r = l / 16):
//  * A operand of a 16x16x32 MFMA wants lane l to hold 8 consecutive
//    contraction values of matrix row c.  The coalesced global load gives a
//    lane a token picked by r and a 16-byte dimension chunk picked by c -- the
//    transpose.  K therefore passes through a per-wave LDS tile (rows padded
//    to 272 B: conflict-free 128-bit writes and reads), written in load layout
//    and read back in operand layout.  Token t is put in LDS row
//    4*(t%4) + t/4, so that result register i of lane l (matrix row 4r+i)
//    belongs to token 4i+r: the token whose V elements the same lane loaded.
//  * B operand = Q^T: lane l holds q[head c][dims of contraction slots]; heads
//    past G are zero columns.
//  * The result S^T has the head on c and tokens on (r, i): a lane owns ONE
//    head, so the online softmax costs the same for any G <= 16.
//  * P^T (B operand of the second MFMA) is exactly what the lane computed:
//    probabilities of its 4 tokens for head c, as two terms hi + lo in the
//    element type (two MFMAs per accumulator), so that the weights keep 16 or
//    more significant bits instead of the 8 of a single bf16.
//  * V needs no LDS: the lane's four loads hold, for each of its 8 dimensions,
//    the 4 tokens (4i+r) -- the A operand (row = dimension 8c+e, 4 contraction
//    values) once the 16-bit halves are gathered with v_perm.  Output register
//    i of accumulator e is dimension 32r+8i+e of head c: the lane that owns a
//    head's softmax state also owns that head's outputs, so rescaling is
//    lane-local.
// The sum l is accumulated from the fp32 probabilities.
constexpr int kLdsRow = 272;                    // 256 B of a K row + 16 B pad
constexpr int kLdsKTile = kBlock * kLdsRow;     // per wave
constexpr int kMfmaHeads = 16;      // query heads per MFMA column block
#ifndef AS_MFMA_MAX_HEADS
#define AS_MFMA_MAX_HEADS 32
#endif
constexpr int kMfmaMaxHeads = AS_MFMA_MAX_HEADS;
#ifndef AS_SHARED_LOADS
#define AS_SHARED_LOADS true
#endif  // query heads one workgroup serves (1 or 2 column blocks)

// The two 16-bit element types differ only in the MFMA opcodes and in how
// probabilities are rounded to the element type and widened back.
template <typename T> struct Mfma;
template <> struct Mfma<bf16_t> {
  __device__ static __forceinline__ f32x4 qk(const u32x4& k, const u32x4& q, const f32x4& s) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, k),
                                                   __builtin_bit_cast(bf16x8_t, q), s, 0, 0, 0);
  }
  __device__ static __forceinline__ f32x4 pv(const u32x2& v, const u32x2& p, const f32x4& o) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, v),
                                                     __builtin_bit_cast(s16x4, p), o, 0, 0, 0);
  }
  // two probabilities rounded to the element type (round to nearest even), packed
  __device__ static __forceinline__ uint32_t pack(float a, float b) {
    const f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
  }
  __device__ static __forceinline__ float first(uint32_t w) { return bf16_lo(w); }
  __device__ static __forceinline__ float second(uint32_t w) { return bf16_hi(w); }
};
template <> struct Mfma<f16_t> {
  __device__ static __forceinline__ f32x4 qk(const u32x4& k, const u32x4& q, const f32x4& s) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h16x8_t, k),
                                                  __builtin_bit_cast(h16x8_t, q), s, 0, 0, 0);
  }
  __device__ static __forceinline__ f32x4 pv(const u32x2& v, const u32x2& p, const f32x4& o) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(h16x4_t, v),
                                                 __builtin_bit_cast(h16x4_t, p), o, 0, 0, 0);
  }
  __device__ static __forceinline__ uint32_t pack(float a, float b) {
    const f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, h16x2_t));
  }
  __device__ static __forceinline__ float first(uint32_t w) {
    return __builtin_convertvector(__builtin_bit_cast(h16x2_t, w), f32x2).x;
  }
  __device__ static __forceinline__ float second(uint32_t w) {
    return __builtin_convertvector(__builtin_bit_cast(h16x2_t, w), f32x2).y;
  }
};

// One tile for NG groups of 16 query heads: the K tile goes through LDS once
// and each A operand read from it feeds NG MFMAs (one per head group); the V
// halves are gathered once and feed NG x 4 MFMAs.  Only the softmax state and
// the probabilities exist per group, so a workgroup of 32 heads reads the K/V
// stream once where two workgroups of 16 would read it twice.
template <typename T, bool MASKED, int NG>
__device__ __forceinline__ void mfma_tile(const u32x4 (&kr)[4], const u32x4 (&vr)[4],
                                          const u32x4 (&qb)[NG][4], char* lds, f32x4 (&acc)[NG][8],
                                          float (&m_run)[NG], float (&l_run)[NG], float c, int first_token,
                                          int kv_len, int lane) {
  const int col = lane & 15;
  const int rg = lane >> 4;
  // K: load layout -> LDS (row 4*rg+i holds token 4*i+rg), then operand layout
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<u32x4*>(lds + (4 * rg + i) * kLdsRow + col * 16) = kr[i];
  __builtin_amdgcn_wave_barrier();
  f32x4 s[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) s[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const u32x4 ku = *reinterpret_cast<const u32x4*>(lds + col * kLdsRow + (4 * j + rg) * 16);
#pragma unroll
    for (int g = 0; g < NG; ++g) s[g] = Mfma<T>::qk(ku, qb[g][j], s[g]);
  }
  __builtin_amdgcn_wave_barrier();

  bool valid[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) valid[i] = !MASKED || (first_token + 4 * i + rg < kv_len);

  u32x2 pB[NG], pB2[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    float sv[4] = {s[g].x, s[g].y, s[g].z, s[g].w};
    if (MASKED) {
#pragma unroll
      for (int i = 0; i < 4; ++i) sv[i] = valid[i] ? sv[i] : kNegInf;
    }
    float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));           // max over the tile's 16 tokens, per head
    const float m_new = fmaxf(m_run[g], mx);       // finite: a tile has at least one valid token
    const float alpha = fast_exp2((m_run[g] - m_new) * c);
    const float nref = -m_new * c;
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = fast_exp2(fmaf(sv[i], c, nref));
      if (MASKED) p[i] = valid[i] ? p[i] : 0.f;
    }
    const uint32_t w01 = Mfma<T>::pack(p[0], p[1]);
    const uint32_t w23 = Mfma<T>::pack(p[2], p[3]);
    // second term of the two-term representation p = hi + lo (each in the
    // element type): the matrix cores have cycles to spare next to the K/V
    // stream, and two terms carry 16 (bf16) or 22 (fp16) bits of the fp32 weight
    const uint32_t x01 = Mfma<T>::pack(p[0] - Mfma<T>::first(w01), p[1] - Mfma<T>::second(w01));
    const uint32_t x23 = Mfma<T>::pack(p[2] - Mfma<T>::first(w23), p[3] - Mfma<T>::second(w23));
    const float psum = (p[0] + p[1]) + (p[2] + p[3]);
    l_run[g] = fmaf(l_run[g], alpha, psum);
    m_run[g] = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
    }
    pB[g] = u32x2{w01, w23};
    pB2[g] = u32x2{x01, x23};
  }

  // V: gather the 16-bit halves of the 4 tokens for each of the lane's 8 dims
  u32x4 v0 = vr[0], v1 = vr[1], v2 = vr[2], v3 = vr[3];
  if (MASKED) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    v0 = valid[0] ? v0 : zero; v1 = valid[1] ? v1 : zero;
    v2 = valid[2] ? v2 : zero; v3 = valid[3] ? v3 : zero;
  }
  const uint32_t a0[4] = {v0.x, v0.y, v0.z, v0.w};
  const uint32_t a1[4] = {v1.x, v1.y, v1.z, v1.w};
  const uint32_t a2[4] = {v2.x, v2.y, v2.z, v2.w};
  const uint32_t a3[4] = {v3.x, v3.y, v3.z, v3.w};
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const u32x2 lo = {__builtin_amdgcn_perm(a1[w], a0[w], 0x05040100u),
                      __builtin_amdgcn_perm(a3[w], a2[w], 0x05040100u)};
    const u32x2 hi = {__builtin_amdgcn_perm(a1[w], a0[w], 0x07060302u),
                      __builtin_amdgcn_perm(a3[w], a2[w], 0x07060302u)};
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      acc[g][2 * w] = Mfma<T>::pv(lo, pB[g], acc[g][2 * w]);
      acc[g][2 * w + 1] = Mfma<T>::pv(hi, pB[g], acc[g][2 * w + 1]);
      acc[g][2 * w] = Mfma<T>::pv(lo, pB2[g], acc[g][2 * w]);
      acc[g][2 * w + 1] = Mfma<T>::pv(hi, pB2[g], acc[g][2 * w + 1]);
    }
  }
}

// G = query heads per workgroup (<= 16 * NG), D = 128, T = bf16_t or f16_t.
template <typename T, int NG, bool SHARED = false>
__global__ __launch_bounds__(kThreads) void attn_mfma_kernel(AttnArgs a, int G, InlinePlan ip) {
  constexpr int D = 128;
  constexpr int kHeads = kMfmaHeads * NG;
  constexpr size_t kSlabBytes = static_cast<size_t>(kBlock) * D * 2;
  // the K transpose tiles (loop) and the cross-wave merge buffers (epilogue)
  // share one allocation; a barrier separates the two uses
  // merge rows are padded by 4 floats: a lane's 8 x 128-bit writes of its 32
  // consecutive output dimensions then fall on distinct banks across the 8
  // lanes (neighbouring heads) that one LDS cycle serves
  constexpr int kMergeRow = D + 4;
  constexpr int kMergeBytes = kWaves * kHeads * kMergeRow * 4;
  __shared__ __attribute__((aligned(16))) char smem[kMergeBytes];
  __shared__ float sm_m[kWaves][kHeads];
  __shared__ float sm_l[kWaves][kHeads];
  static_assert(kWaves * kLdsKTile <= kMergeBytes, "K tiles must fit the shared buffer");

  const int Hkv = a.num_kv_heads;
  const int task = task_of_workgroup(blockIdx.x, gridDim.x);
  const int item = task / a.head_groups;
  const int hg = task - item * a.head_groups;
  const int h = hg / a.kv_div;
  if (!a.exact_grid && item >= a.hdr->total_items) return;
  // (request, chunk) of this item.  The block ids of the chunk are requested
  // before the length is known (index clamped into the table row), so that the
  // length and the ids arrive together instead of one after the other.
  int4 it = make_int4(item, 0, 0, 0);
  int slot = item;  // where this item's partial result goes
  if (a.inline_plan) {
    const uint32_t w = ip.item[item];
    it.x = static_cast<int>(w >> 20);
    it.y = static_cast<int>((w >> 10) & 0x3FFu);
    slot = static_cast<int>(w & 0x3FFu);
  } else if (!a.direct) {
    it = a.items[item];
    slot = it.w;
  }
  const int b = it.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int t0 = it.y * a.chunk;
  // lane i holds the id of tile wave + 4*i of the chunk
  int my_id = a.block_table[static_cast<size_t>(b) * a.max_blocks_per_seq +
                            min(t0 / kBlock + wave + kWaves * lane, a.max_blocks_per_seq - 1)];
  my_id = min(max(my_id, 0), a.num_blocks - 1);
  const int kv_len = (a.direct || a.inline_plan) ? min(a.kv_lens[b], a.max_blocks_per_seq * kBlock)
                                                 : it.z;  // cut to the block_table row
  const int Hq = a.head_groups * G;
  const int col = lane & 15;
  const int rg = lane >> 4;
  const int ntok = min(kv_len - t0, a.chunk);
  if (ntok <= 0) {
    for (int i = tid; i < G * D; i += kThreads) {
      const size_t o = (static_cast<size_t>(b) * Hq + hg * G) * D + i;
      store_out(a.out, o, 0.f, a.out_dtype);
    }
    return;
  }
  const int ntiles = (ntok + kBlock - 1) / kBlock;
  const bool single = kv_len <= a.chunk;
  const int my_tiles = ntiles > wave ? (ntiles - wave + kWaves - 1) / kWaves : 0;

  // Q^T operands: group g, head 16*g + col, dims 8*(4j+rg) .. +8 for MFMA j; zero past G
  u32x4 qb[NG][4];
  {
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int head = kMfmaHeads * g + col;
      const char* qrow = a.q + (static_cast<size_t>(b) * Hq + hg * G + (head < G ? head : 0)) * D * 2;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x4 w = *reinterpret_cast<const u32x4*>(qrow + (4 * j + rg) * 16);
        w = head < G ? w : zero;
        qb[g][j] = w;
      }
    }
  }

  f32x4 acc[NG][8];
  float m_run[NG], l_run[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    m_run[g] = kNegInf;
    l_run[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float c = a.c;
  char* lds = smem + wave * kLdsKTile;
  const size_t head_off = static_cast<size_t>(h) * kSlabBytes;
  const size_t block_stride = static_cast<size_t>(Hkv) * kSlabBytes;

  u32x4 kA[4], vA[4], kB[4], vB[4];
  auto ld = [&](u32x4 (&r)[4], const char* slab) {
    if constexpr (SHARED) load_tile_shared<T, D>(r, slab, lane);
    else load_tile<T, D>(r, slab, lane);
  };
  auto tile_off = [&](int i) {
    return static_cast<size_t>(__builtin_amdgcn_readlane(my_id, i)) * block_stride + head_off;
  };
  if (my_tiles > 0) {
    const size_t off = tile_off(0);
    ld(kA, a.k_blocks + off);
    ld(vA, a.v_blocks + off);
  }
  // Only the chunk's last tile can be partial.  The hot loop takes pairs of
  // full tiles with the unmasked code; at most two tiles are left for the
  // masked code after it.
  const bool owns_partial = (ntok % kBlock) != 0 && ((ntiles - 1) % kWaves) == wave;
  const int full_tiles = my_tiles - (owns_partial ? 1 : 0);
  int i = 0;
  for (; i + 2 <= full_tiles; i += 2) {
    {
      const size_t off = tile_off(i + 1);
      ld(kB, a.k_blocks + off);
      ld(vB, a.v_blocks + off);
    }
    mfma_tile<T, false, NG>(kA, vA, qb, lds, acc, m_run, l_run, c, 0, 0, lane);
    if (i + 2 < my_tiles) {
      const size_t off = tile_off(i + 2);
      ld(kA, a.k_blocks + off);
      ld(vA, a.v_blocks + off);
    }
    mfma_tile<T, false, NG>(kB, vB, qb, lds, acc, m_run, l_run, c, 0, 0, lane);
  }
  if (i < my_tiles) {
    const bool haveB = i + 1 < my_tiles;
    if (haveB) {
      const size_t off = tile_off(i + 1);
      ld(kB, a.k_blocks + off);
      ld(vB, a.v_blocks + off);
    }
    mfma_tile<T, true, NG>(kA, vA, qb, lds, acc, m_run, l_run, c, t0 + (wave + kWaves * i) * kBlock, kv_len, lane);
    if (haveB)
      mfma_tile<T, true, NG>(kB, vB, qb, lds, acc, m_run, l_run, c, t0 + (wave + kWaves * (i + 1)) * kBlock, kv_len, lane);
  }

  // each row group summed its own 4 tokens per tile; m is already common
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    l_run[g] += __shfl_xor(l_run[g], 16);
    l_run[g] += __shfl_xor(l_run[g], 32);
  }

  __syncthreads();  // every wave is done with its K tile: the buffer becomes merge space
  float* sm_o = reinterpret_cast<float*>(smem);  // [wave][head][kMergeRow]
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int head = kMfmaHeads * g + col;
    if (head < G) {
      if (rg == 0) { sm_m[wave][head] = m_run[g]; sm_l[wave][head] = l_run[g]; }
      // register i of accumulator e is dimension 32*rg + 8*i + e: the lane owns
      // 32 consecutive dimensions of its head, written as 8 float4
      float* row = sm_o + (wave * kHeads + head) * kMergeRow + 32 * rg;
#pragma unroll
      for (int i2 = 0; i2 < 4; ++i2) {
        const f32x4 lo4 = {acc[g][0][i2], acc[g][1][i2], acc[g][2][i2], acc[g][3][i2]};
        const f32x4 hi4 = {acc[g][4][i2], acc[g][5][i2], acc[g][6][i2], acc[g][7][i2]};
        *reinterpret_cast<f32x4*>(row + 8 * i2) = lo4;
        *reinterpret_cast<f32x4*>(row + 8 * i2 + 4) = hi4;
      }
    }
  }
  __syncthreads();

  for (int idx = tid; idx < G * D; idx += kThreads) {
    const int g = idx / D;
    const int d = idx - g * D;
    float M = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][g]);
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float f = fast_exp2((sm_m[w][g] - M) * c);
      l = fmaf(sm_l[w][g], f, l);
      o = fmaf(sm_o[(w * kHeads + g) * kMergeRow + d], f, o);
    }
    const int hq = hg * G + g;
    if (single) {
      const float r = o / l;
      const size_t oi = (static_cast<size_t>(b) * Hq + hq) * D + d;
      store_out(a.out, oi, r, a.out_dtype);
    } else {
      const size_t pi = static_cast<size_t>(slot) * Hq + hq;
      __builtin_nontemporal_store(o, a.part_acc + pi * D + d);
      if (d == 0) {
        __builtin_nontemporal_store(M * c, &a.part_ml[pi].x);
        __builtin_nontemporal_store(l, &a.part_ml[pi].y);
      }
    }
  }
}

// ------------------------------------------------------------------ combine
// Exact merge of a request's chunk partials (the re-association identity of
// the online softmax): with M = max_i m_i,
//   out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i.
// D/4 lanes per (request, query head); each lane owns 4 output dimensions.
struct InlineFirst {
  uint16_t first[2 * kInlineItems];  // first item of each request, batch + 1 entries
};

template <int D>
__global__ __launch_bounds__(256) void combine_kernel(const int32_t* __restrict__ cu_chunks,
                                                      InlineFirst icu, int use_inline,
                                                      const float2* __restrict__ part_ml,
                                                      const float* __restrict__ part_acc,
                                                      char* __restrict__ out, int batch, int Hq,
                                                      int out_dtype, int max_items) {
  constexpr int LPP = D / 4;  // lanes per (request, head): an aligned group inside one wavefront
  const int pair = blockIdx.x * (256 / LPP) + threadIdx.x / LPP;
  const int sub = threadIdx.x % LPP;
  if (pair >= batch * Hq) return;  // the whole lane group leaves together
  const int b = pair / Hq;
  const int hq = pair - b * Hq;
  const int first = use_inline ? icu.first[b] : cu_chunks[b];
  int n = (use_inline ? icu.first[b + 1] : cu_chunks[b + 1]) - first;
  if (n <= 1) return;  // finished by the attention kernel itself
  if (first >= max_items) return;      // only when a caller's bound on the lengths did not hold:
  n = min(n, max_items - first);       // stay inside the partial-result arrays
  // Few dependent memory round trips instead of one per chunk: lane `sub` fetches (m, l) of chunk
  // `sub`, the group's maximum and weights come from cross-lane steps, and the accumulator rows are
  // requested eight at a time before any of them is used.  More than LPP chunks: further rounds,
  // rescaled like an online softmax.
  float M = kNegInf, l = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int base = 0; base < n; base += LPP) {
    const int cnt = min(n - base, LPP);
    const bool have = sub < cnt;
    const float2 ml = have ? part_ml[static_cast<size_t>(first + base + sub) * Hq + hq] : make_float2(kNegInf, 0.f);
    float mx = ml.x;
#pragma unroll
    for (int off = LPP / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, LPP));
    const float Mn = fmaxf(M, mx);                    // finite: every chunk holds at least one token
    const float resc = fast_exp2(M - Mn);             // 0 in the first round (M = -inf)
    acc.x *= resc; acc.y *= resc; acc.z *= resc; acc.w *= resc;
    l *= resc;
    M = Mn;
    const float f = have ? fast_exp2(ml.x - M) : 0.f;
    float lw = ml.y * f;
#pragma unroll
    for (int off = LPP / 2; off > 0; off >>= 1) lw += __shfl_xor(lw, off, LPP);
    l += lw;
    for (int j0 = 0; j0 < cnt; j0 += 8) {
      float4 v[8];
      float fj[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int jc = min(j0 + u, cnt - 1);          // clamped: rows past the end get weight 0
        const float w = __shfl(f, jc, LPP);
        fj[u] = (j0 + u < cnt) ? w : 0.f;
        v[u] = *reinterpret_cast<const float4*>(part_acc + (static_cast<size_t>(first + base + jc) * Hq + hq) * D + sub * 4);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc.x = fmaf(v[u].x, fj[u], acc.x); acc.y = fmaf(v[u].y, fj[u], acc.y);
        acc.z = fmaf(v[u].z, fj[u], acc.z); acc.w = fmaf(v[u].w, fj[u], acc.w);
      }
    }
  }
  const float inv = 1.f / l;
  const size_t oi = (static_cast<size_t>(b) * Hq + hq) * D + sub * 4;
  const float o0 = acc.x * inv, o1 = acc.y * inv, o2 = acc.z * inv, o3 = acc.w * inv;
  if (out_dtype != AS_DTYPE_F32) {
    uint2 w;
    w.x = f32_to_out16(o0, out_dtype) | (static_cast<uint32_t>(f32_to_out16(o1, out_dtype)) << 16);
    w.y = f32_to_out16(o2, out_dtype) | (static_cast<uint32_t>(f32_to_out16(o3, out_dtype)) << 16);
    *reinterpret_cast<uint2*>(out + oi * 2) = w;
  } else {
    *reinterpret_cast<float4*>(out + oi * 4) = make_float4(o0, o1, o2, o3);
  }
}

// ------------------------------------------------------------------ read sweep
// Streams the same K/V bytes with the same work split and folds them with
// XOR: the bandwidth ceiling of this access pattern.
template <int NLD>
__global__ __launch_bounds__(kThreads) void sweep_kernel(AttnArgs a, InlinePlan ip, size_t slab_bytes,
                                                         uint32_t* __restrict__ wg_sums) {
  const int Hkv = a.num_kv_heads;
  const int task = task_of_workgroup(blockIdx.x, gridDim.x);
  const int item = task / Hkv;
  const int h = task - item * Hkv;
  if (!a.exact_grid && item >= a.hdr->total_items) {
    if (threadIdx.x == 0) wg_sums[blockIdx.x] = 0;
    return;
  }
  // the same three sources of the work plan as the attention kernels
  int4 it = make_int4(item, 0, 0, 0);
  if (a.inline_plan) {
    const uint32_t w = ip.item[item];
    it.x = static_cast<int>(w >> 20);
    it.y = static_cast<int>((w >> 10) & 0x3FFu);
  } else if (!a.direct) {
    it = a.items[item];
  }
  const int b = it.x;
  const int kv_len = (a.direct || a.inline_plan) ? min(a.kv_lens[b], a.max_blocks_per_seq * kBlock)
                                                 : it.z;  // cut to the block_table row
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int t0 = it.y * a.chunk;
  const int ntok = max(min(kv_len - t0, a.chunk), 0);
  const int ntiles = (ntok + kBlock - 1) / kBlock;
  const int my_tiles = ntiles > wave ? (ntiles - wave + kWaves - 1) / kWaves : 0;
  int my_id = 0;
  if (lane < my_tiles) {
    my_id = a.block_table[static_cast<size_t>(b) * a.max_blocks_per_seq + t0 / kBlock + wave + kWaves * lane];
    my_id = min(max(my_id, 0), a.num_blocks - 1);
  }
  const size_t head_off = static_cast<size_t>(h) * slab_bytes;
  const size_t block_stride = static_cast<size_t>(Hkv) * slab_bytes;
  u32x4 x = {0, 0, 0, 0};
  // same software pipeline as the attention kernel: the K and V slabs of the
  // next tile are requested before the current tile is folded
  u32x4 rA[2 * NLD], rB[2 * NLD];
  auto issue = [&](u32x4 (&r)[2 * NLD], int i) {
    const size_t off = static_cast<size_t>(__builtin_amdgcn_readlane(my_id, i)) * block_stride + head_off;
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      r[j] = load128(a.k_blocks + off + lane * 16 + j * 1024);
      r[NLD + j] = load128(a.v_blocks + off + lane * 16 + j * 1024);
    }
  };
  if (my_tiles > 0) issue(rA, 0);
  for (int i = 0; i < my_tiles; i += 2) {
    const bool haveB = i + 1 < my_tiles;
    if (haveB) issue(rB, i + 1);
#pragma unroll
    for (int j = 0; j < 2 * NLD; ++j) x ^= rA[j];
    if (i + 2 < my_tiles) issue(rA, i + 2);
    if (haveB) {
#pragma unroll
      for (int j = 0; j < 2 * NLD; ++j) x ^= rB[j];
    }
  }
  uint32_t r = x.x ^ x.y ^ x.z ^ x.w;
  for (int off = 32; off > 0; off >>= 1) r ^= __shfl_xor(r, off);
  // one word per workgroup, folded into the caller's 256 slots by a second
  // small kernel (an atomic per workgroup next to the saturated read stream
  // costs several per cent of the bandwidth this kernel exists to measure)
  __shared__ uint32_t wave_sum[kWaves];
  if (lane == 0) wave_sum[wave] = r;
  __syncthreads();
  if (tid == 0) {
    uint32_t t = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) t ^= wave_sum[w];
    __builtin_nontemporal_store(t, wg_sums + blockIdx.x);
  }
}

// checksum[s] ^= XOR of wg_sums[i] over i = s (mod 256)
__global__ __launch_bounds__(256) void sweep_fold_kernel(const uint32_t* __restrict__ wg_sums, int64_t n,
                                                         uint32_t* __restrict__ checksum) {
  uint32_t t = 0;
  for (int64_t i = threadIdx.x; i < n; i += 256) t ^= wg_sums[i];
  checksum[threadIdx.x] ^= t;
}

// ------------------------------------------------------------------ host side
// Which kernel serves these parameters and how many query heads one workgroup
// takes.  Matrix-core path: 16-bit inputs, D = 128, grouped-query shapes where
// the vector-ALU kernel is bound by its own arithmetic; one workgroup takes up
// to 32 heads of a group (two MFMA column blocks fed by one K/V read), wider
// groups are cut into 32s, 16s or 8s.  Vector-ALU
// path: the largest divisor of the group up to 8, so that one K/V read serves
// as many heads as possible; what is left of a wider group is covered by
// several workgroups reading the same KV head.
struct KernelChoice {
  bool mfma;
  int heads;  // query heads per workgroup
};
KernelChoice choose_kernel(const as_attn_params& p) {
  const int group = p.num_q_heads / p.num_kv_heads;
  if (p.dtype != AS_DTYPE_F32 && p.head_dim == 128 && group >= 4 && !(p.flags & AS_ATTN_NO_MFMA)) {
    if (group <= kMfmaMaxHeads) return {true, group};       // the whole group: one read of the KV head
    if (group % kMfmaMaxHeads == 0) return {true, kMfmaMaxHeads};
    if (group % 16 == 0) return {true, 16};
    if (group % 8 == 0) return {true, 8};
  }
  int g = 1;
  for (int d = 2; d <= 8; ++d)
    if (group % d == 0) g = d;
  return {false, g};
}

int pick_chunk(const as_attn_params& p, int64_t total_tokens) {
  if (p.chunk_tokens > 0) return p.chunk_tokens;
  // Long chunks amortise what a workgroup pays once (its start-up, its merge
  // and above all the stores of its result, which cost far more than their
  // bytes next to a saturated read stream); short chunks shorten the tail of
  // the launch, where the last workgroups run next to idle compute units.
  // With a per-item overhead worth o tokens, S concurrently resident
  // workgroups and a tail that grows with the chunk, the cost
  //   o * (T / chunk) / S + tail(chunk)          (T = tokens * KV heads)
  // is smallest at chunk = sqrt(k T).  Because items run longest-first the
  // tail term is small; sweeps on MI355X put k at 1.5 (optimum ~2048 tokens
  // for a 90 k-token ragged MHA batch, the 4096 maximum from ~110 k tokens).
  const double t = static_cast<double>(total_tokens) * p.num_kv_heads;
  // the grouped-query (matrix-core) kernel merges and writes up to 16 heads
  // per item: its per-item overhead is about 4x, so its best chunk about 2x
  const bool wide = choose_kernel(p).mfma;
  int chunk = static_cast<int>(std::sqrt(wide ? 6.0 * t : 1.5 * t));
  chunk = (chunk + 63) / 64 * 64;
  if (chunk < 256) chunk = 256;
  if (chunk > kMaxChunk) chunk = kMaxChunk;
  return chunk;
}

struct Checked {
  bool use_inline;       // plan travels in kernel arguments (no plan kernel)
  InlinePlan ip;
  InlineFirst icu;
  int chunk;
  int64_t total_tokens;  // exact when host lens are given, else worst case
  int64_t items;         // exact or upper bound
  bool exact;
  bool any_split;
  WorkspaceLayout w;
};

as_status validate(const char* what, const as_attn_params* p, const int32_t* kv_lens_host,
                   size_t workspace_bytes, const void* workspace, Checked* out) {
  if (!p) return als::fail(AS_EINVAL, "%s: params is null", what);
  if (p->batch < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1 || p->num_blocks < 1 ||
      p->max_blocks_per_seq < 1)
    return als::fail(AS_EINVAL, "%s: batch, head counts, num_blocks and max_blocks_per_seq must be positive", what);
  if (p->num_q_heads % p->num_kv_heads)
    return als::fail(AS_EINVAL, "%s: num_q_heads %d is not a multiple of num_kv_heads %d", what,
                     p->num_q_heads, p->num_kv_heads);
  if (p->block_size != kBlock)
    return als::fail(AS_EUNSUPPORTED, "%s: block_size %d (only 16 is built)", what, p->block_size);
  if (p->head_dim != 64 && p->head_dim != 128)
    return als::fail(AS_EUNSUPPORTED, "%s: head_dim %d (64 and 128 are built)", what, p->head_dim);
  if (p->dtype < AS_DTYPE_F32 || p->dtype > AS_DTYPE_F16 || p->out_dtype < AS_DTYPE_F32 ||
      p->out_dtype > AS_DTYPE_F16)
    return als::fail(AS_EUNSUPPORTED, "%s: dtype %d / out_dtype %d", what, p->dtype, p->out_dtype);
  if (!(p->scale >= 0.f) || std::isinf(p->scale))
    return als::fail(AS_EINVAL, "%s: scale must be finite and >= 0 (0 selects 1/sqrt(head_dim))", what);
  if (p->total_blocks_bound < 0)
    return als::fail(AS_EINVAL, "%s: total_blocks_bound %d is negative", what, p->total_blocks_bound);
  if (p->chunk_tokens != 0 &&
      (p->chunk_tokens < kBlock || p->chunk_tokens > kMaxChunk || p->chunk_tokens % kBlock))
    return als::fail(AS_EINVAL, "%s: chunk_tokens %d must be 0 or a multiple of 16 in [16, %d]", what,
                     p->chunk_tokens, kMaxChunk);
  const int64_t cap = static_cast<int64_t>(p->max_blocks_per_seq) * kBlock;
  int64_t total = 0;
  if (kv_lens_host) {
    for (int b = 0; b < p->batch; ++b) {
      if (kv_lens_host[b] < 1 || kv_lens_host[b] > cap)
        return als::fail(AS_ERANGE, "%s: kv_lens_host[%d] = %d outside [1, %lld]", what, b,
                         kv_lens_host[b], static_cast<long long>(cap));
      total += kv_lens_host[b];
    }
  } else {
    total = cap * p->batch;
    // the caller's promise on the sum of the lengths (in blocks) sizes the launch instead of the worst case
    if (p->total_blocks_bound > 0 && static_cast<int64_t>(p->total_blocks_bound) * kBlock < total)
      total = static_cast<int64_t>(p->total_blocks_bound) * kBlock;
  }
  out->total_tokens = total;
  out->chunk = pick_chunk(*p, total);
  if (kv_lens_host && p->chunk_tokens == 0) {
    // One chunk per request needs neither the plan nor the combine kernel.
    // Taken when requests are short, or not much longer than the chunk the
    // cost model picked, or when the batch is length-aligned (longest request
    // within 1.5x of the mean: workgroups then finish together anyway).
    int max_len = 0;
    for (int b = 0; b < p->batch; ++b) max_len = kv_lens_host[b] > max_len ? kv_lens_host[b] : max_len;
    const bool aligned = static_cast<double>(max_len) * p->batch <= 1.5 * static_cast<double>(total);
    // ... provided the requests alone make enough workgroups: with fewer
    // than one per compute unit a launch is bound by what a single workgroup
    // can stream, and splitting pays.  Such small launches get chunks sized
    // for about one workgroup per compute unit (fewer for the matrix-core
    // kernel, whose items cost more), but not below 512 tokens; fitted to
    // sweeps over 1-16 requests of 512 to 131072 tokens.
    const KernelChoice kc = choose_kernel(*p);
    const int64_t head_groups = p->num_q_heads / kc.heads;
    if (p->batch * head_groups >= 256) {
      if (out->chunk < max_len &&
          (max_len <= 1024 || (max_len <= kMaxChunk && (max_len <= 2 * out->chunk || aligned))))
        out->chunk = (max_len + kBlock - 1) / kBlock * kBlock;
    } else {
      int64_t par = total * head_groups / (kc.mfma ? 192 : 256);
      par = (par + 63) / 64 * 64;
      if (par < 512) par = 512;
      if (par > kMaxChunk) par = kMaxChunk;
      out->chunk = static_cast<int>(par);
      if (out->chunk > max_len) out->chunk = (max_len + kBlock - 1) / kBlock * kBlock;
    }
  }
  out->exact = kv_lens_host != nullptr;
  out->any_split = true;
  if (kv_lens_host) {
    int64_t items = 0;
    bool split = false;
    for (int b = 0; b < p->batch; ++b) {
      items += (kv_lens_host[b] + out->chunk - 1) / out->chunk;
      split |= kv_lens_host[b] > out->chunk;
    }
    out->items = items;
    out->any_split = split;
  } else {
    // every request contributes ceil(L / chunk) <= L / chunk + 1 items
    out->items = std::min(static_cast<int64_t>(p->batch) * ((cap + out->chunk - 1) / out->chunk),
                          total / out->chunk + p->batch);
  }
  out->w = layout_for(*p, out->items);
  // small launches with known lengths: build the plan here and ship it in the
  // kernel arguments (also when no request is split: the table then only puts
  // the requests in longest-first order)
  out->use_inline = false;
  if (kv_lens_host && out->items <= kInlineItems) {
    // canonical slots, request-major; full chunks go to the front of the
    // execution order as they are met
    uint32_t n = 0, pos = 0;
    struct Last { int32_t tokens; uint32_t word; };
    Last last[kInlineItems];
    int nlast = 0;
    for (int b = 0; b < p->batch; ++b) {
      const int nch = (kv_lens_host[b] + out->chunk - 1) / out->chunk;
      out->icu.first[b] = static_cast<uint16_t>(n);
      for (int c = 0; c < nch; ++c, ++n) {
        const uint32_t word = (static_cast<uint32_t>(b) << 20) | (static_cast<uint32_t>(c) << 10) | n;
        if (c + 1 < nch) out->ip.item[pos++] = word;
        else last[nlast++] = Last{kv_lens_host[b] - c * out->chunk, word};
      }
    }
    out->icu.first[p->batch] = static_cast<uint16_t>(n);
    // last chunks from long to short, equal lengths in request order: a
    // counting sort over the 1..chunk tokens a last chunk can hold (on the
    // stack: this path allocates nothing)
    uint16_t start[kMaxChunk + 2] = {};
    for (int i = 0; i < nlast; ++i) ++start[last[i].tokens];
    uint32_t run = pos;
    for (int t = out->chunk; t >= 1; --t) {
      const uint16_t c = start[t];
      start[t] = static_cast<uint16_t>(run);
      run += c;
    }
    for (int i = 0; i < nlast; ++i) out->ip.item[start[last[i].tokens]++] = last[i].word;
    out->use_inline = true;
  }
  if (out->items * p->num_q_heads > 0x7FFFFFFFLL)
    return als::fail(AS_ERANGE, "%s: %lld work items exceed the launch limit", what,
                     static_cast<long long>(out->items * p->num_q_heads));
  if (workspace) {
    if (reinterpret_cast<uintptr_t>(workspace) % 256)
      return als::fail(AS_EINVAL, "%s: workspace is not 256-byte aligned", what);
    if (workspace_bytes < out->w.total)
      return als::fail(AS_EWORKSPACE, "%s: workspace has %zu bytes, needs %zu", what, workspace_bytes,
                       out->w.total);
  }
  return AS_OK;
}

template <typename T, int D>
void launch_attn(int G, dim3 grid, hipStream_t s, const AttnArgs& a, const InlinePlan& ip) {
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_kernel<T, D, 1>), grid, dim3(kThreads), 0, s, a, ip); break;
    case 2: hipLaunchKernelGGL((attn_kernel<T, D, 2>), grid, dim3(kThreads), 0, s, a, ip); break;
    case 3: hipLaunchKernelGGL((attn_kernel<T, D, 3>), grid, dim3(kThreads), 0, s, a, ip); break;
    case 4: hipLaunchKernelGGL((attn_kernel<T, D, 4>), grid, dim3(kThreads), 0, s, a, ip); break;
    case 5: hipLaunchKernelGGL((attn_kernel<T, D, 5>), grid, dim3(kThreads), 0, s, a, ip); break;
    case 6: hipLaunchKernelGGL((attn_kernel<T, D, 6>), grid, dim3(kThreads), 0, s, a, ip); break;
    case 7: hipLaunchKernelGGL((attn_kernel<T, D, 7>), grid, dim3(kThreads), 0, s, a, ip); break;
    default: hipLaunchKernelGGL((attn_kernel<T, D, 8>), grid, dim3(kThreads), 0, s, a, ip); break;
  }
}

AttnArgs make_args(const as_attn_params& p, const Checked& ck, const void* q, const void* k,
                   const void* v, const int32_t* bt, const int32_t* lens, void* out, char* ws) {
  AttnArgs a;
  a.q = static_cast<const char*>(q);
  a.k_blocks = static_cast<const char*>(k);
  a.v_blocks = static_cast<const char*>(v);
  a.block_table = bt;
  a.kv_lens = lens;
  a.out = static_cast<char*>(out);
  a.hdr = reinterpret_cast<const PlanHeader*>(ws);
  a.items = reinterpret_cast<const int4*>(ws + ck.w.items_off);
  a.part_ml = reinterpret_cast<float2*>(ws + ck.w.ml_off);
  a.part_acc = reinterpret_cast<float*>(ws + ck.w.acc_off);
  a.num_kv_heads = p.num_kv_heads;
  a.head_groups = p.num_kv_heads;
  a.kv_div = 1;
  a.num_blocks = p.num_blocks;
  a.max_blocks_per_seq = p.max_blocks_per_seq;
  a.chunk = ck.chunk;
  a.out_dtype = p.out_dtype;
  a.exact_grid = ck.exact;
  a.direct = ck.exact && !ck.any_split;
  a.inline_plan = ck.use_inline;
  const float scale = p.scale > 0.f ? p.scale : 1.0f / std::sqrt(static_cast<float>(p.head_dim));
  a.c = scale * 1.4426950408889634f;
  return a;
}

as_status run_plan(const as_attn_params& p, const Checked& ck, const int32_t* lens, char* ws,
                   hipStream_t s) {
  const int64_t wgs = (ck.w.max_items + 2047) / 2048;
  hipLaunchKernelGGL(plan_kernel, dim3(static_cast<unsigned>(wgs < 1 ? 1 : wgs > 32 ? 32 : wgs)), dim3(256), 0, s,
                     lens, p.batch, ck.chunk,
                     p.max_blocks_per_seq * kBlock,
                     reinterpret_cast<PlanHeader*>(ws), reinterpret_cast<int32_t*>(ws + ck.w.cu_off),
                     reinterpret_cast<int4*>(ws + ck.w.items_off), ck.w.max_items);
  ALS_HIP_CHECK(hipGetLastError());
  return AS_OK;
}

}  // namespace

extern "C" size_t as_decode_attention_workspace(const as_attn_params* p, int64_t total_kv_tokens) {
  Checked ck;
  if (validate("as_decode_attention_workspace", p, nullptr, 0, nullptr, &ck) != AS_OK) return 0;
  // Upper bound on the items of any call that fits these parameters: every
  // request contributes ceil(L/chunk) <= L/chunk + 1 items, and the smallest
  // chunk the library picks by itself is 256 tokens.
  const int64_t worst = static_cast<int64_t>(p->batch) * p->max_blocks_per_seq * kBlock;
  if (total_kv_tokens < 0 || total_kv_tokens > worst) total_kv_tokens = worst;
  const int chunk = p->chunk_tokens > 0 ? p->chunk_tokens : 256;
  return layout_for(*p, total_kv_tokens / chunk + p->batch).total;
}

namespace {

// Shared body of as_decode_attention and as_decode_attention_static: argument
// checks, then the plan / attention / combine launches on `ws`.
// Host-side argument checks of a decode-attention call (no GPU call is made); fills `ck`.
as_status check_decode_args(const char* what, const void* q, const void* k_blocks, const void* v_blocks,
                            const int32_t* block_table, const int32_t* kv_lens,
                            const int32_t* kv_lens_host, const void* out, const as_attn_params* p,
                            Checked* ck) {
  if (!q || !k_blocks || !v_blocks || !block_table || !kv_lens || !out)
    return als::fail(AS_EINVAL, "%s: a required pointer is null", what);
  // the kernels move q, K, V and the result with 128-bit accesses
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_blocks) |
       reinterpret_cast<uintptr_t>(v_blocks) | reinterpret_cast<uintptr_t>(out)) % 16)
    return als::fail(AS_EINVAL, "%s: q, k_blocks, v_blocks and out must be 16-byte aligned", what);
  if ((reinterpret_cast<uintptr_t>(block_table) | reinterpret_cast<uintptr_t>(kv_lens)) % 4)
    return als::fail(AS_EINVAL, "%s: block_table and kv_lens must be 4-byte aligned", what);
  return validate(what, p, kv_lens_host, 0, nullptr, ck);
}

as_status run_decode_attention(const char* what, const void* q, const void* k_blocks,
                               const void* v_blocks, const int32_t* block_table,
                               const int32_t* kv_lens, const int32_t* kv_lens_host, void* out,
                               const as_attn_params* p, void* workspace, size_t workspace_bytes,
                               void* hip_stream, const Checked* checked = nullptr) {
  if (!workspace)
    return als::fail(AS_EINVAL, "%s: a required pointer is null", what);
  Checked local;
  if (!checked) {
    const as_status st0 = check_decode_args(what, q, k_blocks, v_blocks, block_table, kv_lens, kv_lens_host, out, p,
                                            &local);
    if (st0 != AS_OK) return st0;
    checked = &local;
  }
  const Checked& ck = *checked;
  if (reinterpret_cast<uintptr_t>(workspace) % 256)
    return als::fail(AS_EINVAL, "%s: workspace is not 256-byte aligned", what);
  if (workspace_bytes < ck.w.total)
    return als::fail(AS_EWORKSPACE, "%s: workspace has %zu bytes, needs %zu", what, workspace_bytes, ck.w.total);
  as_status st = AS_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  // When the host lengths show that no request needs more than one chunk,
  // item i is request i and neither the plan nor the combine kernel runs.
  const bool direct = ck.exact && !ck.any_split;
  if (!direct && !ck.use_inline && !(p->flags & AS_ATTN_REUSE_PLAN)) {
    st = run_plan(*p, ck, kv_lens, ws, s);
    if (st != AS_OK) return st;
  }
  AttnArgs a = make_args(*p, ck, q, k_blocks, v_blocks, block_table, kv_lens, out, ws);

  const int group = p->num_q_heads / p->num_kv_heads;
  const KernelChoice kc = choose_kernel(*p);
  const int mfma_heads = kc.mfma ? kc.heads : 0;
  if (mfma_heads) {
    a.head_groups = p->num_q_heads / mfma_heads;
    a.kv_div = group / mfma_heads;
    const dim3 grid(static_cast<unsigned>(ck.items * a.head_groups));
    if (mfma_heads <= kMfmaHeads && a.kv_div == 1) {
      if (p->dtype == AS_DTYPE_BF16)
        hipLaunchKernelGGL((attn_mfma_kernel<bf16_t, 1>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
      else
        hipLaunchKernelGGL((attn_mfma_kernel<f16_t, 1>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
    } else if (mfma_heads <= kMfmaHeads) {  // slices of 16 or 8 heads side by side on one KV head
      if (p->dtype == AS_DTYPE_BF16)
        hipLaunchKernelGGL((attn_mfma_kernel<bf16_t, 1, AS_SHARED_LOADS>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
      else
        hipLaunchKernelGGL((attn_mfma_kernel<f16_t, 1, AS_SHARED_LOADS>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
    } else if (a.kv_div == 1) {
      if (p->dtype == AS_DTYPE_BF16)
        hipLaunchKernelGGL((attn_mfma_kernel<bf16_t, 2>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
      else
        hipLaunchKernelGGL((attn_mfma_kernel<f16_t, 2>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
    } else {  // several slices of 32 heads read the same KV head: loads that the caches may keep
      if (p->dtype == AS_DTYPE_BF16)
        hipLaunchKernelGGL((attn_mfma_kernel<bf16_t, 2, AS_SHARED_LOADS>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
      else
        hipLaunchKernelGGL((attn_mfma_kernel<f16_t, 2, AS_SHARED_LOADS>), grid, dim3(kThreads), 0, s, a, mfma_heads, ck.ip);
    }
  } else {
    const int G = kc.heads;
    a.head_groups = p->num_q_heads / G;
    a.kv_div = group / G;
    const dim3 grid(static_cast<unsigned>(ck.items * a.head_groups));
    if (p->dtype == AS_DTYPE_BF16) {
      if (p->head_dim == 128) launch_attn<bf16_t, 128>(G, grid, s, a, ck.ip);
      else launch_attn<bf16_t, 64>(G, grid, s, a, ck.ip);
    } else if (p->dtype == AS_DTYPE_F16) {
      if (p->head_dim == 128) launch_attn<f16_t, 128>(G, grid, s, a, ck.ip);
      else launch_attn<f16_t, 64>(G, grid, s, a, ck.ip);
    } else {
      if (p->head_dim == 128) launch_attn<float, 128>(G, grid, s, a, ck.ip);
      else launch_attn<float, 64>(G, grid, s, a, ck.ip);
    }
  }
  ALS_HIP_CHECK(hipGetLastError());
  if (ck.any_split) {
    const int lpp = p->head_dim / 4;
    const int pairs_per_block = 256 / lpp;
    const int pairs = p->batch * p->num_q_heads;
    const dim3 cgrid((pairs + pairs_per_block - 1) / pairs_per_block);
    const int32_t* cu = reinterpret_cast<const int32_t*>(ws + ck.w.cu_off);
    const int max_items = static_cast<int>(ck.w.max_items < 0x7FFFFFFF ? ck.w.max_items : 0x7FFFFFFF);
    if (p->head_dim == 128)
      hipLaunchKernelGGL(combine_kernel<128>, cgrid, dim3(256), 0, s, cu, ck.icu, int(ck.use_inline), a.part_ml, a.part_acc,
                         a.out, p->batch, p->num_q_heads, a.out_dtype, max_items);
    else
      hipLaunchKernelGGL(combine_kernel<64>, cgrid, dim3(256), 0, s, cu, ck.icu, int(ck.use_inline), a.part_ml, a.part_acc,
                         a.out, p->batch, p->num_q_heads, a.out_dtype, max_items);
    ALS_HIP_CHECK(hipGetLastError());
  }
  return AS_OK;
}

}  // namespace

extern "C" as_status as_decode_attention(const void* q, const void* k_blocks, const void* v_blocks,
                                         const int32_t* block_table, const int32_t* kv_lens,
                                         const int32_t* kv_lens_host, void* out,
                                         const as_attn_params* p, void* workspace,
                                         size_t workspace_bytes, void* hip_stream) {
  return run_decode_attention("as_decode_attention", q, k_blocks, v_blocks, block_table, kv_lens,
                              kv_lens_host, out, p, workspace, workspace_bytes, hip_stream);
}

// ------------------------------------------------------------------ static scratch
// The variant for callers that cannot allocate: the plan and the split-KV
// partials live in one file-scope device array instead of a caller workspace.
// `scratch` names the array for the compiler only -- in host code it is a
// stand-in, not a device address; the address on each device comes from
// hipGetSymbolAddress, once per device, and that pointer is what the kernels
// get.
static __device__ __align__(256) unsigned char scratch[AS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // per device: each GPU holds its own copy of the array

as_status static_scratch(void** out) {
  int dev = -1;
  ALS_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices)
    return als::fail(AS_EUNSUPPORTED, "as_decode_attention_static: device index %d is beyond %d", dev,
                     kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    ALS_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256)
      return als::fail(AS_EHIP, "as_decode_attention_static: bad address %p for the scratch array", ptr);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return AS_OK;
}

}  // namespace

extern "C" size_t as_decode_attention_static_capacity(void) { return AS_STATIC_SCRATCH_BYTES; }

extern "C" as_status as_decode_attention_static(const void* q, const void* k_blocks,
                                                const void* v_blocks, const int32_t* block_table,
                                                const int32_t* kv_lens, const int32_t* kv_lens_host,
                                                void* out, const as_attn_params* p, void* hip_stream) {
  // argument errors, and a plan + partials larger than the array, are reported before any GPU call
  Checked ck;
  as_status st = check_decode_args("as_decode_attention_static", q, k_blocks, v_blocks, block_table, kv_lens,
                                   kv_lens_host, out, p, &ck);
  if (st != AS_OK) return st;
  if (ck.w.total > AS_STATIC_SCRATCH_BYTES)
    return als::fail(AS_EWORKSPACE, "as_decode_attention_static: plan and partials need %zu bytes, the static array has %u",
                     ck.w.total, static_cast<unsigned>(AS_STATIC_SCRATCH_BYTES));
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != AS_OK) return st;
  return run_decode_attention("as_decode_attention_static", q, k_blocks, v_blocks, block_table, kv_lens,
                              kv_lens_host, out, p, ws, AS_STATIC_SCRATCH_BYTES, hip_stream, &ck);
}

extern "C" as_status as_kv_read_sweep(const void* k_blocks, const void* v_blocks,
                                      const int32_t* block_table, const int32_t* kv_lens,
                                      const int32_t* kv_lens_host, uint32_t* checksum,
                                      const as_attn_params* p, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (!k_blocks || !v_blocks || !block_table || !kv_lens || !workspace)
    return als::fail(AS_EINVAL, "as_kv_read_sweep: a required pointer is null");
  if ((reinterpret_cast<uintptr_t>(k_blocks) | reinterpret_cast<uintptr_t>(v_blocks)) % 16)
    return als::fail(AS_EINVAL, "as_kv_read_sweep: k_blocks and v_blocks must be 16-byte aligned");
  if ((reinterpret_cast<uintptr_t>(block_table) | reinterpret_cast<uintptr_t>(kv_lens) |
       reinterpret_cast<uintptr_t>(checksum)) % 4)
    return als::fail(AS_EINVAL, "as_kv_read_sweep: block_table, kv_lens and checksum must be 4-byte aligned");
  Checked ck;
  as_status st = validate("as_kv_read_sweep", p, kv_lens_host, workspace_bytes, workspace, &ck);
  if (st != AS_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  if (!(ck.exact && !ck.any_split) && !ck.use_inline) {
    st = run_plan(*p, ck, kv_lens, ws, s);
    if (st != AS_OK) return st;
  }
  AttnArgs a = make_args(*p, ck, k_blocks, k_blocks, v_blocks, block_table, kv_lens, checksum, ws);
  const size_t esz = p->dtype == AS_DTYPE_F32 ? 4 : 2;
  const size_t slab = static_cast<size_t>(kBlock) * p->head_dim * esz;
  const int64_t nwg = ck.items * p->num_kv_heads;
  const dim3 grid(static_cast<unsigned>(nwg));
  // per-workgroup words go where the attention call keeps its partial sums:
  // items * H_q * D floats, never fewer than items * H_kv words
  uint32_t* wg_sums = reinterpret_cast<uint32_t*>(a.part_acc);
  switch (slab / 1024) {
    case 2: hipLaunchKernelGGL(sweep_kernel<2>, grid, dim3(kThreads), 0, s, a, ck.ip, slab, wg_sums); break;
    case 4: hipLaunchKernelGGL(sweep_kernel<4>, grid, dim3(kThreads), 0, s, a, ck.ip, slab, wg_sums); break;
    default: hipLaunchKernelGGL(sweep_kernel<8>, grid, dim3(kThreads), 0, s, a, ck.ip, slab, wg_sums); break;
  }
  ALS_HIP_CHECK(hipGetLastError());
  if (checksum) {  // null: timing only, one launch like the attention call of an unsplit batch
    hipLaunchKernelGGL(sweep_fold_kernel, dim3(1), dim3(256), 0, s, wg_sums, nwg, checksum);
    ALS_HIP_CHECK(hipGetLastError());
  }
  return AS_OK;
}
