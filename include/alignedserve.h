/*
 * alignedserve.h -- C ABI of the MI355X (gfx950) decode-attention hot path of
 * AlignedServe: length-aligned batch formation, host-to-HBM staging of a
 * batch's paged KV blocks, and batched single-query attention over the paged
 * KV cache for requests of different KV length.
 *
 * Conventions that hold for every entry point
 *   - plain C types only; "device" pointers are HIP device pointers owned by
 *     the caller, "host" pointers are ordinary host memory unless stated to
 *     be pinned;
 *   - the library never allocates or frees caller-visible memory;
 *   - every call returns an as_status and never throws (a C++ exception
 *     raised inside, such as std::bad_alloc, comes back as AS_ENOMEM); on
 *     failure nothing has been enqueued unless the status is AS_EHIP, and
 *     as_last_error() returns a thread-local, library-owned description;
 *   - calls that take a stream are asynchronous on it and return after
 *     enqueueing; a null stream is the HIP default stream.
 *
 * Paged KV layout (the library's contract; the paper only speaks of "memory
 * blocks", Section 3.3):
 *   k_blocks, v_blocks : [num_blocks][num_kv_heads][block_size][head_dim]
 *                        row-major, block_size == 16, fp32, bf16 or fp16;
 *   block_table        : int32 [batch][max_blocks_per_seq];
 *   logical token t of request b is row t % 16 of physical block
 *   block_table[b][t / 16].  Rows at or past kv_lens[b] in a request's last
 *   block, unused block_table entries and blocks nobody owns are don't-care:
 *   they may hold NaN/Inf and never influence a result.
 */
#ifndef ALIGNEDSERVE_H
#define ALIGNEDSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AS_OK = 0,
  AS_EINVAL = 1,       /* null pointer, non-positive size, inconsistent shape   */
  AS_ERANGE = 2,       /* a value outside what the arguments allow              */
  AS_EWORKSPACE = 3,   /* workspace smaller than as_decode_attention_workspace  */
  AS_EUNSUPPORTED = 4, /* dtype / head_dim / block_size the kernels do not have */
  AS_EHIP = 5,         /* a HIP runtime call failed (message has its string)    */
  AS_ENOMEM = 6        /* host memory ran out inside the library; the object the
                          call was to change is as it was before the call        */
} as_status;

#define AS_DTYPE_F32 0
#define AS_DTYPE_BF16 1
#define AS_DTYPE_F16 2 /* IEEE binary16: the precision the paper runs its models in (Section 4.1) */

/* Library version (major*10000 + minor*100 + patch). */
int32_t as_version(void);

/* Description of the last failure on the calling thread ("" if none). */
const char* as_last_error(void);

/* --------------------------------------------------------------------------
 * Batch formation (host only; no GPU is touched).
 *
 * The paper's prefix-aware batching (Sections 2.4 and 3.3) groups requests
 * whose prefixes have similar length, because a decode iteration lasts as
 * long as its longest member (Section 2.3).  With a fixed batch size this is
 * the partition into ceil(n / batch_size) batches that minimises the sum of
 * per-batch maximum KV lengths; sorting by length and cutting consecutive
 * chunks reaches it.  Canonical result:
 *   order          request indices sorted by (kv_len descending, index
 *                  ascending), int32[n], caller-allocated;
 *   batch_offsets  int32[ceil(n/batch_size) + 1], caller-allocated; batch j is
 *                  order[batch_offsets[j] .. batch_offsets[j+1]); all batches
 *                  hold batch_size requests except possibly the last, which
 *                  then holds the shortest ones;
 *   num_batches    ceil(n / batch_size) (0 when n == 0; batch_offsets = {0}).
 * kv_lens: host int32[n], each >= 1.  All pointers are host pointers.
 * Errors: AS_EINVAL for null pointers (kv_lens/order may be null only when
 * n == 0), n < 0, batch_size <= 0 or a kv_len < 1.
 * -------------------------------------------------------------------------- */
as_status as_aligned_batch(const int32_t* kv_lens, int32_t n, int32_t batch_size,
                           int32_t* order, int32_t* batch_offsets, int32_t* num_batches);

/* --------------------------------------------------------------------------
 * The paper's own batch generator (Section 3.3, Algorithm 1): a quad-tree over
 * prefix lengths [1, max_len] (longer prefixes are clamped, Section 4.1) whose
 * internal nodes carry (request counter, block counter), and Density First
 * Search over it.  Host only.
 *   as_qtree_create      max_len / leaf_width must be a power of four (the
 *                        paper's range is 65536; leaf_width is this library's
 *                        parameter, e.g. 16 tokens = one KV block)
 *   as_qtree_insert      adds request (id, prefix_len >= 1, blocks >= 1);
 *                        `now` stamps sub-trees that were empty (Section 3.5)
 *   as_qtree_remove      removes a request by id
 *   as_qtree_size        request / block counters of the root
 *   as_qtree_next_batch  one search: case 1 (sub-tree fits b_max and holds
 *                        >= k_min requests: taken whole), case 2 (exceeds
 *                        b_max: descend into the child with the most requests,
 *                        leftmost on ties; at a leaf, requests are taken in
 *                        (length, id) order while they fit, at least one),
 *                        case 3 (fits but < k_min: widened with at most
 *                        k_min - |batch| requests of the nearest siblings --
 *                        left siblings if any, else right -- stopping at the
 *                        first that exceeds the remaining budget).  With
 *                        starve_after >= 0 the search starts at the non-empty
 *                        internal node whose age now - stamp is largest and
 *                        above starve_after (pass a negative value to switch
 *                        this off).  The batch's requests are removed from
 *                        the tree; their ids are written to out_ids[0..*out_n)
 *                        (node's own requests by (length, id), then the
 *                        additions); *out_case (optional) is 1, 2 or 3.
 *                        *out_n = 0 when the tree is empty.
 *   as_dfs_batches       convenience: insert n requests (id = index), generate
 *                        batches until the tree is empty; order[n],
 *                        batch_offsets[n + 1] caller-allocated.
 * Errors: AS_EINVAL (null, bad geometry, duplicate / unknown id, non-positive
 * values), AS_ERANGE (capacity too small; nothing is removed then).
 * -------------------------------------------------------------------------- */
typedef struct as_qtree as_qtree;
as_status as_qtree_create(as_qtree** out, int32_t max_len, int32_t leaf_width);
as_status as_qtree_destroy(as_qtree* t);
as_status as_qtree_insert(as_qtree* t, int32_t request_id, int32_t prefix_len, int32_t blocks,
                          double now);
as_status as_qtree_remove(as_qtree* t, int32_t request_id);
as_status as_qtree_size(const as_qtree* t, int64_t* requests, int64_t* blocks);
as_status as_qtree_next_batch(as_qtree* t, int64_t b_max, int32_t k_min, double now,
                              double starve_after, int32_t* out_ids, int32_t capacity,
                              int32_t* out_n, int32_t* out_case);
as_status as_dfs_batches(const int32_t* kv_lens, const int32_t* blocks, int32_t n, int64_t b_max,
                         int32_t k_min, int32_t max_len, int32_t leaf_width, int32_t* order,
                         int32_t* batch_offsets, int32_t* num_batches);

/* --------------------------------------------------------------------------
 * Decode-iteration attention (paper Section 2.2, Eq. 2):
 *   out[b][h] = softmax(q[b][h] . K_b^T / sqrt(d_k)) V_b
 * for the newest token's query of every request b against all kv_lens[b]
 * cached keys / values of that request (the newest token's own k, v are
 * already in the cache; there is no causal mask).  Query head h reads KV head
 * h / (num_q_heads / num_kv_heads).  Accumulation is fp32 for every input
 * type; 16-bit inputs are widened exactly.
 * -------------------------------------------------------------------------- */
typedef struct {
  int32_t dtype;              /* AS_DTYPE_* of q, k_blocks, v_blocks                */
  int32_t out_dtype;          /* AS_DTYPE_* of out                                   */
  int32_t batch;              /* B >= 1                                              */
  int32_t num_q_heads;        /* multiple of num_kv_heads                            */
  int32_t num_kv_heads;
  int32_t head_dim;           /* 64 or 128                                           */
  int32_t block_size;         /* must be 16                                          */
  int32_t num_blocks;         /* pool size; block ids are clamped into [0, this)     */
  int32_t max_blocks_per_seq; /* row stride of block_table                           */
  float scale;                /* 0 => 1/sqrt(head_dim)                               */
  int32_t chunk_tokens;       /* split-KV granularity in tokens: a request's KV is
                                 cut into chunks of this many tokens, one workgroup
                                 each, merged exactly afterwards.  0 => chosen by
                                 the library.  Otherwise a multiple of 16 in
                                 [16, 4096].                                         */
  int32_t flags;              /* AS_ATTN_* bits                                      */
  int32_t total_blocks_bound; /* for calls WITHOUT kv_lens_host: the caller's upper
                                 bound on the sum over the batch of ceil(kv_len / 16)
                                 (a block allocator knows it exactly); the launch is
                                 then sized for it instead of batch *
                                 max_blocks_per_seq blocks.  0 => no bound.  If the
                                 device lengths exceed it, the requests that do not
                                 fit get wrong results (never a fault).  Ignored
                                 when kv_lens_host is given.                         */
} as_attn_params;

/* The work plan in `workspace` was written by an earlier call with the same
 * kv_lens, batch, chunk_tokens and head counts (e.g. the previous layer of
 * the same decode iteration): skip rebuilding it. */
#define AS_ATTN_REUSE_PLAN 1
/* Force the vector-ALU kernel even where the matrix-core (MFMA) kernel would
 * be selected for grouped-query shapes. */
#define AS_ATTN_NO_MFMA 2

/* Bytes of device workspace as_decode_attention needs for these parameters
 * when the batch holds at most total_kv_tokens tokens in all (sum of
 * kv_lens) AND the call either passes kv_lens_host or sets
 * total_blocks_bound <= total_kv_tokens / 16.  Pass total_kv_tokens < 0 to
 * size for the worst case batch * max_blocks_per_seq * 16, which covers every
 * call.  Returns 0 on invalid parameters. */
size_t as_decode_attention_workspace(const as_attn_params* p, int64_t total_kv_tokens);

/* q            device [batch][num_q_heads][head_dim], dtype
 * k_blocks     device paged pool (layout above), dtype
 * v_blocks     device paged pool, dtype
 * block_table  device int32 [batch][max_blocks_per_seq]
 * kv_lens      device int32 [batch]; a request with kv_len <= 0 gets zeros
 * kv_lens_host optional host copy of kv_lens (may be null).  When given the
 *              launch is sized exactly and the lengths are validated
 *              (1 <= kv_len <= max_blocks_per_seq * 16) before anything is
 *              enqueued; when null the launch is sized for the worst case
 *              and nothing is validated.
 * out          device [batch][num_q_heads][head_dim], out_dtype
 * workspace    device scratch of at least as_decode_attention_workspace()
 *              bytes, 256-byte aligned; its contents are only meaningful to
 *              the library (plan + split-KV partials) and may be reused by
 *              the next call.
 * q, k_blocks, v_blocks and out must be 16-byte aligned (AS_EINVAL otherwise).
 * Under HIP graph capture a call made with kv_lens_host bakes the work plan
 * derived from those lengths into the captured launches: replay it only while
 * the device lengths equal them.  A call without kv_lens_host plans on the
 * device at every replay and follows kv_lens as it changes (up to
 * max_blocks_per_seq * 16 tokens per request).
 * Inputs are read-only; out and workspace are the only memory written.
 * Device-side contents of block_table are not validated on the hot path;
 * ids are clamped into the pool so that a bad id yields a wrong result, not
 * a fault.  Two calls sharing one workspace must be ordered on one stream.
 * Errors: AS_EINVAL, AS_ERANGE (host lens out of range), AS_EUNSUPPORTED,
 * AS_EWORKSPACE, AS_EHIP. */
as_status as_decode_attention(const void* q, const void* k_blocks, const void* v_blocks,
                              const int32_t* block_table, const int32_t* kv_lens,
                              const int32_t* kv_lens_host, void* out,
                              const as_attn_params* p, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/* --------------------------------------------------------------------------
 * as_decode_attention for callers that cannot allocate device memory or
 * bring a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result as as_decode_attention, minus the workspace: the work plan and the
 * split-KV partials go to a static device array of AS_STATIC_SCRATCH_BYTES
 * that is part of the library's code object (every GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees
 * nothing, on the host or on the device.
 *   - A call whose plan and partials need more than the array (the figure
 *     as_decode_attention_workspace gives for the same parameters and
 *     total) is rejected with AS_EWORKSPACE before anything is enqueued;
 *     32 MiB holds e.g. 128 requests x 64 query heads x 8 chunks.
 *   - All calls on one GPU share that GPU's array, which keeps the previous
 *     call's contents.  Nothing in it has to start at zero: a call reads only
 *     what it has written itself (with AS_ATTN_REUSE_PLAN: what the previous
 *     static call on this GPU, made with the same lengths and shape, wrote).
 *     Calls that overlap on one GPU -- two streams, two threads, or a captured
 *     graph replayed next to an eager call -- race on it: order them on one
 *     stream or with events.
 *   - The array's address is looked up on the first call on each device
 *     (with that device current); later calls only read it.
 * as_decode_attention_static_capacity returns AS_STATIC_SCRATCH_BYTES.
 * Errors: those of as_decode_attention.
 * -------------------------------------------------------------------------- */
#define AS_STATIC_SCRATCH_BYTES (32u << 20)
size_t as_decode_attention_static_capacity(void);
as_status as_decode_attention_static(const void* q, const void* k_blocks, const void* v_blocks,
                                     const int32_t* block_table, const int32_t* kv_lens,
                                     const int32_t* kv_lens_host, void* out,
                                     const as_attn_params* p, void* hip_stream);

/* --------------------------------------------------------------------------
 * KV append (paper Section 2.1: a generated token's key and value join the
 * request's KVCache and take part in every later iteration).
 * For every request b of the batch, writes k_new[b] and v_new[b]
 * (device, [batch][num_kv_heads][head_dim], dtype) to position kv_lens[b] of
 * its paged cache -- row kv_lens[b] % 16 of block
 * block_table[b][kv_lens[b] / 16] -- and increments kv_lens[b] (device,
 * in place).  The block-table entry must already be allocated by the caller.
 * A request whose table row is full is left untouched.  Uses dtype, batch,
 * num_kv_heads, head_dim, block_size, num_blocks and max_blocks_per_seq of
 * the params.  Asynchronous on the stream.
 * Errors: AS_EINVAL, AS_EUNSUPPORTED, AS_EHIP.
 * -------------------------------------------------------------------------- */
as_status as_kv_append(const void* k_new, const void* v_new, void* k_blocks, void* v_blocks,
                       const int32_t* block_table, int32_t* kv_lens, const as_attn_params* p,
                       void* hip_stream);

/* --------------------------------------------------------------------------
 * Batch-level scheduling policy (paper Section 3.4, Algorithm 2).  Host only;
 * purely logical (ids, lengths, block counts): the caller moves the KV data
 * the returned events imply (as_stage_kv for admissions, as_unstage_kv for
 * evictions).
 *   as_sched_create   total_blocks of HBM, block_size tokens per block,
 *                     max_batch = cap on the running batch
 *   as_sched_push_candidate_batch    fill the candidate-batch buffer with a
 *                     generated batch (origin = its batch number)
 *   as_sched_push_candidate_request  add one request to the candidate-requests
 *                     buffer (late arrivals of the running batch's length)
 *   as_sched_step     one pass after a decode iteration.  advance != 0: every
 *                     running request has produced a token (kv_len + 1,
 *                     remaining - 1).  Then: completed requests are released;
 *                     if the next iteration (one fresh block per running
 *                     request whose kv_len is a multiple of block_size) does
 *                     not fit -> case 3: evict the longest request (while two
 *                     original batches coexist: the longest of the one with
 *                     the smaller batch number) to the tail of the
 *                     candidate-requests buffer, repeatedly until it fits;
 *                     else admit, in buffer order, from the candidate-requests
 *                     buffer (case 1) or, if that is empty, from the
 *                     candidate-batch buffer (case 2), while the batch is
 *                     below max_batch and the request's blocks plus the next
 *                     iteration's growth fit; stops at the first that does
 *                     not.  Outputs: ids of completed / evicted / admitted
 *                     requests (arrays of `capacity` >= max(max_batch, running
 *                     size) entries each) and the case (0 = nothing admitted
 *                     or evicted).
 *   as_sched_state / as_sched_running   inspection.
 * Errors: AS_EINVAL, AS_ERANGE (capacity).
 * -------------------------------------------------------------------------- */
typedef struct as_sched as_sched;
as_status as_sched_create(as_sched** out, int64_t total_blocks, int32_t block_size, int32_t max_batch);
as_status as_sched_destroy(as_sched* s);
as_status as_sched_push_candidate_batch(as_sched* s, int32_t origin, const int32_t* ids,
                                        const int32_t* kv_lens, const int32_t* remaining, int32_t n);
as_status as_sched_push_candidate_request(as_sched* s, int32_t origin, int32_t id, int32_t kv_len,
                                          int32_t remaining);
as_status as_sched_step(as_sched* s, int32_t advance, int32_t* completed, int32_t* n_completed,
                        int32_t* evicted, int32_t* n_evicted, int32_t* admitted, int32_t* n_admitted,
                        int32_t capacity, int32_t* which_case);
as_status as_sched_state(const as_sched* s, int64_t* free_blocks, int32_t* n_running,
                         int32_t* n_candidate_requests, int32_t* n_candidate_batch);
as_status as_sched_running(const as_sched* s, int32_t* ids, int32_t* kv_lens, int32_t* origins,
                           int32_t capacity, int32_t* n);

/* --------------------------------------------------------------------------
 * KV staging: host KV pool -> HBM block pool (paper Section 3.2: the KV pool
 * lives in host memory and a scheduled batch's KVCache is migrated to the
 * decoding GPU, directly over PCIe when no peer GPU serves as a buffer; the
 * batch to run next is prefetched asynchronously, Fig. 4 step 4, so that the
 * transfer overlaps the running batch's decoding, Section 4.4).
 *
 * Enqueues, on `hip_stream`, copies of m blocks of block_bytes bytes each:
 *   host_k + src_ids[i] * block_bytes  ->  dev_k + dst_ids[i] * block_bytes
 * and the same for host_v -> dev_v (host_v/dev_v may both be null to move one
 * pool only).  Runs in which src and dst ids both advance by one are merged
 * into a single DMA copy; when the runs are short (a paged host pool hands out
 * scattered blocks) the blocks are instead moved by a small copy kernel that
 * reads the pinned host memory over the link (see as_stage_set_policy).  The
 * result is the same either way.  host_* must be pinned (hipHostMalloc)
 * memory; the id arrays are host arrays and are consumed before the call
 * returns.  Blocks within one call must not overlap each other.
 * num_src_blocks / num_dst_blocks bound the ids.  The caller orders the
 * copies against consumers with events (see as_pipeline_* below).
 * Errors: AS_EINVAL (null, m < 0, block_bytes == 0 or not a multiple of 16,
 * unpinned host pointer), AS_ERANGE (an id out of range), AS_EHIP.
 * -------------------------------------------------------------------------- */
as_status as_stage_kv(const void* host_k, const void* host_v, const int64_t* src_ids,
                      int64_t num_src_blocks, void* dev_k, void* dev_v,
                      const int32_t* dst_ids, int32_t num_dst_blocks, int32_t m,
                      size_t block_bytes, void* hip_stream);

/* How as_stage_kv / as_unstage_kv move blocks (process-wide, default AUTO):
 *   AS_STAGE_AUTO    DMA copies when a run averages >= 8 MiB, else the kernel
 *   AS_STAGE_DMA     always one hipMemcpyAsync per run (SDMA engines)
 *   AS_STAGE_KERNEL  always the copy kernel (64 workgroups on the given stream)
 * Errors: AS_EINVAL for any other value. */
#define AS_STAGE_AUTO 0
#define AS_STAGE_DMA 1
#define AS_STAGE_KERNEL 2
as_status as_stage_set_policy(int32_t policy);

/* The reverse direction (eviction of a request's blocks to the host pool,
 * Section 3.4 case 3): dev + src_ids[i] -> host + dst_ids[i]. */
as_status as_unstage_kv(void* host_k, void* host_v, const int64_t* dst_ids,
                        int64_t num_host_blocks, const void* dev_k, const void* dev_v,
                        const int32_t* src_ids, int32_t num_dev_blocks, int32_t m,
                        size_t block_bytes, void* hip_stream);

/* --------------------------------------------------------------------------
 * Copy / compute handshake for a multi-buffered HBM block pool (paper
 * Section 4.4: batch generation and prefetch are pipelined with decoding).
 * The pipeline owns one side stream (default priority) and, per buffer, a
 * "ready" event (copies into the buffer are complete) and a "free" event
 * (the last attention that read the buffer is complete).
 *   as_pipeline_create   num_buffers in [1, 8]
 *   as_pipeline_stream   the side stream, to pass to as_stage_kv
 *   as_pipeline_begin_stage(buf)    side stream waits for buf's "free"
 *   as_pipeline_end_stage(buf)      records buf's "ready" on the side stream
 *   as_pipeline_acquire(buf, s)     stream s waits for buf's "ready"
 *   as_pipeline_release(buf, s)     records buf's "free" on stream s
 *   as_pipeline_query(buf, &ready)  host-side poll, no wait: *ready = 1 when
 *                        the copies last closed by end_stage(buf) have
 *                        finished (or none were ever staged), else 0; lets a
 *                        scheduler admit only what is already resident
 *   as_pipeline_destroy  synchronises the side stream, destroys everything
 * Errors: AS_EINVAL (null pipeline, buf out of range), AS_EHIP.
 * -------------------------------------------------------------------------- */
typedef struct as_pipeline as_pipeline;
as_status as_pipeline_create(as_pipeline** out, int32_t num_buffers);
void* as_pipeline_stream(as_pipeline* p);
as_status as_pipeline_begin_stage(as_pipeline* p, int32_t buf);
as_status as_pipeline_end_stage(as_pipeline* p, int32_t buf);
as_status as_pipeline_acquire(as_pipeline* p, int32_t buf, void* hip_stream);
as_status as_pipeline_release(as_pipeline* p, int32_t buf, void* hip_stream);
as_status as_pipeline_query(as_pipeline* p, int32_t buf, int32_t* ready);
as_status as_pipeline_destroy(as_pipeline* p);

/* --------------------------------------------------------------------------
 * Measurement aid: streams every K and V byte the attention call with the
 * same arguments would read (same block table, same lengths, same work
 * split) and folds them into a checksum, with no other arithmetic.  Its
 * bandwidth is the ceiling the attention kernel is compared with.
 * checksum: device uint32[256], XOR-accumulated (slot = workgroup index mod
 * 256, folded in by a second small kernel); the XOR of the 256 slots equals
 * the XOR of every 32-bit word of every K and V block the batch references
 * (whole blocks), for the slots' initial contents zero.  checksum may be null:
 * the folding kernel is then left out and the call is a single launch, the
 * read-only counterpart of an attention call on a batch that is not split
 * (what the per-launch cost of such a call is compared with).  Same errors as
 * as_decode_attention.
 * -------------------------------------------------------------------------- */
as_status as_kv_read_sweep(const void* k_blocks, const void* v_blocks,
                           const int32_t* block_table, const int32_t* kv_lens,
                           const int32_t* kv_lens_host, uint32_t* checksum,
                           const as_attn_params* p, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ALIGNEDSERVE_H */
