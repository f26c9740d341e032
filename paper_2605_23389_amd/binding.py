"""Thin ctypes binding over the C-ABI library (include/alignedserve.h).

Argument marshalling only: every step of the hot path runs inside the
library.  PyTorch tensors are used as device memory (their data_ptr() is
handed over) and torch streams as HIP streams.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libalignedserve.so")

AS_OK, AS_EINVAL, AS_ERANGE, AS_EWORKSPACE, AS_EUNSUPPORTED, AS_EHIP, AS_ENOMEM = range(7)
STATUS_NAMES = {0: "AS_OK", 1: "AS_EINVAL", 2: "AS_ERANGE", 3: "AS_EWORKSPACE",
                4: "AS_EUNSUPPORTED", 5: "AS_EHIP", 6: "AS_ENOMEM"}
DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
ATTN_REUSE_PLAN, ATTN_NO_MFMA = 1, 2
STAGE_AUTO, STAGE_DMA, STAGE_KERNEL = 0, 1, 2

EXPORTS = [
    "as_version", "as_last_error", "as_aligned_batch", "as_decode_attention_workspace",
    "as_decode_attention", "as_stage_kv", "as_unstage_kv", "as_pipeline_create",
    "as_pipeline_stream", "as_pipeline_begin_stage", "as_pipeline_end_stage",
    "as_pipeline_acquire", "as_pipeline_release", "as_pipeline_destroy", "as_kv_read_sweep",
    "as_qtree_create", "as_qtree_destroy", "as_qtree_insert", "as_qtree_remove", "as_qtree_size",
    "as_qtree_next_batch", "as_dfs_batches", "as_kv_append", "as_sched_create", "as_sched_destroy",
    "as_sched_push_candidate_batch", "as_sched_push_candidate_request", "as_sched_step",
    "as_sched_state", "as_sched_running", "as_stage_set_policy",
    "as_decode_attention_static", "as_decode_attention_static_capacity", "as_pipeline_query",
]


class AttnParams(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("out_dtype", C.c_int32), ("batch", C.c_int32),
        ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("block_size", C.c_int32), ("num_blocks", C.c_int32), ("max_blocks_per_seq", C.c_int32),
        ("scale", C.c_float), ("chunk_tokens", C.c_int32), ("flags", C.c_int32),
        ("total_blocks_bound", C.c_int32),
    ]


class AlignedServeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Load the built library; raises if it is missing (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_23389_amd.build` "
            "(hipcc, gfx950). There is no CPU or PyTorch fallback for the hot path.")
    # PyTorch ships its own HIP runtime (same soname as the system one).  It
    # must be the one already mapped when this library is loaded, otherwise the
    # process ends up with two runtimes and the second one sees no device.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    i32p, i64p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.c_void_p
    lib.as_version.restype = C.c_int32
    lib.as_last_error.restype = C.c_char_p
    lib.as_aligned_batch.restype = C.c_int
    lib.as_aligned_batch.argtypes = [i32p, C.c_int32, C.c_int32, i32p, i32p, i32p]
    lib.as_decode_attention_workspace.restype = C.c_size_t
    lib.as_decode_attention_workspace.argtypes = [C.POINTER(AttnParams), C.c_int64]
    lib.as_decode_attention.restype = C.c_int
    lib.as_decode_attention.argtypes = [vp, vp, vp, vp, vp, i32p, vp, C.POINTER(AttnParams), vp,
                                        C.c_size_t, vp]
    lib.as_decode_attention_static.restype = C.c_int
    lib.as_decode_attention_static.argtypes = [vp, vp, vp, vp, vp, i32p, vp, C.POINTER(AttnParams), vp]
    lib.as_decode_attention_static_capacity.restype = C.c_size_t
    lib.as_decode_attention_static_capacity.argtypes = []
    lib.as_kv_read_sweep.restype = C.c_int
    lib.as_kv_read_sweep.argtypes = [vp, vp, vp, vp, i32p, vp, C.POINTER(AttnParams), vp,
                                     C.c_size_t, vp]
    lib.as_stage_kv.restype = C.c_int
    lib.as_stage_kv.argtypes = [vp, vp, i64p, C.c_int64, vp, vp, i32p, C.c_int32, C.c_int32,
                                C.c_size_t, vp]
    lib.as_unstage_kv.restype = C.c_int
    lib.as_unstage_kv.argtypes = [vp, vp, i64p, C.c_int64, vp, vp, i32p, C.c_int32, C.c_int32,
                                  C.c_size_t, vp]
    lib.as_stage_set_policy.restype = C.c_int
    lib.as_stage_set_policy.argtypes = [C.c_int32]
    lib.as_pipeline_create.restype = C.c_int
    lib.as_pipeline_create.argtypes = [C.POINTER(vp), C.c_int32]
    lib.as_pipeline_stream.restype = vp
    lib.as_pipeline_stream.argtypes = [vp]
    for name in ("as_pipeline_begin_stage", "as_pipeline_end_stage"):
        getattr(lib, name).restype = C.c_int
        getattr(lib, name).argtypes = [vp, C.c_int32]
    for name in ("as_pipeline_acquire", "as_pipeline_release"):
        getattr(lib, name).restype = C.c_int
        getattr(lib, name).argtypes = [vp, C.c_int32, vp]
    lib.as_pipeline_query.restype = C.c_int
    lib.as_pipeline_query.argtypes = [vp, C.c_int32, i32p]
    lib.as_pipeline_destroy.restype = C.c_int
    lib.as_pipeline_destroy.argtypes = [vp]
    lib.as_kv_append.restype = C.c_int
    lib.as_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, C.POINTER(AttnParams), vp]
    lib.as_sched_create.restype = C.c_int
    lib.as_sched_create.argtypes = [C.POINTER(vp), C.c_int64, C.c_int32, C.c_int32]
    lib.as_sched_destroy.restype = C.c_int
    lib.as_sched_destroy.argtypes = [vp]
    lib.as_sched_push_candidate_batch.restype = C.c_int
    lib.as_sched_push_candidate_batch.argtypes = [vp, C.c_int32, i32p, i32p, i32p, C.c_int32]
    lib.as_sched_push_candidate_request.restype = C.c_int
    lib.as_sched_push_candidate_request.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.as_sched_step.restype = C.c_int
    lib.as_sched_step.argtypes = [vp, C.c_int32, i32p, i32p, i32p, i32p, i32p, i32p, C.c_int32, i32p]
    lib.as_sched_state.restype = C.c_int
    lib.as_sched_state.argtypes = [vp, i64p, i32p, i32p, i32p]
    lib.as_sched_running.restype = C.c_int
    lib.as_sched_running.argtypes = [vp, i32p, i32p, i32p, C.c_int32, i32p]
    lib.as_qtree_create.restype = C.c_int
    lib.as_qtree_create.argtypes = [C.POINTER(vp), C.c_int32, C.c_int32]
    lib.as_qtree_destroy.restype = C.c_int
    lib.as_qtree_destroy.argtypes = [vp]
    lib.as_qtree_insert.restype = C.c_int
    lib.as_qtree_insert.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_double]
    lib.as_qtree_remove.restype = C.c_int
    lib.as_qtree_remove.argtypes = [vp, C.c_int32]
    lib.as_qtree_size.restype = C.c_int
    lib.as_qtree_size.argtypes = [vp, i64p, i64p]
    lib.as_qtree_next_batch.restype = C.c_int
    lib.as_qtree_next_batch.argtypes = [vp, C.c_int64, C.c_int32, C.c_double, C.c_double, i32p,
                                        C.c_int32, i32p, i32p]
    lib.as_dfs_batches.restype = C.c_int
    lib.as_dfs_batches.argtypes = [i32p, i32p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                   i32p, i32p, i32p]
    _lib = lib
    return lib


def _check(status: int):
    if status != AS_OK:
        raise AlignedServeError(status, load().as_last_error().decode("utf-8", "replace"))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray], ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def version() -> int:
    return int(load().as_version())


# ---------------------------------------------------------------------------
# aligned_batch
# ---------------------------------------------------------------------------
def aligned_batch(kv_lens, batch_size: int):
    """Length-aligned batches.  Returns (order int32[n], batch_offsets
    int32[num_batches + 1])."""
    lib = load()
    lens = _i32(kv_lens)
    n = int(lens.shape[0])
    nb_cap = (n + max(int(batch_size), 1) - 1) // max(int(batch_size), 1)
    order = np.empty(max(n, 1), dtype=np.int32)
    offsets = np.empty(nb_cap + 1, dtype=np.int32)
    nb = C.c_int32(0)
    _check(lib.as_aligned_batch(_ptr(lens, C.c_int32), n, int(batch_size), _ptr(order, C.c_int32),
                                _ptr(offsets, C.c_int32), C.byref(nb)))
    return order[:n], offsets[: nb.value + 1]


# ---------------------------------------------------------------------------
# decode_attention
# ---------------------------------------------------------------------------
def _torch_dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    if t.dtype == torch.float16:
        return DTYPE_F16
    raise AlignedServeError(AS_EUNSUPPORTED, f"tensor dtype {t.dtype}")


def attn_params(q, k_blocks, block_table, out, scale: float = 0.0, chunk_tokens: int = 0,
                flags: int = 0, total_blocks_bound: int = 0) -> AttnParams:
    B, Hq, D = q.shape
    NB, Hkv, bs, D2 = k_blocks.shape
    assert D == D2
    return AttnParams(dtype=_torch_dtype_code(k_blocks), out_dtype=_torch_dtype_code(out), batch=B,
                      num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, block_size=bs, num_blocks=NB,
                      max_blocks_per_seq=block_table.shape[1], scale=float(scale),
                      chunk_tokens=int(chunk_tokens), flags=int(flags),
                      total_blocks_bound=int(total_blocks_bound))


def decode_attention_workspace(params: AttnParams, total_kv_tokens: int = -1) -> int:
    return int(load().as_decode_attention_workspace(C.byref(params), int(total_kv_tokens)))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def decode_attention(q, k_blocks, v_blocks, block_table, kv_lens, out, kv_lens_host=None,
                     workspace=None, scale: float = 0.0, chunk_tokens: int = 0, flags: int = 0,
                     stream=None, params: Optional[AttnParams] = None):
    """Enqueue decode attention for one batch.  All tensor arguments are
    torch CUDA tensors (contiguous); kv_lens_host is an optional int32 NumPy
    array.  `workspace` is a torch uint8 CUDA tensor; one is allocated when
    omitted (callers on a hot loop pass their own).  Returns `out`."""
    import torch
    lib = load()
    for t in (q, k_blocks, v_blocks, block_table, kv_lens, out):
        if not t.is_cuda or not t.is_contiguous():
            raise AlignedServeError(AS_EINVAL, "tensors must be contiguous CUDA tensors")
    if block_table.dtype != torch.int32 or kv_lens.dtype != torch.int32:
        raise AlignedServeError(AS_EINVAL, "block_table and kv_lens must be int32")
    if q.dtype != k_blocks.dtype or v_blocks.dtype != k_blocks.dtype or v_blocks.shape != k_blocks.shape:
        raise AlignedServeError(AS_EINVAL, "q / k_blocks / v_blocks disagree in dtype or shape")
    if out.shape != q.shape or kv_lens.shape[0] != q.shape[0] or block_table.shape[0] != q.shape[0]:
        raise AlignedServeError(AS_EINVAL, "out / kv_lens / block_table disagree with q in shape")
    if params is None:
        params = attn_params(q, k_blocks, block_table, out, scale, chunk_tokens, flags)
    host = None
    if kv_lens_host is not None:
        host = _i32(kv_lens_host)
        if host.shape[0] != q.shape[0]:
            raise AlignedServeError(AS_EINVAL, "kv_lens_host has the wrong length")
    if workspace is None:
        # The temporary below belongs to torch's caching allocator on the CURRENT stream and is
        # released when this call returns; that is safe only for work enqueued on that same stream.
        if _stream_ptr(stream) != torch.cuda.current_stream().cuda_stream:
            raise AlignedServeError(AS_EINVAL, "pass a workspace when launching on a stream other than "
                                               "torch's current stream")
        total = int(host.sum()) if host is not None else -1
        nbytes = decode_attention_workspace(params, total)
        if nbytes == 0:
            _check(AS_EINVAL if not lib.as_last_error() else AS_EINVAL)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    _check(lib.as_decode_attention(q.data_ptr(), k_blocks.data_ptr(), v_blocks.data_ptr(),
                                   block_table.data_ptr(), kv_lens.data_ptr(),
                                   _ptr(host, C.c_int32), out.data_ptr(), C.byref(params),
                                   workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out


def decode_attention_static_capacity() -> int:
    return int(load().as_decode_attention_static_capacity())


def decode_attention_static(q, k_blocks, v_blocks, block_table, kv_lens, out, kv_lens_host=None,
                            scale: float = 0.0, chunk_tokens: int = 0, flags: int = 0, stream=None,
                            params: Optional[AttnParams] = None):
    """decode_attention without a workspace: plan and partials go to the
    library's static device array (no allocation anywhere).  Returns `out`."""
    if params is None:
        params = attn_params(q, k_blocks, block_table, out, scale, chunk_tokens, flags)
    host = None if kv_lens_host is None else _i32(kv_lens_host)
    _check(load().as_decode_attention_static(q.data_ptr(), k_blocks.data_ptr(), v_blocks.data_ptr(),
                                             block_table.data_ptr(), kv_lens.data_ptr(),
                                             _ptr(host, C.c_int32), out.data_ptr(), C.byref(params),
                                             _stream_ptr(stream)))
    return out


def kv_read_sweep(k_blocks, v_blocks, block_table, kv_lens, checksum, params: AttnParams,
                  workspace, kv_lens_host=None, stream=None):
    """Measurement aid: stream the K/V bytes the attention call would read."""
    host = None if kv_lens_host is None else _i32(kv_lens_host)
    _check(load().as_kv_read_sweep(k_blocks.data_ptr(), v_blocks.data_ptr(), block_table.data_ptr(),
                                   kv_lens.data_ptr(), _ptr(host, C.c_int32),
                                   None if checksum is None else checksum.data_ptr(),
                                   C.byref(params), workspace.data_ptr(), workspace.numel(),
                                   _stream_ptr(stream)))


# ---------------------------------------------------------------------------
# stage_kv / unstage_kv / pipeline
# ---------------------------------------------------------------------------
def _move(fn, host_k, host_v, host_ids, dev_k, dev_v, dev_ids, block_bytes, stream):
    hid = np.ascontiguousarray(host_ids, dtype=np.int64)
    did = _i32(dev_ids)
    if hid.shape != did.shape:
        raise AlignedServeError(AS_EINVAL, "id lists differ in length")
    n_host = host_k.numel() * host_k.element_size() // block_bytes
    n_dev = dev_k.numel() * dev_k.element_size() // block_bytes
    _check(fn(host_k.data_ptr(), None if host_v is None else host_v.data_ptr(),
              _ptr(hid, C.c_int64), n_host, dev_k.data_ptr(),
              None if dev_v is None else dev_v.data_ptr(), _ptr(did, C.c_int32), n_dev,
              int(hid.shape[0]), int(block_bytes), _stream_ptr(stream)))


def stage_set_policy(policy: int):
    """How stage_kv / unstage_kv move blocks: STAGE_AUTO, STAGE_DMA or STAGE_KERNEL."""
    _check(load().as_stage_set_policy(int(policy)))


def stage_kv(host_k, host_v, src_ids, dev_k, dev_v, dst_ids, block_bytes: int, stream=None):
    """Enqueue host-pool -> HBM-pool block copies (host tensors pinned)."""
    _move(load().as_stage_kv, host_k, host_v, src_ids, dev_k, dev_v, dst_ids, block_bytes, stream)


def unstage_kv(host_k, host_v, dst_ids, dev_k, dev_v, src_ids, block_bytes: int, stream=None):
    """Enqueue HBM-pool -> host-pool block copies (eviction)."""
    _move(load().as_unstage_kv, host_k, host_v, dst_ids, dev_k, dev_v, src_ids, block_bytes, stream)


class Pipeline:
    """Copy/compute handshake of a multi-buffered HBM block pool."""

    def __init__(self, num_buffers: int = 2):
        self._h = C.c_void_p()
        _check(load().as_pipeline_create(C.byref(self._h), int(num_buffers)))

    @property
    def stream(self) -> int:
        return int(load().as_pipeline_stream(self._h))

    def begin_stage(self, buf: int):
        _check(load().as_pipeline_begin_stage(self._h, buf))

    def end_stage(self, buf: int):
        _check(load().as_pipeline_end_stage(self._h, buf))

    def acquire(self, buf: int, stream=None):
        _check(load().as_pipeline_acquire(self._h, buf, _stream_ptr(stream)))

    def release(self, buf: int, stream=None):
        _check(load().as_pipeline_release(self._h, buf, _stream_ptr(stream)))

    def query(self, buf: int) -> bool:
        """True when the copies last closed by end_stage(buf) have finished."""
        r = C.c_int32(0)
        _check(load().as_pipeline_query(self._h, buf, C.byref(r)))
        return bool(r.value)

    def destroy(self):
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(load().as_pipeline_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ---------------------------------------------------------------------------
# quad-tree + Density First Search batch generator
# ---------------------------------------------------------------------------
class QuadTree:
    """The paper's batch generator: quad-tree over prefix lengths + Density
    First Search (argument marshalling over as_qtree_*)."""

    def __init__(self, max_len: int = 65536, leaf_width: int = 16):
        self._h = C.c_void_p()
        _check(load().as_qtree_create(C.byref(self._h), int(max_len), int(leaf_width)))

    def insert(self, request_id: int, prefix_len: int, blocks: int, now: float = 0.0):
        _check(load().as_qtree_insert(self._h, int(request_id), int(prefix_len), int(blocks), float(now)))

    def remove(self, request_id: int):
        _check(load().as_qtree_remove(self._h, int(request_id)))

    def size(self):
        r, b = C.c_int64(), C.c_int64()
        _check(load().as_qtree_size(self._h, C.byref(r), C.byref(b)))
        return r.value, b.value

    def __len__(self):
        return self.size()[0]

    def next_batch(self, b_max: int, k_min: int, now: float = 0.0, starve_after=None):
        """Returns (ids, case) of one generated batch; ([], 0) when empty."""
        cap = max(len(self), 1)
        ids = np.empty(cap, dtype=np.int32)
        n, case = C.c_int32(0), C.c_int32(0)
        _check(load().as_qtree_next_batch(self._h, int(b_max), int(k_min), float(now),
                                          -1.0 if starve_after is None else float(starve_after),
                                          _ptr(ids, C.c_int32), cap, C.byref(n), C.byref(case)))
        return ids[: n.value].tolist(), case.value

    def destroy(self):
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(load().as_qtree_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def dfs_batches(kv_lens, blocks, b_max: int, k_min: int, max_len: int = 65536, leaf_width: int = 16):
    """All requests through the quad-tree generator; returns (order, batch_offsets)."""
    lens, blk = _i32(kv_lens), _i32(blocks)
    n = int(lens.shape[0])
    order = np.empty(max(n, 1), dtype=np.int32)
    offsets = np.empty(n + 1, dtype=np.int32)
    nb = C.c_int32(0)
    _check(load().as_dfs_batches(_ptr(lens, C.c_int32), _ptr(blk, C.c_int32), n, int(b_max), int(k_min),
                                 int(max_len), int(leaf_width), _ptr(order, C.c_int32),
                                 _ptr(offsets, C.c_int32), C.byref(nb)))
    return order[:n], offsets[: nb.value + 1]


# ---------------------------------------------------------------------------
# decode loop: KV append and the batch-level scheduler
# ---------------------------------------------------------------------------
def kv_append(k_new, v_new, k_blocks, v_blocks, block_table, kv_lens, stream=None):
    """Append one token's K/V per request to the paged cache; kv_lens (device
    int32) is incremented in place."""
    NB, Hkv, bs, D = k_blocks.shape
    params = AttnParams(dtype=_torch_dtype_code(k_blocks), out_dtype=_torch_dtype_code(k_blocks),
                        batch=kv_lens.shape[0], num_q_heads=Hkv, num_kv_heads=Hkv, head_dim=D,
                        block_size=bs, num_blocks=NB, max_blocks_per_seq=block_table.shape[1],
                        scale=0.0, chunk_tokens=0, flags=0, total_blocks_bound=0)
    _check(load().as_kv_append(k_new.data_ptr(), v_new.data_ptr(), k_blocks.data_ptr(), v_blocks.data_ptr(),
                               block_table.data_ptr(), kv_lens.data_ptr(), C.byref(params),
                               _stream_ptr(stream)))


class Scheduler:
    """Batch-level scheduling policy (marshalling over as_sched_*)."""

    def __init__(self, total_blocks: int, block_size: int = 16, max_batch: int = 64):
        self._h = C.c_void_p()
        self.max_batch = int(max_batch)
        _check(load().as_sched_create(C.byref(self._h), int(total_blocks), int(block_size), int(max_batch)))

    def push_candidate_batch(self, origin, ids, kv_lens, remaining):
        i, l, r = _i32(ids), _i32(kv_lens), _i32(remaining)
        _check(load().as_sched_push_candidate_batch(self._h, int(origin), _ptr(i, C.c_int32),
                                                    _ptr(l, C.c_int32), _ptr(r, C.c_int32), int(i.shape[0])))

    def push_candidate_request(self, origin, rid, kv_len, remaining):
        _check(load().as_sched_push_candidate_request(self._h, int(origin), int(rid), int(kv_len), int(remaining)))

    def state(self):
        f, a, b, c = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32()
        _check(load().as_sched_state(self._h, C.byref(f), C.byref(a), C.byref(b), C.byref(c)))
        return dict(free_blocks=f.value, running=a.value, candidate_requests=b.value, candidate_batch=c.value)

    def running(self):
        cap = max(self.state()["running"], 1)
        ids, lens, org = (np.empty(cap, dtype=np.int32) for _ in range(3))
        n = C.c_int32()
        _check(load().as_sched_running(self._h, _ptr(ids, C.c_int32), _ptr(lens, C.c_int32),
                                       _ptr(org, C.c_int32), cap, C.byref(n)))
        return ids[: n.value].copy(), lens[: n.value].copy(), org[: n.value].copy()

    def step(self, advance: bool = True):
        cap = max(self.state()["running"], self.max_batch)
        done, ev, ad = (np.empty(cap, dtype=np.int32) for _ in range(3))
        nd, ne, na, case = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        _check(load().as_sched_step(self._h, 1 if advance else 0, _ptr(done, C.c_int32), C.byref(nd),
                                    _ptr(ev, C.c_int32), C.byref(ne), _ptr(ad, C.c_int32), C.byref(na),
                                    cap, C.byref(case)))
        return done[: nd.value].tolist(), ev[: ne.value].tolist(), ad[: na.value].tolist(), case.value

    def destroy(self):
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(load().as_sched_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
