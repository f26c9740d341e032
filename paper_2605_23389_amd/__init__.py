"""MI355X-native decode-attention hot path of AlignedServe: length-aligned
batch formation, host-to-HBM KV block staging, and batched single-query
attention over a paged KV cache (hand-written HIP for gfx950) behind a C-ABI
library.  `binding` is the thin ctypes layer over that library; `workloads`
draws the seeded synthetic inputs."""

__all__ = ["binding", "workloads", "traffic"]
