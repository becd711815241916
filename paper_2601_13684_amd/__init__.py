"""HeteroCache decode hot path for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI.

  include/hc.h      the boundary (hc_decode_attn, hc_rep_topk_drift, hc_gather_retrieve, ...)
  csrc/             HIP kernels and host-side planning
  binding.py        ctypes binding with the same names (argument marshalling only)
  runtime.py        HBM / pinned-host layout of a layer and the per-step call order
  inputs.py         seeded synthetic workloads (shared with the CPU oracle; no method arithmetic)
  build.py          hipcc build of libhc.so, in-tree

There is no CPU execution path: without the built library every call raises.
"""
__all__ = ["binding", "runtime", "inputs", "build"]
