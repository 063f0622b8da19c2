"""MI355X-native paged-KV attention hot path (decode, append-prefill, KV page restore).

The compute lives in the HIP library under csrc/ behind the C ABI of
include/ta.h; `binding` marshals torch tensors into it and `workloads` builds
seeded synthetic batches.  Nothing here falls back to a CPU implementation.
"""
__all__ = ["binding", "workloads"]
