"""MI355X-native KVCache-reuse hot path: prefix-reused paged prefill attention and
layer-wise KV page pack/unpack, as hand-written HIP kernels behind a C ABI.

``workloads`` (seeded synthetic inputs) imports without the HIP library; the
entry points in ``binding`` load ``libmooncake_hip.so`` on first use and raise
if it has not been built.
"""
__all__ = ["workloads", "binding", "build"]
