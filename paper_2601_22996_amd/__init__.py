"""MI355X-native batched evaluation of KV-cache scheduling policies.

`kvsched` is the binding of the C ABI (include/kvsched.h); `workloads` holds
the seeded synthetic instances; `build` compiles the HIP library in-tree.
Submodules are imported on demand so that the input generators can be used
without loading the GPU library.
"""
__all__ = ["kvsched", "workloads", "build"]
