"""MI355X-native prefill KV-eviction path of CodeComp (score -> select -> gather).

`binding` wraps the C ABI of libcodecomp.so (hand-written HIP for gfx950); `workloads` draws
the seeded synthetic inputs; `build` compiles the library in-tree.  Nothing is imported eagerly.
"""
__all__ = ["binding", "workloads", "build"]
