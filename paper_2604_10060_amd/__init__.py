"""MI355X-native hot path of cluster-driven KV-cache management for streaming
long-video VLM inference: online frame clustering, query-to-cluster scoring,
top-k cluster selection, cluster-granular gather and GQA attention over the
retrieved KV, as hand-written HIP kernels behind the C ABI in include/mosaic.h.

`binding` loads the built library lazily (first use); `inputs` only draws
synthetic streams and loads nothing.
"""
__all__ = ["binding", "inputs", "build"]
