"""NAtS-L hybrid attention for AMD MI355X (gfx950): thin Python binding over the C ABI in
include/nats.h.  All arithmetic runs in the HIP kernels of libnats.so; this package only
marshals arguments (device pointers of torch tensors, the current HIP stream)."""
from .binding import (NatsError, decode, fwd_workspace_bytes, hybrid_attn_decode, hybrid_attn_decode_chunk,
                      hybrid_attn_bwd, hybrid_attn_decode_commit, hybrid_attn_fwd, hybrid_attn_fwd_ex, hybrid_attn_fwd_noalloc, library_path, load_library,
                      merge_weights, route_chunks)
from .autograd import hybrid_attn

__all__ = ["NatsError", "decode", "fwd_workspace_bytes", "hybrid_attn_decode", "hybrid_attn_decode_chunk",
           "hybrid_attn_bwd", "hybrid_attn_decode_commit", "hybrid_attn_fwd", "hybrid_attn_fwd_ex", "hybrid_attn_fwd_noalloc", "library_path", "load_library",
           "merge_weights", "route_chunks", "hybrid_attn"]
