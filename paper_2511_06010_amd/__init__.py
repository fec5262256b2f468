"""MI355X-native MoSKA decode-attention path: HIP kernels behind a C interface (include/moska.h)
and a thin ctypes binding with the same call names."""
from .binding import (MoskaError, Buffers, LIB_PATH, EXPORTS, load_library, problem_t, workspace_bytes, route,
                      bucket, shared_attn, unique_attn, merge, decode_step, decode_step_static, STATIC_SCRATCH_BYTES,
                      chunk_embeddings, quantize_shared)

__all__ = ["MoskaError", "Buffers", "LIB_PATH", "EXPORTS", "load_library", "problem_t", "workspace_bytes", "route",
           "bucket", "shared_attn", "unique_attn", "merge", "decode_step", "decode_step_static", "STATIC_SCRATCH_BYTES",
           "chunk_embeddings", "quantize_shared"]
