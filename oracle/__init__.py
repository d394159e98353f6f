"""fp64 CPU oracle of the MatKV hot path (test infrastructure only; see matkv_oracle.c)."""
from .matkv_oracle import (assemble, attn, build, chunk_attn, compress, decode_attn, decompress,
                           e4m3_decode, e4m3_encode, kv_scale, materialize, prefill_attn, rope, threads)

__all__ = ["assemble", "attn", "build", "chunk_attn", "compress", "decode_attn", "decompress",
           "e4m3_decode", "e4m3_encode", "kv_scale", "materialize", "prefill_attn", "rope", "threads"]
