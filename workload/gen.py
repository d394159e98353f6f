"""Seeded synthetic RAG-shaped inputs.  Holds no arithmetic of the method.

Both the fp64 oracle and the HIP path read tensors made here, so that they see
identical bytes: bf16 tensors are rounded once (round-to-nearest-even, by torch)
in this module and the oracle widens those same values to float64.

Shapes follow the paper's workloads (Section V-A: LLaMA-3 8B / 70B, chunks of
about a thousand tokens, a handful of retrieved chunks, short questions, tens to
hundreds of generated tokens).  Values are N(0,1) times a scale; nothing here is
an item of any dataset.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass

import numpy as np
import torch

MASTER_SEED = 251222195


@dataclass(frozen=True)
class Shape:
    """One benchmark configuration (sizes only)."""
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    hidden: int
    dtype: str            # "f32" | "bf16"
    batch: int
    n_chunks: int         # chunks retrieved per instance
    chunk_tokens: int
    q_len_min: int
    q_len_max: int
    decode_steps: int
    rope_base: float
    pool: int = 0         # size of the materialized-chunk pool (0: private chunks)
    value_scale: float = 1.0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def max_tail(self) -> int:
        return self.q_len_max + self.decode_steps

    def kv_bytes_per_token_layer(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    def blob_bytes(self, n_tokens: int | None = None) -> int:
        n = self.chunk_tokens if n_tokens is None else n_tokens
        return self.n_layers * self.kv_bytes_per_token_layer() * n


CONFIGS = {
    1: Shape("tiny-f32", 1, 4, 2, 64, 256, "f32", 1, 2, 256, 32, 32, 8, 10000.0,
             value_scale=1.0 / 8.0),
    2: Shape("llama3-8b-b1", 32, 32, 8, 128, 4096, "bf16", 1, 10, 1000, 64, 64, 128, 500000.0,
             value_scale=128 ** -0.5),
    3: Shape("llama3-8b-b16-pool200", 32, 32, 8, 128, 4096, "bf16", 16, 5, 1000, 32, 128, 64,
             500000.0, pool=200, value_scale=128 ** -0.5),
    4: Shape("llama3-70b-b4", 80, 64, 8, 128, 8192, "bf16", 4, 20, 1000, 128, 128, 256,
             500000.0, value_scale=128 ** -0.5),
    5: Shape("llama3-8b-stream64", 32, 32, 8, 128, 4096, "bf16", 1, 10, 1000, 64, 64, 128,
             500000.0, value_scale=128 ** -0.5),
}


def seed_for(*names) -> int:
    """Stable 63-bit seed for a named tensor, derived from the master seed."""
    h = hashlib.blake2b(repr((MASTER_SEED,) + tuple(names)).encode(), digest_size=8).digest()
    return int.from_bytes(h, "little") & ((1 << 63) - 1)


def normal(names, shape, scale: float = 1.0, dtype=torch.float32, device="cpu") -> torch.Tensor:
    """N(0,1)*scale tensor named by ``names``.  On the CPU it comes from numpy's
    Philox generator; on a GPU from torch's device generator (large tensors, where
    the oracle later reads back the slices it samples).  Rounded once to ``dtype``."""
    seed = seed_for(*names)
    dev = torch.device(device)
    if dev.type == "cpu":
        rng = np.random.Generator(np.random.Philox(seed))
        a = rng.standard_normal(size=tuple(shape), dtype=np.float32)
        t = torch.from_numpy(a)
        if scale != 1.0:
            t = t * float(scale)
        return t.to(dtype).contiguous()
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    t = torch.empty(tuple(shape), dtype=dtype, device=dev)
    t.normal_(0.0, float(scale), generator=g)
    return t


def question_lengths(cfg: Shape, tag="qlen") -> list[int]:
    """Question length of each instance of the batch, uniform in [q_len_min, q_len_max]."""
    rng = np.random.Generator(np.random.Philox(seed_for(cfg.name, tag)))
    return [int(x) for x in rng.integers(cfg.q_len_min, cfg.q_len_max + 1, size=cfg.batch)]


def retrieved_chunks(cfg: Shape, tag="retrieval") -> list[list[int]]:
    """Chunk ids retrieved by each instance.  With a pool, ids are drawn uniformly
    without replacement inside an instance (a chunk is never retrieved twice by one
    instance) and independently across instances, so pages are shared; without a
    pool every instance owns its chunks."""
    if cfg.pool <= 0:
        return [[b * cfg.n_chunks + c for c in range(cfg.n_chunks)] for b in range(cfg.batch)]
    rng = np.random.Generator(np.random.Philox(seed_for(cfg.name, tag)))
    return [[int(x) for x in rng.choice(cfg.pool, size=cfg.n_chunks, replace=False)]
            for _ in range(cfg.batch)]


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Widen a tensor (any device, f32 or bf16) to a float64 numpy array, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()
