"""Seeded synthetic inputs shared by the oracle-side and HIP-side tests (no method arithmetic)."""
from .gen import (CONFIGS, MASTER_SEED, Shape, normal, question_lengths, retrieved_chunks,
                  seed_for, to_f64)

__all__ = ["CONFIGS", "MASTER_SEED", "Shape", "normal", "question_lengths",
           "retrieved_chunks", "seed_for", "to_f64"]
