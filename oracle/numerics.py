"""Storage / accumulation policies of the oracle (test infrastructure only).

Section 3.1 of the paper fixes the arithmetic of mixed precision: operands
live in fp16, products are accumulated and kept in fp32, and activations,
activation gradients and weight gradients are stored back in fp16.  A Policy
says which type a tensor is *stored* in between operations (`store`) and which
type the arithmetic between two storage points runs in (`acc`).

  MIXED : store = IEEE binary16 with round-to-nearest-even, acc = fp32
          (the method itself).
  FP32  : store = acc = fp32 (the all-fp32 training the paper compares to).
  FP64  : store = acc = fp64 (the mathematical definition; used to pin the
          layer maths by finite differences).

Every tensor the oracle hands around is an array of dtype `acc` whose values
are exactly representable in the storage type.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Policy:
    name: str
    acc: type
    half_storage: bool

    def island(self, x) -> np.ndarray:
        """Bring a value into the arithmetic type (exact for stored values)."""
        return np.asarray(x, dtype=self.acc)

    def store(self, x) -> np.ndarray:
        """Round to the storage type; the result is held in the arithmetic type.

        For MIXED this is the single round-to-nearest-even to binary16 that
        happens at each storage point; values beyond the fp16 range become
        +-inf (that overflow is what dynamic loss scaling watches for) and
        tiny values become fp16 subnormals or zero.
        """
        x = np.asarray(x, dtype=self.acc)
        if self.half_storage:
            with np.errstate(over="ignore", invalid="ignore"):
                return x.astype(np.float16).astype(self.acc)
        return x

    def scalar(self, v):
        return self.acc(v)


MIXED = Policy("mixed", np.float32, True)
FP32 = Policy("fp32", np.float32, False)
FP64 = Policy("fp64", np.float64, False)


def half_bits(x) -> np.ndarray:
    """binary16 bit patterns (uint16) of values that are already fp16-representable."""
    with np.errstate(over="ignore", invalid="ignore"):
        return np.asarray(x).astype(np.float16).view(np.uint16)


def from_half_bits(bits, dtype=np.float32) -> np.ndarray:
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(dtype)
