"""CPU oracle for the mixed-precision training step (TEST INFRASTRUCTURE ONLY).

A plain, slow, step-by-step NumPy statement of what the paper's method
computes (Section 3.1: fp16 maths with fp32 accumulation, loss scaling, fp32
master weights; Section 3.2: the optimizer wrapper), used only by `tests/`,
by `__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`.
The product (the HIP library and its Python binding) never imports it, and
it never imports the product; the two share no code.

Parity status of its parts (what pins each is in tests/test_oracle_*.py):
  * storage rounding, linear / attention / LayerNorm / LSTM forward+backward,
    MSE and softmax cross-entropy, SGD / Adam on masters, the Backoff scale
    state machine: pinned (finite differences in fp64 storage, closed forms,
    invariants, brute force, hand-derived scale sequences).
  * whole multi-step training trajectories: parity unpinned against anything
    external; pinned only through the composition of the parts above.
  * the "LogMax" scaling policy the paper names without defining: not built,
    parity unpinned.
"""
from .numerics import Policy, MIXED, FP32, FP64  # noqa: F401
