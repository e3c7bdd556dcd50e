"""Optimizer wrapper and loss-scale policy of the oracle (test infrastructure only).

Section 3.2 of the paper: the wrapper takes the fp16 gradients, converts them
to fp32, hands them to an ordinary optimizer that updates the fp32 master
weights, and converts the updated masters back to fp16 for the next
iteration.  Section 3.1, item 1: the optimizer inspects the gradients every
iteration and sets the loss scale of the next one ("Backoff" policy; the
paper gives the name only - halve on overflow, skip that step, double after
`growth_interval` consecutive clean steps is the reading taken here).
Section 3.3: a weight-decay regulariser acts on the fp32 copy, its gradient
being added to the unscaled fp32 gradient.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

from .numerics import Policy, half_bits


@dataclass
class ScaleState:
    mode: str = "backoff"            # "static" | "backoff"
    scale: float = 2.0 ** 15
    growth_interval: int = 10
    min_scale: float = 1.0
    max_scale: float = 2.0 ** 24
    good_steps: int = 0
    opt_step: int = 0                # t of Adam: counts applied steps only
    total_steps: int = 0
    skipped_steps: int = 0
    history: List[Tuple[float, int]] = field(default_factory=list)  # (scale used, found_inf)


def has_nonfinite(P: Policy, grads) -> bool:
    """True iff any stored gradient value is inf or NaN.  Under MIXED the test
    is on the binary16 encoding: exponent field all ones."""
    for g in grads:
        if P.half_storage:
            if np.any((half_bits(g) & 0x7C00) == 0x7C00):
                return True
        elif not np.all(np.isfinite(g)):
            return True
    return False


def unscale_check_update(P: Policy, tensors: List[Dict[str, np.ndarray]], opt, st: ScaleState) -> int:
    """One optimizer-wrapper call over every parameter tensor.

    `tensors` is a list of dicts with keys g16 (stored gradient, loss-scaled),
    w32 (master), w16 (stored copy), m, v (Adam moments; absent for SGD); the
    arrays are updated in place.  If any gradient holds inf/NaN nothing is
    touched and 1 is returned.  Otherwise, per element, in the arithmetic type:
        g   = g16 * (1/S)  [+ weight_decay * w32]
        SGD : w32 -= lr * g
        Adam: m = b1 m + (1-b1) g ; v = b2 v + (1-b2) g^2 ;  t = opt_step + 1
              w32 -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
        w16 = store(w32)
    Scalars (1-b1, 1-b2, bias corrections) are formed in double and cast.
    """
    if has_nonfinite(P, [t["g16"] for t in tensors]):
        return 1
    A = P.scalar
    inv_s = A(1) / A(st.scale)
    lr, wd = A(opt.lr), A(opt.weight_decay)
    if opt.kind == "adam":
        t = st.opt_step + 1
        b1, b2, eps = A(opt.beta1), A(opt.beta2), A(opt.eps)
        omb1, omb2 = A(1.0 - opt.beta1), A(1.0 - opt.beta2)
        bc1, bc2 = A(1.0 - float(opt.beta1) ** t), A(1.0 - float(opt.beta2) ** t)
    for tn in tensors:
        g = tn["g16"] * inv_s
        if opt.weight_decay != 0.0:
            g = g + wd * tn["w32"]
        if opt.kind == "sgd":
            tn["w32"][...] = tn["w32"] - lr * g
        elif opt.kind == "adam":
            tn["m"][...] = b1 * tn["m"] + omb1 * g
            tn["v"][...] = b2 * tn["v"] + omb2 * (g * g)
            mhat = tn["m"] / bc1
            vhat = tn["v"] / bc2
            tn["w32"][...] = tn["w32"] - lr * mhat / (np.sqrt(vhat) + eps)
        else:
            raise ValueError(opt.kind)
        tn["w16"][...] = P.store(tn["w32"])
    return 0


def loss_scale_update(st: ScaleState, found_inf: int) -> None:
    """Record the step and set the scale of the next iteration.

    overflow : scale <- max(scale/2, min), good_steps <- 0, step counted as skipped
    clean    : opt_step += 1, good_steps += 1; when good_steps reaches
               growth_interval: scale <- min(2 scale, max), good_steps <- 0
    static   : the scale never changes; an overflowing step is still skipped.
    """
    st.history.append((float(st.scale), int(found_inf)))
    st.total_steps += 1
    if found_inf:
        st.skipped_steps += 1
        st.good_steps = 0
        if st.mode == "backoff":
            st.scale = max(st.scale / 2.0, st.min_scale)
    else:
        st.opt_step += 1
        st.good_steps += 1
        if st.mode == "backoff" and st.good_steps >= st.growth_interval:
            st.scale = min(st.scale * 2.0, st.max_scale)
            st.good_steps = 0
