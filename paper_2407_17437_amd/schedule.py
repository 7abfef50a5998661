"""Learning-rate schedule of the paper's experiments (Section 5.1, Table 1): host-side scalars.

The learning rate is an argument of every training step, so a schedule is nothing but the
number handed to `mlp_train_step`; no kernel is involved.
"""
from __future__ import annotations

# Table 1: initial learning rate by global density
INITIAL_LR_BY_DENSITY = {1.0: 0.01, 0.5: 0.01, 0.2: 0.01, 0.1: 0.03, 0.05: 0.03, 0.01: 0.1, 0.005: 0.1, 0.001: 0.1}


def initial_learning_rate(density: float) -> float:
    """Table 1 for the densities it lists; in between, the entry of the nearest listed density below
    (the table is a step function of the density: 0.01 down to 0.2, 0.03 down to 0.05, 0.1 below)."""
    if not 0.0 < density <= 1.0:
        raise ValueError("density must be in (0, 1]")
    listed = sorted(INITIAL_LR_BY_DENSITY)
    below = [d for d in listed if d <= density * (1 + 1e-12)]
    return INITIAL_LR_BY_DENSITY[below[-1] if below else listed[0]]


def learning_rate(epoch: int, epochs: int, lr0: float, factor: float = 0.1) -> float:
    """Decayed twice, by `factor`, after 50 % and after 75 % of the epochs (Section 5.1); the rate is
    fixed at the start of an epoch (Appendix B listing)."""
    if not 0 <= epoch < epochs:
        raise ValueError("epoch out of range")
    drops = int(2 * epoch >= epochs) + int(4 * epoch >= 3 * epochs)
    return lr0 * factor ** drops
