"""Learning-rate policy of large mini-batch detector training (MegDet, section 3.2
"Learning Rate for Large Mini-Batch" and the training policies of section 4).

Host-side scalar code; nothing here touches the GPU.

What the paper fixes:
  * Linear Scaling Rule: a mini-batch k times larger takes a learning rate k times larger;
    the base rate is 0.02 at mini-batch size 16 (section 4);
  * Linear Gradual Warmup: start from a small rate r and raise it by the same amount after
    every iteration until the scaled rate is reached;
  * "normal" policy: the rate is multiplied by 0.1 at epochs 8 and 10, training ends at
    epoch 11; "long" policy: multiplied by 0.1 at epochs 11 and 14, halved at epoch 17,
    training ends at epoch 18.

Readings where the paper is silent:
  * the length of the warmup is not given: it is the caller's `warmup_iters`;
  * the warmup's starting rate "such as r" is read as the unscaled base rate by default;
  * epochs are counted from 0 and "at epoch e" means from the first iteration of epoch e on.
"""

from __future__ import annotations

BASE_LR = 0.02          # section 4: base learning rate ...
BASE_BATCH = 16         # ... for a mini-batch of 16 images

# policy -> ((epoch, factor applied from that epoch on), ...), epochs in the run
POLICIES = {
    "normal": (((8, 0.1), (10, 0.1)), 11),
    "long": (((11, 0.1), (14, 0.1), (17, 0.5)), 18),
}


def scaled_lr(batch: int, base_lr: float = BASE_LR, base_batch: int = BASE_BATCH) -> float:
    """Linear Scaling Rule (section 3.2): k = batch / base_batch times the base rate."""
    if batch < 1 or base_batch < 1:
        raise ValueError("batch sizes must be positive")
    return base_lr * batch / base_batch


def warmup_lr(iteration: int, warmup_iters: int, start_lr: float, target_lr: float) -> float:
    """Linear Gradual Warmup (section 3.2): `start_lr` at iteration 0, a constant increment
    per iteration, `target_lr` from iteration `warmup_iters` on."""
    if iteration < 0 or warmup_iters < 0:
        raise ValueError("iteration and warmup_iters must be non-negative")
    if iteration >= warmup_iters:
        return target_lr
    return start_lr + (target_lr - start_lr) * iteration / warmup_iters


def policy_factor(epoch: int, policy: str = "normal") -> float:
    """Product of the decay factors in force during `epoch` (section 4)."""
    steps, end = POLICIES[policy]
    if not 0 <= epoch < end:
        raise ValueError(f"the {policy!r} policy runs epochs 0..{end - 1}")
    f = 1.0
    for at, factor in steps:
        if epoch >= at:
            f *= factor
    return f


def total_epochs(policy: str = "normal") -> int:
    return POLICIES[policy][1]


def learning_rate(iteration: int, iters_per_epoch: int, batch: int, policy: str = "normal",
                  warmup_iters: int = 0, start_lr: float | None = None,
                  base_lr: float = BASE_LR, base_batch: int = BASE_BATCH) -> float:
    """Rate for one iteration: the scaled rate, warmed up linearly, times the policy's factor."""
    if iters_per_epoch < 1:
        raise ValueError("iters_per_epoch must be positive")
    target = scaled_lr(batch, base_lr, base_batch)
    start = base_lr if start_lr is None else start_lr
    return warmup_lr(iteration, warmup_iters, start, target) * policy_factor(iteration // iters_per_epoch, policy)
