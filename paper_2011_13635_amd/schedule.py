"""The whole multi-stage schedule driven through the C ABI (Section 3.2, Figure 1; k and the layers per stage
from Section 4.1, step counts and warm-up from Section 4.2).

The training of an N-layer encoder is cut into k stages.  Stage 1 trains a stack of N/k layers completely
(embeddings included).  Every later stage grows the stack by N/k layers, initialised as copies of the N/k
layers below them, and trains only those new layers and the output layer; everything underneath runs
forward only.  A last retraining stage updates all layers together for a few steps with a small learning
rate.  The learning rate warms up linearly over the first steps of the run.

This module holds no arithmetic of the method: it decides which call to make with which layer split and
learning rate; every step runs in the library (mslt_train_step, mslt_grow).
"""
from __future__ import annotations

import inspect
import math
from dataclasses import dataclass, replace
from typing import Callable, List, Optional

from . import binding


@dataclass(frozen=True)
class Stage:
    """One entry of the schedule: layers [0, frozen) forward only, [frozen, frozen+trainable) trained."""
    name: str
    frozen: int
    trainable: int
    train_embeddings: bool
    steps: int
    lr: float
    grow_first: int = 0     # layers to add (by copying the top ones) before the stage starts
    seq_len: int = 0        # sequence length of this entry's batches; 0 = the run's ordinary length


def mslt_schedule(n_layers: int, k: int, steps_per_stage: int, retrain_steps: int, lr: float,
                  retrain_lr: Optional[float] = None) -> List[Stage]:
    """Stages of Section 3.2 for an n_layers encoder trained in k stages plus joint retraining.

    With k = 4 (Section 4.1) and the step counts of Section 4.2 (200 000 steps per stage, 200 000 retraining
    steps) this gives
    3 layers per stage for BERT-Base and 6 for BERT-Large, 1 000 000 steps in total.
    """
    if k < 1 or n_layers % k:
        raise ValueError("the number of layers must be a multiple of the number of stages")
    per = n_layers // k
    stages = [Stage("stage1", 0, per, True, steps_per_stage, lr)]
    for i in range(1, k):
        stages.append(Stage(f"stage{i + 1}", i * per, per, False, steps_per_stage, lr, grow_first=per))
    if retrain_steps > 0:
        stages.append(Stage("retrain", 0, n_layers, True, retrain_steps, lr if retrain_lr is None else retrain_lr))
    return stages


def long_sequence_tail(stages: List[Stage], fraction: float, seq_len: int) -> List[Stage]:
    """The last `fraction` of all steps on sequences of length `seq_len` (Section 4.2: the last 10 % of the
    steps use sequences of 512 so that the position embeddings beyond the ordinary length get trained).
    Entries that straddle the boundary are split in two; a split-off second half does not grow again."""
    total = sum(st.steps for st in stages)
    tail = int(math.ceil(fraction * total))
    out: List[Stage] = []
    for st in reversed(stages):
        if tail <= 0:
            out.append(st)
        elif st.steps <= tail:
            out.append(replace(st, seq_len=seq_len))
            tail -= st.steps
        else:
            out.append(replace(st, name=st.name + "-long", steps=tail, seq_len=seq_len, grow_first=0))
            out.append(replace(st, steps=st.steps - tail))
            tail = 0
    return list(reversed(out))


def warmup_factor(global_step: int, warmup_steps: int) -> float:
    """Linear warm-up over the first warmup_steps steps of the run (Section 4.2), 1 afterwards."""
    if warmup_steps <= 0 or global_step >= warmup_steps:
        return 1.0
    return (global_step + 1) / float(warmup_steps)


def run_schedule(model: "binding.Model", stages: List[Stage], next_batch: Callable[[int], "binding.Batch"],
                 make_opt: Callable[[float], "binding.Opt"], warmup_steps: int = 0,
                 on_step: Optional[Callable[[Stage, int, float], None]] = None) -> List[List[float]]:
    """Runs the stages in order on `model`; returns the losses per stage.

    next_batch(global_step) or next_batch(global_step, stage) hands out a device batch
    (binding.Model.device_batch), of length stage.seq_len where that is set;
    make_opt(lr) builds the optimizer settings for one step (binding.adam / binding.lamb).
    """
    wants_stage = len(inspect.signature(next_batch).parameters) >= 2
    losses: List[List[float]] = []
    present = 0
    step = 0
    for st in stages:
        if st.grow_first:
            model.mslt_grow(present, st.grow_first)
        present = max(present, st.frozen + st.trainable)
        out = []
        for i in range(st.steps):
            lr = st.lr * warmup_factor(step, warmup_steps)
            batch = next_batch(step, st) if wants_stage else next_batch(step)
            loss = model.mslt_train_step(st.frozen, st.trainable, st.train_embeddings, batch, make_opt(lr))
            out.append(loss)
            if on_step is not None:
                on_step(st, i, loss)
            step += 1
        losses.append(out)
    return losses
