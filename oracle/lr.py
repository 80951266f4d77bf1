"""Oracle: the learning-rate schedules of the paper's experiments (test infrastructure).

Section IV, experimental setup: the single-learner baseline starts at 0.1 and is
annealed by 1/sqrt(2) every epoch after the 10th epoch (16 epochs in all).
Section IV, large batch size: with 8192-segment batches the rate is 3.2 (32 times
the rate of 256-segment batches); training starts from 0.32, warms up linearly
over the first 10 epochs to reach 3.2, and is annealed by 1/sqrt(2) in each epoch
afterwards.

Reading where the paper is silent: the rate is constant within an epoch; "linear
over the first 10 epochs" places the start value on epoch 1 and the peak on epoch
10 (with the paper's numbers that is 0.32 * epoch); the first annealed epoch is
the one after `hold_until`.
"""
import math


def lr_at_epoch(epoch, peak, start=None, warmup_epochs=0, hold_until=10):
    """Learning rate of the 1-based `epoch`."""
    if epoch < 1:
        raise ValueError("epochs count from 1")
    if warmup_epochs >= 2 and epoch <= warmup_epochs:
        return start + (peak - start) * (epoch - 1) / (warmup_epochs - 1)
    if epoch <= hold_until:
        return peak
    return peak * math.sqrt(0.5) ** (epoch - hold_until)
