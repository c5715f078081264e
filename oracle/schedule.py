"""CPU oracle (test infrastructure) for the learning-rate schedule of Section 5.

The paper: the rate starts at 0.1, is ramped linearly to 0.1*k*n/256 (k = batch per GPU,
n = number of workers = nodes x GPUs per node), and is divided by 10 after every 30 epochs of
a 90-epoch run.  The length of the ramp is not stated (the schedule the paper cites ramps over
5 epochs), so it is an argument.  Plain float64 arithmetic.
"""
import math


def target_lr(base_lr: float, batch_per_gpu: int, n_workers: int) -> float:
    return base_lr * batch_per_gpu * n_workers / 256.0


def lr_at(epoch: float, base_lr: float = 0.1, batch_per_gpu: int = 64, n_workers: int = 128,
          warmup_epochs: float = 5.0, drop_every_epochs: float = 30.0) -> float:
    top = target_lr(base_lr, batch_per_gpu, n_workers)
    if epoch < warmup_epochs:
        return base_lr + (top - base_lr) * (epoch / warmup_epochs)
    drops = math.floor(epoch / drop_every_epochs)
    return top / (10.0 ** drops)
