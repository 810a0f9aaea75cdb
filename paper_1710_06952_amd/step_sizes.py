"""Per-event step sizes for the ``gamma`` array of a schedule.

The experiments of the paper (Sec. 5.2 and the scaling study of Sec. 5.3) hold the
step size constant within an epoch and change it at epoch boundaries: halved every 25
epochs for one network, divided by 10 at two fixed epochs for the other, and for many
workers a linear warm-up to a step size scaled with the number of workers.  In the
event view an epoch is ``events_per_epoch`` consecutive events (one pass over all
workers' data: total samples / M), so the rules below map an event number to its epoch
and the epoch to a step size.  Host-side only: the library just reads the array.
"""
import numpy as np


def epoch_of_events(K, events_per_epoch, k_begin=0):
    """Epoch number (from 0, fractional) at which each of the events k_begin .. k_begin + K - 1 starts."""
    if events_per_epoch <= 0:
        raise ValueError("events_per_epoch must be positive")
    return (k_begin + np.arange(K, dtype=np.float64)) / float(events_per_epoch)


def step_decay(K, events_per_epoch, base, factor=0.5, every=25, milestones=None, k_begin=0):
    """base * factor^(number of decays so far): a decay every ``every`` epochs, or at the listed
    ``milestones`` (the step changes at the START of that epoch, counting epochs from 1 as the paper
    does: milestone 81 means epochs 1..80 run at the old value)."""
    epoch = np.floor(epoch_of_events(K, events_per_epoch, k_begin))
    if milestones is None:
        decays = np.floor(epoch / every)
    else:
        decays = np.zeros_like(epoch)
        for m in milestones:
            decays += epoch >= (m - 1)
    return (base * np.power(float(factor), decays)).astype(np.float32)


def with_linear_warmup(gamma, events_per_epoch, warmup_epochs, start, k_begin=0):
    """Replace the first ``warmup_epochs`` epochs of ``gamma`` by a per-event linear ramp from ``start``
    to the value ``gamma`` has when the warm-up ends (gradual warm-up for large total batch sizes)."""
    gamma = np.array(gamma, np.float32)
    K = len(gamma)
    end_event = warmup_epochs * events_per_epoch
    k = k_begin + np.arange(K, dtype=np.float64)
    inside = k < end_event
    if inside.any():
        after = np.nonzero(~inside)[0]
        target = float(gamma[after[0]]) if len(after) else float(gamma[-1])
        gamma[inside] = (start + (target - start) * k[inside] / float(end_event)).astype(np.float32)
    return gamma
