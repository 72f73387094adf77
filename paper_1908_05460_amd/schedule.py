"""Approximation schedules (Section 2.5): which gradient method each convolution
layer uses on each training batch.  Host-side masks only; the library's
``conv_wgrad_schedule_run`` consumes one row (one batch) at a time.

Layers are numbered from 1 as in the paper ("starting from the second
convolutional layer"); batches from 0.
"""
import numpy as np

EXACT, APPROX, ZERO, RANDOM = 0, 1, 2, 3
METHOD_NAMES = {EXACT: "exact", APPROX: "approx", ZERO: "zero", RANDOM: "random"}


def _row(nlayers, chosen_layers, method):
    row = np.full(nlayers, EXACT, np.uint8)
    for l in chosen_layers:            # 1-based layer numbers
        row[l - 1] = method
    return row


def schedule1(nlayers, batch, method=APPROX):
    """Every fourth convolution starting from the second, on every batch (Section 3):
    four layers of a 16-convolution VGG-19, five of a 19-convolution ResNet-20."""
    return _row(nlayers, range(2, nlayers + 1, 4), method)


def schedule2(nlayers, batch, method=APPROX):
    """Every other layer on every other batch (Section 3.4)."""
    return _row(nlayers, range(2, nlayers + 1, 2) if batch % 2 == 1 else (), method)


def schedule3(nlayers, batch, method=APPROX):
    """Every layer on every fourth batch (Section 3.4)."""
    return _row(nlayers, range(1, nlayers + 1) if batch % 4 == 3 else (), method)


def all_exact(nlayers, batch, method=APPROX):
    return _row(nlayers, (), method)


def every_other_layer(nlayers, batch, method=APPROX):
    """Layers 2, 4, 6, ... on every batch (the first convolution is never approximated,
    following Section 3)."""
    return _row(nlayers, range(2, nlayers + 1, 2), method)


def all_but_first_and_last(nlayers, batch, method=APPROX):
    return _row(nlayers, range(2, nlayers), method)


def alternate_batches(nlayers, batch, method=APPROX):
    """Every layer approximated on odd batches, none on even ones."""
    return _row(nlayers, range(1, nlayers + 1) if batch % 2 == 1 else (), method)


SWEEP_MASKS = {
    "all_exact": all_exact,
    "every_other_layer": every_other_layer,
    "all_but_first_and_last": all_but_first_and_last,
    "alternate_batches": alternate_batches,
}
PAPER_SCHEDULES = {"schedule1": schedule1, "schedule2": schedule2, "schedule3": schedule3}


def fraction_approximated(fn, nlayers, nbatches):
    rows = np.stack([fn(nlayers, b) for b in range(nbatches)])
    return float((rows != EXACT).mean())
