"""Communication volume and scalability estimate of arXiv 1712.02546, Section 4.2
("Scalability", Eq. (2)) and the Amdahl bounds quoted in Sections 1 and 4.2 -- TEST
INFRASTRUCTURE.  Exact rational arithmetic, no code shared with the library; only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may use it.

A layer is ``(inp, in_ch, k, num_k, out)``: square input width, input channels, square
kernel width, kernels, square output width (the symbols in, inCh, k, numK, out of Eq. (2)).

What the paper fixes: Eq. (2) -- per distributed layer the master exchanges the input maps
(in^2 * inCh * batch), the kernels (k^2 * numK * inCh) and the output maps (out^2 * numK *
batch); a constant bandwidth turns elements into time; the training time of one batch is
communication + convolution (slowest node) + computation of the other layers; Amdahl's law
bounds the speed-up by 1 / (1 - convolution fraction).

What it leaves open and this file decides (``partition_elements``): with several slaves every
slave receives all input maps, but only its own kernels, and returns only its own maps; the
master's own block is not transmitted.  With one slave that holds every kernel this is Eq. (2).
"""
from __future__ import annotations

from fractions import Fraction
from typing import Sequence, Tuple

Layer = Tuple[int, int, int, int, int]


def upload_elements(layers: Sequence[Layer], batch: int) -> int:
    """Eq. (2): elements exchanged between master and slaves for one batch."""
    total = 0
    for inp, in_ch, k, num_k, out in layers:
        total += inp * inp * in_ch * batch          # input maps
        total += k * k * num_k * in_ch              # kernels
        total += out * out * num_k * batch          # output maps
    return total


def partition_elements(layer: Layer, batch: int, bounds: Sequence[int], master: int) -> int:
    """Elements the master exchanges for one layer split at ``bounds`` (device ``master`` keeps
    its block at home): inputs to every other device, kernels out and maps back per block."""
    inp, in_ch, k, num_k, out = layer
    assert bounds[0] == 0 and bounds[-1] == num_k
    total = 0
    for dev in range(len(bounds) - 1):
        if dev == master:
            continue
        own = bounds[dev + 1] - bounds[dev]
        total += inp * inp * in_ch * batch
        total += k * k * own * in_ch
        total += out * out * own * batch
    return total


def transfer_seconds(elements: int, bytes_per_element: int, bits_per_second) -> Fraction:
    """Constant-bandwidth model of Section 4.2 (the paper: doubles, about 5 Mbps)."""
    return Fraction(elements * bytes_per_element * 8) / Fraction(bits_per_second)


def amdahl_limit(parallel_fraction) -> Fraction:
    """Largest speed-up when only ``parallel_fraction`` of the time is distributed."""
    return 1 / (1 - Fraction(parallel_fraction))


def batch_seconds(t_conv: Sequence, shares: Sequence, t_comp, t_comm) -> Fraction:
    """Comm. time + Conv. time of the slowest node + Comp. time (Section 4.2, Figure 5 legend)."""
    conv = max(Fraction(a) * Fraction(b) for a, b in zip(t_conv, shares))
    return Fraction(t_comm) + conv + Fraction(t_comp)


def speedup(t_conv: Sequence, shares: Sequence, t_comp, t_comm, master: int = 0) -> Fraction:
    """Against the master alone (no communication, all convolutions at home)."""
    alone = Fraction(t_conv[master]) + Fraction(t_comp)
    return alone / batch_seconds(t_conv, shares, t_comp, t_comm)
