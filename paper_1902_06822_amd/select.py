"""Host-side choice of the layers that get a second INT4 tensor.

Section 3.5 calls a layer "key" when its MSE exceeds a threshold tau; the
workloads of this build rank layers by normalised error instead (sum of the
per-kernel squared errors over the layer's sum of squares) and take a fixed
share, ties going to the earlier layer.  Both rules are offered; neither is a
kernel.
"""
from __future__ import annotations

from typing import List, Sequence


def normalized_mse(sse_per_layer: Sequence[float], energy_per_layer: Sequence[float]) -> List[float]:
    """sum_k sse_lk / sum x^2 for every layer (0 for an all-zero layer)."""
    return [float(s) / float(e) if e > 0 else 0.0 for s, e in zip(sse_per_layer, energy_per_layer)]


def select_top_fraction(nmse: Sequence[float], fraction: float) -> List[int]:
    """Indices of the max(1, round(fraction*L)) layers with the largest NMSE, ascending."""
    L = len(nmse)
    if L == 0:
        return []
    count = max(1, int(round(fraction * L)))
    order = sorted(range(L), key=lambda i: (-nmse[i], i))
    return sorted(order[:count])


def select_above_threshold(mse: Sequence[float], tau: float) -> List[int]:
    """The rule of Section 3.5: layers whose (mean) squared error exceeds tau."""
    return [i for i, v in enumerate(mse) if v > tau]
