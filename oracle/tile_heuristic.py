"""Oracle of the tile-volume heuristic (paper Sec. IV-C, Eq. (heuristic)).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/`` may import this
module.  Exact rational arithmetic; shares no code with the HIP library.

The equation takes the (d-1)-th root of (s_LM / 4) / (s_f * c / 2), raises it
to the power d-1 again and caps the result by (min_n I_n)^(d-1).  Tiles are
regular (integer width along each of the d-1 modes, Sec. IV-C: "our
implementation assumes that the tile size is regular"), so the root is rounded
down to an integer width before it is raised again; the paper's own values
(216 = 6^3 for its 4-way tensor, 256 = 4^4 for its 5-way tensor) confirm the
rounding.
"""
from fractions import Fraction
from typing import Sequence, Tuple


def tile_volume(dims: Sequence[int], cache_bytes: int, value_bytes: int,
                tiles_per_unit: int) -> Tuple[int, int]:
    """Returns (width, N_T) of Eq. (heuristic)."""
    d = len(dims)
    if d < 2:
        raise ValueError("need at least two modes")
    budget = Fraction(cache_bytes, 4) / (Fraction(value_bytes) * Fraction(tiles_per_unit, 2))
    width = 1
    while Fraction((width + 1) ** (d - 1)) <= budget:
        width += 1
    width = min(width, min(dims))
    return width, width ** (d - 1)
