"""Oracle: the balls-into-bins expectation and the a_max bound (Appendix A, Eq. 4-5).
Used to pin the scheduler's load counting against a closed form.

Test infrastructure only.
"""
from __future__ import annotations

import math
from typing import Sequence

import numpy as np


def expected_activated(p: np.ndarray, hosted: Sequence[int], B: int) -> float:
    """Right-hand side of Eq. 4: sum over hosted experts of 1-(1-p_e)^B, where p_e is the
    probability that one token selects expert e (the p_e sum to K).  Equality holds when
    no hosted expert has a replica elsewhere."""
    return float(sum(1.0 - (1.0 - float(p[e])) ** B for e in hosted))


def a_max_bound(a_bar_max: float, C: int, n_inst: int) -> int:
    """Eq. 5: floor(min(C, a + sqrt(2 a ln n_e)) + 1)."""
    return int(math.floor(min(float(C), a_bar_max + math.sqrt(2.0 * a_bar_max * math.log(n_inst))) + 1.0))
