"""CPU oracle, part 5: chunk-size selection by multiplicative increase, additive
decrease (paper section 4.2.1, "Automatic chunk size selection").

TEST INFRASTRUCTURE ONLY (see oracle/graph.py).  Shares no code with the
library's tuner.

What the paper fixes: start from a small chunk; multiply it by a factor from one
iteration to the next as long as the measured throughput increases; once the
throughput decreases, decrease the chunk additively until a steady state is
reached.  Its example starts at 1 MB with factor 2 and is stable after four
iterations.

Reading where the paper is silent:
  * "increases" means: exceeds the previous measurement by more than rel_tol;
  * the additive step is a parameter (the example's natural choice is the
    initial chunk);
  * in the decrease phase the chunk keeps shrinking while that still raises the
    throughput; the first step that does not ends the search;
  * the steady state is the best chunk measured so far (ties: the earlier one);
  * chunk sizes are clamped to [lo, hi]; hitting a bound ends the phase.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Tuple

INCREASE, DECREASE, STEADY = 0, 1, 2


class Miad:
    def __init__(self, initial: int, factor: float = 2.0, step: Optional[int] = None,
                 lo: int = 1, hi: int = 1 << 40, rel_tol: float = 0.0):
        if initial < 1 or factor <= 1.0 or lo < 1 or hi < lo or rel_tol < 0:
            raise ValueError("bad MIAD parameters")
        self.chunk = min(max(initial, lo), hi)
        self.factor = factor
        self.step = initial if step is None else step
        if self.step < 1:
            raise ValueError("bad MIAD step")
        self.lo, self.hi, self.rel_tol = lo, hi, rel_tol
        self.phase = INCREASE
        self.prev: Optional[float] = None
        self.best: Optional[Tuple[float, int]] = None   # (throughput, chunk)

    def report(self, throughput: float) -> None:
        """Throughput measured with the current ``chunk``; moves to the next chunk."""
        if self.phase == STEADY:
            return
        if self.best is None or throughput > self.best[0]:
            self.best = (throughput, self.chunk)
        rising = self.prev is None or throughput > self.prev * (1.0 + self.rel_tol)
        self.prev = throughput
        if self.phase == INCREASE:
            if rising:
                nxt = min(int(self.chunk * self.factor), self.hi)
                if nxt == self.chunk:
                    self._settle()
                else:
                    self.chunk = nxt
            else:
                self.phase = DECREASE
                self._shrink()
        else:
            if rising:
                self._shrink()
            else:
                self._settle()

    def _shrink(self) -> None:
        nxt = self.chunk - self.step
        if nxt < self.lo:
            self._settle()
        else:
            self.chunk = nxt

    def _settle(self) -> None:
        self.phase = STEADY
        self.chunk = self.best[1]


def run(miad: Miad, throughput_of: Callable[[int], float], max_iters: int = 10_000) -> List[int]:
    """Chunk sizes tried, iteration by iteration, until the steady state (whose
    chunk is appended last)."""
    tried = []
    for _ in range(max_iters):
        if miad.phase == STEADY:
            break
        tried.append(miad.chunk)
        miad.report(throughput_of(miad.chunk))
    tried.append(miad.chunk)
    return tried
