"""Chunk-size selection (paper section 4.2.1): pins for the oracle's state
machine and host-side parity of the library's against it.  CPU only."""
import math

import numpy as np
import pytest

import paper_1910_04940_amd as bl
from oracle import miad as om

MB = 1 << 18      # 1 MiB of 4-byte elements


def unimodal(peak, width=2.0):
    """Throughput curve with a single maximum at `peak` (log-parabola)."""
    return lambda c: 1e6 - (math.log2(c / peak) / width) ** 2 * 10.0


def lib_run(initial, factor, step, lo, hi, tol, curve, max_iters=10_000):
    m = bl.Miad(initial, factor, step, lo, hi, tol)
    tried = []
    for _ in range(max_iters):
        if m.steady:
            break
        tried.append(m.chunk)
        m.report(curve(m.chunk))
    tried.append(m.chunk)
    return tried


def test_paper_example_doubles_from_1MB_and_is_stable_after_four_iterations(paper_pins):
    """Start at 1 MB, factor 2; with a throughput curve that stops rising at 8 MB the
    first four iterations are 1, 2, 4, 8 MB and the search ends on 8 MB."""
    assert paper_pins["miad_initial_chunk_MB"] == "1" and paper_pins["miad_factor"] == "2"
    curve = unimodal(8 * MB)
    tried = om.run(om.Miad(1 * MB, factor=2.0, step=1 * MB), curve)
    assert tried[:4] == [1 * MB, 2 * MB, 4 * MB, 8 * MB]
    assert tried[4] == 16 * MB                      # first measurement that is worse ...
    assert tried[5] == 15 * MB                      # ... then additive decrease by the step
    assert tried[-1] == 8 * MB                      # steady state = best chunk measured
    best = max(tried[:-1], key=curve)
    assert curve(tried[-1]) == curve(best)


def test_increase_phase_is_multiplicative_and_decrease_phase_additive():
    for factor, step, peak in [(2.0, MB, 32 * MB), (3.0, MB // 2, 9 * MB), (1.5, 1000, 5 * MB)]:
        curve = unimodal(peak)
        tried = om.run(om.Miad(MB, factor=factor, step=step), curve)
        turn = next(i for i in range(1, len(tried)) if tried[i] < tried[i - 1])
        for i in range(1, turn):
            assert tried[i] == int(tried[i - 1] * factor)
        for i in range(turn, len(tried) - 1):
            assert tried[i] == tried[i - 1] - step
        assert curve(tried[-1]) == max(curve(c) for c in tried[:-1])


def test_monotone_curves_end_at_the_bounds():
    up = om.run(om.Miad(MB, hi=64 * MB), lambda c: float(c))
    assert up[-1] == 64 * MB and up[:7] == [MB << i for i in range(7)]
    down = om.run(om.Miad(4 * MB, step=MB, lo=MB), lambda c: 1.0 / c)
    assert down == [4 * MB, 8 * MB, 7 * MB, 6 * MB, 5 * MB, 4 * MB, 3 * MB, 2 * MB, 1 * MB, 1 * MB]
    flat = om.run(om.Miad(MB), lambda c: 5.0)
    assert flat[-1] == MB                     # nothing ever rises: the first chunk stays


def test_tolerance_ignores_noise():
    noisy = {MB: 10.0, 2 * MB: 10.05, 4 * MB: 10.02}
    tried = om.run(om.Miad(MB, rel_tol=0.02, step=MB), lambda c: noisy.get(c, 1.0))
    assert tried[:2] == [MB, 2 * MB] and tried[-1] == 2 * MB


CURVES = [unimodal(8 * MB), unimodal(3 * MB, 1.0), unimodal(100 * MB), lambda c: float(c),
          lambda c: 1.0 / c, lambda c: 5.0, lambda c: math.sin(c / MB) + 2.0]


@pytest.mark.parametrize("ci", range(len(CURVES)))
@pytest.mark.parametrize("params", [(MB, 2.0, MB, 1, 1 << 40, 0.0), (MB // 4, 2.0, MB // 4, MB // 8, 64 * MB, 0.01),
                                    (3 * MB, 1.5, 777, 1000, 50 * MB, 0.0), (MB, 4.0, 2 * MB, MB, 16 * MB, 0.05)])
def test_library_state_machine_matches_oracle(ci, params):
    initial, factor, step, lo, hi, tol = params
    curve = CURVES[ci]
    want = om.run(om.Miad(initial, factor, step, lo, hi, tol), curve)
    assert lib_run(initial, factor, step, lo, hi, tol, curve) == want


def test_library_rejects_bad_parameters():
    for args in [(0, 2.0, 1, 1, 10, 0.0), (1, 1.0, 1, 1, 10, 0.0), (1, 2.0, 0, 1, 10, 0.0),
                 (1, 2.0, 1, 0, 10, 0.0), (1, 2.0, 1, 5, 4, 0.0), (1, 2.0, 1, 1, 10, -0.1),
                 (1, float("nan"), 1, 1, 10, 0.0)]:
        from paper_1910_04940_amd import binding
        import ctypes as C
        out = C.c_void_p()
        assert binding.lib().blink_miad_create(*args, C.byref(out)) == bl.BLINK_EINVAL
    m = bl.Miad(MB)
    with pytest.raises(bl.BlinkError):
        m.report(float("nan"))
    with pytest.raises(bl.BlinkError):
        m.report(-1.0)
