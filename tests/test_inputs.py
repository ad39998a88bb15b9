"""The shared input generators (no method arithmetic in them).  CPU only."""
import numpy as np
import pytest

import synth_inputs as si


def test_payload_slices_are_consistent():
    full = si.payload(3, 2, si.BLOCK + 5000, "uniform", "fp32")
    part = si.payload(3, 2, 7000, "uniform", "fp32", start=si.BLOCK - 3000)
    assert np.array_equal(full[si.BLOCK - 3000:si.BLOCK + 4000], part)
    assert full.min() >= -1.0 and full.max() <= 1.0
    assert not np.array_equal(si.payload(3, 1, 100, "uniform", "fp32"), si.payload(3, 2, 100, "uniform", "fp32"))


def test_hash_payload_matches_torch_generator_and_slices():
    torch = pytest.importorskip("torch")
    for dtype in ("fp32", "int32"):
        n = 100_003
        a = si.hash_payload(5, 3, 0, n, dtype)
        b = si.hash_payload_torch(5, 3, n, dtype, "cpu", block=4096).numpy()
        assert a.dtype == b.dtype and np.array_equal(a, b)
        assert np.array_equal(a[777:9999], si.hash_payload(5, 3, 777, 9999 - 777, dtype))
        assert not np.array_equal(a, si.hash_payload(5, 4, 0, n, dtype))
    f = si.hash_payload(1, 0, 0, 1 << 16, "fp32")
    assert -1.0 <= f.min() < -0.99 and 0.99 < f.max() < 1.0 and abs(float(f.mean())) < 0.02
    i = si.hash_payload(1, 0, (1 << 33) + 5, 1 << 16, "int32")     # large offsets keep working
    assert (i < 0).any() and (i > 0).any()


def test_bucket_sizes():
    b = si.bucket_sizes()
    assert len(b) == 16 and sum(b) == 138_000_000 and all(x % 4 == 0 for x in b)
    assert min(b) * 4 >= 64 << 10 and max(b) * 4 <= (400 << 20) + 16 * 4 * 16
    assert b == si.bucket_sizes()


def test_topologies():
    assert si.complete_graph(4).m == 12 and si.hybrid_cube_mesh().m == 32
    d = si.hybrid_cube_mesh(doubled=True)
    assert d.cap.sum() == 2 * (8 * 1 + 8 * 2)
    sub = si.induced(d, (0, 1, 4))
    assert sub.k == 3 and sorted(sub.arcs()) == [(0, 1, 2.0), (0, 2, 2.0), (1, 0, 2.0), (2, 0, 2.0)]
