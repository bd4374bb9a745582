"""The synthetic inputs have the sizes and value structure the workloads call for."""
import numpy as np

from paper_1511_04561_amd import workloads as w


def test_config_sizes():
    assert w.config_numel(1) == 1863690
    assert w.config_numel(2) == 1756426
    assert w.config_numel(3) == w.C3_NUMEL == 61100840
    assert w.config_numel(4) == 128 * 4096 + 1024 * 4096
    assert (w.C3_NUMEL + w.C3_BLOCK - 1) // w.C3_BLOCK == 14918 and w.C3_NUMEL % w.C3_BLOCK == 808


def test_seeding_is_reproducible_and_worker_dependent():
    a = w.tensor(3, 1)
    assert a.dtype == np.float32 and a.size == 64
    assert np.array_equal(a, w.tensor(3, 1))
    assert not np.array_equal(a, w.tensor(5, 1, worker=1))
    assert np.array_equal(w.tensor(3, 2, limit=100), w.tensor(3, 2)[:100])


def test_value_structure():
    g = w.tensor(1, 2)
    assert abs(float(np.std(g)) - 1e-3) < 2e-5
    c2 = w.tensor(2, 4)
    assert np.max(np.abs(c2)) > 20 * np.median(np.abs(c2))  # outliers at 50x
    act = w.tensor(4, 0)
    zeros = np.mean(act == 0)
    assert 0.48 < zeros < 0.52 and np.all(act >= 0) and not np.any(np.signbit(act))
    t = w.tensor(3, 8, limit=200000)
    assert np.max(np.abs(t)) > 10 * np.std(t) * 0.5  # heavy tails
