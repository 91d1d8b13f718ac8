"""Seeded random walk over the parameter space (n, d, s, code, norm, K, value distribution):
every case goes through the same GPU-vs-oracle comparison as the named cases."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_1610_02132_amd as q  # noqa: E402
from paper_1610_02132_amd import workloads as W  # noqa: E402
from test_gpu_parity import run_case  # noqa: E402

DISTS = ["normal", "laplace_lognormal", "normal_loguniform", "student_t", "normal_outliers"]


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    kind = rng.integers(0, 5)
    if kind == 0:      # bucket path, d a multiple of 4
        d = int(rng.integers(1, 2049)) * 4
    elif kind == 1:    # small buckets
        d = int(rng.choice([4, 8, 12, 16, 32, 64, 100, 128, 256, 260, 512]))
    elif kind == 2:    # general path: odd bucket sizes
        d = int(rng.integers(1, 3000)) * 2 + 1
    elif kind == 3:    # general path: long buckets with entry lists
        d = int(rng.integers(8193, 40000))
    else:              # one bucket of n
        d = 1 << 30
    nb = int(rng.integers(1, 12)) if d > 4096 else int(rng.integers(1, 60))
    n = min(d, 150_000) * nb if d < (1 << 30) else int(rng.integers(1, 120_000))
    n = max(1, n - int(rng.integers(0, max(1, min(d, n)))))       # ragged last bucket
    s = int(rng.choice([1, 2, 3, 4, 7, 15, 16, 255, 256, 1000, 4097, 65535]))
    code = int(rng.integers(0, 3))
    norm = int(rng.integers(0, 2))
    K = int(rng.choice([1, 2, 3, 4, 8, 16, 17, 40, 64]))
    if n * K > 6_000_000:
        K = max(1, 6_000_000 // n)
    dist = DISTS[int(rng.integers(0, len(DISTS)))]
    w = W.Workload(f"r{seed}", n, s, min(d, n) if d >= (1 << 30) else d, code, K, 0.1, dist, (n,),
                   seed=int(rng.integers(0, 2**31)))
    return w, norm


@pytest.mark.parametrize("seed", range(int(__import__("os").environ.get("QSGD_RANDOM_CASES", "48"))))
def test_random_config(seed):
    w, norm = random_case(seed)
    run_case(w, norm=norm)
