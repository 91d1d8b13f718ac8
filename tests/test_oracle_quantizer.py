"""Pins for the oracle's Q_s (Sec. 3.1, Eq. 2; Lemma 3.1 and its proof; Sec. 4).

The expected values are computed here in float64 straight from the paper's
formulas; the oracle is driven through its public entry points only (draws are
injected where an exact enumeration needs them)."""
import itertools
import math

import numpy as np
import pytest

from conftest import read_golden


def probs64(v, s):
    """a_i, l_i, p_i of Eq. (2) in float64."""
    v = np.asarray(v, dtype=np.float64)
    nrm = math.sqrt(float((v * v).sum()))
    a = np.abs(v) / nrm
    l = np.minimum(np.floor(a * s), s - 1)
    p = a * s - l
    return nrm, a, l, p


VECTORS = [
    [0.3, -0.7],
    [1.0, 2.0, -3.0],
    [0.11, -0.52, 0.33, 0.77],
    [5e-4, -1.2e-3, 7e-4, 2.4e-3],
    [-2.5],
    [1.0, 1.0, 1.0, 1.0],
]


@pytest.mark.parametrize("v", VECTORS)
@pytest.mark.parametrize("s", [1, 2, 4, 7, 16])
def test_exact_enumeration_small_vectors(qo, v, s):
    """All 2^n rounding outcomes: probabilities sum to 1, the mean is v (Lemma
    3.1 (i)), the second moment matches the closed form in the lemma's proof,
    and the variance bound (ii) holds."""
    v32 = np.asarray(v, dtype=np.float32)
    n = v32.size
    nrm, a, l, p = probs64(v32, s)
    P = qo.Params(n=n, s=s, d=n, code=qo.CODE_SPARSE)
    eps = 1e-4
    mean = np.zeros(n)
    second = 0.0
    total = 0.0
    for up in itertools.product([0, 1], repeat=n):
        prob = 1.0
        u = np.zeros(n, dtype=np.float32)
        for i, b in enumerate(up):
            prob *= p[i] if b else 1.0 - p[i]
            # a draw just below p rounds up, just above rounds down
            u[i] = max(p[i] - eps, 0.0) if b else min(p[i] + eps, 1.0 - 2**-24)
        if prob == 0.0:
            continue
        # skip outcomes that the +-eps nudge cannot realise (p within eps of 0 or 1)
        if any((b and p[i] <= eps) or ((not b) and p[i] >= 1 - eps) for i, b in enumerate(up)):
            pytest.skip("threshold too close to 0/1 for the nudge")
        q = qo.quantize(P, v32, u=u)
        want = l + np.array(up)
        assert list(q["levels"]) == list(want.astype(int))
        dec = qo.decode(qo.encode(P, v32, u=u)).astype(np.float64)
        np.testing.assert_allclose(dec, nrm * np.sign(v32 + 0.0) * want / s, rtol=2e-7, atol=0)
        total += prob
        mean += prob * dec
        second += prob * float(((dec - v32.astype(np.float64)) ** 2).sum())
    assert abs(total - 1.0) < 1e-12
    np.testing.assert_allclose(mean, v32.astype(np.float64), rtol=1e-6, atol=1e-12)
    closed = nrm**2 / s**2 * float((p * (1 - p)).sum())  # proof of Lemma 3.1
    assert second == pytest.approx(closed, rel=1e-5, abs=1e-18)
    assert second <= min(n / s**2, math.sqrt(n) / s) * nrm**2 * (1 + 1e-9)


def test_round_up_threshold_is_p_to_24_bits(qo):
    """With u on the 2^-24 grid, the set of draws that round up is {u < p}: its
    measure differs from p = a s - l by less than 2^-24 (+ fp32 rounding of p)."""
    rng = np.random.default_rng(3)
    for s in (1, 4, 16, 256):
        v = rng.normal(size=8).astype(np.float32)
        nrm, a, l, p = probs64(v, s)
        P = qo.Params(n=8, s=s, d=8)
        for i in range(8):
            lo, hi = 0, 1 << 24  # smallest grid index that does NOT round up
            while lo < hi:
                mid = (lo + hi) // 2
                u = np.zeros(8, dtype=np.float32)
                u[i] = mid * 2.0**-24
                if qo.quantize(P, v, u=u)["levels"][i] == l[i] + 1:
                    lo = mid + 1
                else:
                    hi = mid
            assert abs(lo * 2.0**-24 - p[i]) <= 2.0**-24 + 4e-7 * s


def test_monte_carlo_unbiased_over_streams(qo):
    """E[Q_s(v)] = v with the Philox draws: mean over 10^5 streams within 3 sigma
    per coordinate (sigma from the exact per-coordinate variance), and the mean
    number of nonzeros equals its closed form and respects Lemma 3.1 (iii)."""
    rng = np.random.default_rng(0)
    n, s, T = 12, 4, 100_000
    v = (rng.normal(size=n) * 1e-3).astype(np.float32)
    nrm, a, l, p = probs64(v, s)
    acc = np.zeros(n)
    nnz = 0
    for t in range(T):
        P = qo.Params(n=n, s=s, d=n, seed=2024, stream_id=t)
        q = qo.quantize(P, v)
        acc += q["levels"]
        nnz += int(np.count_nonzero(q["levels"]))
    mean_level = acc / T
    sigma = np.sqrt(p * (1 - p) / T)
    assert np.all(np.abs(mean_level - a * s) <= 3 * sigma + 1e-7)
    exp_nnz = float(np.where(a * s >= 1, 1.0, a * s).sum())
    assert abs(nnz / T - exp_nnz) <= 4 * math.sqrt(n / T)
    assert exp_nnz <= s * (s + math.sqrt(n))


@pytest.mark.parametrize("s,d", [(1, 4096), (4, 512), (16, 512), (256, 512), (64, 4096)])
def test_variance_and_sparsity_bounds_closed_form(qo, s, d):
    """Lemma 3.1 (ii), (iii) from the oracle's own round-up probabilities."""
    rng = np.random.default_rng(s * 1000 + d)
    for dist in ("normal", "laplace", "outliers"):
        v = rng.normal(size=d)
        if dist == "laplace":
            v = rng.laplace(size=d)
        if dist == "outliers":
            v[rng.integers(0, d, 3)] *= 100
        v = (v * 1e-3).astype(np.float32)
        q = qo.quantize(qo.Params(n=d, s=s, d=d), v, want_draws=True)
        nrm, a, l, p = probs64(v, s)
        po = q["p"].astype(np.float64)
        decided = po >= 0
        np.testing.assert_allclose(po[decided], p[decided], atol=2e-6 * s + 1e-6)
        assert float(q["norms"][0]) == pytest.approx(nrm, rel=1e-7)
        var = nrm**2 / s**2 * float((po[decided] * (1 - po[decided])).sum())
        assert var <= min(d / s**2, math.sqrt(d) / s) * nrm**2
        exp_nnz = float(np.where(a * s >= 1, 1.0, a * s).sum())
        assert exp_nnz <= s * (s + math.sqrt(d))


def test_paper_worked_example_bucket512_4bits(qo):
    """Sec. 4: bucket 512 and 4 bits give a variance factor of sqrt(512)/2^4 ~= 1.41;
    the exact variance of the oracle's quantizer stays under it."""
    want = {r[0]: float(r[1]) for r in read_golden("paper_worked_values.txt")}
    d, s = 512, 2**4
    factor = min(d / s**2, math.sqrt(d) / s)
    assert round(factor, 2) == want["bucket512_4bit_variance_factor"]
    rng = np.random.default_rng(1)
    v = rng.normal(size=d).astype(np.float32)
    q = qo.quantize(qo.Params(n=d, s=s, d=d), v, want_draws=True)
    po = q["p"].astype(np.float64)
    nrm = float(q["norms"][0])
    assert nrm**2 / s**2 * float((po * (1 - po)).sum()) <= factor * nrm**2


def test_bucket_of_one_is_no_quantization(qo):
    """Sec. 4: d = 1 is vanilla SGD -- every value comes back exactly."""
    rng = np.random.default_rng(2)
    v = np.concatenate([rng.normal(size=50), [0.0, -0.0, 1e-30, -3e30]]).astype(np.float32)
    for s in (1, 4, 255):
        for code in (qo.CODE_SPARSE, qo.CODE_DENSE, qo.CODE_FIXED):
            P = qo.Params(n=v.size, s=s, d=1, code=code)
            q = qo.quantize(P, v)
            assert np.all(q["levels"][v != 0] == s)
            dec = qo.decode(qo.encode(P, v))
            # scale*s: fl(|v|/s)*s can be an ulp off for s not a power of two
            np.testing.assert_allclose(dec, v, rtol=1.2e-7 if s & (s - 1) else 0, atol=0)


def test_one_hot_zero_and_signs(qo):
    v = np.zeros(512, dtype=np.float32)
    P = qo.Params(n=512, s=4, d=512)
    q = qo.quantize(P, v)
    assert not q["levels"].any() and q["norms"][0] == 0  # Q_s(0) = 0
    assert not qo.decode(qo.encode(P, v)).any()
    v[77] = -0.25
    q = qo.quantize(P, v)
    assert q["levels"][77] == 4 and q["neg"][77] == 1 and np.count_nonzero(q["levels"]) == 1
    assert qo.decode(qo.encode(P, v))[77] == np.float32(-0.25)
    w = np.array([0.0, -0.0, 1.0, -1.0], dtype=np.float32)
    assert list(qo.quantize(qo.Params(n=4, s=2, d=4), w)["neg"]) == [0, 0, 0, 1]  # sgn(0) = +1


def test_buckets_are_independent_and_tail_is_short(qo):
    """Sec. 4: each run of d values is quantized on its own scale; the last bucket
    may be shorter."""
    rng = np.random.default_rng(4)
    n, d, s = 1000, 128, 8
    v = (rng.normal(size=n) * np.repeat(10.0 ** rng.integers(-4, 2, size=8), 128)[:n]).astype(np.float32)
    P = qo.Params(n=n, s=s, d=d, seed=5)
    q = qo.quantize(P, v, want_draws=True)
    assert qo.num_buckets(P) == 8 and q["norms"].size == 8
    for b in range(8):
        seg = v[b * d:(b + 1) * d].astype(np.float64)
        assert float(q["norms"][b]) == pytest.approx(math.sqrt((seg * seg).sum()), rel=1e-7)
        # the same bucket quantized alone, with its own draws, gives the same levels
        alone = qo.quantize(qo.Params(n=seg.size, s=s, d=seg.size), seg.astype(np.float32),
                            u=q["u"][b * d:(b + 1) * d])
        assert np.array_equal(alone["levels"], q["levels"][b * d:(b + 1) * d])
    assert np.all(q["levels"] <= s)


def test_max_scaling_variant(qo):
    """Sec. 4, second variation: scale by max |v_i|; the largest entry sits on level s
    and the quantizer stays unbiased (levels' mean is a s with a = |v_i| / max)."""
    rng = np.random.default_rng(6)
    v = rng.normal(size=256).astype(np.float32)
    P = qo.Params(n=256, s=7, d=256, norm=qo.NORM_MAX, seed=1)
    q = qo.quantize(P, v, want_draws=True)
    assert q["norms"][0] == np.abs(v).max()
    assert q["levels"][np.argmax(np.abs(v))] == 7
    a = np.abs(v).astype(np.float64) / float(np.abs(v).max())
    po = q["p"].astype(np.float64)
    dec = po >= 0
    np.testing.assert_allclose(np.floor(a * 7)[dec] + po[dec], (a * 7)[dec], atol=2e-5)
