"""Pins for the oracle calls that work on a PART of a vector (the references of the
full-size GPU checks): encode of a slice with the draws of the whole vector's
positions, the step on a run of buckets (Sec. 4: buckets are quantized and coded
independently), the entry list of long buckets as pure metadata, and the oracle under
the address and undefined-behaviour sanitizers."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from test_oracle_codes import read_omega, words_to_bits
from test_oracle_elias_philox import py_philox4x32_10

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gradient(n, seed):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal(n).astype(np.float32) * 1e-3
    g[rng.random(n) < 0.01] *= 100
    return g


CODES = [(0, 4), (1, 5), (2, 16)]   # (code, s)


@pytest.mark.parametrize("code,s", CODES)
@pytest.mark.parametrize("n,d", [(10_000, 512), (40_000, 8192), (3000, 100)])
def test_slice_reproduces_the_buckets_of_the_whole_message(qo, code, s, n, d):
    """Buckets i..j of Encode(whole) are word for word the message of the slice that
    starts at position i*d, encoded with the draws of its positions in the whole vector."""
    g = _gradient(n, 1)
    p = qo.Params(n=n, s=s, d=d, code=code, seed=11, stream_id=2, iteration=9)
    whole = qo.encode(p, g)
    nb = qo.num_buckets(p)
    pay = qo.payload_offset_words(whole)
    for b0, b1 in [(0, nb), (1, nb), (2, 3), (nb - 1, nb), (nb // 2, nb - 1)]:
        lo, hi = b0 * d, min(b1 * d, n)
        ps = qo.Params(n=hi - lo, s=s, d=d, code=code, seed=11, stream_id=2, iteration=9)
        part = qo.encode_slice(ps, g[lo:hi], lo)
        ppay = qo.payload_offset_words(part)
        o0, _ = qo.bucket_extent(whole, b0)
        o1, c1 = qo.bucket_extent(whole, b1 - 1)
        assert np.array_equal(part[ppay:], whole[pay + o0: pay + o1 + c1])
        if code != 2:   # the slice's table is the whole one's, rebased
            assert np.array_equal(part[16:16 + (b1 - b0) + 1].astype(np.int64),
                                  whole[16 + b0:16 + b1 + 1].astype(np.int64) - o0)
        # a slice that is NOT drawn at its own positions differs (the offset matters)
        if hi - lo >= 64 and lo > 0:
            assert not np.array_equal(qo.encode_slice(ps, g[lo:hi], 0)[ppay:], part[ppay:])


@pytest.mark.parametrize("code,s", CODES)
def test_slice_far_into_a_long_vector_uses_the_high_counter_word(qo, code, s):
    """Positions beyond 2^34 put a nonzero word into the block counter (i / 4 >= 2^32).
    The draws are recomputed here with the big-integer generator and handed to the
    encoder that takes its draws from the caller."""
    n, d = 2048 + 300, 512
    g = _gradient(n, 2)
    seed = 0x0123456789ABCDEF
    for offset in [2**34 - 1024, 2**34 + 4096, 3 * 2**34 + 512 * 7]:
        ps = qo.Params(n=n, s=s, d=d, code=code, seed=seed, stream_id=5, iteration=1)
        part = qo.encode_slice(ps, g, offset)
        u = np.empty(n, dtype=np.float32)
        for i in range(n):
            idx = offset + i
            if i == 0 or idx % 4 == 0:
                q = idx >> 2
                block = py_philox4x32_10([q & 0xFFFFFFFF, q >> 32, 5, 1],
                                         [seed & 0xFFFFFFFF, seed >> 32])
            u[i] = np.float32((block[idx & 3] >> 8) / 2.0**24)
        assert np.array_equal(qo.encode(ps, g, u=u), part)


@pytest.mark.parametrize("code,s", CODES)
@pytest.mark.parametrize("n,d,K", [(10_000, 512, 3), (40_000, 8192, 16), (3000, 100, 2)])
def test_step_on_a_run_of_buckets_is_the_whole_step_restricted(qo, code, s, n, d, K):
    msgs = [qo.encode(qo.Params(n=n, s=s, d=d, code=code, seed=4, stream_id=k), _gradient(n, 10 + k))
            for k in range(K)]
    x0 = np.random.default_rng(3).uniform(-1, 1, n).astype(np.float32)
    want = qo.sgd_step(msgs, 0.1, x0)
    nb = (n + d - 1) // d
    prep = qo.prepare_messages(msgs)
    got = x0.copy()
    for b0 in range(0, nb, 3):
        cnt = min(3, nb - b0)
        lo, hi = b0 * d, min((b0 + cnt) * d, n)
        got[lo:hi] = qo.sgd_step_buckets(prep, 0.1, got[lo:hi], b0, cnt)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(qo.sgd_step_buckets(msgs, 0.1, x0[:0], nb, 0), x0[:0])
    with pytest.raises(qo.OracleError):
        qo.sgd_step_buckets(msgs, 0.1, x0[:d], nb, 1)


@pytest.mark.parametrize("s,density,n", [(1, 0.01, 2_000_000), (3, 0.2, 60_000)])
def test_entry_list_of_a_long_bucket_is_metadata(qo, s, density, n):
    """A reader that knows nothing of the entry list (it reads the Code_s string from its
    first bit to the stop mark, as the decoder of Sec. 3.1 does) gets the tuple that the
    oracle's reader returns: the list behind the string carries no part of the code."""
    rng = np.random.default_rng(8)
    g = (rng.standard_normal(n) * ((rng.random(n) < density) * 50.0 + 0.01)).astype(np.float32)
    p = qo.Params(n=n, s=s, d=n, code=0, seed=3)
    msg = qo.encode(p, g)
    tup = qo.decode_tuple(msg)
    words = qo.bucket_words(msg, 0)
    entries = int(words[-1])
    assert entries >= 2
    string = words[: len(words) - 2 * entries - 1]
    bits = words_to_bits(string)
    end = len(bits) - 1 - bits[::-1].index("1")       # the stop mark: the last 1 bit
    assert np.float32(tup["norms"][0]).view(np.uint32) == int(bits[:32], 2)
    lev = np.zeros(n, dtype=np.uint32)
    neg = np.zeros(n, dtype=np.uint8)
    i, pos = 32, 0
    while i < end:
        gap, i = read_omega(bits, i)
        sign = bits[i] == "1"
        level, i = read_omega(bits, i + 1)
        pos += gap
        lev[pos - 1], neg[pos - 1] = level, sign
    assert i == end
    assert np.array_equal(lev, tup["levels"])
    nz = lev != 0
    assert np.array_equal(neg[nz], tup["neg"][nz])


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """Builds the oracle with -fsanitize=address,undefined and runs its driver: every code,
    both scalings, ragged and long buckets, slices, bucket ranges, tensor-aware messages,
    with buffers of exactly the advertised sizes."""
    exe = str(tmp_path / "sanitize_check")
    src = [os.path.join(ROOT, "oracle", f) for f in ("sanitize_check.c", "qsgd_oracle.c")]
    subprocess.check_call(["gcc", "-g", "-O1", "-std=c99", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-ffp-contract=off",
                           *src, "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "sanitize_check: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
