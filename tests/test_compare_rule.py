"""The GPU-vs-oracle comparison rule itself, exercised on the CPU: messages that differ
from the oracle's in a planted way (made with the oracle's own encoder from altered
draws, or patched) must be classified as the rule says: near-ties counted, anything
else refused."""
import numpy as np
import pytest

from oracle import compare


def _case(qo, code, s, n=400_000, d=512):
    rng = np.random.default_rng(21)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    p = qo.Params(n=n, s=s, d=d, code=code, seed=6, stream_id=1)
    qz = qo.quantize(p, g, want_draws=True)
    return p, g, qz


@pytest.mark.parametrize("code,s", [(0, 4), (1, 5), (2, 16)])
def test_identical_and_near_tie_messages(qo, code, s):
    p, g, qz = _case(qo, code, s)
    ref = qo.encode(p, g)
    r = compare.compare_encode(p, g, ref)
    assert r["identical"] and r["near_ties"] == 0
    compare.structure_check(ref, p)
    # elements whose draw lies within 1e-5 of the threshold: flip exactly those
    u, pr = qz["u"].astype(np.float64), qz["p"].astype(np.float64)
    near = np.flatnonzero((pr > 0) & (np.abs(u - pr) <= 0.9e-5))
    assert near.size >= 3
    u2 = qz["u"].copy()
    u2[near] = np.where(u[near] < pr[near], pr[near] + 1e-6, pr[near] - 1e-6).astype(np.float32)
    fake = qo.encode(p, g, u=u2)
    assert not np.array_equal(fake, ref)
    r = compare.compare_encode(p, g, fake)
    assert not r["identical"] and r["near_ties"] == near.size and r["norm_mismatches"] == 0
    # one flip away from a threshold is refused
    far = np.flatnonzero((pr > 0.2) & (pr < 0.8) & (np.abs(u - pr) > 0.05))[0]
    u3 = qz["u"].copy()
    u3[far] = np.float32(pr[far] + (0.01 if u[far] < pr[far] else -0.01))
    with pytest.raises(AssertionError):
        compare.compare_encode(p, g, qo.encode(p, g, u=u3))


def test_scale_one_rounding_apart_is_counted_two_are_refused(qo):
    p, g, _ = _case(qo, 0, 4, n=20_000)
    ref = qo.encode(p, g)
    pay = qo.payload_offset_words(ref)
    off, _ = qo.bucket_extent(ref, 7)
    one = ref.copy()
    one[pay + off] += 1                      # the scale word of bucket 7, one ulp up
    r = compare.compare_encode(p, g, one)
    assert r["norm_mismatches"] == 1 and r["near_ties"] == 0
    two = ref.copy()
    two[pay + off] += 2
    with pytest.raises(AssertionError):
        compare.compare_encode(p, g, two)


def test_damaged_strings_and_tables_are_refused(qo):
    p, g, qz = _case(qo, 0, 4, n=20_000)
    ref = qo.encode(p, g)
    pay = qo.payload_offset_words(ref)
    # a sign bit flipped inside a string: levels agree, signs do not
    off, cnt = qo.bucket_extent(ref, 3)
    bad = ref.copy()
    nz = np.flatnonzero(qz["levels"][3 * 512:4 * 512])
    assert nz.size
    tup = None
    for bit in range(32, cnt * 32 - 2):      # find a bit whose flip only changes a sign
        t = ref.copy()
        t[pay + off + bit // 32] ^= np.uint32(1 << (31 - bit % 32))
        try:
            tup = qo.decode_tuple(t)
        except qo.OracleError:
            continue
        if np.array_equal(tup["levels"], qz["levels"]):
            bad = t
            break
    assert tup is not None and not np.array_equal(bad, ref)
    with pytest.raises(AssertionError):
        compare.compare_encode(p, g, bad)
    # a table entry moved: the structure check and the comparison both notice
    t2 = ref.copy()
    t2[16 + 5] += 1
    with pytest.raises((AssertionError, qo.OracleError)):
        compare.compare_encode(p, g, t2)
    t3 = ref.copy()
    t3[16 + 5] = t3[16 + 4]
    with pytest.raises(AssertionError):
        compare.structure_check(t3, p)


def test_run_of_buckets_from_a_longer_message(qo):
    """compare_bucket_run: buckets [b0, b1) cut out of a whole message."""
    p, g, qz = _case(qo, 0, 4)
    whole = qo.encode(p, g)
    pay = qo.payload_offset_words(whole)
    b0, b1, d = 10, 760, 512
    tab = whole[16 + b0:16 + b1 + 1]
    strings = whole[pay + int(tab[0]):pay + int(tab[-1])]
    pr = qo.Params(n=(b1 - b0) * d, s=4, d=d, code=0, seed=6, stream_id=1)
    r = compare.compare_bucket_run(pr, g[b0 * d:b1 * d], b0 * d, tab, strings)
    assert r["identical"]
    # the same run with a near-tie flipped
    u, prob = qz["u"].astype(np.float64), qz["p"].astype(np.float64)
    sl = slice(b0 * d, b1 * d)
    cand = np.flatnonzero((prob[sl] > 0) & (np.abs(u[sl] - prob[sl]) <= 0.9e-5)) + b0 * d
    assert cand.size
    u2 = qz["u"].copy()
    i = cand[0]
    u2[i] = np.float32(prob[i] + (1e-6 if u[i] < prob[i] else -1e-6))
    fake = qo.encode(p, g, u=u2)
    fpay = qo.payload_offset_words(fake)
    ftab = fake[16 + b0:16 + b1 + 1]
    r = compare.compare_bucket_run(pr, g[sl], b0 * d, ftab, fake[fpay + int(ftab[0]):fpay + int(ftab[-1])])
    assert not r["identical"] and r["near_ties"] == 1


@pytest.mark.parametrize("code,s", [(0, 4), (2, 16)])
def test_tensor_aware_message_with_a_planted_near_tie(qo, code, s):
    """compare_layout: a tensor-aware message put together here from per-tensor messages
    (each tensor is a vector of its own, drawn at its arena positions), one of them with
    its near-tie elements flipped."""
    d, bypass = 512, 600
    tensors = [(0, 37), (40, 300_000), (300_040, 9), (300_052, 777), (300_832, 2049)]
    n = 300_832 + 2049
    rng = np.random.default_rng(2)
    arena = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    p = qo.Params(n=n, s=s, d=d, code=code, seed=13, stream_id=2)
    ref = qo.encode_layout(p, tensors, bypass, arena)
    assert compare.compare_layout(p, tensors, bypass, arena, ref)["identical"]
    nb, raw = qo.layout_counts(p, tensors, bypass)
    full = (qo.max_encoded_bytes(qo.Params(n=d, s=s, d=d, code=code)) - 64) // 4
    strings, table, planted = [], [0], 0
    for off, size in tensors:
        if size < bypass:
            continue
        pt = qo.Params(n=size, s=s, d=d, code=code, seed=13, stream_id=2)
        g_t = arena[off:off + size]
        qz = qo.quantize(pt, g_t, want_draws=True, index_offset=off)
        u, pr = qz["u"].astype(np.float64), qz["p"].astype(np.float64)
        near = np.flatnonzero((pr > 0) & (np.abs(u - pr) <= 0.9e-5))
        u2 = qz["u"].copy()
        u2[near] = np.where(u[near] < pr[near], pr[near] + 1e-6, pr[near] - 1e-6).astype(np.float32)
        planted += near.size
        m = qo.encode(pt, g_t, u=u2)
        pay = qo.payload_offset_words(m)
        body = m[pay:]
        nbt = (size + d - 1) // d
        if code == 2:   # every bucket owns a full slot
            body = np.concatenate([body, np.zeros(nbt * full - body.size, dtype=np.uint32)])
        else:
            table += [table[-1] + int(v) for v in m[17:17 + nbt]]
        strings.append(body)
    assert planted >= 2
    strings = np.concatenate(strings)
    tw = 0 if code == 2 else (nb + 1 + 3) // 4 * 4
    tabw = np.zeros(tw, dtype=np.uint32)
    tabw[:len(table) if tw else 0] = table if tw else []
    fake = np.concatenate([ref[:16], tabw, strings, ref[ref.size - raw:]])
    fake[12] = strings.size + raw
    r = compare.compare_layout(p, tensors, bypass, arena, fake)
    assert not r["identical"] and r["near_ties"] == planted
    # a raw value off by one bit is refused
    bad = fake.copy()
    bad[-1] ^= 1
    with pytest.raises(AssertionError):
        compare.compare_layout(p, tensors, bypass, arena, bad)
