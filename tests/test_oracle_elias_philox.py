"""Pins for the oracle's scalar parts: the recursive Elias code (App. A.2,
Definition and Lemma) and the Philox-4x32-10 generator behind the draws."""
import math
import random

import numpy as np

from conftest import read_golden


# -- an independent reading of the Definition, written on strings -------------
def py_omega(k: int) -> str:
    code = "0"
    while k > 1:
        b = bin(k)[2:]
        code = b + code
        k = len(b) - 1
    return code


def py_omega_decode(bits: str):
    n, i = 1, 0
    while True:
        if bits[i] == "0":
            return n, i + 1
        n, i = int(bits[i:i + n + 1], 2), i + n + 1


def test_textbook_codewords(qo):
    for k, word in read_golden("elias_omega_codewords.txt"):
        assert qo.omega_string(int(k)) == word
        assert qo.omega_len(int(k)) == len(word)
        assert qo.omega_decode_string(word) == (int(k), len(word))


def test_length_of_one_is_one(qo):
    want = {r[0]: float(r[1]) for r in read_golden("paper_worked_values.txt")}
    assert qo.omega_len(1) == int(want["elias_len_of_one"])


def test_round_trip_all_up_to_2_pow_20(qo):
    assert qo.omega_roundtrip_failures(1, 1 << 20) == 0


def test_round_trip_large_values(qo):
    rnd = random.Random(5)
    ks = [2**32 - 1, 2**32, 2**40 + 12345, 13_000_000, 2**63] + \
         [rnd.getrandbits(rnd.randint(21, 63)) | 1 for _ in range(2000)]
    for k in ks:
        w = qo.omega_string(k)
        assert w == py_omega(k)
        assert qo.omega_decode_string(w) == (k, len(w))
        assert qo.omega_decode_string(w + "1101") == (k, len(w))  # self-delimiting


def test_matches_independent_definition(qo):
    rnd = random.Random(7)
    for k in list(range(1, 5000)) + [rnd.randrange(1, 1 << 20) for _ in range(5000)]:
        w = qo.omega_string(k)
        assert w == py_omega(k)
        assert py_omega_decode(w) == (k, len(w))


def test_length_formula(qo):
    # |Elias(k)| = 1 + (floor(log k)+1) + (floor(log floor(log k))+1) + ... (Lemma, item 1)
    for k in list(range(1, 70000, 7)) + [2**j for j in range(1, 33)] + [2**j - 1 for j in range(2, 33)]:
        n, total = k, 1
        while n > 1:
            total += n.bit_length()
            n = n.bit_length() - 1
        assert qo.omega_len(k) == total
        # Lemma item 1 with real logarithms: every group is at most log(.) + 1 bits
        t, bound = k, 1.0
        while t > 1:
            bound += math.log2(t) + 1
            t = int(math.floor(math.log2(t)))
        assert total <= bound + 1e-9


def test_prefix_free_and_kraft(qo):
    words = [qo.omega_string(k) for k in range(1, 1 << 12)]
    s = sorted(words)
    for a, b in zip(s, s[1:]):
        assert not b.startswith(a)
    assert sum(2.0 ** -len(w) for w in words) <= 1.0


def test_truncated_code_is_rejected(qo):
    for k in (2, 9, 100, 70000):
        w = qo.omega_string(k)
        for cut in range(len(w)):
            assert qo.omega_decode_string(w[:cut])[1] == 0


def test_lengths_are_monotone(qo):
    prev = 0
    for k in range(1, 1 << 16):
        cur = qo.omega_len(k)
        assert cur >= prev
        prev = cur


# -- Philox ---------------------------------------------------------------------
def py_philox4x32_10(ctr, key):
    c, k = list(ctr), list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers(qo):
    for row in read_golden("philox4x32_10_kat.txt"):
        v = [int(x, 16) for x in row]
        assert list(qo.philox4x32_10(v[0:4], v[4:6])) == v[6:10]
        assert py_philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_philox_against_big_integer_version(qo):
    rnd = random.Random(11)
    for _ in range(3000):
        ctr = [rnd.getrandbits(32) for _ in range(4)]
        key = [rnd.getrandbits(32) for _ in range(2)]
        assert list(qo.philox4x32_10(ctr, key)) == py_philox4x32_10(ctr, key)


def test_draw_mapping(qo):
    """Element i uses word i%4 of the block with counter (i/4, stream, iteration), key=seed."""
    p = qo.Params(n=1 << 40, s=4, d=512, seed=0x0123456789ABCDEF, stream_id=7, iteration=3)
    for idx in [0, 1, 2, 3, 4, 5, 1023, 2**33 + 6, 2**34 + 3]:
        q = idx >> 2
        out = py_philox4x32_10([q & 0xFFFFFFFF, q >> 32, 7, 3],
                               [0x89ABCDEF, 0x01234567])
        u = (out[idx & 3] >> 8) / 2.0**24
        assert qo.draw(p, idx) == np.float32(u)
        assert 0.0 <= qo.draw(p, idx) < 1.0


def test_draws_look_uniform(qo):
    p = qo.Params(n=1 << 20, s=4, d=512, seed=99)
    u = np.array([qo.draw(p, i) for i in range(40000)])
    assert abs(u.mean() - 0.5) < 4 * (1 / math.sqrt(12 * u.size))
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    exp = u.size / 16
    assert ((hist - exp) ** 2 / exp).sum() < 45  # chi^2, 15 dof, far tail
