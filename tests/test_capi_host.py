"""CPU-side checks of the C ABI: the library loads, exports every declared
symbol, and its host-only entry points agree with the oracle's container."""
import ctypes
import os
import re

import numpy as np
import pytest

from conftest import ROOT

LIB = os.path.join(ROOT, "paper_1610_02132_amd", "libqsgd.so")
pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libqsgd.so not built")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "qsgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qsgd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    names = declared_functions()
    assert len(names) >= 13
    for name in names:
        assert hasattr(lib, name), name
    from paper_1610_02132_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_sizes_agree_with_oracle(qo):
    import paper_1610_02132_amd as q
    for n in (0, 1, 5, 511, 512, 513, 4096, 100_000, 13_000_000):
        for s in (1, 4, 16, 256, 65535):
            for d in (1, 4, 512, 8192, 10**10):
                for code in (0, 1, 2):
                    for norm in (0, 1):
                        a = q.qsgd_max_encoded_bytes(q.Params(n=n, s=s, d=d, code=code, norm=norm))
                        b = qo.max_encoded_bytes(qo.Params(n=n, s=s, d=d, code=code, norm=norm))
                        assert a == b, (n, s, d, code, norm)
    assert q.qsgd_max_encoded_bytes(q.Params(n=10, s=0, d=4)) == 0
    assert q.qsgd_workspace_bytes(q.Params(n=1 << 20, s=4, d=512), 2) >= 256


def test_message_info_reads_oracle_headers(qo):
    import paper_1610_02132_amd as q
    g = np.random.default_rng(0).normal(size=3000).astype(np.float32)
    for code in (0, 1, 2):
        msg = qo.encode(qo.Params(n=3000, s=16, d=512, code=code, stream_id=4, iteration=2), g)
        rc, p, total = q.qsgd_message_info(msg.tobytes()[:64])
        assert rc == 0 and total == msg.nbytes
        assert (p.n, p.s, p.d, p.code, p.stream_id, p.iteration) == (3000, 16, 512, code, 4, 2)
    bad = msg.copy(); bad[0] = 0
    assert q.qsgd_message_info(bad.tobytes()[:64])[0] == -3
    bad = msg.copy(); bad[14] = np.uint32(-2 & 0xFFFFFFFF)
    assert q.qsgd_message_info(bad.tobytes()[:64])[0] == -2


def test_error_strings():
    import paper_1610_02132_amd as q
    assert q.qsgd_version() >= 100
    texts = {q.qsgd_strerror(e) for e in (0, -1, -2, -3, -4, -5)}
    assert len(texts) == 6


def test_encode_workspace_sized_from_the_message_capacity():
    """Host arithmetic only: for the stress shape (n = 1e9, s = 4, d = 8192) a message buffer
    of 28 MB needs a fraction of the worst-case staging, and never more than it."""
    import paper_1610_02132_amd as q
    P = q.Params(n=1_000_000_000, s=4, d=8192)
    worst = q.qsgd_workspace_bytes(P, 1)
    assert worst > 1_000_000_000
    small = q.qsgd_encode_workspace_bytes(P, 28_000_000)
    assert 0 < small <= worst // 4
    assert q.qsgd_encode_workspace_bytes(P, q.qsgd_max_encoded_bytes(P)) == worst
    for P2 in (q.Params(n=13_000_000, s=1, d=13_000_000), q.Params(n=10**6, s=256, d=512, code=q.CODE_FIXED)):
        assert q.qsgd_encode_workspace_bytes(P2, 1 << 20) == q.qsgd_workspace_bytes(P2, 1)
