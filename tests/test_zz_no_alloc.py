"""The entry point that allocates nothing (qsgd_encode_static: scratch inside the library
image instead of a caller's workspace) against qsgd_encode, through the C ABI: same
message, bit for bit, on two calls in a row, the second with a smaller input; requests
beyond the built-in scratch are refused."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1610_02132_amd as q  # noqa: E402
from oracle import qsgd_oracle as qo  # noqa: E402


def gradient(n, seed, scale=1e-3):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, scale, generator=g)


def both(P, g):
    cap = q.qsgd_max_encoded_bytes(P)
    ws = torch.zeros(q.qsgd_workspace_bytes(P, 1) // 4, dtype=torch.int32, device="cuda")
    a = torch.full((cap // 4 + 16,), -1, dtype=torch.int32, device="cuda")
    b = torch.full((cap // 4 + 16,), -1, dtype=torch.int32, device="cuda")
    q.qsgd_encode(P, g, a[: cap // 4], ws)
    q.qsgd_encode_static(P, g, b[: cap // 4])
    sa, ta = q.qsgd_message_status(a)
    sb, tb = q.qsgd_message_status(b)
    assert sa == 0 and sb == 0 and ta == tb
    wa = a.cpu().numpy().view(np.uint32)
    wb = b.cpu().numpy().view(np.uint32)
    assert np.array_equal(wa[: ta // 4], wb[: tb // 4]), "messages differ"
    assert np.all(wb[cap // 4:] == 0xFFFFFFFF), "write past the message capacity"
    return wb[: tb // 4].copy()


CASES = [  # (n of the first call, n of the second, s, d, code)
    (512 * 3000 + 100, 512 * 100 + 52, 4, 512, q.CODE_SPARSE),
    (8192 * 40 + 2560, 8192 * 3, 4, 8192, q.CODE_SPARSE),
    (256 * 900 + 7, 256 * 30, 7, 256, q.CODE_DENSE),
    (512 * 2000 + 448, 512 * 64, 256, 512, q.CODE_FIXED),
    (700_000, 50_000, 1, 10**9, q.CODE_SPARSE),            # one long bucket: the general path
]


@pytest.mark.parametrize("n1,n2,s,d,code", CASES)
def test_static_scratch_encode_equals_encode(n1, n2, s, d, code):
    for rep, n in enumerate((n1, n2, n1)):
        P = q.Params(n=n, s=s, d=d, code=code, seed=17, stream_id=3, iteration=rep)
        g = gradient(n, 40 + rep)
        words = both(P, g)
        want = qo.encode(qo.Params(n=n, s=s, d=d, code=code, seed=17, stream_id=3, iteration=rep),
                         g.cpu().numpy())
        assert np.array_equal(words, want), "message differs from the oracle"


def test_static_scratch_limit_is_enforced():
    assert q.qsgd_static_scratch_bytes() == 64 << 20
    big = q.Params(n=1_000_000_000, s=4, d=8192)
    assert q.qsgd_workspace_bytes(big, 1) > q.qsgd_static_scratch_bytes()
    g = torch.zeros(16, dtype=torch.float32, device="cuda")
    msg = torch.zeros(1024, dtype=torch.int32, device="cuda")
    # refused on the host before any buffer is looked at, nothing queued (the raw C call: the
    # binding would refuse the short gradient first)
    import ctypes
    from paper_1610_02132_amd import binding
    cp = big.c()
    rc = binding._load().qsgd_encode_static(ctypes.byref(cp), g.data_ptr(), msg.data_ptr(),
                                            msg.numel() * 4, None)
    assert rc == -6 and "scratch" in q.qsgd_strerror(rc)
    torch.cuda.synchronize()
    assert not msg.any()
    with pytest.raises(q.QsgdError):
        q.qsgd_encode_static(q.Params(n=16, s=0, d=4), g, msg)
