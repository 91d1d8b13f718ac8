"""Pins for the oracle's tensor-aware messages (Sec. 5, "Protocol": small matrices
travel unquantized, buckets are laid out per matrix).

What pins them: a message of one large tensor must carry exactly the strings of
the flat encoder (which has its own pins); every large tensor must decode to
what the flat encoder gives for that tensor alone with the draws of its arena
positions; small tensors must come back bit for bit; positions outside every
tensor must not be touched; the step must equal the plain definition computed
with numpy from the per-message decodes.
"""
import numpy as np
import pytest


def _arena(tensors, n, seed=0):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n).astype(np.float32) * 1e-2
    return a


def _tensors(sizes, align=4):
    out, off = [], 0
    for sz in sizes:
        out.append((off, sz))
        off += (sz + align - 1) // align * align
    return out, off


@pytest.mark.parametrize("code", [0, 1, 2])
def test_single_large_tensor_equals_flat_message(qo, code):
    n, d = 5000, 512
    g = _arena(None, n, 1)
    p = qo.Params(n=n, s=16, d=d, code=code, seed=7, stream_id=3)
    flat = qo.encode(p, g)
    lay = qo.encode_layout(p, [(0, n)], 100, g)
    assert lay[1] == 2 and flat[1] == 1           # header version
    if code == 2:
        # fixed width keeps one full-size slot per bucket, also for the short last bucket
        # of a tensor (the flat message ends with the short string): same words, zero padded
        assert lay.size >= flat.size and not lay[flat.size:].any()
        assert int(lay[12]) == int(flat[12]) + (lay.size - flat.size)
        lay = lay[:flat.size].copy()
        lay[12] = flat[12]
    assert np.array_equal(lay[2:], flat[2:]) and lay[0] == flat[0]
    lay = qo.encode_layout(p, [(0, n)], 100, g)
    assert np.array_equal(qo.decode_layout([(0, n)], 100, lay, n), qo.decode(flat))


@pytest.mark.parametrize("code", [0, 1, 2])
def test_each_tensor_is_quantized_alone_with_its_arena_draws(qo, code):
    sizes = [37, 1300, 9, 512, 2050, 700]
    tensors, n = _tensors(sizes)
    g = _arena(tensors, n, 2)
    d, bypass = 512, 600
    p = qo.Params(n=n, s=7, d=d, code=code, seed=11, stream_id=1, iteration=5)
    msg = qo.encode_layout(p, tensors, bypass, g)
    nb, raw = qo.layout_counts(p, tensors, bypass)
    assert raw == 37 + 9 + 512 and nb == 3 + 5 + 2
    out = qo.decode_layout(tensors, bypass, msg, n)
    touched = np.zeros(n, dtype=bool)
    for off, sz in tensors:
        touched[off:off + sz] = True
        if sz < bypass:   # raw passthrough, bit for bit
            assert np.array_equal(out[off:off + sz].view(np.uint32), g[off:off + sz].view(np.uint32))
        else:             # the flat encoder on this tensor alone, draws of positions off..off+sz
            ps = qo.Params(n=sz, s=7, d=d, code=code, seed=11, stream_id=1, iteration=5)
            want = qo.decode(qo.encode_slice(ps, g[off:off + sz], off))
            assert np.array_equal(out[off:off + sz].view(np.uint32), want.view(np.uint32))
    assert not out[~touched].any()           # padding between tensors is left alone


def test_size_accounting_and_capacity(qo):
    sizes = [100, 4096, 3, 5000]
    tensors, n = _tensors(sizes)
    g = _arena(tensors, n, 3)
    p = qo.Params(n=n, s=4, d=1024, code=0)
    msg = qo.encode_layout(p, tensors, 1000, g)
    nb, raw = qo.layout_counts(p, tensors, 1000)
    assert (nb, raw) == (4 + 5, 103)
    table_words = (nb + 1 + 3) // 4 * 4
    strings = int(msg[16 + nb])
    assert msg.size == 16 + table_words + strings + raw
    assert int(msg[12]) == strings + raw      # payload words in the header
    with pytest.raises(qo.OracleError):
        qo.encode_layout(p, tensors, 1000, g, capacity=4 * (msg.size - 1))
    # overlapping or out-of-arena tensors are rejected
    with pytest.raises(qo.OracleError):
        qo.layout_counts(p, [(0, 10), (5, 10)], 1000)
    with pytest.raises(qo.OracleError):
        qo.layout_counts(p, [(n - 4, 10)], 1000)


def test_step_is_the_plain_definition(qo):
    sizes = [50, 2000, 640, 7]
    tensors, n = _tensors(sizes)
    K, eta = 5, 0.25
    p0 = dict(n=n, s=3, d=256, code=0, seed=5)
    msgs, decs = [], []
    for k in range(K):
        g = _arena(tensors, n, 10 + k)
        m = qo.encode_layout(qo.Params(stream_id=k, **p0), tensors, 100, g)
        msgs.append(m)
        decs.append(qo.decode_layout(tensors, 100, m, n))
    x0 = np.random.default_rng(99).uniform(-1, 1, n).astype(np.float32)
    x1 = qo.sgd_step_layout(tensors, 100, msgs, eta, x0)
    acc = qo.decode_accumulate_layout(tensors, 100, msgs, x0)
    s = np.zeros(n, dtype=np.float32)
    for k in range(K):
        s = (s + decs[k]).astype(np.float32)
    c = np.float32(eta) / np.float32(K)
    want = (x0.astype(np.float64) - np.float64(c) * s.astype(np.float64))   # one rounding: fma
    mask = np.zeros(n, dtype=bool)
    for off, sz in tensors:
        mask[off:off + sz] = True
    assert np.array_equal(x1[mask], want.astype(np.float32)[mask])
    assert np.array_equal(acc[mask], (x0 + s)[mask])
    assert np.array_equal(x1[~mask], x0[~mask]) and np.array_equal(acc[~mask], x0[~mask])
