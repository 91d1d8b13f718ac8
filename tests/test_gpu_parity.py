"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Bar: levels, signs and packed words bit-exact (counted
near-ties aside), fp32 results within 1e-6 relative."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1610_02132_amd as q  # noqa: E402
from paper_1610_02132_amd import workloads as W  # noqa: E402
from oracle import qsgd_oracle as qo  # noqa: E402
from gpu_harness import Device, check_step, compare_encode, oracle_params  # noqa: E402


def run_case(w: W.Workload, norm=q.NORM_L2, code=None, expect_exact_step=True):
    code = w.code if code is None else code
    msgs_dev, msgs_host, near = [], [], 0
    for k in range(w.K):
        P = q.Params(n=w.n, s=w.s, d=w.d, code=code, norm=norm, seed=w.seed, stream_id=k,
                     iteration=3)
        g = W.gradient(w, k, device="cuda")
        dev = Device(P)
        status, words, msg = dev.encode(g)
        assert status == 0
        near += compare_encode(P, g.cpu().numpy(), words)
        msgs_dev.append(msg)
        msgs_host.append(words)
    assert near <= 1e-6 * w.n * w.K + 1
    P0 = q.Params(n=w.n, s=w.s, d=w.d, code=code, norm=norm, seed=w.seed)
    x = W.parameters(w).numpy()
    mism = check_step(P0, msgs_dev, msgs_host, w.eta, x, w.K)
    if expect_exact_step:
        assert mism == 0, f"{mism} values of x not bit-identical"
    return near


SMALL = [
    W.C1,                                   # 2048 full buckets of 512
    W.scaled(W.C2, 200_000 + 132),          # 161 tensors, ragged tail bucket of 324
    W.scaled(W.C5, 8192 * 9 + 2560),        # bucket 8192 (4 wavefronts per bucket), tail 2560
    W.scaled(W.C3, 512 * 300 + 448),        # fixed width, tail 448
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_configs_small(w):
    run_case(w)


@pytest.mark.parametrize("d", [4, 64, 100, 256, 260, 1024, 1500, 2048, 4096, 6000])
@pytest.mark.parametrize("code", [q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED])
def test_bucket_sizes(d, code):
    n = d * 37 + (d // 4) * 3 + 1 if d > 4 else 150  # ragged tail bucket
    w = W.Workload(f"d{d}", n, 16, d, code, 3, 0.1, "normal", (n,))
    run_case(w)


GENERAL = [  # d > 8192, d not a multiple of 4, d = n: the segmented path
    (W.scaled(W.C4, 200_003), None),                                             # s=1, one bucket of n
    (W.Workload("g10000", 10000 * 7 + 4321, 4, 10000, q.CODE_SPARSE, 3, 0.1, "normal_outliers", (74321,)), None),
    (W.Workload("g8196", 8196 * 5 + 100, 16, 8196, q.CODE_SPARSE, 8, 0.1, "laplace_lognormal", (20000, 21080)), None),
    (W.Workload("g130", 130 * 301 + 77, 4, 130, q.CODE_SPARSE, 4, 0.1, "normal", (130 * 301 + 77,)), None),
    (W.Workload("g1", 333, 7, 1, q.CODE_SPARSE, 2, 0.1, "normal", (333,)), None),
    (W.Workload("g9999", 9999 * 4 + 5, 3, 9999, q.CODE_SPARSE, 5, 0.1, "student_t", (40001,)), None),
    (W.Workload("g70001", 70001, 256, 70001, q.CODE_SPARSE, 2, 0.1, "normal", (70001,)), None),
    # more than 1024 segments: the single-workgroup scan takes several passes, and buckets
    # (5 and 9 segments each, entry lists) straddle its pass boundaries
    (W.Workload("g10000x300", 10000 * 300 + 77, 4, 10000, q.CODE_SPARSE, 2, 0.1, "student_t", (3000077,)), None),
    (W.Workload("g17000x150", 17000 * 150 + 5, 16, 17000, q.CODE_SPARSE, 2, 0.1, "normal", (2550005,)), None),
]


@pytest.mark.parametrize("w", [g[0] for g in GENERAL], ids=lambda w: w.name)
@pytest.mark.parametrize("code", [q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED])
def test_general_path(w, code):
    # this path too adds every coordinate's terms in message order: x must be bit-identical
    run_case(w, code=code)
    if code == q.CODE_SPARSE:
        run_case(w, code=code, norm=q.NORM_MAX)


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5, 16, 17, 255, 256, 1000, 65535])
@pytest.mark.parametrize("code", [q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED])
def test_levels(s, code):
    n = 512 * 20 + 36
    w = W.Workload(f"s{s}", n, s, 512, code, 2, 0.05, "normal_outliers", (n,))
    run_case(w)


@pytest.mark.parametrize("K", [1, 2, 5, 16, 33, 64])
def test_peer_counts(K):
    n = 512 * 40 + 100
    w = W.Workload(f"K{K}", n, 4, 512, q.CODE_SPARSE, K, 0.1, "normal", (n,))
    run_case(w)
    w = W.Workload(f"K{K}f", n, 256, 512, q.CODE_FIXED, K, 0.1, "normal", (n,))
    run_case(w)


@pytest.mark.parametrize("K", [1, 2, 3, 5, 16, 33, 64])
@pytest.mark.parametrize("d,s", [(2048, 2), (260, 1), (8192, 7), (1024, 3)])
def test_sparse_messages_counting_apply(K, d, s):
    """Few records per window (64 s^2 <= d): the Elias decoder counts a position's terms
    first.  Heavy-tailed data makes positions hit by three and more messages common."""
    n = d * 9 + d // 3 + 2
    w = W.Workload(f"cnt{d}_{s}_{K}", n, s, d, q.CODE_SPARSE, K, 0.1, "student_t", (n,))
    run_case(w)
    if K == 16:
        run_case(w, norm=q.NORM_MAX)


@pytest.mark.parametrize("scale", [1e-3, 3e-39])
@pytest.mark.parametrize("d,s", [(2048, 2), (8192, 4), (512, 16)])
def test_cancelling_and_tiny_terms(d, s, scale):
    """Peers that carry g and -g (terms of one position cancel, sums pass through zero), and
    magnitudes so small that scales and terms are subnormal: x must still be the oracle's,
    bit for bit (the accumulating adds neither reorder three terms nor flush small ones)."""
    n, K = d * 7 + d // 2 + 4, 6
    gen = torch.Generator().manual_seed(5)
    base = torch.distributions.StudentT(3.0).sample((n,)).float() * scale
    base[torch.rand(n, generator=gen) < 0.01] *= 30.0
    msgs_dev, msgs_host = [], []
    for k in range(K):
        g = (base if k % 2 == 0 else -base).clone()
        P = q.Params(n=n, s=s, d=d, code=q.CODE_SPARSE, seed=3, stream_id=k // 2, iteration=k % 2 * 0)
        status, words, msg = Device(P).encode(g.cuda())
        assert status == 0
        assert compare_encode(P, g.numpy(), words) == 0
        msgs_dev.append(msg)
        msgs_host.append(words)
    P0 = q.Params(n=n, s=s, d=d, code=q.CODE_SPARSE, seed=3)
    for x in (np.zeros(n, dtype=np.float32), np.linspace(-1, 1, n, dtype=np.float32) * np.float32(scale)):
        assert check_step(P0, msgs_dev, msgs_host, 0.1, x, K) == 0


@pytest.mark.parametrize("s,d", [(10, 8192), (4, 8192), (5, 8192), (7, 4096), (2, 2048)])
def test_dense_chunks_inside_sparse_buckets(s, d):
    """Parameters that promise few nonzero levels (Lemma 3.1 (iii)) with data that breaks the
    promise: all of a bucket's mass in one to three chunks of 256 values, or spread evenly
    over the 2048 values of one wavefront (s sqrt(2048) expected survivors there: more than
    its list of 256 holds for s = 7, about as many for s = 5).  A wavefront of the team
    encoder whose survivor list overflows starts over with the direct coder."""
    nb = 25
    n = nb * d + d // 2
    gen = torch.Generator().manual_seed(1234 + s)
    g = torch.zeros(n)
    for b in range(nb + 1):
        m = min(d, n - b * d)
        kind = b % 5
        if kind == 3:                                   # an ordinary bucket
            g[b * d:b * d + m] = torch.randn(m, generator=gen) * 1e-3
            continue
        if kind == 4:                                   # one wavefront's share, evenly
            w0 = 2048 * ((b // 5) % max(1, m // 2048))
            wl = min(2048, m - w0)
            mag = 0.9 + 0.2 * torch.rand(wl, generator=gen)
            sign = torch.where(torch.rand(wl, generator=gen) < 0.5, -1.0, 1.0)
            g[b * d + w0: b * d + w0 + wl] = mag * sign
            continue
        chunks = torch.randperm(m // 256, generator=gen)[: 1 + kind].tolist()
        for c in chunks:                                # full chunks of similar magnitudes
            mag = 0.5 + torch.rand(256, generator=gen)
            sign = torch.where(torch.rand(256, generator=gen) < 0.5, -1.0, 1.0)
            g[b * d + c * 256: b * d + (c + 1) * 256] = mag * sign
        g[b * d + (b * 37) % m] = 0.75                  # and a lone value somewhere
    msgs_dev, msgs_host = [], []
    for k in range(3):
        P = q.Params(n=n, s=s, d=d, code=q.CODE_SPARSE, seed=77, stream_id=k, iteration=1)
        status, words, msg = Device(P).encode(g.cuda())
        assert status == 0
        assert compare_encode(P, g.numpy(), words) == 0
        msgs_dev.append(msg)
        msgs_host.append(words)
    P0 = q.Params(n=n, s=s, d=d, code=q.CODE_SPARSE, seed=77)
    x = np.linspace(-1, 1, n, dtype=np.float32)
    assert check_step(P0, msgs_dev, msgs_host, 0.1, x, 3) == 0


def test_survivor_list_overflow_takes_the_direct_coder():
    """s = 5, d = 8192 is coded through the survivor list (Lemma 3.1 (iii) promises it half
    full), a list of 256 records per wavefront.  Buckets whose mass lies evenly on one
    wavefront's 2048 values bring s sqrt(2048) = 226 survivors there in expectation, a few
    of them more than 256: the oracle's levels say which (at least one with these seeds),
    and those wavefronts must start over with the direct coder, same bits."""
    s, d, nb = 5, 8192, 400
    n = nb * d
    gen = torch.Generator().manual_seed(99)
    g = torch.zeros(n)
    for b in range(nb):
        w0 = 2048 * (b % 4)
        mag = 0.95 + 0.1 * torch.rand(2048, generator=gen)
        sign = torch.where(torch.rand(2048, generator=gen) < 0.5, -1.0, 1.0)
        g[b * d + w0: b * d + w0 + 2048] = mag * sign
    P = q.Params(n=n, s=s, d=d, code=q.CODE_SPARSE, seed=5, stream_id=2, iteration=7)
    lev = qo.quantize(oracle_params(P), g.numpy())["levels"].reshape(nb, 4, 2048)
    per_wave = (lev != 0).sum(axis=2).max(axis=1)
    assert (per_wave > 256).sum() >= 1 and (per_wave <= 256).sum() >= 1
    status, words, msg = Device(P).encode(g.cuda())
    assert status == 0
    assert compare_encode(P, g.numpy(), words) == 0
    x = np.linspace(-1, 1, n, dtype=np.float32)
    assert check_step(P, [msg], [words], 0.1, x, 1) == 0


@pytest.mark.parametrize("same_gradient", [False, True])
@pytest.mark.parametrize("nb", [1, 3])
def test_long_sparse_buckets_read_all_messages_at_once(same_gradient, nb):
    """Long buckets (d > 8192), s = 1, K = 16: the decoder reads the K messages at the same
    time and sums coordinates that several messages hit from a list, in message order.
    Spikes shared by all peers give coordinates with up to 16 terms; the same gradient for
    every peer makes the messages collide so often that the list overflows and the
    workgroup falls back to reading the messages in turns."""
    d, K = 150_001, 16
    n = nb * d - (7 if nb > 1 else 0)
    gen = torch.Generator().manual_seed(99)
    msgs_dev, msgs_host = [], []
    g0 = torch.distributions.StudentT(3.0).sample((n,)) * 1e-3
    for k in range(K):
        if same_gradient:
            g = g0.clone()
        else:
            g = torch.randn(n, generator=gen) * 1e-3
            g[12345] = 0.5                       # every peer
            g[n - 5] = -0.25 if k % 2 == 0 else 0.25
            if k < 3:
                g[777] = 0.125                   # three peers
        P = q.Params(n=n, s=1, d=d, code=q.CODE_SPARSE, seed=3, stream_id=k, iteration=2)
        status, words, msg = Device(P).encode(g.cuda())
        assert status == 0
        assert compare_encode(P, g.numpy(), words) == 0
        msgs_dev.append(msg)
        msgs_host.append(words)
    P0 = q.Params(n=n, s=1, d=d, code=q.CODE_SPARSE, seed=3)
    x = np.linspace(-1, 1, n, dtype=np.float32)
    assert check_step(P0, msgs_dev, msgs_host, 0.1, x, K) == 0


def test_max_scaling():
    n = 512 * 64 + 12
    for code in (q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED):
        w = W.Workload("max", n, 15, 512, code, 4, 0.1, "laplace_lognormal", (n // 2, n - n // 2))
        run_case(w, norm=q.NORM_MAX)


def test_degenerate_buckets():
    """All-zero buckets, one-hot buckets (level s), negative zero, n < d."""
    n, d = 512 * 8, 512
    g = torch.zeros(n)
    g[512 + 77] = -0.25          # one-hot: level s, negative
    g[1024:1536] = -0.0          # negative zeros: sign bit 0
    g[1536:2048] = torch.randn(512) * 1e-3
    g[2048] = 1.0; g[2049] = 1.0  # two equal entries
    g[4095] = 3e-3               # last element of the last bucket
    for code in (q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED):
        for s in (1, 4, 256):
            P = q.Params(n=n, s=s, d=d, code=code, seed=5)
            status, words, msg = Device(P).encode(g.cuda())
            assert status == 0
            assert compare_encode(P, g.numpy(), words) == 0
            x = np.linspace(-1, 1, n, dtype=np.float32)
            assert check_step(P, [msg], [words], 0.5, x, 1) == 0
    # n < d: one short bucket
    for n2 in (4, 300):
        P = q.Params(n=n2, s=4, d=512, code=q.CODE_SPARSE)
        g2 = torch.randn(n2) * 1e-3
        status, words, msg = Device(P).encode(g2.cuda())
        assert status == 0 and compare_encode(P, g2.numpy(), words) == 0
        assert check_step(P, [msg], [words], 0.5, np.ones(n2, dtype=np.float32), 1) == 0


def test_empty_gradient():
    for code in (q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED):
        P = q.Params(n=0, s=4, d=512, code=code)
        g = torch.zeros(0, device="cuda")
        status, words, msg = Device(P).encode(g)
        assert status == 0
        assert np.array_equal(words, qo.encode(oracle_params(P), np.zeros(0, np.float32)))
        x = torch.zeros(0, device="cuda")
        ws = torch.zeros(q.qsgd_workspace_bytes(P, 1) // 4, dtype=torch.int32, device="cuda")
        q.qsgd_sgd_step(P, [msg], 0.1, x, ws)
        assert q.qsgd_workspace_status(ws) == 0


def test_deterministic_and_seed_sensitive():
    w = W.scaled(W.C2, 100_000)
    g = W.gradient(w, 0, device="cuda")
    P = q.Params(n=w.n, s=w.s, d=w.d, seed=11, stream_id=2, iteration=9)
    dev = Device(P)
    a = dev.encode(g)[1]
    b = dev.encode(g)[1]
    assert np.array_equal(a, b)
    for change in (dict(seed=12), dict(stream_id=3), dict(iteration=10)):
        P2 = q.Params(**{**P.__dict__, **change})
        c = dev.encode(g, P2)[1]
        assert compare_encode(P2, g.cpu().numpy(), c) == 0
        assert c.size != a.size or not np.array_equal(a[16:], c[16:])


def test_capacity_overflow_is_reported_not_overrun():
    w = W.scaled(W.C2, 50_000)
    g = W.gradient(w, 0, device="cuda")
    P = q.Params(n=w.n, s=w.s, d=w.d)
    ref = qo.encode(oracle_params(P), g.cpu().numpy())
    for cap in (ref.nbytes - 4, ref.nbytes // 2, 64 + 4 * 100):
        status, needed, _ = Device(P, capacity=cap).encode(g)
        assert status == -2 and needed == ref.nbytes
    status, words, _ = Device(P, capacity=ref.nbytes).encode(g)  # exactly enough
    assert status == 0 and np.array_equal(words, ref)
    with pytest.raises(q.QsgdError):  # not even room for header + table
        Device(P, capacity=64).encode(g)


def test_corrupt_messages_are_flagged():
    w = W.scaled(W.C1, 512 * 64)
    g = W.gradient(w, 0, device="cuda")
    x0 = W.parameters(w).numpy()
    for code in (q.CODE_SPARSE, q.CODE_DENSE, q.CODE_FIXED):
        P = q.Params(n=w.n, s=w.s, d=w.d, code=code)
        status, words, msg = Device(P).encode(g)
        ws = torch.zeros(max(q.qsgd_workspace_bytes(P, 1), 256) // 4, dtype=torch.int32,
                         device="cuda")
        good = msg.clone()

        def step(m, nbytes=None, params=P):
            x = torch.from_numpy(x0.copy()).cuda()
            q.qsgd_sgd_step(params, [m], 0.1, x, ws, msg_bytes=None if nbytes is None else [nbytes])
            return q.qsgd_workspace_status(ws)

        assert step(good) == 0
        bad = good.clone(); bad[0] ^= 1                      # magic
        assert step(bad) == -3
        assert step(good, nbytes=words.nbytes - 4) == -3     # truncated buffer
        assert step(good, params=q.Params(n=w.n, s=w.s + 1, d=w.d, code=code)) == -3
        bad = good.clone(); bad[14] = 7                      # encoder left an error status
        assert step(bad) == -3
        if code != q.CODE_FIXED:
            base = qo.payload_offset_words(words)
            off, cnt = qo.bucket_extent(words, 5)
            bad = good.clone(); bad[base + off + cnt - 1] = 0  # string with no end
            if code == q.CODE_SPARSE:
                assert step(bad) == -3
            bad = good.clone(); bad[16 + 6] = bad[16 + 5] - 1  # table runs backwards
            assert step(bad) == -3
            bad = good.clone(); bad[base + off + 1: base + off + cnt] = -1  # all ones
            assert step(bad) == -3
        assert step(good) == 0


@pytest.mark.parametrize("K", [1, 32])
def test_corrupt_entry_lists_of_long_buckets_are_flagged(K):
    """Buckets above 8192 values carry a list of entry points behind their string; the
    readers (all messages at once for K = 1, message after message for K = 32) must refuse
    a damaged list, leave x alone and stay inside the buffers."""
    n, s = 3_000_000, 1
    rng = np.random.default_rng(4)
    g_host = (rng.standard_normal(n) * ((rng.random(n) < 0.01) * 50.0 + 0.01)).astype(np.float32)
    g = torch.from_numpy(g_host).cuda()
    P = q.Params(n=n, s=s, d=n, code=q.CODE_SPARSE, seed=3)
    status, words, msg = Device(P).encode(g)
    assert status == 0
    nw = words.size
    ents = int(words[-1])
    assert ents >= 3
    ws = torch.zeros(max(q.qsgd_workspace_bytes(P, K), 256) // 4, dtype=torch.int32, device="cuda")
    x0 = torch.from_numpy(W.parameters(W.scaled(W.C4, n)).numpy())
    good = msg[:nw].clone()

    def step(m):
        x = x0.clone().cuda()
        q.qsgd_sgd_step(P, [good] * (K - 1) + [m], 0.1, x, ws)
        st = q.qsgd_workspace_status(ws)
        return st, x.cpu()

    st, x = step(good)
    assert st == 0 and not torch.equal(x, x0)
    for name, index, value in [
            ("one entry too many", nw - 1, ents + 1),
            ("more entries than words", nw - 1, nw),
            ("entry past the string", nw - 1 - 2 * ents + 2, 32 * nw),         # bit offset of entry 1
            ("entry in the middle of a code word", nw - 1 - 2 * ents + 2, int(words[nw - 1 - 2 * ents + 2]) + 1),
            ("wrong position before an entry", nw - 1 - 2 * ents + 3, int(words[nw - 1 - 2 * ents + 3]) + 1),
            ("entries out of order", nw - 1 - 2 * ents, int(words[nw - 1 - 2 * ents + 2])),
    ]:
        bad = good.clone()
        bad[index] = value
        st, x = step(bad)
        assert st == -3, name
        assert torch.equal(x, x0), name
    st, x = step(good)
    assert st == 0


def test_encode_with_a_workspace_below_the_worst_case():
    """Sparse data: the staging of the bucket strings may be far smaller than the worst
    case (qsgd_encode_workspace_bytes sizes it from the message capacity).  Same message
    as with the worst-case workspace; data that code longer than the regions or the
    message buffer allow end with the capacity status, nothing written past either buffer."""
    n, s, d = 512 * 40_000 + 100, 4, 512
    gen = torch.Generator(device="cuda")
    gen.manual_seed(12)
    g = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 1e-3, generator=gen)
    P = q.Params(n=n, s=s, d=d, code=q.CODE_SPARSE, seed=8)
    worst = q.qsgd_workspace_bytes(P, 1)
    status, ref, _ = Device(P).encode(g)
    assert status == 0
    cap = (int(ref.nbytes * 1.25) + 4096) & ~255
    sized = q.qsgd_encode_workspace_bytes(P, cap)
    assert sized <= worst
    for small in (sized, worst // 3):
        ws = torch.full((small // 4 + 64,), -1, dtype=torch.int32, device="cuda")
        msg = torch.full((cap // 4 + 64,), -1, dtype=torch.int32, device="cuda")
        q.qsgd_encode(P, g, msg[: cap // 4], ws[: small // 4])
        status, total = q.qsgd_message_status(msg)
        assert status == 0 and total == ref.nbytes
        assert np.array_equal(msg.cpu().numpy().view(np.uint32)[: total // 4], ref)
        assert bool((msg[cap // 4:] == -1).all()) and bool((ws[small // 4:] == -1).all())
    # a message buffer that is too small: reported with the size needed, not overrun
    tight = (ref.nbytes * 6 // 10) & ~255
    msg.fill_(-1)
    q.qsgd_encode(P, g, msg[: tight // 4], ws[: small // 4])
    status, need = q.qsgd_message_status(msg)
    assert status == -2 and need == ref.nbytes
    assert bool((msg[tight // 4:] == -1).all()) and bool((ws[small // 4:] == -1).all())
    # regions below what the strings need (the smallest workspace the call takes): the
    # regions run out before the message buffer does; same report
    tiny = 256 + 8192 * 12 + 8192 * 64 * 4
    assert tiny < sized
    msg.fill_(-1)
    ws.fill_(-1)
    q.qsgd_encode(P, g, msg[: cap // 4], ws[: tiny // 4])
    status, need = q.qsgd_message_status(msg)
    assert status == -2 and need == ref.nbytes
    assert bool((msg[cap // 4:] == -1).all()) and bool((ws[tiny // 4:] == -1).all())
    # and once more with enough room: the buffers are reusable after an overflow
    q.qsgd_encode(P, g, msg[: cap // 4], ws[: small // 4])
    status, total = q.qsgd_message_status(msg)
    assert status == 0 and np.array_equal(msg.cpu().numpy().view(np.uint32)[: total // 4], ref)
    with pytest.raises(q.QsgdError):      # regions that could not hold one string
        q.qsgd_encode(P, g, msg[: cap // 4], ws[: 40_000])


def test_argument_checks():
    P = q.Params(n=1024, s=4, d=512)
    g = torch.zeros(1024, device="cuda")
    msg = torch.zeros(q.qsgd_max_encoded_bytes(P) // 4, dtype=torch.int32, device="cuda")
    ws = torch.zeros(q.qsgd_workspace_bytes(P, 1) // 4, dtype=torch.int32, device="cuda")
    for bad in (dict(s=0), dict(s=70000), dict(d=0), dict(code=3), dict(norm=2)):
        with pytest.raises(q.QsgdError):
            q.qsgd_encode(q.Params(**{**P.__dict__, **bad}), g, msg, ws)
    with pytest.raises(q.QsgdError):
        q.qsgd_encode(P, g, msg, ws[:8])              # workspace too small
    with pytest.raises(q.QsgdError):
        q.qsgd_encode(P, g, msg.view(torch.uint8)[4:], ws)  # message not 16-byte aligned
    with pytest.raises(q.QsgdError):
        q.qsgd_sgd_step(P, [], 0.1, g, ws)            # K = 0
