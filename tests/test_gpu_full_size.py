"""GPU parity at the full sizes of the five workloads, through the same calls and
launch configuration that bench.py times.  Where the oracle cannot process the
whole input in reasonable time (n = 143M x 16 peers, n = 1e9 x 16 peers) it
checks sampled runs of consecutive buckets, which it can compute one by one
because buckets are coded independently (Sec. 4): their strings, their table
entries and the updated x over those buckets."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1610_02132_amd as q  # noqa: E402
from paper_1610_02132_amd import workloads as W  # noqa: E402
from oracle import qsgd_oracle as qo  # noqa: E402
from gpu_harness import assert_close, check_step, compare_encode  # noqa: E402


def encode_all(w, keep_host_gradients, sample_runs=None):
    """Encodes the K peers' gradients on the GPU (one gradient resident at a time).
    Returns device messages, their sizes, and either the full host gradients or
    the sampled slices [(start, host array)] per peer."""
    ws = torch.empty(q.qsgd_workspace_bytes(q.Params(n=w.n, s=w.s, d=w.d, code=w.code), w.K) // 4,
                     dtype=torch.int32, device="cuda")
    msgs, sizes, host = [], [], []
    cap = None
    for k in range(w.K):
        P = q.Params(n=w.n, s=w.s, d=w.d, code=w.code, seed=w.seed, stream_id=k)
        g = W.gradient(w, k, device="cuda")
        if cap is None:  # size the buffers from the first message, as bench.py does
            probe = torch.empty(q.qsgd_max_encoded_bytes(P) // 4, dtype=torch.int32, device="cuda")
            q.qsgd_encode(P, g, probe, ws)
            st, total = q.qsgd_message_status(probe)
            assert st == 0
            del probe
            cap = min(q.qsgd_max_encoded_bytes(P), (int(total * 1.25) + 4096) & ~255)
        msg = torch.empty(cap // 4, dtype=torch.int32, device="cuda")
        q.qsgd_encode(P, g, msg, ws)
        st, total = q.qsgd_message_status(msg)
        assert st == 0, (k, st)
        msgs.append(msg)
        sizes.append(total)
        if keep_host_gradients:
            host.append(g.cpu().numpy())
        else:
            host.append([(a, g[a:b].cpu().numpy()) for a, b in sample_runs])
        del g
    return msgs, sizes, host, ws


def full_check(w, exact_step=True):
    msgs, sizes, grads, ws = encode_all(w, True)
    words, near = [], 0
    for k in range(w.K):
        P = q.Params(n=w.n, s=w.s, d=w.d, code=w.code, seed=w.seed, stream_id=k)
        mw = msgs[k][: sizes[k] // 4].cpu().numpy().view(np.uint32)
        near += compare_encode(P, grads[k], mw)
        words.append(mw)
    assert near <= 1e-6 * w.n * w.K
    del grads
    P0 = q.Params(n=w.n, s=w.s, d=w.d, code=w.code)
    mism = check_step(P0, msgs, words, w.eta, W.parameters(w).numpy(), w.K)
    if exact_step:
        assert mism == 0


def sampled_check(w, n_runs=6, run_buckets=12):
    d = min(w.d, w.n)
    nb = (w.n + d - 1) // d
    rng = np.random.default_rng(42)
    starts = sorted(set([0, nb - run_buckets] + [int(v) for v in rng.integers(0, nb - run_buckets, n_runs)]))
    runs = [(b0 * d, min((b0 + run_buckets) * d, w.n)) for b0 in starts]  # last run holds the tail
    msgs, sizes, slices, ws = encode_all(w, False, runs)
    table_words = 0 if w.code == q.CODE_FIXED else ((nb + 1 + 3) // 4) * 4
    x0 = W.parameters(w, device="cuda")
    x_before = [x0[a:b].cpu().numpy() for a, b in runs]
    x = x0
    P0 = q.Params(n=w.n, s=w.s, d=w.d, code=w.code)
    q.qsgd_sgd_step(P0, msgs, w.eta, x, ws)
    assert q.qsgd_workspace_status(ws) == 0
    for ri, (a, b) in enumerate(runs):
        b0 = a // d
        nbr = (b - a + d - 1) // d
        ref_msgs = []
        for k in range(w.K):
            Ps = qo.Params(n=b - a, s=w.s, d=d, code=w.code, seed=w.seed, stream_id=k)
            ref = qo.encode_slice(Ps, slices[k][ri][1], a)
            ref_msgs.append(ref)
            # the same buckets in the GPU message
            if w.code == q.CODE_FIXED:
                full = qo.bucket_extent(ref, 0)[1] if nbr > 1 or (b - a) == d else None
                wfull = full if full is not None else None
                # closed-form placement: bucket b at b * words(full bucket)
                P_full = qo.Params(n=d, s=w.s, d=d, code=w.code)
                wfull = (qo.max_encoded_bytes(P_full) - 64) // 4
                lo = 16 + b0 * wfull
                got = msgs[k][lo: lo + (ref.size - 16)].cpu().numpy().view(np.uint32)
                assert np.array_equal(got, ref[16:]), f"peer {k} buckets {b0}.. differ"
            else:
                tab = msgs[k][16 + b0: 16 + b0 + nbr + 1].cpu().numpy().view(np.uint32).astype(np.int64)
                lo = 16 + table_words + int(tab[0])
                got = msgs[k][lo: lo + int(tab[-1] - tab[0])].cpu().numpy().view(np.uint32)
                ref_tab = ref[16:16 + nbr + 1].astype(np.int64)
                ref_pay = ref[qo.payload_offset_words(ref):]
                assert np.array_equal(tab - tab[0], ref_tab), f"peer {k} table at bucket {b0} differs"
                assert np.array_equal(got, ref_pay), f"peer {k} strings of buckets {b0}.. differ"
        want = qo.sgd_step(ref_msgs, w.eta, x_before[ri])
        got_x = x[a:b].cpu().numpy()
        assert_close(got_x, want, x_before[ri])
        assert np.array_equal(got_x, want), "x over the sampled buckets is not bit-identical"
    # header of every message: the length the encoder reported
    for k in range(w.K):
        st, p, total = q.qsgd_message_info(bytes(msgs[k][:16].cpu().numpy().tobytes()))
        assert st == 0 and total == sizes[k] and p.n == w.n and p.stream_id == k


def test_c2_full():
    full_check(W.C2)


def test_c4_full():
    full_check(W.C4)


def test_c3_full_sampled():
    sampled_check(W.C3)


def test_c5_full_sampled():
    sampled_check(W.C5, n_runs=5, run_buckets=6)
