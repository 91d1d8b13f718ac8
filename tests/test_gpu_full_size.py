"""GPU parity at the full sizes of the five workloads, through the same calls and
launch configuration that bench.py times.  c1, c2 and c4 go through the oracle whole.
c3 (143M x 16 peers) and c5 (1e9 x 16 peers) are too long for one oracle call, but
buckets are quantized and coded independently (Sec. 4): the vector is cut into runs of
whole buckets, the oracle encodes each run as a slice with the draws of its positions
and applies the step to each run of x, on the host cores in parallel, and EVERY bucket
of every message and every value of x is compared."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1610_02132_amd as q  # noqa: E402
from paper_1610_02132_amd import workloads as W  # noqa: E402
from oracle import compare  # noqa: E402
from oracle import qsgd_oracle as qo  # noqa: E402
from gpu_harness import assert_close, check_step, compare_encode  # noqa: E402


def encode_all(w):
    """Encodes the K peers' gradients on the GPU (one gradient resident at a time).
    Returns device messages, their sizes and the host gradients."""
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
        host.append(g.cpu().numpy())
        del g
    return msgs, sizes, host, ws


def full_check(w, exact_step=True):
    msgs, sizes, grads, ws = encode_all(w)
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


HOST_THREADS = 16     # the GPU machine's CPU share (the oracle calls release the interpreter lock)


def whole_check(w, run_elems):
    """Every bucket of every peer's message against the oracle's encode of its run, the
    structure of every message, and every value of x after the fused step against the
    oracle's step over the GPU's messages (which the first part has just tied to the
    oracle's own)."""
    d = min(w.d, w.n)
    nb = (w.n + d - 1) // d
    bper = max(1, run_elems // d)
    runs = [(b0, min(b0 + bper, nb)) for b0 in range(0, nb, bper)]
    fixed = w.code == q.CODE_FIXED
    table_words = 0 if fixed else ((nb + 1 + 3) // 4) * 4
    full = (qo.max_encoded_bytes(qo.Params(n=d, s=w.s, d=d, code=w.code)) - 64) // 4
    ws = torch.empty(q.qsgd_workspace_bytes(q.Params(n=w.n, s=w.s, d=w.d, code=w.code), w.K) // 4,
                     dtype=torch.int32, device="cuda")
    msgs, words, totals = [], [], dict(elements=0, near_ties=0, norm_mismatches=0)
    cap = None
    pool = ThreadPoolExecutor(HOST_THREADS)
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
        mw = msg[: total // 4].cpu().numpy().view(np.uint32)
        Po = qo.Params(n=w.n, s=w.s, d=w.d, code=w.code, seed=w.seed, stream_id=k)
        compare.structure_check(mw, Po)
        st2, hp, htotal = q.qsgd_message_info(bytes(mw[:16].tobytes()))
        assert st2 == 0 and htotal == total and hp.n == w.n and hp.stream_id == k
        g_host = g.cpu().numpy()
        del g
        pay = 16 + table_words

        def one_run(run, mw=mw, g_host=g_host, k=k):
            b0, b1 = run
            lo, hi = b0 * d, min(b1 * d, w.n)
            pr = qo.Params(n=hi - lo, s=w.s, d=d, code=w.code, seed=w.seed, stream_id=k)
            if fixed:
                tab, strings = None, mw[pay + b0 * full: min(pay + b1 * full, mw.size)]
            else:
                tab = mw[16 + b0: 16 + b1 + 1]
                strings = mw[pay + int(tab[0]): pay + int(tab[-1])]
            return compare.compare_bucket_run(pr, g_host[lo:hi], lo, tab, strings)

        for r in pool.map(one_run, runs):
            for key in totals:
                totals[key] += r[key]
        print(f"peer {k}: {nb} buckets compared, totals {totals}", flush=True)
        msgs.append(msg)
        words.append(mw)
        del g_host
    assert totals["elements"] == w.n * w.K
    assert totals["near_ties"] <= 1e-6 * totals["elements"], totals
    assert totals["norm_mismatches"] <= 1e-6 * totals["elements"], totals

    # ---- the fused step over the whole x --------------------------------------------------
    x = W.parameters(w, device="cuda")
    x0 = x.cpu().numpy()
    P0 = q.Params(n=w.n, s=w.s, d=w.d, code=w.code)
    q.qsgd_sgd_step(P0, msgs, w.eta, x, ws)
    assert q.qsgd_workspace_status(ws) == 0
    got = x.cpu().numpy()
    prep = qo.prepare_messages(words)

    def step_run(run):
        b0, b1 = run
        lo, hi = b0 * d, min(b1 * d, w.n)
        want = qo.sgd_step_buckets(prep, w.eta, x0[lo:hi], b0, b1 - b0)
        assert_close(got[lo:hi], want, x0[lo:hi])
        return int(np.count_nonzero(got[lo:hi].view(np.uint32) != want.view(np.uint32)))

    mism = sum(pool.map(step_run, runs))
    pool.shutdown()
    print(f"x: {w.n} values compared, {mism} not bit-identical", flush=True)
    assert mism == 0, f"{mism} values of x are not bit-identical"


def test_c2_full():
    full_check(W.C2)


def test_c4_full():
    full_check(W.C4)


def test_c3_full():
    whole_check(W.C3, run_elems=1 << 21)


def test_c5_full():
    whole_check(W.C5, run_elems=1 << 22)
