"""Helpers of the GPU parity tests: run the HIP path through its C ABI binding and
compare with the CPU oracle on the same inputs."""
from __future__ import annotations

import numpy as np
import torch

import paper_1610_02132_amd as q
from oracle import qsgd_oracle as qo


def oracle_params(P: q.Params) -> qo.Params:
    return qo.Params(n=P.n, s=P.s, d=P.d, code=P.code, norm=P.norm, seed=P.seed,
                     stream_id=P.stream_id, iteration=P.iteration)


class Device:
    """Device buffers for one parameter set (message capacity, workspace)."""

    def __init__(self, P: q.Params, K: int = 1, capacity: int | None = None):
        self.P = P
        self.cap = q.qsgd_max_encoded_bytes(P) if capacity is None else capacity
        self.ws = torch.zeros(max(q.qsgd_workspace_bytes(P, K), 256) // 4, dtype=torch.int32,
                              device="cuda")

    def encode(self, g_dev: torch.Tensor, P: q.Params | None = None):
        """Returns (status, message words as numpy uint32 trimmed to its length)."""
        P = self.P if P is None else P
        msg = torch.full(((self.cap + 3) // 4 + 4,), -1, dtype=torch.int32, device="cuda")
        q.qsgd_encode(P, g_dev, msg[: (self.cap // 4)], self.ws)
        status, total = q.qsgd_message_status(msg)
        host = msg.cpu().numpy().view(np.uint32)
        # nothing may be written past the capacity handed in
        assert np.all(host[self.cap // 4:] == 0xFFFFFFFF), "write past the message capacity"
        if status == 0:
            assert total <= self.cap
            return status, host[: total // 4].copy(), msg
        return status, total, msg


def compare_encode(P: q.Params, g_host: np.ndarray, gpu_words: np.ndarray):
    """GPU message vs oracle on the same input.  Returns the number of near-tie
    elements (draw within 1e-5 of the rounding threshold, or in a bucket whose
    fp32 scale came out one rounding apart); everything else must be identical."""
    Po = oracle_params(P)
    ref = qo.encode(Po, g_host)
    if ref.size == gpu_words.size and np.array_equal(ref, gpu_words):
        return 0
    # not byte-identical: every difference must trace back to a near-tie
    tup = qo.decode_tuple(gpu_words)  # raises if the GPU message does not parse
    qz = qo.quantize(Po, g_host, want_draws=True)
    d = qo.bucket_size(Po)
    nb = qo.num_buckets(Po)
    norm_diff = tup["norms"].view(np.uint32) != qz["norms"].view(np.uint32)
    # a scale may differ by one rounding of the fp64 sum, never more
    rel = np.abs(tup["norms"].astype(np.float64) - qz["norms"]) / np.maximum(qz["norms"], 1e-300)
    assert np.all(rel[norm_diff] <= 1.2e-7), "bucket scale differs by more than one rounding"
    lev_diff = tup["levels"] != qz["levels"]
    sent = np.ones(P.n, dtype=bool) if P.code != q.CODE_SPARSE else (qz["levels"] != 0) & ~lev_diff
    sign_diff = sent & (tup["neg"] != qz["neg"])
    assert not sign_diff.any(), "sign bits differ"
    assert np.all(np.abs(tup["levels"].astype(np.int64) - qz["levels"].astype(np.int64)) <= 1)
    idx = np.flatnonzero(lev_diff)
    bucket_of = idx // d
    tie = np.abs(qz["u"][idx] - qz["p"][idx]) <= 1e-5
    assert np.all(tie | norm_diff[bucket_of]), "level differs away from a rounding threshold"
    near = int(idx.size)
    assert near <= max(1e-6 * P.n, 0) or near <= int(norm_diff.sum()) * 2, \
        f"{near} near-tie elements of {P.n}"
    # buckets without any difference must be byte-identical
    dirty = np.zeros(nb, dtype=bool)
    dirty[bucket_of] = True
    dirty |= norm_diff
    for b in np.flatnonzero(~dirty)[:: max(1, nb // 2000)]:
        assert np.array_equal(qo.bucket_words(ref, int(b)), qo.bucket_words(gpu_words, int(b))), \
            f"bucket {b} strings differ"
    assert dirty.any(), "messages differ but no level or scale does (layout mismatch)"
    return near


def check_step(P: q.Params, msgs_dev, msgs_host, eta, x_host: np.ndarray, K: int):
    """GPU fused step and accumulate vs the oracle on the same messages."""
    ws = torch.zeros(max(q.qsgd_workspace_bytes(P, K), 256) // 4, dtype=torch.int32,
                     device="cuda")
    x = torch.from_numpy(x_host.copy()).cuda()
    q.qsgd_sgd_step(P, msgs_dev, eta, x, ws)
    assert q.qsgd_workspace_status(ws) == 0
    want = qo.sgd_step(msgs_host, eta, x_host)
    got = x.cpu().numpy()
    assert_close(got, want, x_host)
    acc = torch.from_numpy(x_host.copy()).cuda()
    q.qsgd_decode_accumulate(P, msgs_dev, acc, ws)
    assert q.qsgd_workspace_status(ws) == 0
    want_acc = qo.decode_accumulate(msgs_host, x_host)
    assert_close(acc.cpu().numpy(), want_acc, x_host)
    return int(np.count_nonzero(got.view(np.uint32) != want.view(np.uint32)))


def assert_close(got, want, x0):
    """fp32 results: within 1e-6 relative (of the larger of the result and the
    starting value, so that a cancelling update is not held to its own size)."""
    scale = np.maximum(np.abs(want), np.abs(x0)).astype(np.float64)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bad = err > 1e-6 * scale + 1e-30
    assert not bad.any(), f"{int(bad.sum())} values off, max rel {float((err / (scale + 1e-30)).max())}"
