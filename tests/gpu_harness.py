"""Helpers of the GPU parity tests: run the HIP path through its C ABI binding and
compare with the CPU oracle on the same inputs."""
from __future__ import annotations

import numpy as np
import torch

import paper_1610_02132_amd as q
from oracle import compare
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
    """GPU message vs oracle on the same input (oracle/compare.py: identical, except
    counted near-tie elements, the oracle's draw within 1e-5 of its threshold, and counted
    buckets whose scale is one rounding apart).  Returns the number of near-tie elements,
    which may be at most 1e-6 of the elements."""
    r = compare.compare_encode(oracle_params(P), g_host, gpu_words)
    assert r["near_ties"] <= 1e-6 * P.n, f"{r['near_ties']} near-tie elements of {P.n}"
    assert r["norm_mismatches"] <= 1e-6 * P.n, f"{r['norm_mismatches']} bucket scales differ"
    return r["near_ties"]


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
