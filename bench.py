#!/usr/bin/env python3
"""Throughput of the QSGD hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients that
are already resident in HBM: K x qsgd_encode (one message per peer) followed by
one qsgd_sgd_step that decodes the K messages, sums them and updates x.
`value` = fp32 gradient bytes through the path per second = 4*K*n*steps / time.

With no flags the headline workload is c5 (n = 1e9, the largest that fits one GPU); the
other workload of the size the target is quoted on, c3 (n = 143M, fixed width), is then
measured the same way in a second leg and reported under the key "c3".

Prints ONE JSON line (see the keys below); everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, vendor figure


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def source_digest() -> str:
    """Digest of the kernel sources: ties stored counter figures to the code they were
    measured on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1610_02132_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def hbm_traffic(workload: str, n: int):
    """HBM bytes per launch of each kernel, as measured with the hardware counters.

    They cannot be collected from inside this process; they come from the committed
    summary of `rocprofv3 --pmc` runs of this same command (FETCH_SIZE, then
    WRITE_SIZE, each scaled by what the counter reads for the copy kernel of known
    size that this script also launches; a third run gives the rate of vector
    instructions).  The summary is only used for the workload and size it was taken on
    AND for the kernel sources it was taken on (`source_digest` line); otherwise the
    figures are reported as null.  Returns (traffic, valu rate, source file or None).
    """
    rel = os.path.join("profiles", f"hbm_traffic_{workload}.txt")
    out, rate = {}, {}
    try:
        with open(os.path.join(ROOT, rel)) as f:
            lines = f.read().splitlines()
    except OSError:
        return out, rate, None
    size_ok, digest_ok = False, False
    for line in lines:
        tok = line.split()
        if len(tok) == 2 and tok[0] == "n":
            size_ok = int(tok[1]) == n
        elif len(tok) == 2 and tok[0] == "source_digest":
            digest_ok = tok[1] == source_digest()
        elif len(tok) == 4 and tok[0] == "kernel":
            out[tok[1]] = float(tok[2]) + float(tok[3])   # fetched + written bytes
        elif len(tok) == 3 and tok[0] == "valu_rate":
            rate[tok[1]] = float(tok[2])
    if not (size_ok and digest_ok):
        return {}, {}, None
    return out, rate, rel


def measure(args, wname: str, torch, np, q, W, cpu_seconds: float) -> dict:
    """Times --steps steps of one workload and returns its record."""
    w = W.WORKLOADS[wname]
    if args.n:
        w = W.scaled(w, args.n)
    K, n = w.K, w.n
    log(f"workload {w.name}: n={n} s={w.s} d={w.d} code={w.code} K={K} ({w.note})")

    # tensor-aware mode: the tensors sit in an arena, each at a multiple of 4 elements
    tensors, n_values = None, n
    if args.layout:
        tensors, off = [], 0
        for size in w.tensors:
            tensors.append((off, size))
            off += (size + 3) // 4 * 4
        n = off          # arena length; n_values = elements that belong to a tensor
        layout = q.Layout(tensors, min(w.d, 8192), args.bypass)
        nb_l, raw_l, _ = q.qsgd_layout_info(layout)
        log(f"layout: {len(tensors)} tensors in an arena of {n}; {nb_l} buckets, {raw_l} raw values")

    def params(k):
        return q.Params(n=n, s=w.s, d=w.d, code=w.code, seed=w.seed, stream_id=k, iteration=0)

    def to_arena(flat):
        if not args.layout:
            return flat
        a = torch.zeros(n, dtype=torch.float32, device="cuda")
        o = 0
        for off_, size in tensors:
            a[off_:off_ + size] = flat[o:o + size]
            o += size
        return a

    # ---- inputs, resident in HBM ------------------------------------------------
    t0 = time.time()
    grads = [to_arena(W.gradient(w, k, device="cuda")) for k in range(K)]
    x = to_arena(W.parameters(w, device="cuda"))
    torch.cuda.synchronize()
    log(f"inputs generated in {time.time() - t0:.1f}s "
        f"({(K + 1) * 4 * n / 2**30:.1f} GiB resident)")

    if args.layout:
        ws_bytes = q.qsgd_layout_workspace_bytes(params(0), layout, K)
        cap_max = q.qsgd_layout_max_encoded_bytes(params(0), layout)

        def encode(k, msg):
            q.qsgd_encode_layout(params(k), layout, grads[k], msg, ws)

        def step():
            q.qsgd_sgd_step_layout(params(0), layout, msgs, w.eta, x, ws)
    else:
        ws_bytes = q.qsgd_workspace_bytes(params(0), K)
        cap_max = q.qsgd_max_encoded_bytes(params(0))

        def encode(k, msg):
            q.qsgd_encode(params(k), grads[k], msg, ws)

        def step():
            q.qsgd_sgd_step(params(0), msgs, w.eta, x, ws)

    if args.pipeline:
        if args.layout or args.pipeline % min(w.d, n):
            raise SystemExit("bench.py: --pipeline needs a flat workload and a chunk that is a "
                             "multiple of d")
    ws = torch.empty(ws_bytes // 4, dtype=torch.int32, device="cuda")
    # size the message buffers from a first encode into a worst-case buffer
    probe = torch.empty(cap_max // 4, dtype=torch.int32, device="cuda")
    encode(0, probe)
    status, total0 = q.qsgd_message_status(probe)
    assert status == 0, status
    del probe
    cap = min(cap_max, (int(total0 * 1.25) + 4096) & ~255)
    msgs = [torch.empty(cap // 4, dtype=torch.int32, device="cuda") for _ in range(K)]
    log(f"message: {total0} bytes = {8 * total0 / n:.3f} bits/element; capacity {cap} bytes each")

    def one_step():
        for k in range(K):
            encode(k, msgs[k])
        step()

    if args.pipeline:
        chunk = min(args.pipeline, n)
        pc = q.Params(n=chunk, s=w.s, d=w.d, code=w.code)
        cap_c = min(q.qsgd_max_encoded_bytes(pc), (int(total0 * 1.3 * chunk / n) + 65536) & ~255)
        del msgs
        msgs = [torch.empty(cap_c // 4, dtype=torch.int32, device="cuda") for _ in range(2 * K)]
        ws2 = torch.empty(ws_bytes // 4, dtype=torch.int32, device="cuda")
        pipe = q.Pipeline()

        def one_step():   # noqa: F811
            q.qsgd_pipeline_step(pipe, params(0), chunk, grads, w.eta, x, msgs, ws, ws2)

    for _ in range(max(args.warmup, 1)):   # at least one untimed pass fills the messages
        one_step()
    torch.cuda.synchronize()
    sizes = []
    for k in range(len(msgs)):
        st, tot = q.qsgd_message_status(msgs[k])
        assert st == 0, (k, st)
        sizes.append(tot)
    assert q.qsgd_workspace_status(ws2 if args.pipeline else ws) == 0
    # (pipelined: the buffers hold the last two chunks; scale to the whole vector)
    msg_bytes_avg = float(total0) if args.pipeline else float(np.mean(sizes))

    # ---- timed region: exactly --steps steps ---------------------------------------
    q.qsgd_timing_reset()
    if args.graph:
        if args.pipeline:
            raise SystemExit("bench.py: --graph and --pipeline do not combine (the pass uses "
                             "its own streams)")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_step()
        graph.replay()                      # one untimed replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        q.qsgd_timing_enable(True)          # kernel times: one eager step outside the timed region
        one_step()
        torch.cuda.synchronize()
        q.qsgd_timing_enable(False)
        steps_timed = 1
    else:
        q.qsgd_timing_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        q.qsgd_timing_enable(False)
        steps_timed = args.steps
    assert q.qsgd_workspace_status(ws2 if args.pipeline else ws) == 0

    ms_per_step = 1e3 * elapsed / args.steps
    n_arena, n = n, n_values      # throughput counts the values that belong to a tensor
    value = 4.0 * K * n * args.steps / elapsed / 1e9

    kern = {}
    for name in ("encode_bucket", "encode_compact", "encode_general", "encode_raw", "decode_check",
                 "decode_raw", "decode_fixed", "decode_elias", "decode_general"):
        ms, cnt = q.qsgd_timing_get(name)
        if cnt:
            kern[name] = {"ms_total": ms, "launches": cnt, "ms_avg": ms / cnt}
    q.qsgd_timing_reset()
    enc_ms = sum(v["ms_total"] for k_, v in kern.items() if k_.startswith("encode")) / (steps_timed * K)
    dec_ms = sum(v["ms_total"] for k_, v in kern.items() if k_.startswith("decode")) / steps_timed
    enc_gbps = 4.0 * n / (enc_ms * 1e-3) / 1e9
    dec_gbps = 4.0 * K * n / (dec_ms * 1e-3) / 1e9

    # ---- roofline of the dominant kernel (HBM bound: a streaming codec) ---------------
    enc_alg = 4.0 * n + msg_bytes_avg                       # read g once, write the message once
    dec_alg = K * msg_bytes_avg + 8.0 * n                   # read K messages, read + write x
    if args.pipeline:   # a launch covers one chunk (kernels of the two streams overlap in time)
        nchunks = (n + args.pipeline - 1) // args.pipeline
        enc_alg /= nchunks
        dec_alg /= nchunks
    enc_main = "encode_bucket" if "encode_bucket" in kern else "encode_general"
    dec_main = next((k_ for k_ in ("decode_elias", "decode_fixed", "decode_general") if k_ in kern), None)
    enc_total = kern[enc_main]["ms_total"]
    dec_total = kern[dec_main]["ms_total"] if dec_main else 0.0
    if enc_total >= dec_total:
        dom, dom_alg = enc_main, enc_alg
    else:
        dom, dom_alg = dec_main, dec_alg
    traffic, valu_rate, counter_file = ({}, {}, None) if (args.layout or args.pipeline or args.n) \
        else hbm_traffic(w.name, n)

    def roof(kname, alg):
        ach = alg / (kern[kname]["ms_avg"] * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": kname, "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                # the two counter figures are NOT measured by this run: they are read from the
                # committed summary named in counters_source (null when it does not match the
                # workload, its size or the kernel sources)
                "traffic": traffic.get(kname),
                "valu_inst_per_simd_per_4clk": valu_rate.get(kname),
                "counters_source": counter_file,
                "bytes_per_launch": alg,
                "avg_launch_ms": round(kern[kname]["ms_avg"], 4)}

    roofline = roof(dom, dom_alg)
    other, other_alg = (dec_main, dec_alg) if dom == enc_main else (enc_main, enc_alg)
    roofline_other = roof(other, other_alg) if other else None

    # ---- copy ceiling of this machine, for context (the library's copy kernel) ----------------
    src = grads[0]
    dst = torch.empty_like(src)
    for _ in range(2):
        q.qsgd_copy_probe(dst, src)
    torch.cuda.synchronize()
    q.qsgd_timing_reset()
    q.qsgd_timing_enable(True)
    for _ in range(5):
        q.qsgd_copy_probe(dst, src)
    torch.cuda.synchronize()
    q.qsgd_timing_enable(False)
    copy_ms, copy_cnt = q.qsgd_timing_get("copy_probe")
    q.qsgd_timing_reset()
    copy_gbps = copy_cnt * 8.0 * n_arena / (copy_ms * 1e-3) / 1e9
    # the second kernel of known traffic (4-byte requests), so that a hardware-counter run of
    # this command holds both calibration points; on a slice, it is not a bandwidth figure
    nw = min(n_arena, 1 << 26)
    q.qsgd_copy_probe_words(dst[:nw], src[:nw])
    torch.cuda.synchronize()
    del dst

    # ---- the oracle on the host cores, on a bounded sample of the same workload, and the ----
    # ---- GPU results over that sample compared with what the oracle computed ----------------
    cpu, parity = None, None
    if not args.no_cpu_baseline and args.layout:
        from oracle import qsgd_oracle as qo

        def run_oracle_layout(T):   # the first T tensors of the arena
            sub = tensors[:T]
            na = sub[-1][0] + sub[-1][1]
            gs = [grads[k][:na].cpu().numpy() for k in range(K)]
            xs = x[:na].cpu().numpy()
            t0 = time.perf_counter()
            ms_ = [qo.encode_layout(qo.Params(n=na, s=w.s, d=w.d, code=w.code, seed=w.seed,
                                              stream_id=k), sub, args.bypass, gs[k])
                   for k in range(K)]
            qo.sgd_step_layout(sub, args.bypass, ms_, w.eta, xs)
            return sum(t[1] for t in sub), time.perf_counter() - t0

        T, (ns, t_cpu) = 1, run_oracle_layout(1)
        while T < len(tensors) and t_cpu < 0.25 * cpu_seconds:
            T = min(len(tensors), 2 * T)
            ns, t_cpu = run_oracle_layout(T)
        cpu = {"value": round(4.0 * K * ns / t_cpu / 1e9, 5), "unit": "GB/s", "cores": 1,
               "kind": "oracle",
               "sample": f"first {T} tensors ({ns} elements) of each of the {K} gradients: {K} x "
                         f"encode + 1 x decode+step, {t_cpu:.1f} s single-threaded"}
    elif not args.no_cpu_baseline and not args.pipeline:
        from oracle import compare
        from oracle import qsgd_oracle as qo
        d_eff = min(w.d, n)
        nb_all = (n + d_eff - 1) // d_eff
        table_words = 0 if w.code == W.CODE_FIXED else (nb_all + 1 + 3) // 4 * 4

        def run_oracle(ns):
            ns = max(d_eff, ns - ns % d_eff) if ns < n else n
            ws_ = W.scaled(w, ns) if ns < n else w
            gs = [grads[k][:ns].cpu().numpy() for k in range(K)]
            xs = x[:ns].cpu().numpy()
            t0 = time.perf_counter()
            ms_ = [qo.encode(qo.Params(n=ns, s=w.s, d=ws_.d, code=w.code, seed=w.seed,
                                       stream_id=k), gs[k]) for k in range(K)]
            x_want = qo.sgd_step(ms_, w.eta, xs)
            return ns, time.perf_counter() - t0, gs, ms_, x_want

        ns0, t_probe, gs, ms_, x_want = run_oracle(min(n, max(d_eff, 1 << 16)))
        ns = int(min(n, ns0 * cpu_seconds / max(t_probe, 1e-3)))
        if ns > ns0:
            ns, t_cpu, gs, ms_, x_want = run_oracle(ns)
        else:
            ns, t_cpu = ns0, t_probe
        cpu = {"value": round(4.0 * K * ns / t_cpu / 1e9, 5), "unit": "GB/s", "cores": 1,
               "kind": "oracle",
               "sample": f"first {ns} elements of each of the {K} gradients: {K} x encode + 1 x "
                         f"decode+step, {t_cpu:.1f} s single-threaded"}
        # parity over the same sample: the messages the timed steps left behind (buckets
        # 0 .. ns/d of each), and x over those buckets after one more fused step from the
        # state the oracle started from
        nbs = (ns + d_eff - 1) // d_eff
        parity = {"elements": 0, "near_ties": 0, "norm_mismatches": 0, "messages_identical": True}
        full = (qo.max_encoded_bytes(qo.Params(n=d_eff, s=w.s, d=d_eff, code=w.code)) - 64) // 4
        for k in range(K):
            pr = qo.Params(n=ns, s=w.s, d=d_eff if ns < n else w.d, code=w.code, seed=w.seed,
                           stream_id=k)
            if w.code == W.CODE_FIXED:
                tab = None
                hi_w = sizes[k] // 4 if ns == n else 16 + nbs * full
                strings = msgs[k][16:hi_w].cpu().numpy().view(np.uint32)
            else:
                tab = msgs[k][16:16 + nbs + 1].cpu().numpy().view(np.uint32)
                pay = 16 + table_words
                strings = msgs[k][pay + int(tab[0]):pay + int(tab[-1])].cpu().numpy().view(np.uint32)
            ref = ms_[k]              # what the timed oracle leg produced for this sample
            rpay = qo.payload_offset_words(ref)
            same = strings.size == ref.size - rpay and np.array_equal(strings, ref[rpay:]) and \
                (tab is None or np.array_equal(tab.astype(np.int64) - int(tab[0]),
                                               ref[16:16 + nbs + 1].astype(np.int64)))
            if same:
                parity["elements"] += int(ns)
            else:                     # classifies every difference; raises on a real one
                r = compare.compare_bucket_run(pr, gs[k], 0, tab, strings)
                for key in ("elements", "near_ties", "norm_mismatches"):
                    parity[key] += r[key]
                parity["messages_identical"] = False
        step()
        torch.cuda.synchronize()
        assert q.qsgd_workspace_status(ws) == 0
        got = x[:ns].cpu().numpy()
        parity["x_elements"] = int(ns)
        parity["x_mismatches"] = int(np.count_nonzero(got.view(np.uint32) != x_want.view(np.uint32)))
        parity["sample"] = f"first {ns} elements ({nbs} buckets) of each of the {K} messages and of x"
        log(f"parity: {parity}")
        if parity["near_ties"] > 1e-6 * parity["elements"] or \
                parity["norm_mismatches"] > 1e-6 * parity["elements"] or parity["x_mismatches"]:
            raise SystemExit(f"bench.py: GPU results differ from the oracle: {parity}")
        del gs, ms_, x_want, got

    rec = {
        "value": round(value, 2), "unit": "GB/s", "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": f"{w.name}: n={n}, s={w.s}, d={w.d}, "
                               f"code={['sparse Elias', 'dense Elias', 'fixed width'][w.code]}, K={K}"
                               + (f", tensor-aware ({len(tensors)} tensors, raw below {args.bypass})"
                                  if args.layout else "")
                               + (f", double-buffered in chunks of {args.pipeline}"
                                  if args.pipeline else "")
                               + (", step replayed from a HIP graph" if args.graph else ""),
                   "n": n, "s": w.s, "d": w.d, "K": K, "eta": w.eta,
                   "bits_per_element": round(8 * msg_bytes_avg / n, 4),
                   "message_bytes": int(msg_bytes_avg)},
        "encode_GBps": round(enc_gbps, 1), "encode_frac_hbm_peak": round(enc_gbps / HBM_PEAK_GBPS, 4),
        "decode_step_GBps": round(dec_gbps, 1),
        "encode_ms_per_message": round(enc_ms, 4), "decode_step_ms": round(dec_ms, 4),
        "copy_ceiling_GBps": round(copy_gbps, 1),
        "roofline": roofline, "roofline_other": roofline_other,
        "kernels": {k_: {"ms_avg": round(v["ms_avg"], 4), "launches": v["launches"]}
                    for k_, v in kern.items()},
        "parity": parity,
        "cpu_baseline": cpu,
    }
    del grads, x, msgs, ws
    gc.collect()
    torch.cuda.empty_cache()
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None,
                    help="c1..c5; default: c5 (n=1e9, s=4, d=8192, K=16) as the headline and c3 "
                         "(n=143M, fixed width, K=16) as a second leg under the key \"c3\"")
    ap.add_argument("--n", type=int, default=0, help="shrink the workload to n elements (debug)")
    ap.add_argument("--layout", action="store_true",
                    help="tensor-aware messages: the workload's tensors in an arena, tensors "
                         "below --bypass elements sent raw, buckets restart at every tensor")
    ap.add_argument("--bypass", type=int, default=10_000)
    ap.add_argument("--pipeline", type=int, default=0, metavar="CHUNK",
                    help="double-buffered pass: chunks of CHUNK elements (a multiple of d), the "
                         "encodes of one chunk overlapping decode+step of the previous one")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (for the small, "
                         "launch-bound workloads); per-kernel times then come from one extra eager "
                         "step after the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg (its timing and the parity record)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="target CPU time of the oracle baseline sample")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (the K peers' messages are K buffers "
            "resident on it); --gpus must be 1")
        return 2

    import numpy as np
    import torch

    import paper_1610_02132_amd as q
    from paper_1610_02132_amd import workloads as W

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    torch.cuda.set_device(0)

    headline = args.workload or "c5"
    second = None if (args.workload or args.n or args.layout or args.pipeline or args.graph) else "c3"
    rec = measure(args, headline, torch, np, q, W, args.cpu_seconds)
    out = {
        "metric": "Encode and Decode+accumulate GB/s of fp32 gradient; % of MI355X HBM peak",
        "value": rec.pop("value"), "unit": rec.pop("unit"), "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": rec.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    out.update(rec)
    if second:
        r2 = measure(args, second, torch, np, q, W, 0.5 * args.cpu_seconds)
        out[second] = r2
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
