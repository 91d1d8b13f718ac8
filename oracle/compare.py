"""Comparison of a message made by the GPU library with the CPU oracle's message for
the same input -- TEST INFRASTRUCTURE ONLY (tests, the smoke check and the oracle leg of
the benchmark).  Uses the oracle and numpy, nothing of the GPU package.

Rule: levels, signs, scales, strings and the offset table must be identical.  The one
exception is the near-tie element: the oracle's draw u lies within 1e-5 of its round-up
probability p, where the last bit of the bucket scale (summed in another order on the
GPU) may tip the comparison u < p.  Such elements are counted, and so are buckets whose
32-bit scale differs (by one rounding at most); the caller bounds the counts (at most
1e-6 of the elements).  Every other difference raises AssertionError.
"""
from __future__ import annotations

import numpy as np

from . import qsgd_oracle as qo

H_WORDS, H_PW_LO, H_PW_HI = 16, 12, 13
NEAR_TIE = 1e-5


def _strings_and_table(words: np.ndarray, p: qo.Params):
    """(table of nb+1 word offsets, string words) of a complete message."""
    nb = qo.num_buckets(p)
    pay = qo.payload_offset_words(words)
    if p.code == qo.CODE_FIXED:
        d = qo.bucket_size(p)
        full = (qo.max_encoded_bytes(qo.Params(n=d, s=p.s, d=d, code=p.code, norm=p.norm)) - 64) // 4
        table = np.arange(nb + 1, dtype=np.int64) * full
        table[nb] = words.size - pay
    else:
        table = words[H_WORDS:H_WORDS + nb + 1].astype(np.int64)
    return table, words[pay:]


def compare_encode(p: qo.Params, g_host: np.ndarray, gpu_words: np.ndarray,
                   index_offset: int = 0) -> dict:
    """`gpu_words`: a complete message for exactly the parameters p (n = g_host.size), made
    from g_host drawn at positions index_offset.. of a longer vector.  Returns
    dict(elements, near_ties, norm_mismatches, identical)."""
    g_host = np.ascontiguousarray(g_host, dtype=np.float32)
    assert g_host.size == p.n
    ref = qo.encode_slice(p, g_host, index_offset) if index_offset else qo.encode(p, g_host)
    out = dict(elements=int(p.n), near_ties=0, norm_mismatches=0, identical=True)
    if ref.size == gpu_words.size and np.array_equal(ref, gpu_words):
        return out
    out["identical"] = False
    # not byte-identical: every difference must trace back to a near-tie or a scale rounding
    hdr = np.ones(H_WORDS, dtype=bool)
    hdr[[H_PW_LO, H_PW_HI]] = False          # the length may differ with a flipped level
    assert np.array_equal(ref[:H_WORDS][hdr], gpu_words[:H_WORDS][hdr]), "headers differ"
    tup = qo.decode_tuple(gpu_words)          # raises if the GPU message does not parse
    qz = qo.quantize(p, g_host, want_draws=True, index_offset=index_offset)
    d, nb = qo.bucket_size(p), qo.num_buckets(p)
    norm_diff = tup["norms"].view(np.uint32) != qz["norms"].view(np.uint32)
    rel = np.abs(tup["norms"].astype(np.float64) - qz["norms"]) / np.maximum(qz["norms"], 1e-300)
    assert np.all(rel[norm_diff] <= 1.2e-7), "a bucket scale differs by more than one rounding"
    lev_diff = tup["levels"] != qz["levels"]
    sent = (np.ones(p.n, dtype=bool) if p.code != qo.CODE_SPARSE
            else (qz["levels"] != 0) & (tup["levels"] != 0))
    assert not (sent & (tup["neg"] != qz["neg"])).any(), "sign bits differ"
    idx = np.flatnonzero(lev_diff)
    assert np.all(np.abs(tup["levels"][idx].astype(np.int64) - qz["levels"][idx].astype(np.int64)) == 1), \
        "a level differs by more than one step"
    tie = np.abs(qz["u"][idx].astype(np.float64) - qz["p"][idx].astype(np.float64)) <= NEAR_TIE
    assert np.all(tie & (qz["p"][idx] >= 0)), \
        f"{int((~tie).sum())} levels differ away from a rounding threshold"
    out["near_ties"] = int(idx.size)
    out["norm_mismatches"] = int(norm_diff.sum())
    # every bucket without such a difference: same string, same length (so the offset tables
    # agree once the length changes of the other buckets are taken out)
    dirty = norm_diff.copy()
    dirty[idx // d] = True
    assert dirty.any(), "messages differ but no level or scale does (layout mismatch)"
    tab_g, str_g = _strings_and_table(gpu_words, p)
    tab_r, str_r = _strings_and_table(ref, p)
    assert tab_g[0] == tab_r[0] == 0 and np.all(np.diff(tab_g) > 0), "offset table is not increasing"
    assert tab_g[nb] == str_g.size and tab_r[nb] == str_r.size
    clean = ~dirty
    assert np.array_equal(np.diff(tab_g)[clean], np.diff(tab_r)[clean]), "string lengths differ"
    edges = np.flatnonzero(np.diff(np.concatenate(([False], clean, [False])).astype(np.int8)))
    for a, b in zip(edges[0::2], edges[1::2]):     # runs [a, b) of clean buckets
        assert np.array_equal(str_g[tab_g[a]:tab_g[b]], str_r[tab_r[a]:tab_r[b]]), \
            f"strings of buckets {a}..{b - 1} differ"
    return out


def compare_bucket_run(p_run: qo.Params, g_run: np.ndarray, index_offset: int,
                       gpu_table, gpu_strings: np.ndarray) -> dict:
    """Buckets [b0, b1) of a longer GPU message against the oracle's message of the slice
    g_run (which starts at position index_offset = b0 * d of the whole vector).
    gpu_table: the b1 - b0 + 1 table entries of those buckets (None for the fixed width),
    gpu_strings: their string words.  Fast path: words and rebased table equal the
    oracle's; otherwise the run is re-wrapped as a message of its own (the oracle's
    header for the slice, the GPU's table and strings) and goes through compare_encode."""
    g_run = np.ascontiguousarray(g_run, dtype=np.float32)
    ref = qo.encode_slice(p_run, g_run, index_offset)
    pay = qo.payload_offset_words(ref)
    nb = qo.num_buckets(p_run)
    if gpu_table is not None:
        table = np.asarray(gpu_table, dtype=np.int64) - int(gpu_table[0])
        same_table = np.array_equal(table, ref[H_WORDS:H_WORDS + nb + 1].astype(np.int64))
    else:
        table, same_table = None, True
    if same_table and gpu_strings.size == ref.size - pay and np.array_equal(gpu_strings, ref[pay:]):
        return dict(elements=int(p_run.n), near_ties=0, norm_mismatches=0, identical=True)
    wrapped = ref[:pay].copy()
    if table is not None:
        assert table.size == nb + 1 and table[0] == 0 and np.all(np.diff(table) > 0) \
            and table[-1] == gpu_strings.size, "offset table of the run is not consistent"
        wrapped[H_WORDS:H_WORDS + nb + 1] = table.astype(np.uint32)
    wrapped[H_PW_LO] = gpu_strings.size & 0xFFFFFFFF
    wrapped[H_PW_HI] = gpu_strings.size >> 32
    return compare_encode(p_run, g_run, np.concatenate([wrapped, gpu_strings]), index_offset)


def structure_check(words: np.ndarray, p: qo.Params) -> None:
    """Properties every message has, read from the message alone (any size): the header's
    length, an increasing offset table that ends at the payload length, and for Code_s a
    stop mark in the last word of every string."""
    hp, total = qo.message_info(words[:H_WORDS])
    assert (hp.n, hp.s, hp.d, hp.code, hp.norm) == (p.n, p.s, qo.bucket_size(p), p.code, p.norm)
    assert total == 4 * words.size, "header length and message length differ"
    nb = qo.num_buckets(p)
    if p.code == qo.CODE_FIXED:
        return
    pay = H_WORDS + (nb + 1 + 3) // 4 * 4
    table = words[H_WORDS:H_WORDS + nb + 1].astype(np.int64)
    assert table[0] == 0 and np.all(np.diff(table) > 0), "offset table is not increasing"
    assert table[nb] == words.size - pay, "offset table does not end at the payload length"
    assert not words[H_WORDS + nb + 1:pay].any(), "table padding is not zero"
    if p.code == qo.CODE_SPARSE and qo.bucket_size(p) <= 8192:
        assert np.all(words[pay + table[1:] - 1] != 0), "a string has no stop mark in its last word"


def compare_layout(p: qo.Params, tensors, bypass_below: int, arena: np.ndarray,
                   gpu_words: np.ndarray) -> dict:
    """A tensor-aware message (small tensors raw, buckets restart at every tensor) against
    the oracle.  Not identical: the raw values must still be, and every quantized tensor's
    run of buckets goes through compare_bucket_run (a tensor is quantized like a vector of
    its own with the draws of its arena positions)."""
    arena = np.ascontiguousarray(arena, dtype=np.float32)
    ref = qo.encode_layout(p, tensors, bypass_below, arena)
    out = dict(elements=int(sum(sz for _, sz in tensors)), near_ties=0, norm_mismatches=0,
               identical=True)
    if ref.size == gpu_words.size and np.array_equal(ref, gpu_words):
        return out
    out["identical"] = False
    hdr = np.ones(H_WORDS, dtype=bool)
    hdr[[H_PW_LO, H_PW_HI]] = False
    assert np.array_equal(ref[:H_WORDS][hdr], gpu_words[:H_WORDS][hdr]), "headers differ"
    nb, raw = qo.layout_counts(p, tensors, bypass_below)
    d = p.d
    fixed = p.code == qo.CODE_FIXED
    if fixed:
        full = (qo.max_encoded_bytes(qo.Params(n=d, s=p.s, d=d, code=p.code, norm=p.norm)) - 64) // 4
        pay = H_WORDS
        tab = np.arange(nb + 1, dtype=np.int64) * full
    else:
        pay = H_WORDS + (nb + 1 + 3) // 4 * 4
        tab = gpu_words[H_WORDS:H_WORDS + nb + 1].astype(np.int64)
        assert tab[0] == 0 and np.all(np.diff(tab) > 0), "offset table is not increasing"
    strings_len = int(tab[nb])
    assert gpu_words.size == pay + strings_len + raw, "message length does not fit its parts"
    assert np.array_equal(gpu_words[pay + strings_len:], ref[ref.size - raw:]), "raw values differ"
    b = 0
    for off, size in tensors:
        off, size = int(off), int(size)
        if size < bypass_below:
            continue
        nbt = (size + d - 1) // d
        p_t = qo.Params(n=size, s=p.s, d=d, code=p.code, norm=p.norm, seed=p.seed,
                        stream_id=p.stream_id, iteration=p.iteration)
        g_t = arena[off:off + size]
        strings = gpu_words[pay + int(tab[b]):pay + int(tab[b + nbt])]
        if fixed:    # a short last bucket still owns a full slot, zero padded
            used = qo.encode_slice(p_t, g_t, off).size - H_WORDS
            assert not strings[used:].any(), "padding of a short bucket's slot is not zero"
            r = compare_bucket_run(p_t, g_t, off, None, strings[:used])
        else:
            r = compare_bucket_run(p_t, g_t, off, tab[b:b + nbt + 1], strings)
        out["near_ties"] += r["near_ties"]
        out["norm_mismatches"] += r["norm_mismatches"]
        b += nbt
    assert b == nb
    assert out["near_ties"] + out["norm_mismatches"] > 0, \
        "messages differ but no level or scale does (layout mismatch)"
    return out
