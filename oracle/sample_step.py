"""Runs the CPU oracle on a few requests of a large GPU-resident workload.

TEST INFRASTRUCTURE ONLY (tests and the benchmark's CPU-baseline leg).  The inputs are the
host copies that the workload builder kept of its own generated tensors: weights as bf16 bit
patterns, and the cache rows of the sampled requests.  The requests are laid out in a compact
pool of their own: physical page placement never changes the oracle's results (pinned by
tests/test_oracle_step.py), and each request's result is independent of the rest of the batch.
"""
import time

import numpy as np

import chiron_oracle as orc


def pages_needed(lens, bs=16):
    return (np.asarray(lens, np.int64) + 1 + bs - 1) // bs


def run(m, w_host, kv_host, lens, tokens, q_len=1):
    """lens/tokens: the sampled requests' context lengths and input tokens (tokens [n] or, with q_len > 1,
    [n, q_len]); kv_host[l] = (K, V) rows of those requests, sequence-major.
    Returns (logits, pool, block_table, seconds_of_the_step)."""
    cfg = orc.make_config(m, orc.BF16, orc.BF16)
    lens = np.asarray(lens, np.int32)
    need = pages_needed(lens + (q_len - 1))
    bt = np.full((len(lens), int(need.max())), -1, np.int32)
    o = 0
    for r, c in enumerate(need):
        bt[r, :c] = np.arange(o, o + c)
        o += c
    pool = orc.Pool(cfg, o, np.uint16)
    seq_idx = np.repeat(np.arange(len(lens), dtype=np.int32), lens)
    starts = np.concatenate([[0], np.cumsum(lens.astype(np.int64))[:-1]])
    pos = (np.arange(int(lens.sum()), dtype=np.int64) - np.repeat(starts, lens)).astype(np.int32)
    for l, (k, v) in enumerate(kv_host):
        kf = (k.astype(np.uint32) << 16).view(np.float32)
        vf = (v.astype(np.uint32) << 16).view(np.float32)
        orc.append_kv(pool, l, kf, vf, bt, seq_idx, pos)
    t0 = time.perf_counter()
    if q_len > 1:
        logits = orc.decode_step_multi(cfg, w_host, pool, bt, lens, np.asarray(tokens, np.int32).reshape(len(lens), q_len))
    else:
        logits, _ = orc.decode_step(cfg, w_host, pool, bt, lens, np.asarray(tokens, np.int32))
    return logits, pool, bt, time.perf_counter() - t0
