"""Full-size parity: the 8B-shaped decoder in the launch configuration the benchmark times
(batch 64, lognormal contexts), plus the batch-512 mixed population and the 32k-context batch,
checked on sampled requests that the CPU oracle computes one by one, and by properties that hold
for every row.  (The 70B-shaped case lives in test_gpu_3_full_size_70b.py so that this module's 8B
model is released first.)  Needs a real MI355X: run with -m gpu."""
import os
import time

import numpy as np
import pytest
import torch

import chiron_oracle as orc
import sample_step
from helpers import bf16_to_f32, bits
from paper_2501_08090_amd import inputs as I

pytestmark = pytest.mark.gpu
STEP_TOL = 2e-2   # max|dlogit| <= 2e-2 * std(oracle logits); greedy argmax agrees on >= 99% of rows


def _mods():
    from paper_2501_08090_amd import binding as B, workloads as W
    return B, W


@pytest.fixture(scope="module")
def model8b():
    B, W = _mods()
    t0 = time.time()
    model, w_host = W.build_model(I.LLAMA_8B, seed=0, max_batch=4096, max_blocks_per_seq=2049, host_weights=True,
                                  log=lambda *a: print(*a, flush=True))
    print("8B model built in %.1f s" % (time.time() - t0), flush=True)
    yield model, w_host
    model.close()


def check_workload(name, model8b, sample, batches):
    B, W = _mods()
    model, w_host = model8b
    t0 = time.time()
    wl = W.build(name, seed=0, host_seqs=sample, model=model, w_host=w_host, log=lambda *a: print(*a, flush=True))
    print("%s: cache built in %.1f s (%d context tokens)" % (name, time.time() - t0, wl.context_tokens), flush=True)
    B.validate_step_inputs(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens)
    logits = B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens)
    torch.cuda.synchronize()
    got = logits[sample].cpu().numpy()
    print("oracle on requests", sample, "lengths", wl.lens[sample].tolist(), flush=True)
    want, opool, obt, dt = sample_step.run(wl.m, wl.w_host, wl.kv_host, wl.lens[sample], wl.tok[sample])
    sig = want.std()
    err = np.abs(got - want).max() / sig
    agree = (got.argmax(1) == want.argmax(1)).mean()
    print("%s: sampled rows max|d|/sigma = %.3e, argmax agreement %.3f, oracle %.1f s" % (name, err, agree, dt), flush=True)
    assert err <= STEP_TOL and agree >= 0.99
    # every row: finite, and on the scale of the sampled rows
    full = logits.float()
    assert bool(torch.isfinite(full).all())
    rs = full.std(dim=1).cpu().numpy()
    assert np.all(np.abs(rs / rs[sample].mean() - 1) < 0.25)
    # slot contract on the sampled requests: old positions untouched (bit-exact against the generated cache),
    # the new position holds the oracle's k, v up to one bf16 ulp
    starts = np.concatenate([[0], np.cumsum(wl.lens[sample].astype(np.int64))])
    for r, i in enumerate(sample):
        L = int(wl.lens[i])
        for l in (0, wl.m["n_layers"] - 1):
            k, v = wl.pool.gather(l, wl.block_table[i].contiguous(), L + 1)
            ok, ov = orc.gather_kv(opool, l, obt[r], L + 1)
            assert np.array_equal(bits(k)[:L], wl.kv_host[l][0][starts[r]:starts[r + 1]])
            assert np.array_equal(bits(v)[:L], wl.kv_host[l][1][starts[r]:starts[r + 1]])
            for a, b in ((bits(k)[L], ok[L]), (bits(v)[L], ov[L])):
                fa, fb = bf16_to_f32(a), bf16_to_f32(b)
                assert np.all(np.abs(fa - fb) <= np.abs(fb) * 2.0 ** -7 + 1e-3 * np.abs(fb).max())
    # a prefix of the batch gives the same rows (this is how the batch-size sweep is run).  Both runs are within
    # tolerance of the oracle; they differ from each other by the order of partial sums (the tiling depends on the row
    # count), which is ~1e-4 sigma, except in rows where that moves a new k or v element across a bf16 rounding
    # boundary: the element lands on the other bf16 neighbour, and the row moves by a few 1e-3 sigma.  Checked here:
    # every row that differs by more than 2e-3 sigma is a row whose freshly written K/V bits differ between the runs.
    def new_slot_bits(rows):
        out = {}
        for i in rows:
            L = int(wl.lens[i])
            last_page = wl.block_table[i][L // 16:].contiguous()   # the row from the page that holds position L on
            out[i] = [np.concatenate([bits(t)[L % 16].ravel() for t in wl.pool.gather(l, last_page, L % 16 + 1)])
                      for l in range(wl.m["n_layers"])]
        return out
    for b in batches:
        sub = B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, batch=b)
        drow = ((sub - logits[:b]).abs().amax(dim=1) / sig).cpu().numpy()
        moved = [int(i) for i in np.nonzero(drow > 2e-3)[0]]
        print("prefix batch %d vs full batch: max|d|/sigma = %.2e, rows above 2e-3: %s" % (b, drow.max(), moved), flush=True)
        assert drow.max() <= 1e-2
        if moved:
            bits_prefix = new_slot_bits(moved)
            B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens)   # the full batch again: rewrites every new slot
            bits_full = new_slot_bits(moved)
            for i in moved:
                flipped = sum(int((a != c).sum()) for a, c in zip(bits_prefix[i], bits_full[i]))
                print("  row %d: %d new k/v elements on different bf16 neighbours" % (i, flipped), flush=True)
                assert flipped > 0, "row %d moved by %.1e sigma without a differing k/v element" % (i, drow[i])
    wl.pool.close()
    del wl
    torch.cuda.empty_cache()


def test_8b_batch64_lognormal(model8b):
    lens = I.population("b64", 64, 0)
    sample = sorted({0, 1, int(lens.argmin()), int(lens.argmax()), 31, 63} | set(range(5, 64, 7)))   # 15 of the 64 rows
    check_workload("llama8b-b64-lognormal800", model8b, sample, batches=(1, 8, 33))


def test_8b_batch64_multi_token_step(model8b):
    """The verify shape of speculative decoding at full size: 64 requests x 4 new tokens (256 rows; 4 tokens x 4 query
    heads per KV head fill the 16 operand columns of the attention kernel, so a request's pages are read once).
    The last three cached tokens of every request are treated as not yet cached, so that the four new positions
    lie in pages the workload has allocated."""
    B, W = _mods()
    model, w_host = model8b
    T = 4
    sample = [0, 31, 63]
    wl = W.build("llama8b-b64-lognormal800", seed=0, host_seqs=sample, model=model, w_host=w_host)
    lens = (wl.lens - (T - 1)).astype(np.int32)
    toks = I.token_ids(wl.batch * T, wl.m["vocab"], 9).reshape(wl.batch, T)
    logits = B.decode_step_multi(wl.model, wl.pool, wl.block_table, torch.from_numpy(lens).cuda(), torch.from_numpy(toks).cuda())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(logits).all())
    got = logits[sample].cpu().numpy().reshape(len(sample) * T, -1)
    starts = np.concatenate([[0], np.cumsum(wl.lens[sample].astype(np.int64))])
    keep = np.concatenate([np.arange(starts[r], starts[r] + lens[i]) for r, i in enumerate(sample)])
    kv = [(k[keep], v[keep]) for k, v in wl.kv_host]
    want, _, _, dt = sample_step.run(wl.m, wl.w_host, kv, lens[sample], toks[sample], q_len=T)
    want = want.reshape(len(sample) * T, -1)
    err = np.abs(got - want).max() / want.std()
    agree = (got.argmax(1) == want.argmax(1)).mean()
    print("multi-token: sampled rows max|d|/sigma = %.3e, argmax agreement %.3f, oracle %.1f s" % (err, agree, dt), flush=True)
    assert err <= STEP_TOL and agree >= 0.99
    # token 0 of every request is what a single-token step computes at the same state (pool rewritten identically)
    one = B.decode_step(wl.model, wl.pool, wl.block_table, torch.from_numpy(lens).cuda(),
                        torch.from_numpy(np.ascontiguousarray(toks[:, 0])).cuda())
    d = (one - logits[:, 0]).abs().max().item() / want.std()
    print("token 0 vs single-token step: max|d|/sigma = %.2e" % d, flush=True)
    assert d <= 1e-2


def test_8b_batch512_mixed_population(model8b):
    lens = I.population("mixed", 512, 0)
    sample = sorted({0, 3, int(lens.argmin()), 255, 511} | set(range(40, 512, 67)))   # 12 rows across the four 128-row tiles
    check_workload("llama8b-mixed-sweep512", model8b, sample, batches=(1, 128))


def test_8b_batch2048_interactive_population(model8b):
    """The large-batch regime (batch-class instances in the paper run at 2048-4096): 2048 requests with
    interactive-length contexts, 186 GB of cache."""
    free, _ = torch.cuda.mem_get_info()
    if free < 215e9:
        pytest.skip("needs 215 GB of free HBM, %.0f GB available" % (free / 1e9))
    lens = I.population("interactive", 2048, 0)
    sample = sorted({0, int(lens.argmin()), int(lens.argmax()), 1023, 2047})
    check_workload("llama8b-interactive-sweep2048", model8b, sample, batches=(1024,))


def test_8b_batch4096_short_population(model8b):
    """The upper end of the batch sizes the paper reports for batch-class instances (2048-4096): 4096 requests with
    short contexts (lognormal, median 256 tokens), 190 GB of cache; 32 M-tiles of the large-batch projection kernels."""
    free, _ = torch.cuda.mem_get_info()
    if free < 225e9:
        pytest.skip("needs 225 GB of free HBM, %.0f GB available" % (free / 1e9))
    lens = I.population("short", 4096, 0)
    sample = sorted({0, int(lens.argmin()), int(lens.argmax()), 2047, 4095})
    check_workload("llama8b-short-sweep4096", model8b, sample, batches=(3000,))


def test_8b_batch32_long_context(model8b):
    check_workload("llama8b-b32-long32k", model8b, [0, 31], batches=(8,))


def test_8b_width_two_layers_every_row_of_batch512():
    """Every width of the 8B shape (hidden 4096, 32q/8kv heads of 128, FFN 14336, vocabulary 128256) with two layers,
    all 512 requests of the mixed population against the oracle: max|d|/sigma and the argmax agreement are taken
    over 512 rows, and every row tile and row position of the large-batch kernels is compared element by element.
    Prefix batches cross the other row-tile shapes (96-row tiles at 65..96 and 129..192 rows, 128-row tiles above)."""
    B, W = _mods()
    t0 = time.time()
    wl = W.build("llama8b-width-2layers-mixed512", seed=0, host_seqs=list(range(512)), host_weights=True, gain_jitter=0.1,
                 log=lambda *a: print(*a, flush=True))
    print("two-layer 8B-width workload built in %.1f s (%d context tokens)" % (time.time() - t0, wl.context_tokens), flush=True)
    logits = B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens)
    torch.cuda.synchronize()
    got = logits.cpu().numpy()
    want, _, _, dt = sample_step.run(wl.m, wl.w_host, wl.kv_host, wl.lens, wl.tok)
    sig = want.std()
    err = np.abs(got - want).max(axis=1) / sig
    agree = got.argmax(1) == want.argmax(1)
    print("all 512 rows: max|d|/sigma = %.3e (worst row %d), argmax agreement %d/512, oracle %.1f s" % (
        err.max(), int(err.argmax()), int(agree.sum()), dt), flush=True)
    assert err.max() <= STEP_TOL and agree.mean() >= 0.99
    for b in (65, 150, 257, 400):
        sub = B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, batch=b).cpu().numpy()
        e = np.abs(sub - want[:b]).max() / sig
        a = (sub.argmax(1) == want[:b].argmax(1)).mean()
        print("prefix batch %d: max|d|/sigma = %.3e, argmax agreement %.4f" % (b, e, a), flush=True)
        assert e <= STEP_TOL and a >= 0.99
    # the other form of the feed-forward intermediate (tiled bf16 terms written by the gate/up epilogue, which the step
    # takes from 513 rows on at this width), forced here so that all 512 rows and a ragged 300 are checked through it
    B.set_tuning("linear_big_min_m", 97)
    try:
        for b in (512, 300):
            sub = B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, batch=b).cpu().numpy()
            e = np.abs(sub - want[:b]).max() / sig
            a = (sub.argmax(1) == want[:b].argmax(1)).mean()
            print("tiled intermediate, batch %d: max|d|/sigma = %.3e, argmax agreement %.4f" % (b, e, a), flush=True)
            assert e <= STEP_TOL and a >= 0.99
    finally:
        B.set_tuning("linear_big_min_m", 0)
    wl.pool.close()
    wl.model.close()
    del wl
    torch.cuda.empty_cache()


def test_local_autoscaler_closed_loop_on_the_mixed_population(model8b):
    """Alg. 1 driven by the measured curve: ITL = median step latency at the current maximum batch size,
    throughput = batch / ITL, both from chiron_step_latency_profile on prefixes of the 512-request mixed
    population.  The SLO is the measured latency at batch 128.  Asserted here is only what holds for any measured
    curve: every update equals the oracle's for the same observations (exact), the batch size grows or stays when
    the backpressure the library returned is below one and shrinks when it is at or above one, and it stays within
    [1, limit].  Where the loop settles depends on the device's timings and is printed, not asserted (the
    trajectory's shape is tested on fixed curves in test_autoscale.py).  Both caller policies are run: Alg. 1 as
    printed (the previous tick's throughput always enters TBP) and the one the benchmark uses (a tick that did not
    scale up leaves no comparable previous throughput, so the next tick passes none)."""
    B, W = _mods()
    model, w_host = model8b
    wl = W.build("llama8b-mixed-sweep512", seed=0, model=model, w_host=w_host)
    prof = lambda b: B.step_latency_profile(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, [b], warmup=1, iters=3)[0]
    slo = prof(128)["lat_ms_median"] * 1e-3
    limit = 512
    for policy in ("as-printed", "reset-after-no-growth"):
        mbs, tput_prev, traj = 1, 0.0, []
        for tick in range(40):
            pt = prof(mbs)
            itl, tput = pt["lat_ms_median"] * 1e-3, pt["tokens_per_s"]
            assert itl > 0 and tput > 0
            new, lb = B.local_autoscale_step(itl, slo, tput_prev, tput, mbs, limit)
            assert (new, lb) == orc.autoscale_step(itl, slo, tput_prev, tput, 0.5, limit, mbs)
            # the rule, on the exact backpressure the library returned (rounded only for printing below)
            assert 1 <= new <= limit
            assert (new >= mbs) if lb < 1.0 else (new < mbs or mbs == 1)
            traj.append((mbs, round(itl * 1e3, 3), round(lb, 4), new))
            tput_prev = tput if (policy == "as-printed" or new > mbs) else 0.0
            mbs = new
        print("policy %s, SLO %.3f ms; (batch, itl ms, backpressure, next batch):" % (policy, slo * 1e3), traj, flush=True)
    wl.pool.close()
    del wl
    torch.cuda.empty_cache()
