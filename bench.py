#!/usr/bin/env python3
"""Benchmark of the decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--sweep] [--no-cpu-baseline]

A "step" is one chiron_decode_step (every kernel of the path) over one batch of seeded synthetic
requests whose weights, cache and index arrays are already resident in HBM.  Prints ONE JSON line:
whole-job decode tokens/s, the roofline position of the dominant kernel (timed with the start/stop HIP
events that the library attaches to each kernel launch), and the CPU oracle timed on the host cores on a bounded sample of the
same workload.  Everything runs on one GPU; --gpus above 1 is refused.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

DEFAULT_WORKLOAD = "llama8b-b64-lognormal800"
CURVE_WORKLOAD = "llama8b-mixed-sweep512"   # same model shape: the curve the local autoscaler tunes
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/*_hbm_traffic.md), already scaled
# by what the same counters read for a plain 1 GiB copy.  Valid only for the kernel sources they were taken on:
# `sha` is the sha256 of the kernel's source file at that time; with any other source the figure is reported null.
TRAFFIC = {
    # (workload, kernel class): (source file, sha256, fetch bytes, write bytes)
    ("llama8b-b64-lognormal800", "attn"): ("attention.hip", "02217a164f11f306204df37f6e2b724792ba1bdb546d81105e6be8e84d6e4635", 275697032, 4259904),
    ("llama8b-b64-lognormal800", "gateup"): ("linear.hip", "05a738cc438354e18a9eb186fdc7e1c7d3925e12a706b569264088025053acdc", 243439145, 3670016),
    ("llama8b-b64-lognormal800", "down"): ("linear.hip", "05a738cc438354e18a9eb186fdc7e1c7d3925e12a706b569264088025053acdc", 121329453, 16777219),
    ("llama8b-mixed-sweep512", "attn"): ("attention.hip", "02217a164f11f306204df37f6e2b724792ba1bdb546d81105e6be8e84d6e4635", 4197918185, 37881916),
    ("llama8b-b32-long32k", "attn"): ("attention.hip", "02217a164f11f306204df37f6e2b724792ba1bdb546d81105e6be8e84d6e4635", 3723503215, 30211101),
}


def measured_traffic(workload, kclass):
    import hashlib
    ent = TRAFFIC.get((workload, kclass))
    if not ent:
        return None
    src, sha, fetch, write = ent
    path = os.path.join(ROOT, "paper_2501_08090_amd", "csrc", src)
    try:
        cur = hashlib.sha256(open(path, "rb").read()).hexdigest()
    except OSError:
        return None
    return dict(fetch_bytes=fetch, write_bytes=write, total_bytes=fetch + write) if cur == sha else None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


# the paper's inter-token-latency SLOs (Evaluation: workloads and SLOs): interactive requests 200 ms, batch requests 2 s
ITL_SLOS_MS = (("interactive", 200.0), ("batch", 2000.0))


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def kernel_algorithmic(m, batch, ctx_tokens):
    """per-launch algorithmic HBM bytes and flops of each kernel class (weights + fp32 activations in/out for the
    projections, the gate/up projection writing the F columns of silu(gate)*up at 4 bytes each; 4*n_kv*d bytes per
    attended token for attention)"""
    H, d, F, V = m["hidden"], m["head_dim"], m["ffn"], m["vocab"]
    qn, kn = m["n_q_heads"] * d, m["n_kv_heads"] * d
    M = batch

    def gemm(N, K, out_cols=None):
        act = 4 * M * K + 4 * M * (N if out_cols is None else out_cols)
        return dict(bytes=2 * N * K + act, act_bytes=act, flops=2 * M * N * K)

    return {
        "qkv": gemm(qn + 2 * kn, H), "o": gemm(H, qn), "gateup": gemm(2 * F, H, out_cols=F), "down": gemm(H, F),
        "lmhead": gemm(V, H),
        "attn": dict(bytes=4 * m["n_kv_heads"] * d * ctx_tokens, flops=4 * m["n_q_heads"] * d * ctx_tokens),
    }


def time_steps(B, wl, batch, steps, warmup, logits):
    import torch
    for _ in range(warmup):
        B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, logits=logits, batch=batch)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, logits=logits, batch=batch)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kernel_times(B, wl, batch, steps, logits):
    import torch
    torch.cuda.synchronize()
    B.kernel_timing_begin(wl.model)
    for _ in range(steps):
        B.decode_step(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, logits=logits, batch=batch)
    return B.kernel_timing_end(wl.model)


def cpu_baseline(wl, sample, gpu_logits):
    """Times the CPU oracle on the requests in `sample` (whole model) and compares its logits with the GPU's."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import chiron_oracle as orc
    import sample_step
    logits, _, _, dt = sample_step.run(wl.m, wl.w_host, wl.kv_host, wl.lens[sample], wl.tok[sample])
    sig = float(logits.std())
    err = float(np.abs(gpu_logits - logits).max() / sig)
    agree = float((gpu_logits.argmax(1) == logits.argmax(1)).mean())
    return dict(value=len(sample) / dt, unit="tokens/s", cores=orc.num_threads(), cpu=cpu_model(), kind="oracle",
                sample="requests %d..%d of the batch, all %d layers and the LM head, one step (%.1f s)" % (
                    sample[0], sample[-1], wl.m["n_layers"], dt),
                seconds=dt), dict(rows=len(sample), max_abs_err_over_sigma=err, argmax_agreement=agree)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--sweep", action="store_true", help="also time the batch-size sweep (prefixes of the batch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=32)
    ap.add_argument("--autoscale-slo-ms", type=float, default=0.0,
                    help="also run the local autoscaler (Alg. 1) closed loop on the measured curve with this ITL SLO")
    ap.add_argument("--q-len", type=int, default=0, help="also time the multi-token (verify) step with this many new tokens per request")
    ap.add_argument("--swap", action="store_true", help="also time evicting the longest request's cache to pinned host memory and back")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known bytes) so that rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE "
                         "readings of the kernels can be scaled by what the same counter reads for it")
    ap.add_argument("--batch", type=int, default=0, help="time a prefix of the workload's batch instead of all of it")
    ap.add_argument("--no-curve", action="store_true",
                    help="default workload only: skip the latency/throughput curve over batch sizes 1..512 of the mixed "
                         "population that is otherwise measured after the step (kernel profiles of the step use this)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: the library runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "Replicas scale by running one instance per GPU." % a.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2501_08090_amd import binding as B
    from paper_2501_08090_amd import workloads as W
    B.load()   # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")

    m0, kind, full_batch, _ = W.WORKLOADS[a.workload]
    batch = min(a.batch, full_batch) if a.batch > 0 else full_batch
    sample = list(range(min(a.cpu_sample, batch))) if not a.no_cpu_baseline else []
    t0 = time.time()
    curve = a.workload == DEFAULT_WORKLOAD and not a.no_curve and batch == full_batch
    cm, _, cbatch, _ = W.WORKLOADS[CURVE_WORKLOAD]
    wl = W.build(a.workload, seed=0, host_seqs=sample, host_weights=bool(sample), log=log,
                 max_batch=max(full_batch * max(1, a.q_len), cbatch if curve else 0),
                 max_blocks_per_seq=(8192 + 16) // 16 + 1 if curve else None)
    if batch != full_batch:
        wl.context_tokens = int(wl.lens[:batch].astype(np.int64).sum()) + batch
    log("workload %s built in %.1f s: batch %d, %d context tokens, pool %d pages" % (
        a.workload, time.time() - t0, batch, wl.context_tokens, wl.num_blocks))
    m = wl.m
    logits = torch.empty((batch, m["vocab"]), dtype=torch.float32, device="cuda")

    if a.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # 1 GiB read + 1 GiB written by one copy kernel
        torch.cuda.synchronize()
        del src, dst

    sec = time_steps(B, wl, batch, a.steps, a.warmup, logits)
    gpu_logits = logits[:len(sample)].cpu().numpy() if sample else None
    tokens_per_s = batch / sec
    log("step %.3f ms, %.0f tokens/s" % (sec * 1e3, tokens_per_s))

    # per-kernel timing from the launches' own start/stop events (separate steps: timed launches cost host time)
    kt = kernel_times(B, wl, batch, max(2, min(a.steps, 10)), logits)
    alg = kernel_algorithmic(m, batch, wl.context_tokens)
    kernels = {}
    for name, (ms, n) in kt.items():
        if n == 0:
            continue
        avg_us = ms / n * 1e3
        k = dict(avg_us=round(avg_us, 2), launches_per_step=n // max(2, min(a.steps, 10)))
        if name in alg:
            k["GBps"] = round(alg[name]["bytes"] / (avg_us * 1e-6) / 1e9, 1)
            k["TFLOPs"] = round(alg[name]["flops"] / (avg_us * 1e-6) / 1e12, 2)
            # the same two figures against the published peaks (algorithmic work: a product issued for both activation
            # terms counts once)
            k["frac_of_hbm_peak"] = round(k["GBps"] / HBM_PEAK_GBS, 4)
            k["frac_of_mfma_peak"] = round(k["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4)
        kernels[name] = k
    step_kernel_ms = sum(ms for ms, n in kt.values()) / max(2, min(a.steps, 10))
    dom = max((n for n in kernels if n in alg), key=lambda n: kt[n][0])
    d_us = kernels[dom]["avg_us"]
    hbm_frac = alg[dom]["bytes"] / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS
    mfma_frac = alg[dom]["flops"] / (d_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS
    if mfma_frac > hbm_frac:
        roof = dict(bound="mfma", achieved=round(mfma_frac * MFMA_BF16_PEAK_TFLOPS, 2), peak=MFMA_BF16_PEAK_TFLOPS,
                    unit="TFLOP/s", frac=round(mfma_frac, 4), traffic=None)
    else:
        roof = dict(bound="hbm", achieved=round(hbm_frac * HBM_PEAK_GBS, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(hbm_frac, 4), traffic=None)
    roof["kernel"] = {"qkv": "linear_kernel (QKV projection)", "o": "linear_kernel (O projection)",
                      "gateup": "linear_kernel (gate/up projection + SwiGLU)", "down": "linear_kernel (down projection)",
                      "lmhead": "linear_kernel (LM head)", "attn": "paged_attn_kernel"}[dom]
    roof["avg_us"] = d_us
    roof["algorithmic_bytes_per_launch"] = alg[dom]["bytes"]
    if roof["bound"] == "hbm" and dom != "attn":
        # the same kernel priced on its weight bytes alone (2*N*K), the figure for a small-M projection
        wb = alg[dom]["bytes"] - alg[dom]["act_bytes"]
        roof["weight_bytes_per_launch"] = wb
        roof["frac_weights_only"] = round(wb / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
    if batch == full_batch:
        roof["traffic"] = measured_traffic(a.workload, dom)

    step_bytes = W.algorithmic_bytes(m, wl.lens, batch)
    step_flops = W.algorithmic_flops(m, wl.lens, batch)
    out = dict(metric="decode_tokens_per_s", value=round(tokens_per_s, 1), unit="tokens/s", n_gpus=1, steps=a.steps,
               warmup=a.warmup, ms_per_step=round(sec * 1e3, 4), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="bf16", data="synthetic",
               config=dict(workload=a.workload, shape=m["name"], batch=batch, context_tokens=wl.context_tokens,
                           page_tokens=16, pool_pages=wl.num_blocks),
               roofline=roof,
               step=dict(algorithmic_GB=round(step_bytes / 1e9, 3), hbm_floor_ms=round(step_bytes / HBM_PEAK_GBS / 1e6, 3),
                         frac_of_hbm_floor=round(step_bytes / HBM_PEAK_GBS / 1e9 / sec, 4),
                         algorithmic_TFLOP=round(step_flops / 1e12, 3),
                         mfma_floor_ms=round(step_flops / MFMA_BF16_PEAK_TFLOPS / 1e9, 3),
                         frac_of_roofline=round(max(step_bytes / HBM_PEAK_GBS / 1e9, step_flops / MFMA_BF16_PEAK_TFLOPS / 1e12) / sec, 4),
                         sum_of_kernel_ms=round(step_kernel_ms, 3)),
               kernels=kernels)

    if a.sweep:
        sizes = [b for b in W.SWEEP_BATCHES if b <= batch]
        pts = B.step_latency_profile(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, sizes, warmup=2,
                                     iters=max(3, min(a.steps, 10)), logits=logits)
        for p in pts:
            by = W.algorithmic_bytes(m, wl.lens, p["batch"])
            fl = W.algorithmic_flops(m, wl.lens, p["batch"])
            p["frac_of_hbm_floor"] = round(by / HBM_PEAK_GBS / 1e6 / p["lat_ms_median"], 4)
            # the step's roofline: the larger of its HBM time and its matrix-core time at the published peaks
            p["frac_of_roofline"] = round(max(by / HBM_PEAK_GBS / 1e6, fl / MFMA_BF16_PEAK_TFLOPS / 1e9) / p["lat_ms_median"], 4)
            p["context_tokens"] = int(wl.lens[:p["batch"]].astype(np.int64).sum()) + p["batch"]
            log("batch %4d: %.3f ms  %.0f tok/s  (%.1f%% of HBM floor)" % (
                p["batch"], p["lat_ms_median"], p["tokens_per_s"], 100 * p["frac_of_hbm_floor"]))
        out["sweep"] = pts

    if a.autoscale_slo_ms > 0:
        # Alg. 1 closed loop: ITL and throughput observed at the current maximum batch size, one update per tick, under
        # both caller policies: "as-printed" keeps the previous tick's throughput for TBP whatever the tick did;
        # "reset-after-no-growth" passes none after a tick that did not scale up (nothing comparable was observed)
        runs = {}
        for policy in ("as-printed", "reset-after-no-growth"):
            slo, mbs, tput_prev, traj = a.autoscale_slo_ms * 1e-3, 1, 0.0, []
            for tick in range(64):
                pt = B.step_latency_profile(wl.model, wl.pool, wl.block_table, wl.seq_lens, wl.tokens, [mbs], warmup=1, iters=3,
                                            logits=logits)[0]
                new, lb = B.local_autoscale_step(pt["lat_ms_median"] * 1e-3, slo, tput_prev, pt["tokens_per_s"], mbs, batch)
                traj.append(dict(max_batch=mbs, itl_ms=round(pt["lat_ms_median"], 3), tokens_per_s=round(pt["tokens_per_s"], 1),
                                 backpressure=round(lb, 4), next_max_batch=new))
                tput_prev = pt["tokens_per_s"] if (policy == "as-printed" or new > mbs) else 0.0
                mbs = new
            log("autoscale (%s): batch sizes %s" % (policy, [t["max_batch"] for t in traj]))
            runs[policy] = traj
        out["autoscale"] = dict(itl_slo_ms=a.autoscale_slo_ms, alpha=0.5, trajectories=runs)

    if a.q_len > 1:
        # verify step of speculative decoding: q_len new tokens per request in one pass (the last q_len-1 cached
        # tokens are treated as not yet cached so that the new positions lie in allocated pages)
        T = a.q_len
        if batch * T > wl.model.cfg.max_batch:
            log("--q-len %d skipped: batch*q_len exceeds the model's max_batch" % T)
        else:
            lens_m = torch.from_numpy((wl.lens[:batch] - (T - 1)).clip(min=0).astype(np.int32)).cuda()
            from paper_2501_08090_amd import inputs as I
            toks_m = torch.from_numpy(I.token_ids(batch * T, wl.m["vocab"], 9).reshape(batch, T)).cuda()
            lg_m = torch.empty((batch, T, wl.m["vocab"]), dtype=torch.float32, device="cuda")
            bt_m = wl.block_table[:batch].contiguous()
            for _ in range(2):
                B.decode_step_multi(wl.model, wl.pool, bt_m, lens_m, toks_m, logits=lg_m)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(a.steps):
                B.decode_step_multi(wl.model, wl.pool, bt_m, lens_m, toks_m, logits=lg_m)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / a.steps
            out["multi_token"] = dict(q_len=T, ms_per_step=round(dt * 1e3, 4), rows_per_s=round(batch * T / dt, 1),
                                      vs_single_token_step=round(dt * 1e3 / out["ms_per_step"], 3))
            log("multi-token step (q_len %d): %.3f ms = %.2fx the single-token step, %.0f rows/s" % (
                T, dt * 1e3, dt * 1e3 / out["ms_per_step"], batch * T / dt))

    if a.swap:
        # eviction path: the longest request's pages to pinned host memory and back (kernels write/read the host
        # buffer directly over PCIe)
        i = int(np.argmax(wl.lens[:batch]))
        npg = int((int(wl.lens[i]) + 1 + 15) // 16)
        nbytes = npg * wl.model.kv_block_bytes()
        image = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        row = wl.block_table[i].contiguous()
        res = {}
        for name, fn in (("swap_out", wl.pool.swap_out), ("swap_in", wl.pool.swap_in)):
            fn(row, npg, image)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                fn(row, npg, image)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / 5
            res[name] = dict(ms=round(dt * 1e3, 3), GBps=round(nbytes / dt / 1e9, 2))
        out["swap"] = dict(request=i, context_tokens=int(wl.lens[i]), pages=npg, bytes=nbytes, target="pinned host memory", **res)
        log("swap of request %d (%d pages, %.1f MB): out %.2f ms (%.1f GB/s), in %.2f ms (%.1f GB/s)" % (
            i, npg, nbytes / 1e6, res["swap_out"]["ms"], res["swap_out"]["GBps"], res["swap_in"]["ms"], res["swap_in"]["GBps"]))

    if sample:
        log("timing the CPU oracle on %d requests ..." % len(sample))
        out["cpu_baseline"], out["parity_sample"] = cpu_baseline(wl, sample, gpu_logits)
        log("oracle: %.2f tokens/s on %d threads; parity on the sample: max|d|/sigma %.2e, argmax agreement %.3f" % (
            out["cpu_baseline"]["value"], out["cpu_baseline"]["cores"], out["parity_sample"]["max_abs_err_over_sigma"],
            out["parity_sample"]["argmax_agreement"]))
    else:
        out["cpu_baseline"] = None
    if curve:
        # Per-step latency and tokens/s over batch sizes 1..512 of the mixed population (Local Autoscaler: the curve
        # its batch-size updates walk), on the same model: the default workload's cache is released first.
        model, wl_w_host = wl.model, wl.w_host
        del logits
        wl.pool.close()
        del wl
        torch.cuda.empty_cache()
        t0 = time.time()
        w_host = wl_w_host
        oracle_sizes = [b for b in (1, 8, 64) if w_host is not None]
        cw = W.build(CURVE_WORKLOAD, seed=0, model=model, host_seqs=list(range(max(oracle_sizes))) if oracle_sizes else ())
        log("curve workload %s built in %.1f s: %d requests, %d context tokens" % (CURVE_WORKLOAD, time.time() - t0, cbatch, cw.context_tokens))
        clog = torch.empty((cbatch, cm["vocab"]), dtype=torch.float32, device="cuda")
        sizes = [b for b in W.SWEEP_BATCHES if b <= cbatch]
        pts = B.step_latency_profile(model, cw.pool, cw.block_table, cw.seq_lens, cw.tokens, sizes, warmup=2, iters=5, logits=clog)
        for p in pts:
            by, fl = W.algorithmic_bytes(cm, cw.lens, p["batch"]), W.algorithmic_flops(cm, cw.lens, p["batch"])
            p["context_tokens"] = int(cw.lens[:p["batch"]].astype(np.int64).sum()) + p["batch"]
            p["frac_of_roofline"] = round(max(by / HBM_PEAK_GBS / 1e6, fl / MFMA_BF16_PEAK_TFLOPS / 1e9) / p["lat_ms_median"], 4)
            log("curve: batch %4d: %.3f ms  %.0f tok/s  (%.1f%% of the step's roofline)" % (
                p["batch"], p["lat_ms_median"], p["tokens_per_s"], 100 * p["frac_of_roofline"]))
        out["curve"] = dict(workload=CURVE_WORKLOAD, points=pts)
        # the curve against the paper's ITL SLOs: the largest measured batch size whose step stays within each
        slo_rows = []
        for cls, slo_ms in ITL_SLOS_MS:
            ok = [p["batch"] for p in pts if p["lat_ms_p99"] <= slo_ms]
            slo_rows.append(dict(request_class=cls, itl_slo_ms=slo_ms, largest_batch_within_slo=max(ok) if ok else 0,
                                 step_ms_there=round(max(p["lat_ms_p99"] for p in pts if p["batch"] == max(ok)), 3) if ok else None,
                                 bounded_by="largest batch measured" if ok and max(ok) == max(sizes) else "the SLO"))
            log("curve: ITL SLO %.0f ms (%s requests): largest measured batch within it %d" % (slo_ms, cls, max(ok) if ok else 0))
        out["curve"]["itl_slo"] = slo_rows
        if oracle_sizes:
            # the oracle beside the curve's smallest batch sizes, on the host cores
            sys.path.insert(0, os.path.join(ROOT, "oracle"))
            import chiron_oracle as orc
            import sample_step
            orows = []
            for b in oracle_sizes:
                n = int(cw.lens[:b].astype(np.int64).sum())
                _, _, _, dt = sample_step.run(cm, w_host, [(k[:n], v[:n]) for k, v in cw.kv_host], cw.lens[:b], cw.tok[:b])
                orows.append(dict(batch=b, seconds=round(dt, 3), tokens_per_s=round(b / dt, 3), cores=orc.num_threads(), cpu=cpu_model()))
                log("curve: oracle at batch %d: %.2f s = %.2f tokens/s" % (b, dt, b / dt))
            out["curve"]["oracle"] = orows
            out["curve"]["oracle_skipped"] = [b for b in sizes if b not in oracle_sizes]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
