"""GPU-resident synthetic workloads for the decode step: builds the model, the paged cache and
the index arrays of a named configuration on the current GPU, from the seeded generators in
`inputs`.  Only plumbing lives here (torch allocates, the C-ABI library repacks weights and
fills the cache through chiron_append_kv); no arithmetic of the step.

A caller that wants to check results on the host can ask for `host_seqs`: the weights and the
cache rows of those requests are also returned as numpy arrays, taken from the generated
tensors themselves (never read back through the library).
"""
import math

import numpy as np
import torch

from . import binding as B
from . import inputs as I

# name -> (model shape, population kind, batch, pool factor)
WORKLOADS = {
    "tiny-b4": (I.TINY, "tiny", 4, 2.0),
    "llama8b-b64-lognormal800": (I.LLAMA_8B, "b64", 64, 2.0),
    "llama8b-mixed-sweep512": (I.LLAMA_8B, "mixed", 512, 1.15),
    "llama70b-b128-lognormal2048": (I.LLAMA_70B, "b128-70b", 128, 1.0),
    "llama8b-b32-long32k": (I.LLAMA_8B, "long", 32, 1.25),
    # the batch sizes the paper reports for batch-class instances (2048-4096) on what one GPU's HBM holds:
    # interactive-length contexts only (a 2048-request mixed population would need 270 GB of cache)
    "llama8b-interactive-sweep2048": (I.LLAMA_8B, "interactive", 2048, 1.05),
    # 4096 requests, the upper end of the batch sizes the paper reports for batch-class instances: contexts short enough
    # (lognormal median 256) that their caches fit beside the weights
    "llama8b-short-sweep4096": (I.LLAMA_8B, "short", 4096, 1.05),
    # every width of the 8B shape (hidden, heads, FFN, vocabulary) with two layers only, so that a CPU checker can
    # afford all 512 rows of the mixed population: every row tile of the large-batch kernels, element by element
    "llama8b-width-2layers-mixed512": (dict(I.LLAMA_8B, name="llama3-8b-width-2-layers", n_layers=2), "mixed", 512, 1.15),
}
SWEEP_BATCHES = (1, 8, 32, 64, 128, 256, 512, 1024, 2048, 4096)
KV_CHUNK_TOKENS = 1 << 17


class Workload:
    pass


def kv_bytes_per_token(m):
    return m["n_layers"] * m["n_kv_heads"] * m["head_dim"] * 2 * 2


def streamed_params(m):
    """parameters every step reads: all layer matrices plus the LM head (not the embedding table)"""
    s = I.matrix_shapes(m)
    return m["n_layers"] * sum(a * b for a, b in s.values()) + m["vocab"] * m["hidden"]


def build_model(m, seed=0, max_batch=1, max_blocks_per_seq=1, host_weights=False, log=None, gain_jitter=0.0):
    """Random-init model of shape m on the GPU, loaded layer by layer.  Returns (model, w_host or None)."""
    dev = "cuda"
    say = log or (lambda *a: None)
    model = B.Model(m, max_batch, max_blocks_per_seq)
    w_host = {n: [] for n in I.LAYER_MATRICES + ("attn_norm", "ffn_norm")} if host_weights else None
    shp = I.matrix_shapes(m)
    H = m["hidden"]

    def gain(*names):
        if gain_jitter == 0.0:
            return torch.ones(H, device=dev, dtype=torch.bfloat16)
        return I.normal((H,), gain_jitter, seed, *names, device=dev, mean=1.0)

    for l in range(m["n_layers"]):
        lw = {n: I.normal(shp[n], 0.02, seed, n, l, device=dev) for n in I.LAYER_MATRICES}
        lw["attn_norm"], lw["ffn_norm"] = gain("attn_norm", l), gain("ffn_norm", l)
        model.load_layer(l, **lw)
        if host_weights:
            for n, t in lw.items():
                w_host[n].append(I.to_numpy_storage(t))
        torch.cuda.synchronize()
        del lw
        if l % 8 == 7:
            say("weights: layer %d/%d loaded" % (l + 1, m["n_layers"]))
    embed = I.normal((m["vocab"], H), 0.02, seed, "embed", device=dev)
    lm_head = I.normal((m["vocab"], H), 0.02, seed, "lm_head", device=dev)
    fin = gain("final_norm")
    model.load_head(embed, fin, lm_head)
    if host_weights:
        w_host.update(embed=I.to_numpy_storage(embed), lm_head=I.to_numpy_storage(lm_head), final_norm=I.to_numpy_storage(fin))
    torch.cuda.synchronize()
    return model, w_host


def build(name, seed=0, host_seqs=(), host_weights=False, max_batch=None, log=None, gain_jitter=0.0, model=None,
          w_host=None, pool_memory=None, max_blocks_per_seq=None):
    """Returns a Workload with .model .pool .block_table .seq_lens .tokens (GPU) and .lens .bt .tok (numpy).
    host_weights / host_seqs additionally fill .w_host (numpy storage arrays) and .kv_host[l] = (K, V) rows of
    the listed requests, concatenated in the order given.  An existing model of the same shape (created with a
    large enough max_batch and max_blocks_per_seq) can be passed in to skip the weight generation; max_batch and
    max_blocks_per_seq size a new model for more than this workload needs, so that it can serve another one later."""
    m, kind, batch, pool_factor = WORKLOADS[name]
    m = dict(m)
    dev = "cuda"
    say = log or (lambda *a: None)
    wl = Workload()
    wl.name, wl.m, wl.batch = name, m, batch
    wl.lens = I.population(kind, batch, seed)
    mb = model.cfg.max_blocks_per_seq if model is not None else max_blocks_per_seq  # None: as wide as the longest request
    wl.bt, wl.num_blocks = I.make_block_table(wl.lens, seed=seed, pool_factor=pool_factor, max_blocks=mb)
    wl.tok = I.token_ids(batch, m["vocab"], seed)
    wl.block_table = torch.from_numpy(wl.bt).to(dev)
    wl.seq_lens = torch.from_numpy(wl.lens).to(dev)
    wl.tokens = torch.from_numpy(wl.tok).to(dev)
    wl.context_tokens = int(wl.lens.astype(np.int64).sum()) + batch  # tokens attended over, incl. the new ones

    if model is None:
        model, w_host = build_model(m, seed, max_batch or batch, wl.bt.shape[1], host_weights or len(host_seqs) > 0, log,
                                    gain_jitter)
    wl.model, wl.w_host = model, w_host

    wl.pool = B.KVPool(model, num_blocks=wl.num_blocks, memory=pool_memory)
    seq_idx, pos = I.prefill_index(wl.lens)
    total = len(seq_idx)
    starts = np.concatenate([[0], np.cumsum(wl.lens.astype(np.int64))])
    host_rows = np.concatenate([np.arange(starts[i], starts[i + 1]) for i in host_seqs]) if len(host_seqs) else None
    wl.kv_host = []
    si_d, ps_d = torch.from_numpy(seq_idx).to(dev), torch.from_numpy(pos).to(dev)
    for l in range(m["n_layers"]):
        hk, hv = [], []
        for c, t0 in enumerate(range(0, total, KV_CHUNK_TOKENS)):
            t1 = min(total, t0 + KV_CHUNK_TOKENS)
            shape = (t1 - t0, m["n_kv_heads"], m["head_dim"])
            k = I.normal(shape, 1.0, seed, "k_cache", l, c, device=dev)
            v = I.normal(shape, 1.0, seed, "v_cache", l, c, device=dev)
            wl.pool.append(l, k, v, wl.block_table, si_d[t0:t1].contiguous(), ps_d[t0:t1].contiguous())
            if host_rows is not None:
                sel = host_rows[(host_rows >= t0) & (host_rows < t1)] - t0
                if len(sel):
                    sel_d = torch.from_numpy(sel).to(dev)
                    hk.append(I.to_numpy_storage(k[sel_d]))
                    hv.append(I.to_numpy_storage(v[sel_d]))
            torch.cuda.synchronize()
            del k, v
        if host_rows is not None:
            wl.kv_host.append((np.concatenate(hk), np.concatenate(hv)))
        if l % 8 == 7:
            say("cache: layer %d/%d filled (%d tokens)" % (l + 1, m["n_layers"], total))
    return wl


def algorithmic_bytes(m, lens, batch):
    """HBM bytes one step must move: weights once, the K/V of every attended token, the new K/V written,
    and the fp32 logits (activations between kernels are < 1% and left out)."""
    ctx = int(np.asarray(lens[:batch], np.int64).sum()) + batch
    kappa = kv_bytes_per_token(m)
    return 2 * streamed_params(m) + kappa * ctx + kappa * batch + 4 * batch * m["vocab"]


def algorithmic_flops(m, lens, batch):
    """Flops one step must do: two per streamed weight and request, four per query head, head dimension, layer and
    attended token (scores and weighted sum)."""
    ctx = int(np.asarray(lens[:batch], np.int64).sum()) + batch
    return 2 * batch * streamed_params(m) + 4 * m["n_q_heads"] * m["head_dim"] * m["n_layers"] * ctx
