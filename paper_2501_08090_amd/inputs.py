"""Seeded synthetic inputs for the decode step: model shapes, random-init weights,
context-length populations, block tables and cache contents.

This module holds no arithmetic of the decode step itself; it only draws random
data and lays out index arrays.  Both the GPU library's callers and the CPU
checker's callers take their inputs from here, so the two sides see the same
bytes.  Large tensors can be drawn directly on a GPU (torch's device generator)
and copied to the host for whoever needs them there; the values for a given
(seed, name, device type) are reproducible.

The length populations stand in for ShareGPT-shaped requests and for the
interactive/batch request mix of the paper's evaluation (Evaluation: workloads
and SLOs); the dataset itself is not used.
"""
import math
import zlib

import numpy as np
import torch

BLOCK_SIZE = 16

TINY = dict(name="tiny", n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=688, vocab=1024,
            rope_base=10000.0, rms_eps=1e-5, block_size=BLOCK_SIZE)
LLAMA_8B = dict(name="llama3-8b-shape", n_layers=32, hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=14336,
                vocab=128256, rope_base=500000.0, rms_eps=1e-5, block_size=BLOCK_SIZE)
LLAMA_70B = dict(name="llama3-70b-shape", n_layers=80, hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=28672,
                 vocab=128256, rope_base=500000.0, rms_eps=1e-5, block_size=BLOCK_SIZE)

LAYER_MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def matrix_shapes(m):
    """(out_features, in_features) of every per-layer matrix."""
    H, qn, kn, F = m["hidden"], m["n_q_heads"] * m["head_dim"], m["n_kv_heads"] * m["head_dim"], m["ffn"]
    return dict(wq=(qn, H), wk=(kn, H), wv=(kn, H), wo=(H, qn), w_gate=(F, H), w_up=(F, H), w_down=(H, F))


def _sub_seed(seed, *names):
    return (zlib.crc32(("/".join(str(n) for n in names)).encode()) ^ (int(seed) * 0x9E3779B1)) & 0x7FFFFFFF


def normal(shape, std, seed, *names, device="cpu", dtype=torch.bfloat16, mean=0.0):
    """N(mean, std^2) draws in fp32, rounded once (RNE) to `dtype`."""
    g = torch.Generator(device=device)
    g.manual_seed(_sub_seed(seed, *names))
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(dtype)


def make_weights(m, seed=0, device="cpu", dtype=torch.bfloat16, std=0.02, gain_jitter=0.0, layers=None):
    """Random-init weights: matrices and embedding ~ N(0, std^2); norm gains 1 (+ gain_jitter*N(0,1) when a
    test wants the gains to matter).  Matrices are (out, in) row-major.  Returns dict name -> tensor or list."""
    L = m["n_layers"] if layers is None else layers
    H, V = m["hidden"], m["vocab"]
    shp = matrix_shapes(m)

    def gain(*names):
        if gain_jitter == 0.0:
            return torch.ones(H, device=device, dtype=dtype)
        return normal((H,), gain_jitter, seed, *names, device=device, dtype=dtype, mean=1.0)

    w = dict(embed=normal((V, H), std, seed, "embed", device=device, dtype=dtype), final_norm=gain("final_norm"),
             lm_head=normal((V, H), std, seed, "lm_head", device=device, dtype=dtype))
    for n in LAYER_MATRICES:
        w[n] = [normal(shp[n], std, seed, n, l, device=device, dtype=dtype) for l in range(L)]
    w["attn_norm"] = [gain("attn_norm", l) for l in range(L)]
    w["ffn_norm"] = [gain("ffn_norm", l) for l in range(L)]
    return w


def to_numpy_storage(t):
    """torch tensor -> numpy array the CPU checker accepts: float32 as is, bf16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.to(torch.float32).numpy()


def weights_to_numpy(w):
    return {k: ([to_numpy_storage(a) for a in v] if isinstance(v, list) else to_numpy_storage(v)) for k, v in w.items()}


# ---- context-length populations --------------------------------------------------------------

LOGNORMAL_SIGMA = 0.8


def lognormal_lengths(n, median, lo, hi, rng, sigma=LOGNORMAL_SIGMA):
    z = rng.standard_normal(n)
    L = np.rint(np.exp(math.log(median) + sigma * z)).astype(np.int64)
    return np.clip(L, lo, hi).astype(np.int32)


def uniform_lengths(n, lo, hi, rng):
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def population(kind, n, seed=0):
    """Context lengths (tokens already cached) of n requests.
    tiny: U{16..128};  b64: lognormal median 800 in [64,4096];  mixed: 70% interactive (lognormal median 512 in
    [16,8192]) / 30% batch (U{2048..8192}), request j is batch-class iff j mod 10 in {3,6,9};
    interactive: the interactive class alone;  short: lognormal median 256 in [16,2048] (what lets 4096 requests'
    caches fit one GPU);
    b128-70b: lognormal median 2048 in [128,8192];  long: U{24576..32768}."""
    rng = np.random.default_rng(_sub_seed(seed, "population", kind))
    if kind == "tiny":
        return uniform_lengths(n, 16, 128, rng)
    if kind == "b64":
        return lognormal_lengths(n, 800, 64, 4096, rng)
    if kind == "mixed":
        inter = lognormal_lengths(n, 512, 16, 8192, rng)
        batch = uniform_lengths(n, 2048, 8192, rng)
        is_batch = np.isin(np.arange(n) % 10, (3, 6, 9))
        return np.where(is_batch, batch, inter).astype(np.int32)
    if kind == "interactive":
        return lognormal_lengths(n, 512, 16, 8192, rng)
    if kind == "short":
        return lognormal_lengths(n, 256, 16, 2048, rng)
    if kind == "b128-70b":
        return lognormal_lengths(n, 2048, 128, 8192, rng)
    if kind == "long":
        return uniform_lengths(n, 24576, 32768, rng)
    raise ValueError(kind)


# ---- paged layout ------------------------------------------------------------------------------

def pages_needed(seq_lens, block_size=BLOCK_SIZE):
    """pages a sequence needs so that the token at position seq_len has a slot"""
    return (np.asarray(seq_lens, np.int64) + 1 + block_size - 1) // block_size


def make_block_table(seq_lens, seed=0, block_size=BLOCK_SIZE, pool_factor=2.0, shuffle=True, max_blocks=None,
                     num_blocks=None):
    """Distinct pages for every sequence, drawn at random from a pool of pool_factor x the pages in use.
    Returns (block_table int32 [B, max_blocks] with -1 in unused entries, num_blocks)."""
    need = pages_needed(seq_lens, block_size)
    total = int(need.sum())
    if num_blocks is None:
        num_blocks = max(1, int(math.ceil(total * pool_factor)))
    if max_blocks is None:
        max_blocks = int(need.max()) if len(need) else 1
    rng = np.random.default_rng(_sub_seed(seed, "block_table"))
    ids = rng.permutation(num_blocks)[:total] if shuffle else np.arange(total)
    bt = np.full((len(need), max_blocks), -1, np.int32)
    o = 0
    for i, c in enumerate(need):
        bt[i, :c] = ids[o:o + c]
        o += c
    return bt, int(num_blocks)


def token_ids(n, vocab, seed=0):
    rng = np.random.default_rng(_sub_seed(seed, "tokens"))
    return rng.integers(0, vocab, size=n).astype(np.int32)


def prefill_index(seq_lens):
    """(seq_idx, pos) of every already-cached token, sequence-major."""
    seq_lens = np.asarray(seq_lens, np.int64)
    seq_idx = np.repeat(np.arange(len(seq_lens), dtype=np.int32), seq_lens)
    starts = np.concatenate([[0], np.cumsum(seq_lens)[:-1]])
    pos = (np.arange(int(seq_lens.sum()), dtype=np.int64) - np.repeat(starts, seq_lens)).astype(np.int32)
    return seq_idx, pos


def make_kv_layer(m, total_tokens, layer, seed=0, device="cpu", dtype=torch.bfloat16):
    """Synthetic cache content of one layer: K and V ~ N(0,1), [total_tokens, n_kv, d], sequence-major in the
    order of prefill_index()."""
    shape = (int(total_tokens), m["n_kv_heads"], m["head_dim"])
    return (normal(shape, 1.0, seed, "k_cache", layer, device=device, dtype=dtype),
            normal(shape, 1.0, seed, "v_cache", layer, device=device, dtype=dtype))
