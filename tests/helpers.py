"""Shared scenario builders for the tests: small seeded cases handed, as the same
bytes, to the CPU oracle and (in the gpu tests) to the HIP library."""
import numpy as np
import torch

import chiron_oracle as orc
from paper_2501_08090_amd import inputs as I


class Case:
    """One decode-step scenario on the host (numpy), in the oracle's formats."""
    pass


def make_case(m=None, batch=4, kind="tiny", seed=0, storage="f32", gain_jitter=0.0, seq_lens=None, shuffle=True,
              pool_factor=2.0, std=0.02, poison_unused=False):
    """storage 'f32': fp32 weights/cache as generated; 'bf16': the same draws rounded once to bf16."""
    m = dict(I.TINY if m is None else m)
    c = Case()
    c.m = m
    tdt = torch.float32 if storage == "f32" else torch.bfloat16
    c.storage = storage
    c.w_t = I.make_weights(m, seed=seed, dtype=tdt, std=std, gain_jitter=gain_jitter)
    c.w = I.weights_to_numpy(c.w_t)
    c.seq_lens = I.population(kind, batch, seed) if seq_lens is None else np.asarray(seq_lens, np.int32)
    batch = len(c.seq_lens)
    c.batch = batch
    c.block_table, c.num_blocks = I.make_block_table(c.seq_lens, seed=seed, shuffle=shuffle, pool_factor=pool_factor)
    c.tokens = I.token_ids(batch, m["vocab"], seed)
    dt = orc.F32 if storage == "f32" else orc.BF16
    c.cfg = orc.make_config(m, dt, dt)
    c.seq_idx, c.pos = I.prefill_index(c.seq_lens)
    total = int(c.seq_lens.sum())
    c.kv_t = [I.make_kv_layer(m, total, l, seed=seed, dtype=tdt) for l in range(m["n_layers"])]
    c.kv = [(I.to_numpy_storage(k), I.to_numpy_storage(v)) for k, v in c.kv_t]
    c.poison_unused = poison_unused
    return c


def fresh_pool(c, block_table=None, num_blocks=None):
    """Oracle pool pre-filled with the case's cache content (through the oracle's own append)."""
    bt = c.block_table if block_table is None else block_table
    nb = c.num_blocks if num_blocks is None else num_blocks
    pool = orc.Pool(c.cfg, nb, np.float32 if c.storage == "f32" else np.uint16)
    if c.poison_unused:
        # unused slots hold NaN bit patterns: nothing may ever read them
        if c.storage == "f32":
            pool.k[...] = np.nan
            pool.v[...] = np.nan
        else:
            pool.k[...] = 0x7FC0
            pool.v[...] = 0x7FC0
    for l, (k, v) in enumerate(c.kv):
        kf = k if c.storage == "f32" else bf16_to_f32(k)
        vf = v if c.storage == "f32" else bf16_to_f32(v)
        orc.append_kv(pool, l, kf, vf, bt, c.seq_idx, c.pos)
    return pool


def bf16_to_f32(u16):
    return (u16.astype(np.uint32) << 16).view(np.float32)


def as_f64(a):
    """storage array (float32 or bf16 bits) -> float64 values"""
    if a.dtype == np.uint16:
        return bf16_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ---- GPU side (only the gpu tests call these) ----------------------------------------------------

def gpu_setup(c, max_batch=None, poison=False, extra_blocks=0):
    """Build the HIP model and pool for a bf16-storage case and pre-fill the cache through chiron_append_kv."""
    from paper_2501_08090_amd import binding as B
    assert c.storage == "bf16"
    dev = "cuda"
    model = B.Model(c.m, max_batch or max(c.batch, 1), c.block_table.shape[1])
    model.load_weights({k: ([a.to(dev) for a in v] if isinstance(v, list) else v.to(dev)) for k, v in c.w_t.items()})
    nb = c.num_blocks + extra_blocks
    mem = torch.empty(nb * model.kv_block_bytes(), dtype=torch.uint8, device=dev)
    if poison:
        mem.view(torch.int16).fill_(0x7FC0)      # bf16 NaN everywhere: nothing outside live slots may be read
    else:
        mem.zero_()
    pool = B.KVPool(model, memory=mem)
    assert pool.num_blocks == nb
    g = Case()
    g.model, g.pool = model, pool
    g.block_table = torch.from_numpy(c.block_table).to(dev)
    g.seq_lens = torch.from_numpy(c.seq_lens).to(dev)
    g.tokens = torch.from_numpy(c.tokens).to(dev)
    si, ps = torch.from_numpy(c.seq_idx).to(dev), torch.from_numpy(c.pos).to(dev)
    for l, (k, v) in enumerate(c.kv_t):
        pool.append(l, k.to(dev), v.to(dev), g.block_table, si, ps)
    torch.cuda.synchronize()
    return g


def bits(t):
    """bf16 GPU tensor -> numpy uint16 bit patterns"""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
