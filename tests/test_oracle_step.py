"""Pins of the oracle's whole decode step: an independent float64 composition of
torch library ops, layout/permutation invariants, degenerate-weight special cases
that collapse to one library GEMM, and the slot-write contract.  CPU only."""
import math

import numpy as np
import pytest
import torch

import chiron_oracle as orc
from helpers import as_f64, fresh_pool, make_case
from paper_2501_08090_amd import inputs as I


def torch_reference_multi(c, tokens):
    """Second opinion built only from torch float64 library ops on contiguous per-sequence caches (no paging, no
    shared code with the oracle).  tokens [B, T]: request i feeds tokens[i][t] at position seq_lens[i]+t, every
    token's k, v joins the request's cache before the next one is taken.  Returns logits [B, T, V] float64."""
    m = c.m
    H, nq, nkv, d, F = m["hidden"], m["n_q_heads"], m["n_kv_heads"], m["head_dim"], m["ffn"]
    t64 = lambda a: torch.from_numpy(as_f64(a))
    W = {k: ([t64(a) for a in v] if isinstance(v, list) else t64(v)) for k, v in c.w.items()}
    inv_freq = torch.tensor(m["rope_base"], dtype=torch.float64) ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    out = []
    starts = np.concatenate([[0], np.cumsum(c.seq_lens)])
    for i in range(c.batch):
        p0 = int(c.seq_lens[i])
        Kc = [t64(c.kv[l][0][starts[i]:starts[i] + p0]) for l in range(m["n_layers"])]     # [p, nkv, d] per layer
        Vc = [t64(c.kv[l][1][starts[i]:starts[i] + p0]) for l in range(m["n_layers"])]
        row = []
        for t in range(tokens.shape[1]):
            p = p0 + t
            h = W["embed"][int(tokens[i][t])].clone()
            rot = torch.polar(torch.ones_like(inv_freq), p * inv_freq)

            def rope(x):  # x [heads, d]
                z = torch.complex(x[:, :d // 2], x[:, d // 2:]) * rot
                return torch.cat([z.real, z.imag], dim=1)

            for l in range(m["n_layers"]):
                x = torch.nn.functional.rms_norm(h, (H,), W["attn_norm"][l], m["rms_eps"])
                q = rope((W["wq"][l] @ x).view(nq, d))
                k = rope((W["wk"][l] @ x).view(nkv, d))
                v = (W["wv"][l] @ x).view(nkv, d)
                if c.storage == "bf16":  # the cache stores bf16
                    k = k.float().to(torch.bfloat16).double(); v = v.float().to(torch.bfloat16).double()
                Kc[l] = torch.cat([Kc[l], k[None]], 0)                                       # [p+1, nkv, d]
                Vc[l] = torch.cat([Vc[l], v[None]], 0)
                Kh = Kc[l].permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)              # [nq, p+1, d]
                Vh = Vc[l].permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)
                o = torch.nn.functional.scaled_dot_product_attention(q[:, None, :], Kh, Vh)  # [nq,1,d]
                h = h + W["wo"][l] @ o.reshape(nq * d)
                x = torch.nn.functional.rms_norm(h, (H,), W["ffn_norm"][l], m["rms_eps"])
                h = h + W["w_down"][l] @ (torch.nn.functional.silu(W["w_gate"][l] @ x) * (W["w_up"][l] @ x))
            x = torch.nn.functional.rms_norm(h, (H,), W["final_norm"], m["rms_eps"])
            row.append(W["lm_head"] @ x)
        out.append(torch.stack(row))
    return torch.stack(out).numpy()


def torch_reference_step(c):
    return torch_reference_multi(c, np.asarray(c.tokens).reshape(-1, 1))[:, 0, :]


@pytest.mark.parametrize("storage,jitter", [("f32", 0.0), ("f32", 0.2), ("bf16", 0.2)])
def test_step_matches_independent_torch_composition(storage, jitter):
    c = make_case(batch=4, seed=0, storage=storage, gain_jitter=jitter)
    logits, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table, c.seq_lens, c.tokens)
    want = torch_reference_step(c)
    sig = want.std()
    # fp32 rounding at tensor boundaries only (bf16 storage: a rare 1-ulp flip of a stored k/v is allowed for)
    tol = 2e-5 if storage == "f32" else 2e-3
    assert np.abs(logits - want).max() <= tol * sig
    assert np.array_equal(logits.argmax(1), want.argmax(1))


def test_paged_equals_contiguous_bit_identical():
    c = make_case(batch=4, seed=5, shuffle=True)
    l1, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table, c.seq_lens, c.tokens)
    bt2, nb2 = I.make_block_table(c.seq_lens, shuffle=False, pool_factor=1.0)
    assert not np.array_equal(bt2, c.block_table)
    l2, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c, bt2, nb2), bt2, c.seq_lens, c.tokens)
    assert np.array_equal(l1, l2)


def test_batch_permutation_permutes_logits_bit_exactly():
    c = make_case(batch=5, seed=6)
    l1, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table, c.seq_lens, c.tokens)
    perm = np.array([3, 0, 4, 2, 1])
    l2, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table[perm], c.seq_lens[perm], c.tokens[perm])
    assert np.array_equal(l2, l1[perm])
    # and a sequence's logits do not depend on who else is in the batch
    l3, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table[2:3], c.seq_lens[2:3], c.tokens[2:3])
    assert np.array_equal(l3[0], l1[2])


def test_zero_output_projections_collapse_to_one_gemm():
    c = make_case(batch=4, seed=7, gain_jitter=0.1)
    for l in range(c.m["n_layers"]):
        c.w["wo"][l] = np.zeros_like(c.w["wo"][l]); c.w["w_down"][l] = np.zeros_like(c.w["w_down"][l])
    logits, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table, c.seq_lens, c.tokens)
    h = as_f64(c.w["embed"])[c.tokens]
    x = h / np.sqrt((h ** 2).mean(1, keepdims=True) + c.m["rms_eps"]) * as_f64(c.w["final_norm"])
    assert np.allclose(logits, x @ as_f64(c.w["lm_head"]).T, rtol=1e-5, atol=1e-7)


def test_zero_gate_kills_the_ffn_branch():
    a = make_case(batch=3, seed=8)
    b = make_case(batch=3, seed=8)
    for l in range(a.m["n_layers"]):
        a.w["w_gate"][l] = np.zeros_like(a.w["w_gate"][l])        # silu(0) = 0
        b.w["w_down"][l] = np.zeros_like(b.w["w_down"][l])
    la, _ = orc.decode_step(a.cfg, a.w, fresh_pool(a), a.block_table, a.seq_lens, a.tokens)
    lb, _ = orc.decode_step(b.cfg, b.w, fresh_pool(b), b.block_table, b.seq_lens, b.tokens)
    assert np.array_equal(la, lb)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_step_writes_exactly_one_slot_per_sequence_layer_and_tensor(storage):
    c = make_case(batch=4, seed=9, storage=storage, seq_lens=[0, 15, 16, 47])   # empty context, page edges
    pool = fresh_pool(c)
    before = pool.copy()
    logits, slots = orc.decode_step(c.cfg, c.w, pool, c.block_table, c.seq_lens, c.tokens)
    want = c.block_table[np.arange(4), c.seq_lens // 16].astype(np.int64) * 16 + c.seq_lens % 16
    assert np.array_equal(slots, want)
    for arr0, arr1 in ((before.k, pool.k), (before.v, pool.v)):
        changed = np.any(arr0 != arr1, axis=(2, 3))              # [layers, slots]
        for l in range(c.m["n_layers"]):
            assert set(np.nonzero(changed[l])[0].tolist()) == set(want.tolist())
    assert np.all(np.isfinite(logits))
    # seq_len 0: the sequence attends only to itself, so its attention output is its own v; the step still
    # agrees with the library composition
    ref = torch_reference_step(c)
    assert np.abs(logits - ref).max() <= (2e-5 if storage == "f32" else 2e-3) * ref.std()


def test_unused_slots_are_never_read():
    c = make_case(batch=3, seed=10, poison_unused=True)
    logits, _ = orc.decode_step(c.cfg, c.w, fresh_pool(c), c.block_table, c.seq_lens, c.tokens)
    assert np.all(np.isfinite(logits))
    c2 = make_case(batch=3, seed=10)
    l2, _ = orc.decode_step(c2.cfg, c2.w, fresh_pool(c2), c2.block_table, c2.seq_lens, c2.tokens)
    assert np.array_equal(logits, l2)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_multi_token_step_matches_library_composition_and_sequential_steps(storage):
    c = make_case(batch=3, seed=11, storage=storage, gain_jitter=0.1, seq_lens=[14, 31, 60], pool_factor=3.0)
    T = 4
    toks = I.token_ids(3 * T, c.m["vocab"], 5).reshape(3, T)
    # room for the T new tokens: extend each row's pages from the pool's unused ones
    bt, nb = I.make_block_table(np.asarray(c.seq_lens) + T - 1, seed=11, pool_factor=3.0)
    pool = fresh_pool(c, bt, nb)
    logits = orc.decode_step_multi(c.cfg, c.w, pool, bt, c.seq_lens, toks)
    want = torch_reference_multi(c, toks)
    tol = 2e-5 if storage == "f32" else 3e-3
    assert np.abs(logits - want).max() <= tol * want.std()
    assert np.array_equal(logits.argmax(2), want.argmax(2))
    # the same thing as T ordinary steps issued by a caller that advances seq_lens itself: bit-identical
    pool2 = fresh_pool(c, bt, nb)
    for t in range(T):
        lt, _ = orc.decode_step(c.cfg, c.w, pool2, bt, np.asarray(c.seq_lens) + t, toks[:, t])
        assert np.array_equal(lt, logits[:, t, :])
    assert np.array_equal(pool.k, pool2.k) and np.array_equal(pool.v, pool2.v)
    # causality: the logits of token t do not depend on the tokens after it
    toks2 = toks.copy(); toks2[:, 2:] = (toks2[:, 2:] + 7) % c.m["vocab"]
    l2 = orc.decode_step_multi(c.cfg, c.w, fresh_pool(c, bt, nb), bt, c.seq_lens, toks2)
    assert np.array_equal(l2[:, :2], logits[:, :2]) and not np.array_equal(l2[:, 2:], logits[:, 2:])
