"""Pins of the CPU oracle against things other than itself: hand-worked values
(tests/golden), closed forms, invariants, brute force, and library routines
(numpy / torch float64).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

import chiron_oracle as orc
from helpers import as_f64, bf16_to_f32, fresh_pool, make_case
from paper_2501_08090_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")
TINY = I.TINY


# ---- bf16 rounding -----------------------------------------------------------------------------

def test_bf16_rounding_matches_library_and_ties_to_even():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(3000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, np.inf, -np.inf, 1e-40, 3.3895e38, 65280.0], np.float32)])
    got = orc.bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # exact ties: 1 + 2^-8 is halfway between 1 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert orc.bf16_bits(np.float32(1 + 2.0 ** -8)) == 0x3F80
    assert orc.bf16_bits(np.float32(1 + 3 * 2.0 ** -8)) == 0x3F82
    assert np.isnan(bf16_to_f32(orc.bf16_bits(np.array([np.nan], np.float32)))[0])


# ---- RMSNorm -----------------------------------------------------------------------------------

def test_rmsnorm_closed_form_and_invariants():
    rng = np.random.default_rng(2)
    n = 256
    ones = np.ones(n, np.float32)
    # constant vector c: out = c / sqrt(c^2 + eps)
    out = orc.rmsnorm(np.full(n, 3.0, np.float32), ones, 1e-5)
    assert np.allclose(out, 3.0 / math.sqrt(9.0 + 1e-5), rtol=1e-7)
    # eps sits inside the root and is added to the MEAN square: h=0 except one entry a -> a/sqrt(a^2/n+eps)
    h = np.zeros(n, np.float32); h[7] = 0.5
    assert np.isclose(orc.rmsnorm(h, ones, 0.25)[7], 0.5 / math.sqrt(0.25 / n + 0.25), rtol=1e-7)
    h = rng.standard_normal(n).astype(np.float32)
    out = orc.rmsnorm(h, ones, 0.0)
    assert np.isclose(np.sqrt(np.mean(out.astype(np.float64) ** 2)), 1.0, rtol=1e-6)      # unit RMS
    assert np.allclose(orc.rmsnorm(8 * h, ones, 0.0), out, rtol=1e-6)                     # scale invariance
    g = rng.standard_normal(n).astype(np.float32)
    assert np.allclose(orc.rmsnorm(h, g, 0.0), out * g, rtol=1e-6)                        # gain is elementwise
    want = torch.nn.functional.rms_norm(torch.from_numpy(h).double(), (n,), torch.from_numpy(g).double(), 1e-5)
    assert np.allclose(orc.rmsnorm(h, g, 1e-5), want.numpy(), rtol=1e-6)                  # library routine
    gb = orc.bf16_bits(g)                                                                 # bf16 gains widen exactly
    assert np.allclose(orc.rmsnorm(h, gb, 0.0), out * bf16_to_f32(gb), rtol=1e-6)


# ---- linear ------------------------------------------------------------------------------------

@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_linear_is_x_times_w_transposed(storage):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 37)).astype(np.float32)
    W = rng.standard_normal((11, 37)).astype(np.float32)
    Ws = W if storage == "f32" else orc.bf16_bits(W)
    want = x.astype(np.float64) @ as_f64(Ws).T
    got = orc.linear(x, Ws)
    assert got.shape == (5, 11)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    # one-hot input picks a weight column exactly
    e = np.zeros((1, 37), np.float32); e[0, 4] = 1
    assert np.array_equal(orc.linear(e, Ws)[0], as_f64(Ws)[:, 4].astype(np.float32))


# ---- RoPE --------------------------------------------------------------------------------------

def _golden_rope():
    for line in open(os.path.join(GOLD, "rope_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, c = line.split("|")
        d, base, pos = a.split()
        yield int(d), float(base), int(pos), np.array(b.split(), np.float32), np.array(c.split(), np.float64)


def test_rope_hand_worked_values():
    n = 0
    for d, base, pos, x, want in _golden_rope():
        got = orc.rope(x.reshape(1, d), pos, base)[0]
        assert np.allclose(got, want, atol=1e-6), (d, base, pos, got, want)
        n += 1
    assert n >= 6


def test_rope_closed_form_complex_rotation():
    rng = np.random.default_rng(4)
    d, heads, base = 64, 3, 10000.0
    x = rng.standard_normal((heads, d)).astype(np.float32)
    for pos in (0, 1, 17, 4095, 32767):
        got = orc.rope(x, pos, base)
        z = x[:, :d // 2].astype(np.float64) + 1j * x[:, d // 2:].astype(np.float64)
        theta = base ** (-2.0 * np.arange(d // 2) / d)
        zr = z * np.exp(1j * pos * theta)
        want = np.concatenate([zr.real, zr.imag], axis=1)
        assert np.allclose(got, want, atol=2e-6)
        if pos == 0:
            assert np.array_equal(got, x)
        # per-pair norm is preserved
        n_in = x[:, :d // 2] ** 2 + x[:, d // 2:] ** 2
        n_out = got[:, :d // 2] ** 2 + got[:, d // 2:] ** 2
        assert np.allclose(n_in, n_out, rtol=1e-5)


def test_rope_inner_product_depends_only_on_distance():
    rng = np.random.default_rng(5)
    d = 64
    q = rng.standard_normal((1, d)).astype(np.float32)
    k = rng.standard_normal((1, d)).astype(np.float32)
    ref = float(orc.rope(q, 9, 1e4)[0].astype(np.float64) @ orc.rope(k, 2, 1e4)[0].astype(np.float64))
    for shift in (5, 100, 1000):
        v = float(orc.rope(q, 9 + shift, 1e4)[0].astype(np.float64) @ orc.rope(k, 2 + shift, 1e4)[0].astype(np.float64))
        assert abs(v - ref) < 1e-4


# ---- slots, append, gather ---------------------------------------------------------------------

def test_slot_formula_brute_force_injective():
    c = make_case(batch=6, seed=3)
    seen = {}
    for i, L in enumerate(c.seq_lens):
        for t in range(int(L) + 1):
            s = orc.slot(c.block_table[i], t, 16)
            assert s == int(c.block_table[i][t // 16]) * 16 + t % 16
            assert 0 <= s < c.num_blocks * 16
            assert s not in seen, "two live tokens share a slot"
            seen[s] = (i, t)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_append_gather_roundtrip_and_only_target_slots_change(storage):
    c = make_case(batch=4, seed=1, storage=storage)
    pool = orc.Pool(c.cfg, c.num_blocks, np.float32 if storage == "f32" else np.uint16)
    sentinel = 0x1234 if storage == "bf16" else np.float32(123.25)
    pool.k[...] = sentinel
    pool.v[...] = sentinel
    k, v = c.kv[1]
    kf = as_f64(k).astype(np.float32); vf = as_f64(v).astype(np.float32)
    slots = orc.append_kv(pool, 1, kf, vf, c.block_table, c.seq_idx, c.pos)
    want_slots = c.block_table[c.seq_idx, c.pos // 16].astype(np.int64) * 16 + c.pos % 16
    assert np.array_equal(slots, want_slots)
    assert len(set(slots.tolist())) == len(slots)
    # plain numpy indexing as the independent statement of where things must be
    assert np.array_equal(pool.k[1, slots], k) and np.array_equal(pool.v[1, slots], v)
    mask = np.ones(pool.num_slots, bool); mask[slots] = False
    assert np.all(pool.k[1, mask] == sentinel) and np.all(pool.v[1, mask] == sentinel)
    assert np.all(pool.k[0] == sentinel) and np.all(pool.v[0] == sentinel)       # other layer untouched
    o = 0
    for i, L in enumerate(c.seq_lens):
        gk, gv = orc.gather_kv(pool, 1, c.block_table[i], int(L))
        assert np.array_equal(gk, k[o:o + L]) and np.array_equal(gv, v[o:o + L])
        o += int(L)


# ---- attention ---------------------------------------------------------------------------------

def _dense_attention_f64(q, K, V, G):
    """brute force: q [nq,d], K,V [len,nkv,d] float64 -> [nq,d]; full score row, softmax, weighted sum"""
    nq, d = q.shape
    out = np.zeros((nq, d))
    for a in range(nq):
        s = K[:, a // G, :] @ q[a] / math.sqrt(d)
        p = np.exp(s - s.max()); p /= p.sum()
        out[a] = p @ V[:, a // G, :]
    return out


def test_attention_hand_worked_value():
    rows = {"q": [], "k": [], "v": [], "o": []}
    for line in open(os.path.join(GOLD, "attention_cases.txt")):
        if line.strip() and not line.startswith("#"):
            t = line.split()
            rows[t[0]].append([float(x) for x in t[1:]])
    m = dict(TINY, n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=4)
    cfg = orc.make_config(m, orc.F32, orc.F32)
    pool = orc.Pool(cfg, 1)
    k = np.array(rows["k"], np.float32).reshape(2, 1, 4); v = np.array(rows["v"], np.float32).reshape(2, 1, 4)
    bt = np.array([[0]], np.int32)
    orc.append_kv(pool, 0, k, v, bt, [0, 0], [0, 1])
    o = orc.paged_attention(pool, 0, bt[0], 2, np.array(rows["q"], np.float32))
    assert np.allclose(o[0], rows["o"][0], atol=1e-7)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_attention_matches_dense_brute_force(storage):
    c = make_case(batch=4, seed=2, storage=storage)
    pool = fresh_pool(c)
    rng = np.random.default_rng(7)
    G = TINY["n_q_heads"] // TINY["n_kv_heads"]
    o0 = 0
    for i, L in enumerate(c.seq_lens):
        L = int(L)
        q = rng.standard_normal((TINY["n_q_heads"], TINY["head_dim"])).astype(np.float32)
        for layer in range(TINY["n_layers"]):
            K = as_f64(c.kv[layer][0][o0:o0 + L]); V = as_f64(c.kv[layer][1][o0:o0 + L])
            got = orc.paged_attention(pool, layer, c.block_table[i], L, q)
            want = _dense_attention_f64(q.astype(np.float64), K, V, G)
            assert np.allclose(got, want, atol=1e-6)
            # convex combination: inside the per-dimension range of V
            for a in range(TINY["n_q_heads"]):
                Va = V[:, a // G, :]
                assert np.all(got[a] <= Va.max(0) + 1e-6) and np.all(got[a] >= Va.min(0) - 1e-6)
        o0 += L


def test_attention_special_cases():
    m = dict(TINY, n_layers=1)
    cfg = orc.make_config(m, orc.F32, orc.F32)
    rng = np.random.default_rng(8)
    nkv, d, nq = m["n_kv_heads"], m["head_dim"], m["n_q_heads"]
    L = 40
    bt = np.array([[2, 0, 1]], np.int32)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    V = rng.standard_normal((L, nkv, d)).astype(np.float32)
    # all keys equal -> uniform softmax -> mean of V
    K = np.repeat(rng.standard_normal((1, nkv, d)).astype(np.float32), L, 0)
    pool = orc.Pool(cfg, 3)
    orc.append_kv(pool, 0, K, V, bt, np.zeros(L, np.int32), np.arange(L, dtype=np.int32))
    o = orc.paged_attention(pool, 0, bt[0], L, q)
    for a in range(nq):
        assert np.allclose(o[a], V[:, a // 2, :].astype(np.float64).mean(0), atol=1e-6)
    # a single token -> output is its value exactly
    o1 = orc.paged_attention(pool, 0, bt[0], 1, q)
    for a in range(nq):
        assert np.array_equal(o1[a], V[0, a // 2])
    # GQA == MHA with every KV head repeated G times
    K = rng.standard_normal((L, nkv, d)).astype(np.float32)
    orc.append_kv(pool, 0, K, V, bt, np.zeros(L, np.int32), np.arange(L, dtype=np.int32))
    og = orc.paged_attention(pool, 0, bt[0], L, q)
    m2 = dict(m, n_kv_heads=nq)
    cfg2 = orc.make_config(m2, orc.F32, orc.F32)
    pool2 = orc.Pool(cfg2, 3)
    orc.append_kv(pool2, 0, np.repeat(K, 2, 1), np.repeat(V, 2, 1), bt, np.zeros(L, np.int32), np.arange(L, dtype=np.int32))
    assert np.array_equal(orc.paged_attention(pool2, 0, bt[0], L, q), og)
    # a very large score does not overflow (max subtraction) and picks that token
    K[5] *= 0; K[5, :, 0] = 1e4
    qb = np.zeros((nq, d), np.float32); qb[:, 0] = 1e3
    orc.append_kv(pool, 0, K, V, bt, np.zeros(L, np.int32), np.arange(L, dtype=np.int32))
    ob = orc.paged_attention(pool, 0, bt[0], L, qb)
    assert np.all(np.isfinite(ob)) and np.allclose(ob[0], V[5, 0], atol=1e-6)


def test_swiglu_matches_library_silu():
    rng = np.random.default_rng(9)
    g = (rng.standard_normal(500) * 4).astype(np.float32); u = rng.standard_normal(500).astype(np.float32)
    want = torch.nn.functional.silu(torch.from_numpy(g).double()) * torch.from_numpy(u).double()
    assert np.allclose(orc.swiglu(g, u), want.numpy(), rtol=1e-6, atol=1e-7)
    assert orc.swiglu(np.zeros(1, np.float32), np.ones(1, np.float32))[0] == 0.0
    assert np.isclose(orc.swiglu(np.array([1.0], np.float32), np.array([2.0], np.float32))[0], 2 / (1 + math.exp(-1)))


# ---- page migration ---------------------------------------------------------------------------------

@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_swap_out_and_in_to_other_pages_is_a_pure_relocation(storage):
    c = make_case(batch=3, seed=21, storage=storage, pool_factor=3.0)
    pool = fresh_pool(c)
    i = 2
    L = int(c.seq_lens[i]); npg = int(I.pages_needed([L])[0])
    want = [orc.gather_kv(pool, l, c.block_table[i], L) for l in range(TINY["n_layers"])]
    others = [[orc.gather_kv(pool, l, c.block_table[r], int(c.seq_lens[r])) for l in range(TINY["n_layers"])] for r in (0, 1)]
    image = orc.swap(pool, c.block_table[i], npg)
    # the image holds exactly the request's slots: plain numpy indexing as the independent statement
    es = image.size // (TINY["n_layers"] * 2 * npg * 16 * TINY["n_kv_heads"] * TINY["head_dim"])
    img = image.view(np.float32 if es == 4 else np.uint16).reshape(TINY["n_layers"], 2, npg * 16, TINY["n_kv_heads"], TINY["head_dim"])
    slots = (c.block_table[i][np.arange(npg * 16) // 16].astype(np.int64) * 16 + np.arange(npg * 16) % 16)
    for l in range(TINY["n_layers"]):
        assert np.array_equal(img[l, 0], pool.k[l, slots]) and np.array_equal(img[l, 1], pool.v[l, slots])
    # scribble over the old pages, restore into pages nobody uses
    pool.k[:, slots] = 77; pool.v[:, slots] = 77
    used = set(c.block_table[c.block_table >= 0].tolist())
    free = [b for b in range(c.num_blocks) if b not in used][:npg]
    assert len(free) == npg
    new_row = np.full_like(c.block_table[i], -1); new_row[:npg] = free[::-1]
    orc.swap(pool, new_row, npg, image)
    for l in range(TINY["n_layers"]):
        k, v = orc.gather_kv(pool, l, new_row, L)
        assert np.array_equal(k, want[l][0]) and np.array_equal(v, want[l][1])
        for n, r in enumerate((0, 1)):     # nobody else moved
            k, v = orc.gather_kv(pool, l, c.block_table[r], int(c.seq_lens[r]))
            assert np.array_equal(k, others[n][l][0]) and np.array_equal(v, others[n][l][1])
