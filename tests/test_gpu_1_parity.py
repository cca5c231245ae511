"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Index work (slots, gathers) must be bit-exact; floating point within the
stated tolerances.  Needs a real MI355X: run with -m gpu."""
import math

import numpy as np
import pytest
import torch

import chiron_oracle as orc
from helpers import as_f64, bf16_to_f32, bits, fresh_pool, gpu_setup, make_case
from paper_2501_08090_amd import inputs as I

pytestmark = pytest.mark.gpu

# bf16 weights/cache are identical on both sides and activations enter the matrix cores as two
# bf16 terms (relative error 2^-17 per term), so a single kernel differs from the fp32/double
# oracle by ~1e-5 of the output scale; 1e-4 leaves an order of magnitude.
KERNEL_TOL = 1e-4
# whole step: the bar is max|dlogit| <= 2e-2 * std(oracle logits) and argmax agreement >= 99% of rows
STEP_TOL = 2e-2


def B():
    from paper_2501_08090_amd import binding
    return binding


def rel_err(got, want):
    return float(np.abs(got - want).max() / (want.std() + 1e-30))


# ---- slots: append / gather are pure index work, bit-exact ---------------------------------------

@pytest.mark.parametrize("m,kind,batch", [(I.TINY, "tiny", 4), (dict(I.TINY, head_dim=128, n_kv_heads=2, n_q_heads=8), "tiny", 3)])
def test_append_gather_bit_exact(m, kind, batch):
    c = make_case(m=m, batch=batch, kind=kind, seed=11, storage="bf16")
    g = gpu_setup(c, poison=True)
    opool = fresh_pool(c)
    o = 0
    for i, L in enumerate(c.seq_lens):
        L = int(L)
        for l in range(m["n_layers"]):
            print("gather seq", i, "layer", l, "len", L, flush=True)
            k, v = g.pool.gather(l, g.block_table[i].contiguous(), L)
            ok, ov = orc.gather_kv(opool, l, c.block_table[i], L)
            assert np.array_equal(bits(k), ok) and np.array_equal(bits(v), ov)
            assert np.array_equal(bits(k), c.kv[l][0][o:o + L])
        # slots of the sequence's pages that were never written still hold the fill pattern
        npages = int(I.pages_needed([L])[0])
        k, v = g.pool.gather(0, g.block_table[i].contiguous(), npages * 16)
        assert np.all(bits(k)[L:] == 0x7FC0) and np.all(bits(v)[L:] == 0x7FC0)
        o += L


def test_append_overwrites_only_its_slot():
    c = make_case(batch=3, seed=12, storage="bf16")
    g = gpu_setup(c)
    before = [[g.pool.gather(l, g.block_table[i].contiguous(), int(c.seq_lens[i])) for i in range(3)] for l in range(2)]
    nkv, d = c.m["n_kv_heads"], c.m["head_dim"]
    newk = I.normal((1, nkv, d), 1.0, 99, "newk").cuda()
    newv = I.normal((1, nkv, d), 1.0, 99, "newv").cuda()
    tgt_seq, tgt_pos = 1, int(c.seq_lens[1]) // 2
    g.pool.append(1, newk, newv, g.block_table, torch.tensor([tgt_seq], dtype=torch.int32, device="cuda"),
                  torch.tensor([tgt_pos], dtype=torch.int32, device="cuda"))
    for l in range(2):
        for i in range(3):
            k, v = g.pool.gather(l, g.block_table[i].contiguous(), int(c.seq_lens[i]))
            bk, bv = bits(before[l][i][0]).copy(), bits(before[l][i][1]).copy()
            if l == 1 and i == tgt_seq:
                bk[tgt_pos] = bits(newk)[0]
                bv[tgt_pos] = bits(newv)[0]
            assert np.array_equal(bits(k), bk) and np.array_equal(bits(v), bv)


@pytest.mark.parametrize("where", ["device", "pinned_host"])
def test_swap_out_in_relocates_a_request_bit_exactly(where):
    """Eviction to (host) memory and restore into other pages: gathers are bit-identical to the oracle's after the
    same migration, and the decode step's logits do not change by a single bit (page placement never matters)."""
    c = make_case(batch=4, seed=15, storage="bf16", pool_factor=3.0)
    g = gpu_setup(c)
    opool = fresh_pool(c)
    before = B().decode_step(g.model, g.pool, g.block_table, g.seq_lens, g.tokens).clone()
    # the step wrote position L of every request: rebuild the cache so that both sides hold the pre-step state
    g = gpu_setup(c)
    i = 3
    L = int(c.seq_lens[i]); npg = int(I.pages_needed([L])[0])
    nbytes = npg * g.model.kv_block_bytes()
    image = (torch.empty(nbytes, dtype=torch.uint8, device="cuda") if where == "device"
             else torch.empty(nbytes, dtype=torch.uint8, pin_memory=True))
    row = g.block_table[i].contiguous()
    g.pool.swap_out(row, npg, image)
    torch.cuda.synchronize()
    oimage = orc.swap(opool, c.block_table[i], npg)
    used = set(c.block_table[c.block_table >= 0].tolist())
    free = [b for b in range(c.num_blocks) if b not in used][:npg]
    new_row = np.full_like(c.block_table[i], -1); new_row[:npg] = free[::-1]
    # poison the old pages on the GPU (through the public append), then restore elsewhere
    nkv, d = c.m["n_kv_heads"], c.m["head_dim"]
    junk = torch.full((L, nkv, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    for l in range(c.m["n_layers"]):
        g.pool.append(l, junk, junk, g.block_table, torch.full((L,), i, dtype=torch.int32, device="cuda"),
                      torch.arange(L, dtype=torch.int32, device="cuda"))
    new_row_d = torch.from_numpy(new_row).cuda()
    g.pool.swap_in(new_row_d, npg, image)
    orc.swap(opool, new_row, npg, oimage)
    for l in range(c.m["n_layers"]):
        k, v = g.pool.gather(l, new_row_d, L)
        ok, ov = orc.gather_kv(opool, l, new_row, L)
        assert np.array_equal(bits(k), ok) and np.array_equal(bits(v), ov)
    bt2 = g.block_table.clone(); bt2[i] = new_row_d
    after = B().decode_step(g.model, g.pool, bt2, g.seq_lens, g.tokens)
    assert torch.equal(after, before)
    assert B().load().chiron_kv_swap_out(g.pool._h, None, 1, None, None) == -1


# ---- single kernels -------------------------------------------------------------------------------

@pytest.mark.parametrize("rows,n", [(1, 256), (5, 4096), (3, 8192), (2, 688)])
def test_rmsnorm(rows, n):
    rng = np.random.default_rng(rows * 1000 + n)
    h = (rng.standard_normal((rows, n)) * 3).astype(np.float32)
    gain = I.normal((n,), 0.3, 5, "gain", n, mean=1.0)
    got = B().op_rmsnorm(torch.from_numpy(h).cuda(), gain.cuda(), 1e-5).cpu().numpy()
    want = np.stack([orc.rmsnorm(h[r], I.to_numpy_storage(gain), 1e-5) for r in range(rows)])
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


@pytest.mark.parametrize("M,N,K", [(1, 256, 256), (4, 512, 256), (4, 1376, 256), (4, 256, 688), (33, 96, 1040),
                                   (64, 1024, 4096), (100, 160, 512), (130, 4096, 1024), (7, 1000, 64),
                                   (400, 8192, 512), (385, 2080, 256), (70, 512, 256), (96, 1376, 4096), (65, 4096, 512),
                                   (150, 1376, 256), (270, 4096, 512), (300, 28672, 256),
                                   # wide unsliced outputs of up to 32 rows take the 16-step weight ring (256-wide chunks):
                                   # one chunk, several chunks, a ragged last chunk
                                   (8, 20000, 256), (1, 17000, 1040), (32, 16416, 784), (17, 28672, 2048)])
def test_linear(M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    x = rng.standard_normal((M, K)).astype(np.float32)
    W = I.normal((N, K), 0.05, 6, "w", N, K)
    print("linear", M, N, K, flush=True)
    lin = B().Linear(W.cuda())
    xg = torch.from_numpy(x).cuda()
    got = lin(xg).cpu().numpy()
    want = orc.linear(x, I.to_numpy_storage(W))
    assert rel_err(got, want) <= KERNEL_TOL
    # residual form: y += x W^T
    y0 = rng.standard_normal((M, N)).astype(np.float32)
    got2 = lin(xg, torch.from_numpy(y0).cuda(), accumulate=True).cpu().numpy()
    assert rel_err(got2, want + y0) <= KERNEL_TOL
    lin.close()


def ffn_case(M, K, F, N, seed, scale=2.0):
    """x [M,K] fp32, Wg, Wu [F,K], Wd [N,F] bf16 and the oracle's act = silu(x Wg^T) * (x Wu^T), y = act Wd^T"""
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((M, K)) * scale).astype(np.float32)
    Wg, Wu = I.normal((F, K), 0.05, 7, "wg", seed), I.normal((F, K), 0.05, 7, "wu", seed)
    Wd = I.normal((N, F), 0.05, 7, "wd", seed)
    act = orc.swiglu(orc.linear(x, I.to_numpy_storage(Wg)), orc.linear(x, I.to_numpy_storage(Wu)))
    return x, Wg, Wu, Wd, act, orc.linear(act, I.to_numpy_storage(Wd))


@pytest.mark.parametrize("M,K,F", [(4, 256, 688), (1, 64, 16), (33, 1040, 48), (64, 512, 1408), (40, 64, 96), (96, 256, 2064),
                                   (130, 512, 704), (390, 256, 1376), (17, 2048, 14336), (300, 256, 14336),
                                   (400, 64, 14336)])  # the 128-row x 4-tile wave shape
def test_gate_up_swiglu(M, K, F):
    """SwiGLU in the gate/up projection's epilogue: every column of silu(gate) * up against the oracle (a slip in the
    interleaved packing would pair a gate column with the wrong up column); widths of one 16-column group, of ragged
    counts of workgroup columns, and the 8B width; rows across the tile shapes."""
    x, Wg, Wu, _, act, _ = ffn_case(M, K, F, 16, M + K + F)
    print("gate_up_swiglu", M, K, F, flush=True)
    gu = B().GateUp(Wg.cuda(), Wu.cuda())
    got = gu.swiglu(torch.from_numpy(x).cuda()).cpu().numpy()
    assert np.all(np.isfinite(got))
    assert rel_err(got, act) <= KERNEL_TOL
    with pytest.raises(TypeError):
        gu(torch.from_numpy(x).cuda())
    gu.close()


@pytest.mark.parametrize("M,K,F,N", [(4, 256, 688, 256), (64, 256, 1408, 512), (40, 64, 64, 96), (390, 128, 704, 512), (80, 512, 704, 512),
                                     (96, 64, 64, 96), (97, 64, 688, 96), (200, 256, 2048, 1024), (513, 128, 688, 512),
                                     (600, 64, 2048, 256), (520, 64, 4096, 64)])  # last: tiled output from the widest wave shape
def test_swiglu_ffn(M, K, F, N):
    """The feed-forward block as the step runs it: gate/up with the SwiGLU epilogue, then the down projection, the
    intermediate as fp32 rows (up to 512 rows at these widths) or as tiled bf16 terms (from 513 rows on; F = 688 leaves
    K padding in the down projection's operand).  test_linear_large_batch_kernel forces the tiled form at other sizes."""
    x, Wg, Wu, Wd, _, want = ffn_case(M, K, F, N, M + K + F + N)
    print("swiglu_ffn", M, K, F, N, flush=True)
    gu, down = B().GateUp(Wg.cuda(), Wu.cuda()), B().Linear(Wd.cuda())
    xg = torch.from_numpy(x).cuda()
    got = gu.ffn(down, xg).cpu().numpy()
    assert rel_err(got, want) <= KERNEL_TOL
    y0 = np.random.default_rng(5).standard_normal((M, N)).astype(np.float32)
    got2 = gu.ffn(down, xg, torch.from_numpy(y0).cuda(), accumulate=True).cpu().numpy()
    assert rel_err(got2, want + y0) <= KERNEL_TOL
    gu.close(); down.close()


def test_linear_over_seeded_random_shapes():
    """The launch shape (rows per tile, column tiles per wave, K-slices, pre-split input) is chosen from M, N and K by
    several rules: 48 seeded random shapes, widths from a few columns to more than two workgroups per CU and rows
    across every tile boundary, each against the oracle; every third shape also as the down projection of a feed-forward
    block behind a gate/up projection with the SwiGLU epilogue."""
    rng = np.random.default_rng(2024)
    for case in range(48):
        M = int(rng.integers(1, 700))
        N = int(rng.choice([rng.integers(1, 200), rng.integers(200, 3000), rng.integers(3000, 40000)]))
        K = 16 * int(rng.integers(1, 1 + (64 if N < 3000 else 16)))
        x = rng.standard_normal((M, K)).astype(np.float32)
        W = I.normal((N, K), 0.05, 9, "wr", case)
        print("random linear", case, M, N, K, flush=True)
        lin = B().Linear(W.cuda())
        want = orc.linear(x, I.to_numpy_storage(W))
        got = lin(torch.from_numpy(x).cuda()).cpu().numpy()
        assert rel_err(got, want) <= KERNEL_TOL, (M, N, K)
        if case % 3 == 0:
            Kin = 16 * int(rng.integers(1, 9))
            xin = (rng.standard_normal((M, Kin)) * 2).astype(np.float32)
            Wg, Wu = I.normal((K, Kin), 0.05, 9, "wrg", case), I.normal((K, Kin), 0.05, 9, "wru", case)
            gu = B().GateUp(Wg.cuda(), Wu.cuda())
            got = gu.ffn(lin, torch.from_numpy(xin).cuda()).cpu().numpy()
            act = orc.swiglu(orc.linear(xin, I.to_numpy_storage(Wg)), orc.linear(xin, I.to_numpy_storage(Wu)))
            want = orc.linear(act, I.to_numpy_storage(W))
            assert rel_err(got, want) <= KERNEL_TOL, (M, N, K, Kin, "ffn")
            gu.close()
        lin.close()


@pytest.mark.parametrize("M,N,K", [(256, 512, 256), (300, 1000, 688), (513, 2080, 1040), (97, 96, 64), (640, 4096, 512)])
def test_linear_large_batch_kernel(M, N, K):
    """the large-batch path (activations pre-split into tiled bf16 terms, copied straight into LDS), forced at any M"""
    rng = np.random.default_rng(M * 5 + N * 3 + K)
    x = rng.standard_normal((M, K)).astype(np.float32)
    W = I.normal((N, K), 0.05, 8, "wb", N, K)
    print("linear big", M, N, K, flush=True)
    b = B()
    b.set_tuning("linear_big_min_m", 1)
    b.set_tuning("linear_big_all", 1)
    try:
        lin = b.Linear(W.cuda())
        xg = torch.from_numpy(x).cuda()
        got = lin(xg).cpu().numpy()
        want = orc.linear(x, I.to_numpy_storage(W))
        assert rel_err(got, want) <= KERNEL_TOL
        y0 = rng.standard_normal((M, N)).astype(np.float32)
        got2 = lin(xg, torch.from_numpy(y0).cuda(), accumulate=True).cpu().numpy()
        assert rel_err(got2, want + y0) <= KERNEL_TOL
        lin.close()
        # the feed-forward block with its intermediate forced into the tiled form at this M: F = K is the width of
        # the gate/up output and of the down projection's input
        xs, Wg, Wu, Wd, _, want3 = ffn_case(M, 64, K, N, M + N + K)
        gu, down = b.GateUp(Wg.cuda(), Wu.cuda()), b.Linear(Wd.cuda())
        got3 = gu.ffn(down, torch.from_numpy(xs).cuda()).cpu().numpy()
        assert rel_err(got3, want3) <= KERNEL_TOL
        gu.close(); down.close()
    finally:
        b.set_tuning("linear_big_min_m", 0)
        b.set_tuning("linear_big_all", 0)


def test_rope_large_positions():
    rng = np.random.default_rng(21)
    pos = np.array([0, 1, 17, 4095, 32767, 131071], np.int32)
    x = rng.standard_normal((len(pos), 3, 128)).astype(np.float32)
    got = B().op_rope(torch.from_numpy(x).cuda(), torch.from_numpy(pos).cuda(), 500000.0).cpu().numpy()
    want = np.stack([orc.rope(x[r], int(pos[r]), 500000.0) for r in range(len(pos))])
    assert np.abs(got - want).max() <= 2e-6
    assert np.array_equal(got[0], x[0])


@pytest.mark.parametrize("d,nq,nkv,lens", [
    (64, 4, 2, [1, 15, 16, 17, 128]),
    (128, 32, 8, [1, 16, 33, 700, 64, 2049]),
    (128, 8, 1, [5, 300]),
    (128, 4, 4, [250]),
])
def test_paged_attention(d, nq, nkv, lens):
    m = dict(I.TINY, n_layers=2, head_dim=d, n_q_heads=nq, n_kv_heads=nkv, hidden=256)
    lens = np.array(lens, np.int32)
    # the case's seq_lens are the cached tokens; attention here spans exactly those
    c = make_case(m=m, seed=13, storage="bf16", seq_lens=lens, poison_unused=True)
    g = gpu_setup(c, poison=True)
    opool = fresh_pool(c)
    rng = np.random.default_rng(14)
    q = (rng.standard_normal((len(lens), nq * d)) * 1.3).astype(np.float32)
    for layer in (0, 1):
        print("attention d", d, "nq", nq, "nkv", nkv, "layer", layer, flush=True)
        got = B().op_paged_attention(g.model, g.pool, layer, torch.from_numpy(q).cuda(), g.block_table, g.seq_lens).cpu().numpy()
        want = np.stack([orc.paged_attention(opool, layer, c.block_table[i], int(lens[i]), q[i].reshape(nq, d)).reshape(-1)
                         for i in range(len(lens))])
        assert np.all(np.isfinite(got))
        assert np.abs(got - want).max() <= KERNEL_TOL * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("grid,chunk", [(4, 0), (4, 3), (2, 1), (0, 5), (8, 2), (24, 1)])
def test_paged_attention_work_list_over_several_rounds(grid, chunk):
    """A small persistent grid (grid workgroups = 4*grid wave slots) makes every wave walk several items of the work
    list: its own first, then items whose indices it draws from ticket counters (one counter below 8 workgroups, eight
    from there on), records fetched one item ahead; forced chunk sizes give items of 1, 2, 3 or 5 pages with ragged
    ends.  24 requests of 1..1500 cached tokens, 4 query heads per KV head.  The call is made twice and must give the
    same bits (the counters' state between the layers of one step is covered by the multi-layer steps at batch 512)."""
    d, nq, nkv = 128, 8, 2
    rng = np.random.default_rng(41)
    lens = rng.integers(1, 1500, size=24).astype(np.int32)
    lens[:4] = [1, 16, 17, 1499]
    m = dict(I.TINY, n_layers=1, head_dim=d, n_q_heads=nq, n_kv_heads=nkv, hidden=256)
    c = make_case(m=m, seed=17, storage="bf16", seq_lens=lens, poison_unused=True)
    g = gpu_setup(c, poison=True)
    opool = fresh_pool(c)
    q = (rng.standard_normal((len(lens), nq * d)) * 1.3).astype(np.float32)
    b = B()
    b.set_tuning("attn_grid", grid)
    b.set_tuning("attn_chunk_pages", chunk)
    try:
        print("attention grid", grid, "chunk", chunk, flush=True)
        got = b.op_paged_attention(g.model, g.pool, 0, torch.from_numpy(q).cuda(), g.block_table, g.seq_lens).cpu().numpy()
        again = b.op_paged_attention(g.model, g.pool, 0, torch.from_numpy(q).cuda(), g.block_table, g.seq_lens).cpu().numpy()
    finally:
        b.set_tuning("attn_grid", 0)
        b.set_tuning("attn_chunk_pages", 0)
    want = np.stack([orc.paged_attention(opool, 0, c.block_table[i], int(lens[i]), q[i].reshape(nq, d)).reshape(-1)
                     for i in range(len(lens))])
    assert np.all(np.isfinite(got))
    assert np.abs(got - want).max() <= KERNEL_TOL * max(1.0, np.abs(want).max())
    assert np.array_equal(got, again)  # which wave takes which item does not enter the result


# ---- the whole step ---------------------------------------------------------------------------------

def run_both(c, g=None, poison=False):
    g = g or gpu_setup(c, poison=poison)
    logits = B().decode_step(g.model, g.pool, g.block_table, g.seq_lens, g.tokens)
    torch.cuda.synchronize()
    opool = fresh_pool(c)
    want, slots = orc.decode_step(c.cfg, c.w, opool, c.block_table, c.seq_lens, c.tokens)
    return g, logits.cpu().numpy(), want, opool


def check_logits(got, want, min_agree=0.99):
    sig = want.std()
    err = np.abs(got - want).max() / sig
    agree = float((got.argmax(1) == want.argmax(1)).mean())
    print("max|d|/sigma = %.3e, argmax agreement = %.4f" % (err, agree), flush=True)
    assert np.all(np.isfinite(got))
    assert err <= STEP_TOL
    assert agree >= min_agree
    return err


@pytest.mark.parametrize("seed,jitter", [(0, 0.0), (1, 0.2)])
def test_decode_step_tiny_config(seed, jitter):
    """Tiny decoder (2 layers, hidden 256, 4q/2kv heads of 64, FFN 688, vocab 1024), batch 4, contexts U{16..128},
    16-token pages, shuffled block table, bf16-rounded copies of the fp32 draws on both sides."""
    c = make_case(batch=4, seed=seed, storage="bf16", gain_jitter=jitter, poison_unused=True)
    g, got, want, opool = run_both(c, poison=True)
    assert got.shape == (4, 1024)
    err = check_logits(got, want, min_agree=1.0)
    assert err <= 2e-3   # what the two-term activation split should deliver on two layers
    B().validate_step_inputs(g.model, g.pool, g.block_table, g.seq_lens, g.tokens)
    # slot contract: position p of every request now holds the new K/V (value within one bf16 ulp of the
    # oracle's, since both sides round their own fp32 k,v), every older position is bit-unchanged
    o = 0
    for i, L in enumerate(c.seq_lens):
        L = int(L)
        for l in range(c.m["n_layers"]):
            k, v = g.pool.gather(l, g.block_table[i].contiguous(), L + 1)
            ok, ov = orc.gather_kv(opool, l, c.block_table[i], L + 1)
            assert np.array_equal(bits(k)[:L], ok[:L]) and np.array_equal(bits(v)[:L], ov[:L])
            assert np.array_equal(bits(k)[:L], c.kv[l][0][o:o + L])
            for a, b in ((bits(k)[L], ok[L]), (bits(v)[L], ov[L])):
                fa, fb = bf16_to_f32(a), bf16_to_f32(b)
                # one bf16 ulp of the element, plus the fp32-level difference of the two k/v (visible where a
                # rotated element nearly cancels)
                assert np.all(np.abs(fa - fb) <= np.abs(fb) * 2.0 ** -7 + 1e-4 * np.abs(fb).max())
                assert np.mean(a == b) > 0.95
        o += L


def test_decode_step_edge_lengths_and_batch_sizes():
    # empty context, page boundaries (the new token opens a fresh page at 16 and 32), a longer one
    c = make_case(seed=3, storage="bf16", seq_lens=[0, 15, 16, 31, 32, 1, 200], poison_unused=True)
    g, got, want, _ = run_both(c, poison=True)
    check_logits(got, want, min_agree=1.0)
    # a request's logits do not depend on the rest of the batch (up to summation order)
    for b in (1, 3):
        g2 = gpu_setup(c, poison=True)
        sub = B().decode_step(g2.model, g2.pool, g2.block_table, g2.seq_lens, g2.tokens, batch=b).cpu().numpy()
        assert np.abs(sub - want[:b]).max() <= STEP_TOL * want.std()
    # batch 0 is a no-op
    B().decode_step(g.model, g.pool, g.block_table, g.seq_lens, g.tokens, batch=0,
                    logits=torch.empty((1, 1024), device="cuda"))


def test_decode_step_batch_permutation_and_layout():
    c = make_case(batch=6, seed=4, storage="bf16")
    g, got, want, _ = run_both(c)
    perm = np.array([4, 2, 0, 5, 1, 3])
    c2 = make_case(batch=6, seed=4, storage="bf16", shuffle=False, pool_factor=1.0)   # contiguous pages
    assert np.array_equal(c2.seq_lens, c.seq_lens)
    g2 = gpu_setup(c2)
    p = torch.from_numpy(perm).cuda()
    got2 = B().decode_step(g2.model, g2.pool, g2.block_table[p].contiguous(), g2.seq_lens[p].contiguous(),
                           g2.tokens[p].contiguous()).cpu().numpy()
    # permuted batch on a different physical layout: same logits, permuted (up to the order of partial sums)
    assert np.abs(got2 - got[perm]).max() <= 1e-4 * want.std()
    check_logits(got2, want[perm], min_agree=1.0)


def test_decode_step_medium_shape_d128():
    """4 layers of the 8B head geometry (32q/8kv heads of 128) at reduced width, batch 70 (two M-tiles, ragged),
    contexts lognormal: exercises the d=128 attention path, G=4, split contexts and M > 64."""
    m = dict(I.LLAMA_8B, name="mid", n_layers=4, hidden=1024, ffn=2816, vocab=4096, n_q_heads=32, n_kv_heads=8)
    lens = I.lognormal_lengths(70, 300, 1, 1500, np.random.default_rng(5))
    c = make_case(m=m, seed=5, storage="bf16", seq_lens=lens, poison_unused=True)
    g, got, want, _ = run_both(c, poison=True)
    check_logits(got, want, min_agree=0.99)


def test_decode_step_over_seeded_random_geometries():
    """Eight seeded random decoders: 1-3 layers, hidden and FFN widths that are multiples of 16 but of nothing larger,
    head dimension 64 or 128, 1..16 query heads per KV head, vocabularies that are not multiples of 32, batches of
    1..90 requests with 0..600 cached tokens.  Every width goes through the K padding, column masking and tile rules of
    the projections, every head grouping through its attention instance."""
    rng = np.random.default_rng(77)
    for case in range(8):
        d = 64 if case % 2 == 0 else 128
        G = int(rng.choice([1, 2, 4, 8, 16]))
        nkv = int(rng.integers(1, 4)) if G <= 4 else 1
        m = dict(I.TINY, name="rand%d" % case, n_layers=int(rng.integers(1, 4)), hidden=16 * int(rng.integers(5, 40)),
                 n_q_heads=G * nkv, n_kv_heads=nkv, head_dim=d, ffn=16 * int(rng.integers(5, 90)),
                 vocab=int(rng.integers(50, 3000)), rope_base=float(rng.choice([1e4, 5e5])))
        batch = int(rng.integers(1, 91))
        lens = rng.integers(0, 600, size=batch).astype(np.int32)
        print("geometry", case, {k: m[k] for k in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")},
              "batch", batch, flush=True)
        c = make_case(m=m, seed=100 + case, storage="bf16", gain_jitter=0.1, seq_lens=lens, poison_unused=True)
        g, got, want, _ = run_both(c, poison=True)
        check_logits(got, want, min_agree=0.99)


G4_D128 = dict(I.TINY, head_dim=128, n_kv_heads=2, n_q_heads=8)
G8_D128 = dict(I.TINY, head_dim=128, n_kv_heads=1, n_q_heads=8)


@pytest.mark.parametrize("m,T", [(I.TINY, 2), (I.TINY, 4), (I.TINY, 8), (I.TINY, 9), (I.TINY, 17), (G4_D128, 4), (G4_D128, 3),
                                 (G4_D128, 5), (G4_D128, 8), (G4_D128, 11), (G8_D128, 2), (G8_D128, 5)])
def test_multi_token_step(m, T):
    """q_len > 1 (speculative-decoding verify shape): causal over the block, all T tokens' K/V appended.
    As many tokens as fit the 16 operand columns (16 / heads-per-KV-head) share one pass over the request's pages
    (operand columns token*G + head); longer blocks take several passes, the last one ragged (9 = 8+1, 17 = 8+8+1,
    11 = 4+4+3, 5 = 2+2+1).  Lengths 15, 31, 63 put the first new token at the end of a page / of a work item, so
    that later tokens open a page or an item in which the earlier ones see nothing."""
    lens = [14, 15, 31, 63, 60, 0, 127, 1]
    c = make_case(m=m, seed=16, storage="bf16", gain_jitter=0.1, seq_lens=lens, pool_factor=3.0)
    toks = I.token_ids(len(lens) * T, c.m["vocab"], 6).reshape(len(lens), T)
    bt, nb = I.make_block_table(np.asarray(lens) + T - 1, seed=16, pool_factor=3.0)
    c.block_table, c.num_blocks = bt, nb
    g = gpu_setup(c, max_batch=len(lens) * T, poison=True)
    B().validate_step_inputs(g.model, g.pool, g.block_table, g.seq_lens, torch.from_numpy(toks).cuda())
    got = B().decode_step_multi(g.model, g.pool, g.block_table, g.seq_lens, torch.from_numpy(toks).cuda()).cpu().numpy()
    opool = fresh_pool(c)
    want = orc.decode_step_multi(c.cfg, c.w, opool, bt, c.seq_lens, toks)
    assert got.shape == (len(lens), T, c.m["vocab"])
    check_logits(got.reshape(-1, c.m["vocab"]), want.reshape(-1, c.m["vocab"]), min_agree=1.0)
    # the T new positions of every request hold the oracle's k, v up to one bf16 ulp; older ones are untouched
    o = 0
    for i, L in enumerate(lens):
        k, v = g.pool.gather(1, g.block_table[i].contiguous(), L + T)
        ok, ov = orc.gather_kv(opool, 1, bt[i], L + T)
        assert np.array_equal(bits(k)[:L], ok[:L]) and np.array_equal(bits(v)[:L], ov[:L])
        fa, fb = bf16_to_f32(bits(k)[L:]), bf16_to_f32(ok[L:])
        assert np.all(np.abs(fa - fb) <= np.abs(fb) * 2.0 ** -7 + 1e-3 * np.abs(fb).max())
        o += L
    with pytest.raises(B().ChironError) as e:
        B().decode_step_multi(g.model, g.pool, g.block_table, g.seq_lens, torch.zeros((len(lens), T + 1), dtype=torch.int32, device="cuda"))
    assert e.value.code == -3


def test_continuous_batching_over_several_iterations():
    """The calls in the use the paper describes (Continuous Batching: requests join and leave the running batch between
    iterations; the queue and its lengths are the caller's): eight requests start, every iteration feeds each running
    request the token the oracle's greedy choice gave it and advances its length, some finish and others take
    their place, lengths cross page boundaries.  Both sides run the same schedule from the same cache content;
    every iteration's logits are compared."""
    lens0 = np.array([13, 15, 30, 47, 5, 64, 0, 95], np.int32)
    n_iter, grow = 7, 8
    c = make_case(seed=21, storage="bf16", gain_jitter=0.1, seq_lens=lens0, pool_factor=3.0)
    bt, nb = I.make_block_table(lens0 + grow, seed=21, pool_factor=3.0)   # pages for the tokens still to come
    c.block_table, c.num_blocks = bt, nb
    g = gpu_setup(c, poison=True)
    opool = fresh_pool(c)
    lens = lens0.copy()
    toks = c.tokens.copy()
    running = list(range(8))
    for it in range(n_iter):
        if it == 2:
            running = [0, 2, 3, 5, 7]          # three requests finish
        if it == 4:
            running = [7, 1, 0, 4, 5, 6]       # two waiting ones (their caches kept) join, order changes
        idx = np.asarray(running)
        B().validate_step_inputs(g.model, g.pool, g.block_table[idx].contiguous(), torch.from_numpy(lens[idx]).cuda(),
                                 torch.from_numpy(toks[idx]).cuda())
        got = B().decode_step(g.model, g.pool, g.block_table[idx].contiguous(), torch.from_numpy(lens[idx]).cuda(),
                              torch.from_numpy(toks[idx]).cuda()).cpu().numpy()
        want, _ = orc.decode_step(c.cfg, c.w, opool, np.ascontiguousarray(bt[idx]), lens[idx], toks[idx])
        print("iteration", it, "batch", running, flush=True)
        check_logits(got, want, min_agree=1.0)
        toks[idx] = want.argmax(1).astype(np.int32)   # greedy continuation, the same on both sides
        lens[idx] += 1
    assert lens.max() <= (lens0 + grow).max()
    # the caches agree afterwards: old content bit-exact, generated positions to one bf16 ulp
    for i in range(8):
        k, v = g.pool.gather(1, g.block_table[i].contiguous(), int(lens[i]))
        ok, ov = orc.gather_kv(opool, 1, bt[i], int(lens[i]))
        L0 = int(lens0[i])
        assert np.array_equal(bits(k)[:L0], ok[:L0]) and np.array_equal(bits(v)[:L0], ov[:L0])
        fa, fb = bf16_to_f32(bits(k)[L0:]), bf16_to_f32(ok[L0:])
        if fb.size:
            assert np.all(np.abs(fa - fb) <= np.abs(fb) * 2.0 ** -6 + 2e-3 * np.abs(fb).max())


def test_repeat_step_is_idempotent_and_profile_runs():
    c = make_case(batch=4, seed=6, storage="bf16")
    g, got, want, _ = run_both(c)
    again = B().decode_step(g.model, g.pool, g.block_table, g.seq_lens, g.tokens).cpu().numpy()
    assert np.abs(again - got).max() <= 1e-4 * want.std()
    pts = B().step_latency_profile(g.model, g.pool, g.block_table, g.seq_lens, g.tokens, [1, 2, 4], warmup=1, iters=3)
    assert [p["batch"] for p in pts] == [1, 2, 4]
    for p in pts:
        assert p["lat_ms_median"] > 0 and p["lat_ms_p99"] >= p["lat_ms_median"] and p["tokens_per_s"] > 0


def test_decode_step_replays_from_a_hip_graph():
    """The step only enqueues kernels, so it can be recorded into a HIP graph.  Three replays, each after eager work of
    the program's own on the same model (a step over another batch size, a host synchronisation) and into a logits
    buffer overwritten in between, must give the bits of the eager step.  A small attention grid makes the waves draw
    work items from the ticket counters, which only kernels of the step itself put back to zero."""
    m = dict(I.LLAMA_8B, name="mid", n_layers=3, hidden=1024, ffn=2816, vocab=4096, n_q_heads=32, n_kv_heads=8)
    lens = I.lognormal_lengths(70, 300, 1, 1500, np.random.default_rng(8))
    c = make_case(m=m, seed=8, storage="bf16", seq_lens=lens, poison_unused=True)
    g = gpu_setup(c, poison=True)
    b = B()
    b.set_tuning("attn_grid", 16)
    try:
        logits = torch.empty((70, 4096), dtype=torch.float32, device="cuda")
        step = lambda: b.decode_step(g.model, g.pool, g.block_table, g.seq_lens, g.tokens, logits=logits, batch=70)
        step()
        torch.cuda.synchronize()
        eager = logits.clone()
        assert torch.isfinite(eager).all()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        torch.cuda.synchronize()
        for replay in range(3):
            print("graph replay", replay, flush=True)
            other = b.decode_step(g.model, g.pool, g.block_table, g.seq_lens, g.tokens, batch=5 + replay)
            torch.cuda.synchronize()
            assert (other - eager[:5 + replay]).abs().max() <= 1e-2 * eager.std()  # other tile shapes: not the same bits
            logits.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(logits, eager), replay
    finally:
        b.set_tuning("attn_grid", 0)


def test_error_paths_on_device():
    c = make_case(batch=4, seed=7, storage="bf16")
    g = gpu_setup(c)
    Bd = B()
    with pytest.raises(Bd.ChironError) as e:
        five = lambda t: torch.cat([t, t[:1]]).contiguous()
        Bd.decode_step(g.model, g.pool, five(g.block_table), five(g.seq_lens), five(g.tokens), batch=5,
                       logits=torch.empty((5, 1024), device="cuda"))
    assert e.value.code == -3
    # the binding itself refuses a block table whose row stride is not the model's, or with too few rows
    with pytest.raises(ValueError):
        Bd.decode_step(g.model, g.pool, g.block_table[:, :-1].contiguous(), g.seq_lens, g.tokens)
    with pytest.raises(ValueError):
        Bd.decode_step(g.model, g.pool, g.block_table[:3].contiguous(), g.seq_lens, g.tokens)
    bad = g.block_table.clone(); bad[2, 0] = g.pool.num_blocks + 3
    with pytest.raises(Bd.ChironError) as e:
        Bd.validate_step_inputs(g.model, g.pool, bad, g.seq_lens, g.tokens)
    assert e.value.code == -4
    badtok = g.tokens.clone(); badtok[1] = 1024
    with pytest.raises(Bd.ChironError) as e:
        Bd.validate_step_inputs(g.model, g.pool, g.block_table, g.seq_lens, badtok)
    assert e.value.code == -7
    # the fused gate/up matrix: widths, pairing and use are checked on the host before anything is launched
    import ctypes as C
    W = I.normal((48, 64), 0.05, 7, "e_w").cuda()
    with pytest.raises(Bd.ChironError) as e:
        Bd.GateUp(W[:40].contiguous(), W[:40].contiguous())  # 40 columns: not a multiple of 16
    assert e.value.code == -2
    gu, plain, narrow = Bd.GateUp(W, W), Bd.Linear(I.normal((32, 48), 0.05, 7, "e_d").cuda()), Bd.Linear(I.normal((32, 64), 0.05, 7, "e_n").cuda())
    x = torch.zeros((3, 64), dtype=torch.float32, device="cuda")
    y = torch.zeros((3, 96), dtype=torch.float32, device="cuda")
    lib = Bd.load()
    ptr = lambda t: C.c_void_p(t.data_ptr())
    assert lib.chiron_op_linear(gu._h, ptr(x), C.c_int32(3), ptr(y), C.c_int32(0), None) == -1      # no plain product of it
    assert lib.chiron_op_gate_up_swiglu(plain._h, ptr(x), C.c_int32(3), ptr(y), None) == -1         # not a gate/up matrix
    with pytest.raises(Bd.ChironError) as e:
        gu.ffn(narrow, x)                                                                            # 48 columns into 64 inputs
    assert e.value.code == -2
    with pytest.raises(Bd.ChironError) as e:
        gu.ffn(gu, x)                                                                                # a gate/up matrix as the down projection
    assert e.value.code == -1
    assert gu.ffn(plain, x).shape == (3, 32) and float(gu.ffn(plain, x).abs().max()) == 0.0        # silu(0) * 0 = 0
    for l in (gu, plain, narrow):
        l.close()
