"""The rotary embedding through the entry point that allocates nothing (its cos/sin table is a fixed device array
inside the library) against the allocating entry point: same kernels, so the results are bit-identical.  Two calls in
a row, the second smaller, so that the second runs on a table that still holds the first call's values.  Needs a
real MI355X: run with -m gpu."""
import numpy as np
import pytest
import torch

import chiron_oracle as orc
from paper_2501_08090_amd import binding as B

pytestmark = pytest.mark.gpu


def test_rope_noalloc_matches_rope_on_two_calls_in_a_row():
    rng = np.random.default_rng(31)
    for rows, nh, d, base in ((1500, 3, 128, 500000.0), (37, 5, 64, 10000.0)):
        pos = rng.integers(0, 40000, size=rows).astype(np.int32)
        x = rng.standard_normal((rows, nh, d)).astype(np.float32)
        print("rope_noalloc rows", rows, "heads", nh, "d", d, flush=True)
        want = B.op_rope(torch.from_numpy(x).cuda(), torch.from_numpy(pos).cuda(), base)
        got = B.op_rope_noalloc(torch.from_numpy(x).cuda(), torch.from_numpy(pos).cuda(), base)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        # and the allocating entry point itself is the oracle's rotation
        ref = np.stack([orc.rope(x[r], int(pos[r]), base) for r in range(0, rows, 97)])
        assert np.abs(got.cpu().numpy()[::97] - ref).max() <= 2e-6


def test_rope_noalloc_rejects_sizes_beyond_its_table():
    x = torch.zeros((2049, 1, 128), dtype=torch.float32, device="cuda")
    pos = torch.zeros(2049, dtype=torch.int32, device="cuda")
    with pytest.raises(B.ChironError) as e:
        B.op_rope_noalloc(x, pos, 10000.0)
    assert e.value.code == -2 and "exceeds" in str(e.value)
    B.op_rope_noalloc(x[:2048].contiguous(), pos[:2048].contiguous(), 10000.0)   # exactly the limit
    torch.cuda.synchronize()
