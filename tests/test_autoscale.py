"""The local autoscaler update (Alg. 1): the oracle against hand-worked values and the properties the paper
states, and the library's host function against the oracle (integer results: exact).  CPU only."""
import os

import numpy as np

import chiron_oracle as orc
from paper_2501_08090_amd import binding as B

GOLD = os.path.join(os.path.dirname(__file__), "golden", "autoscale_cases.txt")


def cases():
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            a, b = line.split("|")
            yield [float(x) for x in a.split()], [float(x) for x in b.split()]


def test_oracle_hand_worked_passes():
    n = 0
    for (itl, slo, tp, tc, alpha, limit, mbs), (want, lb) in cases():
        got, glb = orc.autoscale_step(itl, slo, tp, tc, alpha, limit, mbs)
        assert got == int(want) and abs(glb - lb) < 1e-12, (itl, slo, tp, tc, mbs, got, glb)
        n += 1
    assert n >= 9


def test_oracle_properties_from_the_paper():
    # backpressure at or above one halves the batch size
    for lbp in (1.0, 1.3, 7.0):
        assert orc.autoscale_step(lbp * 0.2, 0.2, 0, 50, 0.5, 10**6, 1000)[0] == 500
    # below one the growth factor is 1 + alpha*(1/LB - 1): it shrinks to 1 as the backpressure approaches one ...
    prev = None
    for lb in (0.2, 0.4, 0.6, 0.8, 0.95, 0.999):
        new = orc.autoscale_step(lb * 0.2, 0.2, 0, 50, 0.5, 10**9, 100000)[0]
        assert abs(new / 100000 - (1 + 0.5 * (1 / lb - 1))) < 1e-4
        assert prev is None or new < prev
        prev = new
    assert abs(prev / 100000 - 1) < 1e-3
    # ... and the larger of the two backpressures decides
    assert orc.autoscale_step(0.1, 0.2, 95, 100, 0.5, 10**6, 1000)[1] == 0.95
    assert orc.autoscale_step(0.19, 0.2, 50, 100, 0.5, 10**6, 1000)[1] == 0.95
    # fixed point: a loop on a latency curve itl(b) = b ms with SLO 100 ms hovers around b = 100
    b, seen = 1, []
    for _ in range(60):
        b, _lb = orc.autoscale_step(b * 1e-3, 0.1, 0, b / (b * 1e-3), 0.5, 4096, b)
        seen.append(b)
    assert max(seen[20:]) <= 150 and min(seen[20:]) >= 50 and any(abs(x - 100) <= 25 for x in seen[20:])


def test_library_matches_oracle_exactly():
    for (itl, slo, tp, tc, alpha, limit, mbs), (want, lb) in cases():
        got, glb = B.local_autoscale_step(itl, slo, tp, tc, int(mbs), int(limit), alpha)
        assert got == int(want) and abs(glb - lb) < 1e-12
    rng = np.random.default_rng(0)
    for _ in range(3000):
        itl = float(rng.uniform(0, 0.5)) if rng.random() > 0.05 else 0.0
        slo = float(rng.uniform(0.01, 0.5))
        tp = float(rng.uniform(0, 2000)) if rng.random() > 0.2 else 0.0
        tc = float(rng.uniform(0, 2000)) if rng.random() > 0.05 else 0.0
        alpha = float(rng.choice([0.0, 0.25, 0.5, 1.0]))
        limit = int(rng.integers(1, 5000))
        mbs = int(rng.integers(1, limit + 1))
        assert B.local_autoscale_step(itl, slo, tp, tc, mbs, limit, alpha) == orc.autoscale_step(itl, slo, tp, tc, alpha, limit, mbs)


def test_library_rejects_bad_arguments():
    import ctypes as C
    lib = B.load()
    mb = C.c_int32(8)
    d = C.c_double
    assert lib.chiron_local_autoscale_step(d(0.1), d(0.0), d(0), d(1), d(0.5), 64, C.byref(mb), None) == -1
    assert lib.chiron_local_autoscale_step(d(0.1), d(0.2), d(0), d(1), d(1.5), 64, C.byref(mb), None) == -1
    assert lib.chiron_local_autoscale_step(d(0.1), d(0.2), d(0), d(1), d(0.5), 0, C.byref(mb), None) == -1
    assert lib.chiron_local_autoscale_step(d(0.1), d(0.2), d(0), d(1), d(0.5), 64, None, None) == -1
    assert mb.value == 8


# ---- the closed loop on fixed curves (deterministic; the measured curve is walked in the GPU tests) --------------

def _loop(itl_of, slo, policy, ticks=80, limit=512):
    """Alg. 1 ticked on a latency curve itl_of(batch) in seconds; throughput = batch / ITL.  policy 'as-printed':
    the previous tick's throughput always enters TBP; 'reset-after-no-growth': a tick that did not scale up leaves
    no comparable previous throughput (the next tick passes none)."""
    mbs, tput_prev, traj = 1, 0.0, []
    for _ in range(ticks):
        itl = itl_of(mbs)
        tput = mbs / itl
        new, lb = orc.autoscale_step(itl, slo, tput_prev, tput, 0.5, limit, mbs)
        traj.append((mbs, lb, new))
        tput_prev = tput if (policy == "as-printed" or new > mbs) else 0.0
        mbs = new
    return traj


def _affine_with_step(b):
    # the shape of a measured decode curve: a weight-streaming floor, a per-request slope, a step where the
    # projections need the next row tile
    return (3.5 + 0.06 * b + (1.0 if b > 64 else 0.0)) * 1e-3


def test_closed_loop_settles_under_the_slo_on_a_fixed_curve():
    slo = _affine_with_step(128)
    traj = _loop(_affine_with_step, slo, "reset-after-no-growth")
    sizes = [b for b, _, _ in traj]
    # climbs monotonically (no observation ever reaches backpressure one on a noise-free curve below the SLO) ...
    assert all(n >= b for b, _, n in traj)
    # ... and settles at the largest batch size whose latency is still under the SLO
    assert sizes[-1] == sizes[-10] and 120 <= sizes[-1] <= 128
    assert _affine_with_step(sizes[-1]) <= slo < _affine_with_step(sizes[-1] + 2)
    # a tighter SLO settles lower, a looser one higher
    lo = _loop(_affine_with_step, _affine_with_step(32), "reset-after-no-growth")[-1][0]
    hi = _loop(_affine_with_step, _affine_with_step(400), "reset-after-no-growth", ticks=200)[-1][0]
    assert lo <= 32 < sizes[-1] < hi <= 400


def test_closed_loop_as_printed_collapses_once_the_batch_size_repeats():
    """With the previous throughput always kept, the first tick whose update rounds to the same batch size is followed
    by TBP = 1 exactly (same batch, same throughput): the batch halves, the lower throughput after the halving reads
    as TBP > 1 and halves again, down to one request, where TBP = 1 keeps it.  This is why the closed loop here
    forgets the previous throughput after a tick that did not scale up."""
    slo = _affine_with_step(128)
    traj = _loop(_affine_with_step, slo, "as-printed")
    sizes = [b for b, _, _ in traj]
    first_repeat = next(i for i, (b, _, n) in enumerate(traj) if n == b)
    assert traj[first_repeat + 1][1] == 1.0 and traj[first_repeat + 1][2] < traj[first_repeat + 1][0]
    assert sizes[-1] == 1 and max(sizes) < 32
