"""CPU checks of the parity harness's own logic (no GPU): the pass that draws queries again behind near-ties."""
import numpy as np

from paper_2501_04987_amd import inputs
from tests import parity_harness as ph


def test_settle_schedule_leaves_no_near_tie_and_is_reproducible(oracle):
    """With a threshold large enough to be met often: afterwards every margin is above it, the recorded results are
    exactly what a fresh oracle run on the final queries gives, and only queries of calls that met a near-tie changed."""
    c, G, d, thresh = 24, 2, 16, 0.08
    sched = [10, 0, 0, 0, 30, 0] + [0] * 700 + [40, 7] + [0] * 30
    T = sum(max(L, 1) for L in sched)
    q, k, v = inputs.stream_lowrank(5, T, G, d, kv_head=1)
    q0 = q.copy()
    ocfg = dict(budget=c, G=G, d=d, n_sink=2, n_recent=5, scale=d ** -0.5, flags=0)
    redraw = lambda t, n, a: inputs.redrawn_queries("lowrank", 5, t, n, a, G, d, kv_head=1)
    ref = ph.settle_schedule(oracle, ocfg, q, k, v, sched, redraw, thresh=thresh)
    assert ref["redraws"] > 5 and ph.near_ties(ref["margins"], thresh) == 0
    assert np.count_nonzero(ref["margins"] >= 0) == T - c
    changed = np.flatnonzero(np.any(q != q0, axis=(1, 2)))
    assert 0 < len(changed) < T // 2
    s = oracle.OracleStream(c, G, d, n_sink=2, n_recent=5)
    t = 0
    for L in sched:
        if L == 0:
            o, e, m, _, _ = s.decode_step(q[t], k[t], v[t])
            assert np.array_equal(o, ref["out"][t]) and e == ref["evicted"][t] and m == ref["margins"][t]
            t += 1
        else:
            r = s.prefill_chunk(q[t:t + L], k[t:t + L], v[t:t + L])
            assert np.array_equal(r["out"], ref["out"][t:t + L]) and np.array_equal(r["evicted"], ref["evicted"][t:t + L])
            t += L
    for a, b in zip(s.state(), ref["stream"].state()):
        assert np.array_equal(a, b)
    # the untouched run meets near-ties at this threshold (so the pass had work to do)
    plain = oracle.run_decode_stream(ocfg, q0, k, v)
    assert ph.near_ties(plain["margins"], thresh) > 0
