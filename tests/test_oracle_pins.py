"""Pins for the CPU oracle: facts the paper prints, closed forms, invariants, a dense
library reference, exact-tie inputs and brute force on tiny inputs.  No GPU needed."""
import math
import os

import numpy as np
import pytest

from paper_2501_04987_amd import inputs
from tests.brute_force import BruteTreeKV
from tests.span_sim import SpanSim

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig3_worked_example.txt")


def _cfg(c, G=1, d=4, n_sink=0, n_recent=0, scale=None, flags=0):
    return dict(budget=c, G=G, d=d, n_sink=n_sink, n_recent=n_recent, scale=scale, flags=flags)


def _rand_stream(seed, T, G, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, G, d)), rng.standard_normal((T, d)), rng.standard_normal((T, d)))


# --------------------------------------------------------------------------- #
# P1: the worked example of Figure 3 / Section 4.1
# --------------------------------------------------------------------------- #
def _read_golden():
    facts = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        facts.setdefault(key, []).append(vals)
    return facts


def test_fig3_worked_example(oracle):
    g = _read_golden()
    c = int(g["cache_size"][0][0])
    T = int(g["sequence_length"][0][0])
    # rig the scores: paper token 2 (0-based position 1) draws nearly all attention at every step
    d = 2
    q = np.tile(np.array([1.0, 0.0]), (T, 1, 1))
    k = np.zeros((T, d))
    k[1, 0] = 8.0
    v = np.arange(T * d, dtype=np.float64).reshape(T, d)
    s = oracle.OracleStream(c, 1, d, scale=1.0)
    idx_before, evicted, caches = {}, {}, {}
    for t in range(T):
        step = t + 1  # the paper counts steps and tokens from 1
        idx_before[step] = s.idx
        before = list(s.retained() + 1) + [step]
        _, ev, _, _, _ = s.decode_step(q[t], k[t], v[t])
        evicted[step] = ev + 1 if ev >= 0 else None
        caches[step] = list(s.retained() + 1)
        if ev >= 0:
            i = idx_before[step] - 1
            assert evicted[step] in before[i:i + 2], "evicted token must lie in scope {idx, idx+1}"
    first = int(g["first_eviction_step"][0][0])
    assert [st for st in range(1, T + 1) if evicted[st] is not None][0] == first
    for st, val in g["idx_at_step"]:
        assert idx_before[int(st)] == int(val)
    st, a, b = map(int, g["scope_at_step"][0])
    assert list(range(1, c + 1))[idx_before[st] - 1: idx_before[st] + 1] == [a, b]
    st, tok = map(int, g["evicted_at_step"][0])
    assert evicted[st] == tok
    st, *toks = map(int, g["cache_after_step"][0])
    assert caches[st] == toks
    cyc = list(map(int, g["idx_cycle"][0]))
    assert [idx_before[first + i] for i in range(2 * len(cyc))] == cyc + cyc
    st, tok = map(int, g["scope_left_at_step"][0])
    before17 = caches[st - 1] + [st]
    assert before17[idx_before[st] - 1] == tok
    assert g["evicted_side_at_step"][0] == [str(st), "right"]
    assert evicted[st] == before17[idx_before[st]] and tok in caches[st]


def test_fig3_scopes_in_spans(oracle):
    """At every step the scope is the pair of spans the tree structure predicts (c=4, 17 tokens):
    5:(1|2) 6:(3|4) 7:(5|6) 8:(7|8) 9:(1-2|3-4) ... 13:(1-4|5-8) ... 17:(1-8|9-12)."""
    expect = {5: ((1, 1), (2, 2)), 6: ((3, 3), (4, 4)), 7: ((5, 5), (6, 6)), 8: ((7, 7), (8, 8)),
              9: ((1, 2), (3, 4)), 10: ((5, 6), (7, 8)), 11: ((9, 9), (10, 10)), 12: ((11, 11), (12, 12)),
              13: ((1, 4), (5, 8)), 14: ((9, 10), (11, 12)), 15: ((13, 13), (14, 14)),
              16: ((15, 15), (16, 16)), 17: ((1, 8), (9, 12))}
    for seed in range(20):
        q, k, v = _rand_stream(seed, 17, 1, 3)
        s = oracle.OracleStream(4, 1, 3)
        sim = SpanSim(4)
        for t in range(17):
            before = list(s.retained()) + [t]
            _, ev, _, _, _ = s.decode_step(q[t], k[t], v[t])
            scope = sim.step()
            if t + 1 < 5:
                assert ev == -1 and scope is None
                continue
            (llo, lhi), (rlo, rhi) = scope
            assert ((llo + 1, lhi + 1), (rlo + 1, rhi + 1)) == expect[t + 1]
            assert llo <= ev <= rhi
            i = before.index(ev)
            partner = before[i + 1] if llo <= ev <= lhi else before[i - 1]
            assert (rlo <= partner <= rhi) if llo <= ev <= lhi else (llo <= partner <= lhi)


# --------------------------------------------------------------------------- #
# P3: span structure (score independent) and P6: budget invariants
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("c,rounds,sizes", [
    (4, 1, [2, 2, 2, 2]), (4, 2, [4, 4, 2, 2]), (4, 3, [8, 4, 2, 2]), (4, 4, [12, 4, 2, 2]),
    (4, 5, [16, 4, 2, 2]), (8, 4, [16, 8, 4, 4, 2, 2, 2, 2]), (6, 3, [8, 6, 4, 2, 2, 2]),
    (5, 3, [8, 5, 3, 2, 2]),
])
def test_span_closed_forms(c, rounds, sizes):
    """s'_j = e_{2j-1} + e_{2j} with e = (spans at round start, then m ones)."""
    sim = SpanSim(c)
    for _ in range(c + rounds * c):
        sim.step()
    assert sim.sizes() == sizes
    e = [1] * c
    for _ in range(rounds):
        e = e + [1] * c
        e = [e[2 * j] + e[2 * j + 1] for j in range(c)]
    assert e == sizes


def test_span_fig1_setting():
    """Cache 128 on a 512-token sequence (the setting of Figure 1): 32 slots of span 8, 32 of 4, 64 of 2."""
    sim = SpanSim(128)
    for _ in range(512):
        sim.step()
    assert sim.sizes() == [8] * 32 + [4] * 32 + [2] * 64


@pytest.mark.parametrize("c,n_sink,n_recent,G", [(4, 0, 0, 1), (8, 0, 0, 2), (13, 0, 0, 1), (16, 2, 5, 1),
                                                  (16, 4, 4, 4), (9, 0, 3, 1), (9, 3, 0, 1), (6, 2, 3, 1)])
def test_retained_in_spans_and_budget(oracle, c, n_sink, n_recent, G):
    T, d = 6 * c + 7, 5
    for seed in range(5):
        q, k, v = _rand_stream(100 + seed, T, G, d)
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent)
        sim = SpanSim(c, n_sink, n_recent)
        for t in range(T):
            _, ev, margin, _, _ = s.decode_step(q[t], k[t], v[t])
            scope = sim.step()
            pos, S, Cn = s.state()
            # budget (the cache keeps a fixed size) and ordering
            assert len(pos) == min(t + 1, c)
            assert np.all(np.diff(pos) > 0)
            assert (ev >= 0) == (t + 1 > c) == (scope is not None)
            # every slot keeps exactly one position of its span; spans shrink towards the right
            for p, (lo, hi) in zip(pos, sim.spans):
                assert lo <= p <= hi
            sizes = sim.sizes()[n_sink:n_sink + sim.m]
            if scope is not None and sim.idx0 == 0:   # at a round boundary the tree region is sorted
                assert all(a >= b for a, b in zip(sizes, sizes[1:]))
            # sinks and the recent window are never evicted
            assert list(pos[:min(n_sink, t + 1)]) == list(range(min(n_sink, t + 1)))
            nr = min(n_recent, t + 1)
            if nr:
                assert list(pos[-nr:]) == list(range(t + 1 - nr, t + 1))
            # C counts the queries since arrival
            assert np.array_equal(Cn, t - pos + 1)
            if ev >= 0:
                assert scope[0][0] <= ev <= scope[1][1] and margin >= 0.0


def test_newest_token_without_recent_window(oracle):
    """Algorithm 1 verbatim (no protected window): token t is attended at step t and can be evicted
    only when the scope has reached the end of the cache (idx = c)."""
    c, T, d = 8, 100, 3
    q, k, v = _rand_stream(7, T, 1, d)
    s = oracle.OracleStream(c, 1, d)
    for t in range(T):
        idx = s.idx
        _, ev, _, _, _ = s.decode_step(q[t], k[t], v[t])
        if ev == t:
            assert idx == c
        else:
            assert s.retained()[-1] == t


# --------------------------------------------------------------------------- #
# P2: the keep-left ablation (Section 5.4) has a closed form
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("c,n_sink,n_recent", [(4, 0, 0), (8, 0, 0), (7, 0, 0), (12, 2, 3)])
def test_keep_left_closed_form(oracle, c, n_sink, n_recent):
    T, d = 9 * c + 3, 3
    q, k, v = _rand_stream(3, T, 1, d)
    s = oracle.OracleStream(c, 1, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.KEEP_LEFT)
    sim = SpanSim(c, n_sink, n_recent)
    for t in range(T):
        s.decode_step(q[t], k[t], v[t])
        sim.step()
        assert list(s.retained()) == [lo for lo, _ in sim.spans]


def test_literal_idx_schedule(oracle):
    """The printed update idx = (idx+1) mod c + 1 visits only every other scope."""
    c, d = 4, 2
    q, k, v = _rand_stream(0, 12, 1, d)
    s = oracle.OracleStream(c, 1, d, flags=oracle.IDX_LITERAL)
    seen = []
    for t in range(12):
        seen.append(s.idx)
        s.decode_step(q[t], k[t], v[t])
    assert seen[c:] == [1, 3, 1, 3, 1, 3, 1, 3]


# --------------------------------------------------------------------------- #
# P4: with no eviction the step is textbook causal softmax attention (Section 3.1)
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("G", [1, 3])
def test_no_eviction_equals_dense_causal_attention(oracle, G):
    import torch

    T, d = 40, 8
    q, k, v = _rand_stream(11, T, G, d)
    res = oracle.run_decode_stream(_cfg(T, G, d), q, k, v)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    logits = torch.einsum("tgd,sd->gts", tq, tk) / math.sqrt(d)
    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    A = torch.softmax(logits.masked_fill(~mask, float("-inf")), dim=-1)      # [G, T, T]
    out = torch.einsum("gts,sd->tgd", A, tv)
    np.testing.assert_allclose(res["out"], out.numpy(), rtol=0, atol=1e-12)
    pos, S, Cn = res["stream"].state()
    colsum = A.sum(dim=(0, 1)).numpy()
    np.testing.assert_allclose(S, colsum, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(Cn, T - np.arange(T))
    assert np.all(res["evicted"] == -1)
    # mass: every query row sums to one
    assert abs(S.sum() - G * T) < 1e-10


def test_prefill_without_eviction_equals_dense(oracle):
    import torch

    T, d, G = 48, 8, 2
    q, k, v = _rand_stream(12, T, G, d)
    s = oracle.OracleStream(T + 5, G, d)
    outs = []
    for lo, hi in [(0, 7), (7, 8), (8, 30), (30, 48)]:
        outs.append(s.prefill_chunk(q[lo:hi], k[lo:hi], v[lo:hi])["out"])
    out = np.concatenate(outs)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    logits = torch.einsum("tgd,sd->gts", tq, tk) / math.sqrt(d)
    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    A = torch.softmax(logits.masked_fill(~mask, float("-inf")), dim=-1)
    np.testing.assert_allclose(out, torch.einsum("gts,sd->tgd", A, tv).numpy(), rtol=0, atol=1e-12)
    pos, S, Cn = s.state()
    np.testing.assert_allclose(S, A.sum(dim=(0, 1)).numpy(), rtol=0, atol=1e-12)
    np.testing.assert_array_equal(Cn, T - np.arange(T))


# --------------------------------------------------------------------------- #
# P7: brute force on tiny inputs
# --------------------------------------------------------------------------- #
def _tiny_cases():
    rng = np.random.default_rng(2025)
    cases = []
    for seed in range(150):
        c = int(rng.integers(2, 9))
        n_sink = int(rng.integers(0, max(1, c // 3)))
        n_recent = int(rng.integers(0, max(1, c - n_sink - 1)))
        if seed % 3 == 0:
            n_sink = n_recent = 0
        cases.append((seed, c, n_sink, n_recent, int(rng.integers(1, 4)), int(rng.integers(1, 5)),
                      int(rng.integers(c + 1, 65))))
    return cases


def test_brute_force_decode(oracle):
    for seed, c, n_sink, n_recent, G, d, T in _tiny_cases():
        q, k, v = _rand_stream(seed, T, G, d)
        flags = [0, oracle.KEEP_LEFT, oracle.IDX_LITERAL][seed % 11 % 3] if seed % 11 < 3 else 0
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=flags)
        b = BruteTreeKV(c, G, d, n_sink, n_recent, keep_left=flags == oracle.KEEP_LEFT,
                        literal_idx=flags == oracle.IDX_LITERAL)
        for t in range(T):
            o, ev, _, _, _ = s.decode_step(q[t], k[t], v[t])
            bo, bev = b.decode_step(q[t].tolist(), k[t].tolist(), v[t].tolist())
            assert ev == bev, (seed, t)
            np.testing.assert_allclose(o, np.array(bo), rtol=0, atol=1e-12)
            assert list(s.retained()) == b.positions()
        pos, S, Cn = s.state()
        bS, bC = b.scores()
        np.testing.assert_allclose(S, bS, rtol=0, atol=1e-12)
        assert list(Cn) == bC


def test_brute_force_prefill(oracle):
    for seed, c, n_sink, n_recent, G, d, T in _tiny_cases()[:100]:
        q, k, v = _rand_stream(1000 + seed, T, G, d)
        rng = np.random.default_rng(seed)
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent)
        b = BruteTreeKV(c, G, d, n_sink, n_recent)
        lo = 0
        while lo < T:
            L = int(rng.integers(1, 2 * c + 2))
            hi = min(T, lo + L)
            if rng.random() < 0.25 and hi - lo == 1:      # mix single decode steps in
                o, ev, _, _, _ = s.decode_step(q[lo], k[lo], v[lo])
                bo, bev = b.decode_step(q[lo].tolist(), k[lo].tolist(), v[lo].tolist())
                assert ev == bev
                np.testing.assert_allclose(o, np.array(bo), rtol=0, atol=1e-12)
            else:
                r = s.prefill_chunk(q[lo:hi], k[lo:hi], v[lo:hi])
                bo, bev = b.prefill_chunk(q[lo:hi].tolist(), k[lo:hi].tolist(), v[lo:hi].tolist())
                assert list(r["evicted"]) == bev, (seed, lo, hi)
                np.testing.assert_allclose(r["out"], np.array(bo), rtol=0, atol=1e-12)
            assert list(s.retained()) == b.positions()
            lo = hi
        pos, S, Cn = s.state()
        bS, bC = b.scores()
        np.testing.assert_allclose(S, bS, rtol=0, atol=1e-12)
        assert list(Cn) == bC


# --------------------------------------------------------------------------- #
# P5: mass conservation with evictions
# --------------------------------------------------------------------------- #
def test_mass_conservation(oracle):
    c, G, d, T = 8, 2, 4, 60
    q, k, v = _rand_stream(5, T, G, d)
    s = oracle.OracleStream(c, G, d)
    lost = 0.0
    for t in range(T):
        pos0, S0, _ = s.state()
        _, ev, _, _, _ = s.decode_step(q[t], k[t], v[t])
        pos1, S1, _ = s.state()
        if ev >= 0:
            # the evicted token took its score with it: old score plus what it got at this step,
            # which is G minus what the survivors got at this step
            gained = {p: S1[i] - (S0[list(pos0).index(p)] if p in pos0 else 0.0) for i, p in enumerate(pos1)}
            got = G - sum(gained.values())
            old = S0[list(pos0).index(ev)] if ev in pos0 else 0.0
            assert got > -1e-12
            lost += old + got
        assert abs(S1.sum() + lost - G * (t + 1)) < 1e-9


# --------------------------------------------------------------------------- #
# P8: exact ties resolve towards evicting the left slot (strict ">")
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("c", [3, 7, 15])
def test_exact_ties(oracle, c):
    """q = 0 gives uniform attention; with c+1 a power of two every token that arrives after the
    cache filled has Sbar = 1/(c+1) exactly, older tokens have strictly larger Sbar."""
    d, T = 2, 6 * c + 5
    rng = np.random.default_rng(0)
    k, v = rng.standard_normal((T, d)), rng.standard_normal((T, d))
    q = np.zeros((T, 1, d))
    s = oracle.OracleStream(c, 1, d)
    cache = []      # reference: left wins iff it arrived while the cache was still filling
    idx0 = 0
    for t in range(T):
        _, ev, margin, _, _ = s.decode_step(q[t], k[t], v[t])
        cache.append(t)
        if len(cache) > c:
            left, right = cache[idx0], cache[idx0 + 1]
            gone = right if left < c else left
            cache.remove(gone)
            idx0 = (idx0 + 1) % c
            assert ev == gone
            if left >= c:
                assert margin == 0.0
        assert list(s.retained()) == cache
    pos, S, Cn = s.state()
    late = pos >= c
    assert np.all(S[late] / Cn[late] == 1.0 / (c + 1))


# --------------------------------------------------------------------------- #
# P9: consistency between the prefill chunk and the decode step
# --------------------------------------------------------------------------- #
def test_prefill_len1_is_decode(oracle):
    c, G, d, T = 10, 2, 6, 50
    q, k, v = _rand_stream(21, T, G, d)
    a = oracle.OracleStream(c, G, d, n_sink=1, n_recent=3)
    b = oracle.OracleStream(c, G, d, n_sink=1, n_recent=3)
    for t in range(T):
        o, ev, mg, _, _ = a.decode_step(q[t], k[t], v[t])
        r = b.prefill_chunk(q[t:t + 1], k[t:t + 1], v[t:t + 1])
        assert np.array_equal(o, r["out"][0]) and ev == r["evicted"][0] and mg == r["margins"][0]
    for x, y in zip(a.state(), b.state()):
        assert np.array_equal(x, y)


def test_prefill_spans_match_decode(oracle):
    """Chunked prefill keeps one position per span, the same spans as token-by-token decoding."""
    c, d = 16, 4
    for n_sink, n_recent in [(0, 0), (2, 4)]:
        q, k, v = _rand_stream(33, 200, 1, d)
        s = oracle.OracleStream(c, 1, d, n_sink=n_sink, n_recent=n_recent)
        sim = SpanSim(c, n_sink, n_recent)
        lo = 0
        for L in [5, 11, 1, 40, 16, 17, 64, 46]:
            s.prefill_chunk(q[lo:lo + L], k[lo:lo + L], v[lo:lo + L])
            for _ in range(L):
                sim.step()
            lo += L
            pos = s.retained()
            assert len(pos) == min(lo, c)
            for p, (a, b) in zip(pos, sim.spans):
                assert a <= p <= b


def test_dry_run_leaves_state(oracle):
    c, d = 5, 3
    q, k, v = _rand_stream(8, 20, 1, d)
    s = oracle.OracleStream(c, 1, d)
    for t in range(20):
        before = [x.copy() for x in s.state()]
        o1, ev1, m1, _, _ = s.decode_step(q[t], k[t], v[t], commit=False)
        for x, y in zip(before, s.state()):
            assert np.array_equal(x, y)
        assert s.t == t
        o2, ev2, m2, _, _ = s.decode_step(q[t], k[t], v[t])
        assert np.array_equal(o1, o2) and ev1 == ev2 and m1 == m2


def test_follow_mode(oracle):
    """The oracle adopts another implementation's choice only inside the near-tie threshold."""
    c, d = 4, 2
    q, k, v = _rand_stream(9, 5, 1, d)
    s = oracle.OracleStream(c, 1, d)
    for t in range(4):
        s.decode_step(q[t], k[t], v[t])
    _, ev, margin, _, _ = s.decode_step(q[4], k[4], v[4], commit=False)
    other = 1 - ev          # the scope at the first eviction is positions (0, 1)
    assert ev in (0, 1) and margin > 1e-6
    _, ev2, _, adopted, disagreed = s.decode_step(q[4], k[4], v[4], forced_pos=other, follow_thresh=1e-9,
                                                  commit=False)
    assert (ev2, adopted, disagreed) == (ev, 0, 1)
    _, ev3, _, adopted, disagreed = s.decode_step(q[4], k[4], v[4], forced_pos=other, follow_thresh=2.0,
                                                  commit=False)
    assert (ev3, adopted, disagreed) == (other, 1, 0)
    _, ev4, _, adopted, disagreed = s.decode_step(q[4], k[4], v[4], forced_pos=3, follow_thresh=2.0)
    assert (ev4, adopted, disagreed) == (ev, 0, 1)


def test_tiny_config_runs_in_seconds(oracle):
    """The tiny decode configuration: 2 heads, d 64, fp32, budget 64, 512 tokens."""
    for h in range(2):
        q, k, v = inputs.stream_iid(0, 512, 1, 64, kv_head=h, k_scale=1.0 / 8.0, dtype="f32")
        res = oracle.run_decode_stream(_cfg(64, 1, 64, 4, 28, scale=1.0), q, k, v)
        assert len(res["stream"]) == 64 and np.count_nonzero(res["evicted"] >= 0) == 512 - 64


# --------------------------------------------------------------------------- #
# One-shot block-level prompt compression (Section 4.2)
# --------------------------------------------------------------------------- #
def _prompt(seed, T, G, d, b):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((b, G, d)), rng.standard_normal((T, d)), rng.standard_normal((T, d))


def _block_layout(c, b, n_sink, n_recent):
    cb, sb, rb = c // b, -(-n_sink // b), -(-n_recent // b)
    return cb, sb, rb, cb - sb - rb


def _final_block_spans(N, c, b, n_sink, n_recent):
    cb, sb, rb, _ = _block_layout(c, b, n_sink, n_recent)
    sim = SpanSim(cb, sb, rb)
    for _ in range(N):
        sim.step()
    return sim.spans


@pytest.mark.parametrize("G", [1, 3])
def test_prompt_scores_equal_dense_window_attention(oracle, G):
    """Token scores are the column means of the window's causal attention matrix (library softmax, fp64);
    block scores are the means of their tokens; each window row carries mass 1."""
    import torch
    T, d, b, c = 96, 8, 8, 32
    Qw, K, V = _prompt(5, T, G, d, b)
    s = oracle.OracleStream(c, G, d, n_sink=2, n_recent=8)
    r = s.prefill_prompt(Qw, K, V, b)
    logits = torch.einsum("igd,jd->gij", torch.tensor(Qw), torch.tensor(K)) / math.sqrt(d)
    rows = torch.arange(b)[:, None] + (T - b)
    mask = torch.arange(T)[None, :] > rows
    A = torch.softmax(logits.masked_fill(mask[None], float("-inf")), dim=-1)     # [G, b, T]
    seen = (~mask).sum(0).double()                                               # window queries that see j
    want = (A.sum((0, 1)) / seen).numpy()
    np.testing.assert_allclose(r["token_scores"], want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r["block_scores"], want.reshape(-1, b).mean(1), rtol=1e-12, atol=1e-15)
    assert abs(float((r["token_scores"] * seen.numpy()).sum()) - G * b) < 1e-9


@pytest.mark.parametrize("c,b,T,n_sink,n_recent", [(16, 4, 64, 0, 0), (16, 4, 100, 0, 4), (32, 4, 256, 4, 8),
                                                   (24, 2, 90, 3, 5), (8, 1, 40, 0, 0), (64, 8, 1024, 4, 28)])
def test_prompt_survivor_is_rightmost_maximum_of_its_span(oracle, c, b, T, n_sink, n_recent):
    """With frozen scores the block a slot keeps is the best block of the slot's span, the rightmost one
    among equals (strict '>' keeps the right member of a tied scope); the spans do not depend on scores."""
    G, d = 1, 4
    Qw, K, V = _prompt(c + T, T, G, d, b)
    s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent)
    r = s.prefill_prompt(Qw, K, V, b)
    beta = r["block_scores"]
    kept = []
    for lo, hi in _final_block_spans(T // b, c, b, n_sink, n_recent):
        seg = beta[lo:hi + 1]
        kept.append(lo + int(np.flatnonzero(seg == seg.max())[-1]))
    want = np.concatenate([np.arange(k * b, (k + 1) * b) for k in kept])
    np.testing.assert_array_equal(s.retained(), want)
    assert len(s) == min(T, c) and s.t == T and s.idx == 1


def test_prompt_keep_left_keeps_first_block_of_every_span(oracle):
    c, b, T, n_sink, n_recent = 32, 4, 200, 4, 8
    Qw, K, V = _prompt(1, T, 1, 4, b)
    s = oracle.OracleStream(c, 1, 4, n_sink=n_sink, n_recent=n_recent, flags=oracle.KEEP_LEFT)
    s.prefill_prompt(Qw, K, V, b)
    want = np.concatenate([np.arange(lo * b, (lo + 1) * b) for lo, _ in _final_block_spans(T // b, c, b, n_sink, n_recent)])
    np.testing.assert_array_equal(s.retained(), want)


def test_prompt_uniform_attention_ties_keep_the_right_block(oracle):
    """q = 0: every token before the window gets bit-identical scores, so every scope before the window is an
    exact tie and the strict comparison evicts its left member: each span keeps its last block."""
    c, b, T = 16, 4, 128
    _, K, V = _prompt(2, T, 1, 4, b)
    s = oracle.OracleStream(c, 1, 4, n_sink=0, n_recent=4)
    r = s.prefill_prompt(np.zeros((b, 1, 4)), K, V, b)
    assert len(set(r["token_scores"][: T - b].tolist())) == 1
    spans = _final_block_spans(T // b, c, b, 0, 4)
    want = np.concatenate([np.arange(hi * b, (hi + 1) * b) for _, hi in spans])
    np.testing.assert_array_equal(s.retained(), want)


def test_prompt_that_fits_is_kept_whole(oracle):
    c, b, T = 32, 4, 24
    Qw, K, V = _prompt(3, T, 2, 4, b)
    s = oracle.OracleStream(c, 2, 4, n_sink=4, n_recent=8)
    r = s.prefill_prompt(Qw, K, V, b)
    np.testing.assert_array_equal(s.retained(), np.arange(T))
    assert (r["evicted_blocks"] == -1).all()
    Kc, Vc = s.kv()
    np.testing.assert_array_equal(Kc, K)
    np.testing.assert_array_equal(Vc, V)


def test_prompt_hands_over_to_decoding(oracle):
    """After the prompt: C = T - position, S / C = the window average, idx = 1; decoding then keeps the budget
    and evicts inside the token-level scope, starting at the first one."""
    c, b, T, n_sink, n_recent, d = 16, 4, 64, 2, 4, 4
    Qw, K, V = _prompt(4, T, 1, d, b)
    s = oracle.OracleStream(c, 1, d, n_sink=n_sink, n_recent=n_recent)
    r = s.prefill_prompt(Qw, K, V, b)
    pos, S, C = s.state()
    np.testing.assert_array_equal(C, T - pos)
    np.testing.assert_allclose(S / C, r["token_scores"][pos], rtol=1e-15)
    Kc, Vc = s.kv()
    np.testing.assert_array_equal(Kc, K[pos])
    np.testing.assert_array_equal(Vc, V[pos])
    q, k, v = _rand_stream(9, 12, 1, d)
    m = c - n_sink - n_recent
    for t in range(12):
        before = list(s.retained()) + [T + t]
        i = n_sink + (t % m)
        _, ev, _, _, _ = s.decode_step(q[t], k[t], v[t])
        assert ev in before[i:i + 2] and len(s) == c
    assert (s.retained()[-n_recent:] == np.arange(T + 12 - n_recent, T + 12)).all()


def test_prompt_brute_force(oracle):
    for seed in range(60):
        rng = np.random.default_rng(seed)
        b = int(rng.integers(1, 4))
        cb = int(rng.integers(3, 7))
        c = cb * b
        n_sink = int(rng.integers(0, b + 1))
        n_recent = int(rng.integers(0, b + 1))
        if cb - (-(-n_sink // b)) - (-(-n_recent // b)) < 1:
            continue
        G, d = int(rng.integers(1, 3)), 3
        T = b * int(rng.integers(1, 14))
        Qw, K, V = _prompt(1000 + seed, T, G, d, b)
        keep_left = seed % 7 == 0
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.KEEP_LEFT if keep_left else 0)
        r = s.prefill_prompt(Qw, K, V, b)
        bf = BruteTreeKV(c, G, d, n_sink=n_sink, n_recent=n_recent, keep_left=keep_left)
        gone, sbar, beta = bf.prefill_prompt(Qw.tolist(), K.tolist(), V.tolist(), b)
        assert list(r["evicted_blocks"]) == gone, seed
        assert list(s.retained()) == bf.positions(), seed
        np.testing.assert_allclose(r["token_scores"], sbar, rtol=1e-12)
        np.testing.assert_allclose(r["block_scores"], beta, rtol=1e-12)
        S_b, C_b = bf.scores()
        _, S, C = s.state()
        np.testing.assert_allclose(S, S_b, rtol=1e-12)
        assert list(C) == C_b
        # and decoding goes on identically
        q, k, v = _rand_stream(seed, 6, G, d)
        for t in range(6):
            o1, e1, _, _, _ = s.decode_step(q[t], k[t], v[t])
            o2, e2 = bf.decode_step(q[t].tolist(), k[t].tolist(), v[t].tolist())
            assert e1 == e2, (seed, t)
            np.testing.assert_allclose(o1, np.array(o2), rtol=1e-10, atol=1e-12)


def test_prompt_rejects_what_does_not_fit(oracle):
    s = oracle.OracleStream(16, 1, 4)
    Qw, K, V = _prompt(0, 30, 1, 4, 4)
    with pytest.raises(ValueError):
        s.prefill_prompt(Qw, K, V, 4)            # 30 is not a multiple of 4
    with pytest.raises(ValueError):
        s.prefill_prompt(Qw[:3], K[:27], V[:27], 3)  # nor is the budget of 3
    s.prefill_prompt(Qw, K[:28], V[:28], 4)
    with pytest.raises(ValueError):
        s.prefill_prompt(Qw, K[:28], V[:28], 4)  # not empty any more


def test_prompt_follow_mode(oracle):
    """A forced block is adopted only when it is the other member of the scope and the margin is small."""
    c, b, T = 16, 4, 64
    Qw, K, V = _prompt(6, T, 1, 4, b)
    ref = oracle.OracleStream(c, 1, 4).prefill_prompt(Qw, K, V, b)
    first = int(np.flatnonzero(ref["evicted_blocks"] >= 0)[0])
    forced = ref["evicted_blocks"].copy()
    forced[first] = 1 - forced[first]            # the first scope is blocks (0, 1)
    s = oracle.OracleStream(c, 1, 4)
    r = s.prefill_prompt(Qw, K, V, b, forced_blocks=forced, follow_thresh=0.0)
    assert r["disagreed"] == 1 and r["adopted"] == 0 and r["evicted_blocks"][first] == ref["evicted_blocks"][first]
    s = oracle.OracleStream(c, 1, 4)
    r = s.prefill_prompt(Qw, K, V, b, forced_blocks=forced, follow_thresh=2.0)
    assert r["adopted"] == 1 and r["evicted_blocks"][first] == forced[first]


# --------------------------------------------------------------------------- #
# The accumulated-weight criterion (Section 4.1, "Importance Score": the variant that was tried next to the average)
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("c,n_sink,n_recent", [(8, 0, 0), (16, 2, 5), (13, 0, 4)])
def test_accumulated_uniform_attention_evicts_the_newer_token(oracle, c, n_sink, n_recent):
    """q = 0: every step adds 1 / len to every cached token, so the older token of a scope has strictly more
    accumulated weight and the right one is always evicted: the retained set is the keep-left closed form."""
    T, d = 6 * c, 3
    _, k, v = _rand_stream(3, T, 1, d)
    s = oracle.OracleStream(c, 1, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.SCORE_ACCUMULATED)
    sim = SpanSim(c, n_sink, n_recent)
    for t in range(T):
        s.decode_step(np.zeros((1, d)), k[t], v[t])
        sim.step()
        assert list(s.retained()) == [lo for lo, _ in sim.spans]


def test_accumulated_differs_from_averaged_only_through_the_counts(oracle):
    """Same stream, both criteria: S and C evolve identically until the first decision that differs; that
    decision is one where S_l > S_r but S_l / C_l <= S_r / C_r (the left token is the older one)."""
    c, G, d, T = 12, 2, 4, 200
    q, k, v = _rand_stream(11, T, G, d)
    a = oracle.OracleStream(c, G, d, flags=oracle.SCORE_ACCUMULATED)
    b = oracle.OracleStream(c, G, d)
    differed = False
    for t in range(T):
        pos_b, S_b, C_b = b.state()
        idx = b.idx
        _, ea, _, _, _ = a.decode_step(q[t], k[t], v[t])
        _, eb, _, _, _ = b.decode_step(q[t], k[t], v[t], commit=False)
        if ea != eb:
            # replay b's step to read the two scope members' S and C after the update
            probe = oracle.OracleStream(c, G, d)
            for u in range(t):
                probe.decode_step(q[u], k[u], v[u])
            before = list(probe.retained()) + [t]
            _, _, _, _, _ = probe.decode_step(q[t], k[t], v[t], commit=True)
            l_pos, r_pos = before[idx - 1], before[idx]
            assert {ea, eb} == {l_pos, r_pos}
            assert ea == r_pos and eb == l_pos          # accumulated keeps the older (left) token here
            differed = True
            break
        b.decode_step(q[t], k[t], v[t])
    assert differed, "the two criteria should part ways within 200 steps of a budget-12 cache"


def test_accumulated_brute_force(oracle):
    for seed in range(40):
        rng = np.random.default_rng(500 + seed)
        c = int(rng.integers(2, 9))
        n_sink = int(rng.integers(0, 2))
        n_recent = int(rng.integers(0, max(1, c - n_sink - 1)))
        G, d = int(rng.integers(1, 3)), 3
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.SCORE_ACCUMULATED)
        bf = BruteTreeKV(c, G, d, n_sink=n_sink, n_recent=n_recent, accumulated=True)
        T = 40
        q, k, v = _rand_stream(seed, T, G, d)
        t = 0
        while t < T:
            L = int(rng.integers(0, 6))
            if L == 0 or t + L > T:
                o1, e1, _, _, _ = s.decode_step(q[t], k[t], v[t])
                o2, e2 = bf.decode_step(q[t].tolist(), k[t].tolist(), v[t].tolist())
                assert e1 == e2, (seed, t)
                t += 1
            else:
                r = s.prefill_chunk(q[t:t + L], k[t:t + L], v[t:t + L])
                _, evs = bf.prefill_chunk(q[t:t + L].tolist(), k[t:t + L].tolist(), v[t:t + L].tolist())
                assert list(r["evicted"]) == evs, (seed, t)
                t += L
        assert list(s.retained()) == bf.positions()


def test_accumulated_prompt_brute_force(oracle):
    for seed in range(30):
        rng = np.random.default_rng(700 + seed)
        b = int(rng.integers(1, 4))
        cb = int(rng.integers(3, 7))
        c = cb * b
        G, d = int(rng.integers(1, 3)), 3
        T = b * int(rng.integers(1, 14))
        Qw, K, V = _prompt(2000 + seed, T, G, d, b)
        s = oracle.OracleStream(c, G, d, flags=oracle.SCORE_ACCUMULATED)
        r = s.prefill_prompt(Qw, K, V, b)
        bf = BruteTreeKV(c, G, d, accumulated=True)
        gone, sbar, beta = bf.prefill_prompt(Qw.tolist(), K.tolist(), V.tolist(), b)
        assert list(r["evicted_blocks"]) == gone, seed
        np.testing.assert_allclose(r["token_scores"], sbar, rtol=1e-12)
        S_b, C_b = bf.scores()
        _, S, C = s.state()
        np.testing.assert_allclose(S, S_b, rtol=1e-12)
        assert list(C) == C_b
        # the token scores are plain column sums of the window's attention
        assert abs(float(r["token_scores"].sum()) - G * b) < 1e-9


# --------------------------------------------------------------------------- #
# Position re-assignment (Section 4.1, "Position Encoding")
# --------------------------------------------------------------------------- #
def _rotary_attention(q, K, V, q_pos, k_pos, scale, base=10000.0):
    """Textbook rotary attention with complex arithmetic: plane i of a row is the complex number
    x[2i] + 1j*x[2i+1], multiplied by exp(1j * position * base**(-2i/d)); logit = Re <q', conj k'>."""
    d = K.shape[1]
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    kc = (K[:, 0::2] + 1j * K[:, 1::2]) * np.exp(1j * np.outer(k_pos, theta))
    out = []
    for qg in q:
        qc = (qg[0::2] + 1j * qg[1::2]) * np.exp(1j * q_pos * theta)
        logits = np.real(kc.conj() @ qc) * scale
        a = np.exp(logits - logits.max())
        a /= a.sum()
        out.append(a @ V)
    return np.array(out)


def test_rerank_paper_example(oracle):
    """The cache of the paper's example ({0,1,2,3,7,8,9}, then token 10) comes out of 3 sinks + 1 tree slot + 3
    recent tokens with the keep-left policy; the step that decodes token 10 must see positions 0..7."""
    facts = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "position_reassignment_example.txt")):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            facts[key] = [int(x) for x in vals]
    G, d = 2, 8
    q, k, v = _rand_stream(31, 11, G, d)
    s = oracle.OracleStream(7, G, d, n_sink=3, n_recent=3, flags=oracle.KEEP_LEFT | oracle.POSITION_RERANK)
    for t in range(10):
        s.decode_step(q[t], k[t], v[t])
    assert list(s.retained()) == facts["cached_tokens"]
    out = s.decode_step(q[10], k[10], v[10], commit=False)[0]
    toks = facts["cached_tokens"] + facts["new_token"]
    want = _rotary_attention(q[10], k[toks], v[toks], facts["assigned_positions"][-1], facts["assigned_positions"],
                             s.scale)
    np.testing.assert_allclose(out, want, rtol=1e-10, atol=1e-12)
    wrong = _rotary_attention(q[10], k[toks], v[toks], facts["original_positions"][-1], facts["original_positions"],
                              s.scale)
    assert np.abs(out - wrong).max() > 1e-3


@pytest.mark.parametrize("c,n_sink,n_recent,G,d", [(12, 0, 0, 1, 4), (16, 2, 5, 2, 6), (9, 1, 0, 3, 8)])
def test_rerank_equals_rotary_attention_over_cache_ranks(oracle, c, n_sink, n_recent, G, d):
    """At every step: outputs equal rotary attention over the retained tokens at positions 0..n-1 (while the cache
    fills these are the original positions: plain causal rotary attention)."""
    T = 5 * c
    q, k, v = _rand_stream(c * 7 + d, T, G, d)
    s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.POSITION_RERANK, rope_base=50.0)
    kept = []
    S = {}
    for t in range(T):
        toks = kept + [t]
        n = len(toks)
        out, ev, *_ = s.decode_step(q[t], k[t], v[t])
        want = _rotary_attention(q[t], k[toks], v[toks], n - 1, np.arange(n), s.scale, base=50.0)
        np.testing.assert_allclose(out, want, rtol=1e-9, atol=1e-12)
        # relative only: any common shift of the positions gives the same output
        np.testing.assert_allclose(out, _rotary_attention(q[t], k[toks], v[toks], n + 2, np.arange(n) + 3, s.scale, 50.0),
                                   rtol=1e-8, atol=1e-11)
        assert (ev >= 0) == (n > c)
        kept = [x for x in toks if x != ev]
        assert list(s.retained()) == kept


def test_rerank_closed_form_single_plane(oracle):
    """d = 2, every key and query (1, 0): the plane's angle is the position itself (base^0 = 1), so the logit of
    the key at cache index j is cos(n - 1 - j) whatever the base."""
    c = 6
    s = oracle.OracleStream(c, 1, 2, scale=1.0, flags=oracle.POSITION_RERANK | oracle.KEEP_LEFT, rope_base=123.0)
    x = np.array([1.0, 0.0])
    for t in range(15):
        out, ev, *_ = s.decode_step(x[None], x, np.array([float(t), 1.0]), commit=False)
        pos = list(s.retained()) + [t]
        w = np.exp(np.cos(len(pos) - 1 - np.arange(len(pos))))
        w /= w.sum()
        np.testing.assert_allclose(out[0], [float(w @ np.array(pos, dtype=np.float64)), 1.0], rtol=1e-12)
        s.decode_step(x[None], x, np.array([float(t), 1.0]))


def test_rerank_off_is_untouched(oracle):
    q, k, v = _rand_stream(5, 30, 1, 4)
    a = oracle.run_decode_stream(_cfg(8), q, k, v)
    b = oracle.run_decode_stream(dict(_cfg(8), rope_base=3.0), q, k, v)       # base without the flag: no effect
    np.testing.assert_array_equal(a["out"], b["out"])
    r = oracle.run_decode_stream(_cfg(8, flags=oracle.POSITION_RERANK), q, k, v)
    assert np.abs(r["out"] - a["out"]).max() > 1e-3


def test_rerank_brute_force(oracle):
    """Evictions, outputs and scores under position re-assignment against the independent re-simulation (which
    uses the relative form of the rotary encoding)."""
    for seed in range(25):
        rng = np.random.default_rng(900 + seed)
        c = int(rng.integers(3, 9))
        n_sink = int(rng.integers(0, 2))
        n_recent = int(rng.integers(0, 2))
        G, d = int(rng.integers(1, 3)), 2 * int(rng.integers(1, 4))
        base = float(rng.choice([10000.0, 7.0]))
        T = 4 * c
        q, k, v = _rand_stream(3000 + seed, T, G, d)
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.POSITION_RERANK, rope_base=base)
        bf = BruteTreeKV(c, G, d, n_sink=n_sink, n_recent=n_recent, rerank_base=base)
        for t in range(T):
            out, ev, *_ = s.decode_step(q[t], k[t], v[t])
            o_b, ev_b = bf.decode_step(q[t].tolist(), k[t].tolist(), v[t].tolist())
            assert ev == ev_b, (seed, t)
            np.testing.assert_allclose(out, np.array(o_b), rtol=1e-9, atol=1e-12)
        S_b, C_b = bf.scores()
        _, S, C = s.state()
        np.testing.assert_allclose(S, S_b, rtol=1e-10)
        assert list(C) == C_b


# --------------------------------------------------------------------------- #
# Wavelet analysis (Sections 3.2-3.3)
# --------------------------------------------------------------------------- #
def _haar_matrix(t, levels):
    """Orthonormal analysis matrix of the multi-level Haar transform, rows ordered [A_L, D_L, .., D_1], built
    from Kronecker products (textbook construction), independent of the filter-bank code."""
    r = math.sqrt(0.5)
    rows_d = []
    avg = np.eye(t)
    for l in range(1, levels + 1):
        n = avg.shape[0] // 2
        lo = np.kron(np.eye(n), np.array([[r, r]])) @ avg
        hi = np.kron(np.eye(n), np.array([[r, -r]])) @ avg
        rows_d.append(hi)
        avg = lo
    return np.vstack([avg] + rows_d[::-1])


@pytest.mark.parametrize("t,d,levels", [(32, 3, 5), (64, 2, 3), (96, 4, 5), (8, 1, 1)])
def test_wavelet_decomposition_is_the_haar_transform(oracle, t, d, levels):
    rng = np.random.default_rng(t + d)
    a = rng.random(t)
    a /= a.sum()
    V = rng.standard_normal((t, d))
    mag, co, rs = oracle.wavelet_components(a, V, levels, want_coeffs=True)
    sig = a[:, None] * V
    # the coefficient list equals the orthonormal Haar matrix applied to the signal (pair (2n-1, 2n), first minus
    # second in the details), energy is preserved, and the components add up to the signal again
    np.testing.assert_allclose(co.T, _haar_matrix(t, levels) @ sig, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose((co ** 2).sum(), (sig ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(rs.T, sig, rtol=1e-12, atol=1e-15)
    # closed form: Rec(D_l) is constant in magnitude over a block of 2^l positions, 2^-l |first half - second half|
    for l in range(1, levels + 1):
        blk = sig.reshape(t >> l, 1 << l, d)
        diff = np.abs(blk[:, : 1 << (l - 1)].sum(1) - blk[:, 1 << (l - 1):].sum(1)) / (1 << l)
        np.testing.assert_allclose(mag[l - 1], np.repeat(diff.mean(-1), 1 << l), rtol=1e-11, atol=1e-16)


def test_wavelet_special_signals(oracle):
    t, levels = 64, 5
    # a constant signal has no detail at any level
    mag = oracle.wavelet_components(np.full(t, 1.0 / t), np.ones((t, 2)), levels)
    assert np.abs(mag).max() < 1e-17
    # an impulse at (1-based) position 1 shows in every level's first block with magnitude 2^-l
    a = np.zeros(t)
    a[0] = 1.0
    mag = oracle.wavelet_components(a, np.ones((t, 1)), levels)
    for l in range(1, levels + 1):
        np.testing.assert_allclose(mag[l - 1, : 1 << l], 2.0 ** -l, rtol=1e-12)
        assert np.all(mag[l - 1, 1 << l:] == 0.0)
    # an alternating signal lives in level 1 only
    mag = oracle.wavelet_components(np.ones(t), np.tile([[1.0], [-1.0]], (t // 2, 1)), levels)
    np.testing.assert_allclose(mag[0], 1.0, rtol=1e-12)
    assert np.abs(mag[1:]).max() < 1e-15
    with pytest.raises(ValueError):
        oracle.wavelet_components(np.ones(48), np.ones((48, 1)), 5)


def test_rerank_prompt_scores_and_hand_over(oracle):
    """One-shot compression of a prompt whose keys carry no positional encoding: the token scores are the column
    averages of textbook rotary attention at the ORIGINAL positions (nothing has been evicted yet), the cache
    keeps the keys unencoded, and the decode steps that follow see the kept tokens at their ranks."""
    rng = np.random.default_rng(77)
    G, d, b, T, c = 2, 8, 4, 40, 16
    Qw, K, V = rng.standard_normal((b, G, d)), rng.standard_normal((T, d)), rng.standard_normal((T, d))
    s = oracle.OracleStream(c, G, d, n_sink=2, n_recent=5, flags=oracle.POSITION_RERANK, rope_base=100.0)
    r = s.prefill_prompt(Qw, K, V, b)
    theta = 100.0 ** (-2.0 * np.arange(d // 2) / d)
    kc = (K[:, 0::2] + 1j * K[:, 1::2]) * np.exp(1j * np.outer(np.arange(T), theta))
    tot, cnt = np.zeros(T), np.zeros(T)
    for i in range(b):
        p = T - b + i
        for g in range(G):
            qc = (Qw[i, g, 0::2] + 1j * Qw[i, g, 1::2]) * np.exp(1j * p * theta)
            lg = np.real(kc[: p + 1].conj() @ qc) / np.sqrt(d)
            w = np.exp(lg - lg.max())
            tot[: p + 1] += w / w.sum()
        cnt[: p + 1] += 1
    np.testing.assert_allclose(r["token_scores"], tot / cnt, rtol=1e-10)
    kept = s.retained()
    Kc, Vc = s.kv()
    np.testing.assert_array_equal(Kc, K[kept])
    q1, k1, v1 = rng.standard_normal((G, d)), rng.standard_normal(d), rng.standard_normal(d)
    out = s.decode_step(q1, k1, v1, commit=False)[0]
    want = _rotary_attention(q1, np.vstack([K[kept], k1]), np.vstack([V[kept], v1]), len(kept), np.arange(len(kept) + 1),
                             s.scale, base=100.0)
    np.testing.assert_allclose(out, want, rtol=1e-9, atol=1e-12)


def test_rerank_prompt_brute_force(oracle):
    for seed in range(20):
        rng = np.random.default_rng(1700 + seed)
        b = int(rng.integers(1, 4))
        cb = int(rng.integers(3, 7))
        c = cb * b
        G, d = int(rng.integers(1, 3)), 2 * int(rng.integers(1, 4))
        T = b * int(rng.integers(1, 14))
        Qw, K, V = _prompt(4000 + seed, T, G, d, b)
        s = oracle.OracleStream(c, G, d, flags=oracle.POSITION_RERANK, rope_base=30.0)
        r = s.prefill_prompt(Qw, K, V, b)
        bf = BruteTreeKV(c, G, d, rerank_base=30.0)
        gone, sbar, beta = bf.prefill_prompt(Qw.tolist(), K.tolist(), V.tolist(), b)
        assert list(r["evicted_blocks"]) == gone, seed
        np.testing.assert_allclose(r["token_scores"], sbar, rtol=1e-10)
        q, k, v = _rand_stream(5000 + seed, 6, G, d)
        for t in range(6):
            out, ev, *_ = s.decode_step(q[t], k[t], v[t])
            o_b, ev_b = bf.decode_step(q[t].tolist(), k[t].tolist(), v[t].tolist())
            assert ev == ev_b, (seed, t)
            np.testing.assert_allclose(out, np.array(o_b), rtol=1e-9, atol=1e-12)


# --------------------------------------------------------------------------- #
# The decision margin |Sbar_l - Sbar_r| / max(Sbar_l, Sbar_r): it gates the near-tie handling of the parity runs
# --------------------------------------------------------------------------- #
class _UniformAttentionExact:
    """Algorithm 1 under uniform attention (q = 0) in exact rational arithmetic: every step adds G / len to every
    cached token, so S_p = G * (P[t] - P[p-1]) with P the running sum of 1 / len.  step() appends the next token and
    returns None, or the scope (left position, right position, Sbar_l, Sbar_r) as Fractions; evict() removes one."""

    def __init__(self, c, n_sink=0, n_recent=0, G=1):
        from fractions import Fraction

        self.F, self.c, self.n_sink, self.m, self.G = Fraction, c, n_sink, c - n_sink - n_recent, G
        self.P, self.cache, self.idx0, self.t = [Fraction(0)], [], 0, -1

    def step(self):
        self.t += 1
        t = self.t
        self.cache.append(t)
        self.P.append(self.P[-1] + self.F(1, len(self.cache)))
        if len(self.cache) <= self.c:
            return None
        sbar = lambda p: self.G * (self.P[t + 1] - self.P[p]) / (t - p + 1)
        l, r = self.cache[self.n_sink + self.idx0], self.cache[self.n_sink + self.idx0 + 1]
        return l, r, sbar(l), sbar(r)

    def evict(self, pos):
        self.cache.remove(pos)
        self.idx0 = (self.idx0 + 1) % self.m


@pytest.mark.parametrize("c,n_sink,n_recent,G,T", [(4, 0, 0, 1, 40), (12, 2, 3, 2, 90), (64, 4, 28, 1, 400),
                                                   (1023, 0, 0, 1, 1100)])
def test_margin_is_the_relative_score_difference(oracle, c, n_sink, n_recent, G, T):
    """With q = 0 the two scores of every scope are known rationals (tokens of unequal age have seen different cache
    lengths), so the evicted position is known and the reported margin must equal |l - r| / max(l, r) to rounding.
    (Where the rationals tie, the fp64 sums may differ in the last bit unless 1 / (c+1) is a binary fraction: the
    reference then takes the oracle's pick of the two.)"""
    d = 2
    rng = np.random.default_rng(1)
    k, v = rng.standard_normal((T, d)), rng.standard_normal((T, d))
    s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent)
    ref = _UniformAttentionExact(c, n_sink, n_recent, G)
    apart = decided = 0
    for t in range(T):
        _, ev, margin, _, _ = s.decode_step(np.zeros((G, d)), k[t], v[t])
        scope = ref.step()
        if scope is None:
            assert ev == -1 and margin == -1.0
            continue
        l, r, sl, sr = scope
        mg = abs(sl - sr) / max(sl, sr)
        assert abs(margin - float(mg)) <= 1e-12, (t, margin, float(mg))
        if mg == 0:
            assert ev in (l, r)
            if (c + 1) & c == 0:
                assert margin == 0.0 and ev == l         # an exact tie: the strict ">" evicts the left slot
        else:
            assert ev == (r if sl > sr else l), t
            decided += 1
            # what the margin is NOT: the absolute difference, or the difference over the smaller score
            absolute, over_min = float(abs(sl - sr)), float(abs(sl - sr) / min(sl, sr))
            if abs(absolute - float(mg)) > 1e-6 and abs(over_min - float(mg)) > 1e-6:
                apart += 1
        ref.evict(ev)
        assert list(s.retained()) == ref.cache
    assert apart > 0 and decided > 0


def test_margin_relative_and_absolute_differ_by_orders_of_magnitude(oracle):
    """Budget 1023, uniform attention: scores are about 1e-3, so a relative margin of a few per cent is an absolute
    difference of order 1e-5 -- below a 1e-4 threshold taken absolutely, far above it taken relatively."""
    c = 1023
    ref = _UniformAttentionExact(c)
    for _ in range(c):
        assert ref.step() is None
    l, r, sl, sr = ref.step()                   # first eviction: tokens 0 and 1, the older one scores higher
    mg = abs(sl - sr) / max(sl, sr)
    assert (l, r) == (0, 1) and sl > sr
    assert float(mg) > 0.05 and float(abs(sl - sr)) < 1e-3 and float(abs(sl - sr)) * 50 < float(mg)
    d = 2
    s = oracle.OracleStream(c, 1, d)
    rng = np.random.default_rng(2)
    for t in range(c + 1):
        _, ev, margin, _, _ = s.decode_step(np.zeros((1, d)), rng.standard_normal(d), rng.standard_normal(d),
                                            forced_pos=0 if t == c else -1, follow_thresh=1e-4)
    # the other implementation's choice (token 0) is NOT adopted: the margin is far above the threshold
    assert ev == 1 and abs(margin - float(mg)) <= 1e-12
    assert s.retained()[0] == 0


def test_margin_in_prefill_chunk_and_prompt_blocks(oracle):
    """The same definition in the chunk replay (frozen scores) and at block level: recomputed from the scores the
    oracle reports."""
    c, G, d = 8, 1, 4
    q, k, v = _rand_stream(77, 60, G, d)
    s = oracle.OracleStream(c, G, d, n_sink=1, n_recent=2)
    s.prefill_chunk(q[:8], k[:8], v[:8])
    pos0, S0, C0 = s.state()
    t = oracle.OracleStream(c, G, d, n_sink=1, n_recent=2)
    t.prefill_chunk(q[:8], k[:8], v[:8])
    res = s.prefill_chunk(q[8:9], k[8:9], v[8:9])         # one token: scope = logical slots (1, 2) = positions 1, 2
    o, ev, mg, _, _ = t.decode_step(q[8], k[8], v[8], commit=False)
    assert res["margins"][0] == mg and res["evicted"][0] == ev
    # rebuild both scores from the state before the step and this step's attention row
    K = np.stack([k[p] for p in pos0] + [k[8]])
    logit = K @ q[8, 0] / math.sqrt(d)
    a = np.exp(logit - logit.max()); a /= a.sum()
    sb = [(S0[i] + a[i]) / (C0[i] + 1) for i in (1, 2)]
    assert abs(mg - abs(sb[0] - sb[1]) / max(sb)) < 1e-12
    assert ev == (pos0[2] if sb[0] > sb[1] else pos0[1])
    # block level
    T, b = 48, 4
    qw, kp, vp = q[T - b:T], k[:T], v[:T]
    u = oracle.OracleStream(16, G, d, n_sink=0, n_recent=4)
    r = u.prefill_prompt(qw, kp, vp, b)
    beta = r["block_scores"]
    first = int(np.flatnonzero(r["evicted_blocks"] >= 0)[0])     # block capacity 4: first eviction when block 4 arrives
    assert first == 4
    want = abs(beta[0] - beta[1]) / max(beta[0], beta[1])        # tree region = 3 blocks, scope (0, 1)
    assert abs(r["margins"][first] - want) < 1e-12
    assert r["evicted_blocks"][first] == (1 if beta[0] > beta[1] else 0)


# --------------------------------------------------------------------------- #
# Position re-assignment in the prefill chunk: ranks at the moment the chunk is scored
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("c,n_sink,n_recent,G,d", [(12, 0, 0, 1, 4), (16, 2, 5, 2, 6), (10, 1, 3, 3, 8)])
def test_rerank_chunk_equals_rotary_attention_over_ranks(oracle, c, n_sink, n_recent, G, d):
    """Row i of a chunk sees the n0 cached tokens at positions 0..n0-1 and chunk tokens 0..i at n0..n0+i: its output is
    textbook rotary attention (complex arithmetic) over exactly those tokens, its probabilities are what the scores
    grow by, and nothing depends on the tokens' original positions."""
    sched = [5, 9, 1, 2 * c + 3, 4, 1, c]
    T = sum(sched)
    q, k, v = _rand_stream(c * 11 + d, T, G, d)
    s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.POSITION_RERANK, rope_base=40.0)
    t = 0
    for L in sched:
        kept = list(s.retained())
        pos0, S0, C0 = s.state()
        n0 = len(kept)
        res = s.prefill_chunk(q[t:t + L], k[t:t + L], v[t:t + L])
        add = np.zeros(n0 + L)
        for i in range(L):
            toks = kept + list(range(t, t + i + 1))
            want = _rotary_attention(q[t + i], k[toks], v[toks], n0 + i, np.arange(n0 + i + 1), s.scale, base=40.0)
            np.testing.assert_allclose(res["out"][i], want, rtol=1e-9, atol=1e-12)
            # the probabilities behind the scores, from the same textbook formula
            theta = 40.0 ** (-2.0 * np.arange(d // 2) / d)
            kc = (k[toks][:, 0::2] + 1j * k[toks][:, 1::2]) * np.exp(1j * np.outer(np.arange(n0 + i + 1), theta))
            for g in range(G):
                qc = (q[t + i, g, 0::2] + 1j * q[t + i, g, 1::2]) * np.exp(1j * (n0 + i) * theta)
                lg = np.real(kc.conj() @ qc) * s.scale
                a = np.exp(lg - lg.max())
                add[:n0 + i + 1] += a / a.sum()
        pos1, S1, C1 = s.state()
        before = dict(zip(list(pos0) + list(range(t, t + L)), list(S0) + [0.0] * L))
        idx = {p: j for j, p in enumerate(kept + list(range(t, t + L)))}
        for p, sc in zip(pos1, S1):
            assert abs(sc - (before[p] + add[idx[p]])) < 1e-10
        t += L


def test_rerank_chunk_of_one_token_is_the_decode_step(oracle):
    c, G, d, T = 9, 2, 6, 40
    q, k, v = _rand_stream(77, T, G, d)
    a = oracle.OracleStream(c, G, d, n_sink=1, n_recent=2, flags=oracle.POSITION_RERANK)
    b = oracle.OracleStream(c, G, d, n_sink=1, n_recent=2, flags=oracle.POSITION_RERANK)
    for t in range(T):
        o, ev, mg, _, _ = a.decode_step(q[t], k[t], v[t])
        r = b.prefill_chunk(q[t:t + 1], k[t:t + 1], v[t:t + 1])
        assert np.array_equal(o, r["out"][0]) and ev == r["evicted"][0] and mg == r["margins"][0]
    for x, y in zip(a.state(), b.state()):
        assert np.array_equal(x, y)


def test_rerank_chunk_brute_force(oracle):
    """Chunks and decode steps mixed, against the independent re-simulation (relative form of the encoding)."""
    for seed in range(20):
        rng = np.random.default_rng(4100 + seed)
        c = int(rng.integers(3, 9))
        n_sink, n_recent = int(rng.integers(0, 2)), int(rng.integers(0, 3))
        if c - n_sink - n_recent < 1:
            n_recent = 0
        G, d = int(rng.integers(1, 3)), 2 * int(rng.integers(1, 4))
        base = float(rng.choice([10000.0, 5.0]))
        sched = [int(x) for x in rng.integers(0, 2 * c, size=6)]
        T = sum(max(L, 1) for L in sched)
        q, k, v = _rand_stream(5200 + seed, T, G, d)
        s = oracle.OracleStream(c, G, d, n_sink=n_sink, n_recent=n_recent, flags=oracle.POSITION_RERANK, rope_base=base)
        bf = BruteTreeKV(c, G, d, n_sink=n_sink, n_recent=n_recent, rerank_base=base)
        t = 0
        for L in sched:
            if L == 0:
                out, ev, *_ = s.decode_step(q[t], k[t], v[t])
                o_b, ev_b = bf.decode_step(q[t].tolist(), k[t].tolist(), v[t].tolist())
                outs, evs, outs_b, evs_b = out[None], [ev], [o_b], [ev_b]
                t += 1
            else:
                r = s.prefill_chunk(q[t:t + L], k[t:t + L], v[t:t + L])
                outs_b, evs_b = bf.prefill_chunk(q[t:t + L].tolist(), k[t:t + L].tolist(), v[t:t + L].tolist())
                outs, evs = r["out"], list(r["evicted"])
                t += L
            assert list(evs) == list(evs_b), (seed, t)
            np.testing.assert_allclose(outs, np.array(outs_b), rtol=1e-9, atol=1e-12)
        S_b, C_b = bf.scores()
        _, S, C = s.state()
        np.testing.assert_allclose(S, S_b, rtol=1e-10)
        assert list(C) == C_b
