"""Drives the HIP path through the C ABI and the CPU oracle on the same inputs, and compares.

Retained-index sets must match bit for bit.  The two sides accumulate scores in different
precision (fp32 on the GPU, fp64 in the oracle), so a comparison whose relative margin is
below FOLLOW_THRESH can legitimately fall either way: there the oracle adopts the GPU's
choice, the event is counted, and everything after it is still compared exactly.  A
disagreement at a larger margin is a failure.
"""
from __future__ import annotations

import os

import numpy as np

FOLLOW_THRESH = 1e-4          # relative score margin below which a decision is "flagged"
TOL = {"bf16": 2e-3, "f32": 1e-5}


def to_device(x: np.ndarray, dtype: str):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x))
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda()


def gpu_decode_run(kv, Qd, Kd, Vd, sample_steps=()):
    """Run T decode steps.  Qd [T,B,H,d], Kd/Vd [T,B,Hkv,d] device tensors in storage dtype.

    Returns dict(out [T,B,H,d] f32 cpu, evicted [T,B,Hkv] cpu, n_retained [T,B,Hkv] cpu,
    retained {step: [B,Hkv,c] cpu}).
    """
    import torch

    T = Qd.shape[0]
    c = kv.cfg
    out = torch.empty(T, c.batch, c.q_heads, c.head_dim, dtype=torch.float32, device=kv.device)
    ev = torch.empty(T, c.batch, c.kv_heads, dtype=torch.int32, device=kv.device)
    nret = torch.empty(T, c.batch, c.kv_heads, dtype=torch.int32, device=kv.device)
    sample_steps = sorted(set(int(s) for s in sample_steps))
    ret_s = torch.empty(max(len(sample_steps), 1), c.batch, c.kv_heads, c.budget, dtype=torch.int32, device=kv.device)
    scratch = torch.empty(c.batch, c.kv_heads, c.budget, dtype=torch.int32, device=kv.device)
    where = {s: i for i, s in enumerate(sample_steps)}
    for t in range(T):
        r = ret_s[where[t]] if t in where else scratch
        kv.decode_step(Qd[t], Kd[t], Vd[t], out[t], r, nret[t], ev[t])
    torch.cuda.synchronize()
    return dict(out=out.cpu().numpy(), evicted=ev.cpu().numpy(), n_retained=nret.cpu().numpy(),
                retained={s: ret_s[i].cpu().numpy() for s, i in where.items()})


def oracle_cfg(kv, **over):
    c = kv.cfg
    d = dict(budget=c.budget, G=c.q_heads // c.kv_heads, d=c.head_dim, n_sink=c.n_sink, n_recent=c.n_recent,
             scale=float(c.softmax_scale), flags=int(c.flags), rope_base=float(c.rope_base))
    d.update(over)
    return d


def retained_from_evictions(evicted: np.ndarray, upto: int) -> np.ndarray:
    """Ascending positions alive after step `upto` given the per-step evicted positions."""
    alive = np.ones(upto + 1, bool)
    ev = evicted[: upto + 1]
    alive[ev[ev >= 0]] = False
    return np.flatnonzero(alive)


def compare_decode(oracle, kv, Q, K, V, gpu, units=None, dtype="bf16", every_step_retained=False, workers=None):
    """Q [T,B,H,d], K/V [T,B,Hkv,d] float arrays holding the values the GPU consumed.

    Runs the oracle (follow mode) on the chosen units and checks outputs, evictions, retained
    sets.  Returns dict(flagged, max_err, decisions).
    """
    c = kv.cfg
    G = c.q_heads // c.kv_heads
    T = Q.shape[0]
    if units is None:
        units = [(b, h) for b in range(c.batch) for h in range(c.kv_heads)]
    cfg = oracle_cfg(kv)
    tol = TOL[dtype]

    def job(u):
        b, h = u
        return oracle.run_decode_stream(cfg, Q[:, b, h * G:(h + 1) * G, :], K[:, b, h, :], V[:, b, h, :],
                                        forced=gpu["evicted"][:, b, h], follow_thresh=FOLLOW_THRESH)

    results = oracle.run_many(job, units, workers=workers or min(len(units), os.cpu_count() or 1, 16))
    flagged = 0
    decisions = 0
    max_err = 0.0
    for (b, h), res in zip(units, results):
        assert res["disagreed"] == 0, f"unit {(b, h)}: {res['disagreed']} eviction decisions differ outside the near-tie margin"
        np.testing.assert_array_equal(res["evicted"], gpu["evicted"][:, b, h], err_msg=f"evicted positions, unit {(b, h)}")
        flagged += res["adopted"]
        decisions += int(np.count_nonzero(res["evicted"] >= 0))
        err = np.abs(res["out"] - gpu["out"][:, b, h * G:(h + 1) * G, :]).max()
        max_err = max(max_err, float(err))
        assert err <= tol, f"unit {(b, h)}: attention output differs by {err} > {tol}"
        want_n = np.minimum(np.arange(1, T + 1), c.budget)
        np.testing.assert_array_equal(gpu["n_retained"][:, b, h], want_n)
        steps = gpu["retained"].keys()
        for s in steps:
            want = retained_from_evictions(res["evicted"], s)
            got = gpu["retained"][s][b, h]
            assert np.array_equal(got[: len(want)], want), f"retained set, unit {(b, h)}, step {s}"
            assert np.all(got[len(want):] == -1)
        # the oracle's own final state agrees with the reconstruction
        assert np.array_equal(res["stream"].retained(), retained_from_evictions(res["evicted"], T - 1))
    return dict(flagged=flagged, max_err=max_err, decisions=decisions, results=dict(zip(units, results)))


def compare_scores(kv, results, dtype="bf16"):
    """Averaged scores Sbar = S / C of the retained tokens, GPU vs oracle, at the current step."""
    import torch

    S = kv.scores()
    torch.cuda.synchronize()
    S = S.cpu().numpy()
    tol = TOL[dtype]
    worst = 0.0
    for (b, h), res in results.items():
        pos, So, Co = res["stream"].state()
        n = len(pos)
        sbar_o = So / Co
        sbar_g = S[b, h, :n].astype(np.float64) / Co
        worst = max(worst, float(np.abs(sbar_o - sbar_g).max()))
        assert np.all(S[b, h, n:] == 0)
    assert worst <= tol, f"averaged scores differ by {worst} > {tol}"
    return worst


# --------------------------------------------------------------------------- #
# mixed prefill / decode schedules
# --------------------------------------------------------------------------- #
def run_schedule(oracle, kv, Q, K, V, schedule, dtype="bf16", units=None, check_every_call=True, streams=None,
                 t_start=0):
    """Drive GPU and oracle through `schedule`, a list of chunk lengths (0 = one decode step).

    Q [T,B,H,d], K/V [T,B,Hkv,d]: float arrays of the values the GPU consumes, T = total tokens.
    After every call compares outputs, evicted positions (follow mode) and the retained list.
    `streams` / `t_start`: continue from oracle streams (and a token offset) an earlier call left.
    """
    import torch

    c = kv.cfg
    G = c.q_heads // c.kv_heads
    if units is None:
        units = [(b, h) for b in range(c.batch) for h in range(c.kv_heads)]
    ocfg = oracle_cfg(kv)
    if streams is None:
        streams = {u: oracle.OracleStream(ocfg["budget"], G, c.head_dim, n_sink=ocfg["n_sink"],
                                          n_recent=ocfg["n_recent"], scale=ocfg["scale"], flags=ocfg["flags"],
                                          rope_base=ocfg["rope_base"])
                   for u in units}
    tol = TOL[dtype]
    Qd, Kd, Vd = to_device(Q, dtype), to_device(K, dtype), to_device(V, dtype)
    t = t_start
    stats = dict(flagged=0, decisions=0, max_err=0.0, calls=0)
    for L in schedule:
        if L == 0:
            out, ret, nret, ev = kv.new_outputs()
            kv.decode_step(Qd[t], Kd[t], Vd[t], out, ret, nret, ev)
            torch.cuda.synchronize()
            o_g = out.cpu().numpy()[:, None]                      # [B,1,H,d]
            ev_g = ev.cpu().numpy()[:, :, None]                   # [B,Hkv,1]
            n_tok = 1
        else:
            qc = Qd[t:t + L].permute(1, 0, 2, 3).contiguous()     # [B,L,H,d]
            kc = Kd[t:t + L].permute(1, 0, 2, 3).contiguous()
            vc = Vd[t:t + L].permute(1, 0, 2, 3).contiguous()
            out, ret, nret, ev = kv.new_outputs(L)
            kv.prefill_chunk(qc, kc, vc, L, out, ret, nret, ev)
            torch.cuda.synchronize()
            o_g, ev_g = out.cpu().numpy(), ev.cpu().numpy()
            n_tok = L
        ret_g, nret_g = ret.cpu().numpy(), nret.cpu().numpy()

        def job(u):
            b, h = u
            s = streams[u]
            qs, ks, vs = Q[t:t + n_tok, b, h * G:(h + 1) * G, :], K[t:t + n_tok, b, h, :], V[t:t + n_tok, b, h, :]
            if L == 0:
                o, e, mg, ad, dis = s.decode_step(qs[0], ks[0], vs[0], forced_pos=int(ev_g[b, h, 0]),
                                                  follow_thresh=FOLLOW_THRESH)
                return dict(out=o[None], evicted=np.array([e]), adopted=np.array([ad]), disagreed=np.array([dis]))
            return s.prefill_chunk(qs, ks, vs, forced_pos=ev_g[b, h], follow_thresh=FOLLOW_THRESH)

        results = oracle.run_many(job, units, workers=min(len(units), os.cpu_count() or 1, 16))
        for (b, h), res in zip(units, results):
            where = f"call {stats['calls']} (len {L}, t={t}), unit {(b, h)}"
            assert int(np.sum(res["disagreed"])) == 0, f"{where}: eviction decisions differ outside the near-tie margin"
            np.testing.assert_array_equal(res["evicted"], ev_g[b, h], err_msg=where)
            err = float(np.abs(res["out"] - o_g[b, :, h * G:(h + 1) * G, :]).max())
            assert err <= tol, f"{where}: attention output differs by {err} > {tol}"
            stats["max_err"] = max(stats["max_err"], err)
            stats["flagged"] += int(np.sum(res["adopted"]))
            stats["decisions"] += int(np.count_nonzero(res["evicted"] >= 0))
            want = streams[(b, h)].retained()
            assert nret_g[b, h] == len(want), where
            assert np.array_equal(ret_g[b, h, :len(want)], want), f"{where}: retained set"
            assert np.all(ret_g[b, h, len(want):] == -1)
        t += n_tok
        stats["calls"] += 1
    stats["results"] = {u: dict(stream=streams[u]) for u in units}
    return stats


# --------------------------------------------------------------------------- #
# one-shot prompt compression, then decoding
# --------------------------------------------------------------------------- #
def run_prompt(oracle, kv, Q, K, V, T, block, decode_steps, units=None, dtype="bf16"):
    """Compress the first T tokens in one shot on both sides, compare, then decode `decode_steps` more tokens.

    Q [T + decode_steps, B, H, d], K/V [.., B, Hkv, d]: float arrays of the values the GPU consumes.
    Compared: the block evicted at every step (follow mode), every token's score, the retained list, the
    averaged scores and the cache rows of the retained tokens, then every decode step as in run_schedule.
    """
    import torch

    c = kv.cfg
    G = c.q_heads // c.kv_heads
    if units is None:
        units = [(b, h) for b in range(c.batch) for h in range(c.kv_heads)]
    ocfg = oracle_cfg(kv)
    streams = {u: oracle.OracleStream(ocfg["budget"], G, c.head_dim, n_sink=ocfg["n_sink"], n_recent=ocfg["n_recent"],
                                      scale=ocfg["scale"], flags=ocfg["flags"], rope_base=ocfg["rope_base"])
               for u in units}
    N = T // block
    Qd, Kd, Vd = to_device(Q[:T], dtype), to_device(K[:T], dtype), to_device(V[:T], dtype)
    qw = Qd[T - block:T].permute(1, 0, 2, 3).contiguous()          # [B, block, H, d]
    kp = Kd.permute(1, 0, 2, 3).contiguous()                       # [B, T, Hkv, d]
    vp = Vd.permute(1, 0, 2, 3).contiguous()
    _, ret, nret, _ = kv.new_outputs()
    evb = torch.empty(c.batch, c.kv_heads, N, dtype=torch.int32, device=kv.device)
    tok = torch.empty(c.batch, c.kv_heads, T, dtype=torch.float32, device=kv.device)
    kv.prefill_prompt(qw, kp, vp, T, block, ret, nret, evb, tok)
    torch.cuda.synchronize()
    ret_g, nret_g, evb_g, tok_g = ret.cpu().numpy(), nret.cpu().numpy(), evb.cpu().numpy(), tok.cpu().numpy()

    def job(u):
        b, h = u
        return streams[u].prefill_prompt(Q[T - block:T, b, h * G:(h + 1) * G, :], K[:T, b, h, :], V[:T, b, h, :], block,
                                         forced_blocks=evb_g[b, h], follow_thresh=FOLLOW_THRESH)

    results = oracle.run_many(job, units, workers=min(len(units), os.cpu_count() or 1, 16))
    stats = dict(flagged=0, decisions=0, tok_err=0.0)
    for (b, h), res in zip(units, results):
        where = f"prompt of {T} in blocks of {block}, unit {(b, h)}"
        assert res["disagreed"] == 0, f"{where}: block evictions differ outside the near-tie margin"
        np.testing.assert_array_equal(res["evicted_blocks"], evb_g[b, h], err_msg=where)
        # both sides consume the same bf16 values; the scores differ by fp32 accumulation only
        np.testing.assert_allclose(tok_g[b, h], res["token_scores"], rtol=2e-4, atol=1e-9, err_msg=where)
        stats["tok_err"] = max(stats["tok_err"], float(np.abs(tok_g[b, h] / res["token_scores"] - 1).max()))
        stats["flagged"] += res["adopted"]
        stats["decisions"] += int(np.count_nonzero(res["evicted_blocks"] >= 0))
        want = streams[(b, h)].retained()
        assert nret_g[b, h] == len(want), where
        assert np.array_equal(ret_g[b, h, :len(want)], want), f"{where}: retained set"
        assert np.all(ret_g[b, h, len(want):] == -1)
    res_map = {u: dict(stream=streams[u]) for u in units}
    stats["score_err"] = compare_scores(kv, res_map, dtype)
    Kc, Vc = kv.gather_kv()
    torch.cuda.synchronize()
    for (b, h) in units:
        pos = streams[(b, h)].retained()
        np.testing.assert_array_equal(Kc[b, h, :len(pos)].float().cpu().numpy(), K[pos, b, h])
        np.testing.assert_array_equal(Vc[b, h, :len(pos)].float().cpu().numpy(), V[pos, b, h])
    stats["streams"] = streams
    if decode_steps:
        st = run_schedule(oracle, kv, Q, K, V, [0] * decode_steps, dtype=dtype, units=units, streams=streams, t_start=T)
        stats["decode"] = st
        stats["score_err_after"] = compare_scores(kv, st["results"], dtype)
    return stats


def smoke_prefill(oracle, binding):
    """Two prefill chunks and two decode steps on a small GQA configuration, checked against the oracle."""
    from paper_2501_04987_amd import inputs

    T, B, H, Hkv, d, budget = 150, 1, 4, 2, 128, 40
    Q, K, V = inputs.batch_streams("lowrank", 1, T, B, Hkv, H // Hkv, d, dtype="bf16")
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype="bf16", n_sink=2, n_recent=10, max_chunk=128)
    st = run_schedule(oracle, kv, Q, K, V, [30, 100, 0, 18, 0], dtype="bf16")
    err = compare_scores(kv, st["results"], "bf16")
    print(f"smoke: prefill ok, {st['decisions']} evictions, {st['flagged']} near-ties, "
          f"max |out err| {st['max_err']:.2e}, max |score err| {err:.2e}")


def smoke_prompt(oracle, binding):
    """A one-shot prompt compression followed by decode steps, on a small configuration, against the oracle."""
    from paper_2501_04987_amd import inputs

    T, block, steps, B, H, Hkv, d, budget = 16 * 23, 16, 6, 1, 4, 2, 128, 96
    Q, K, V = inputs.batch_streams("lowrank", 2, T + steps, B, Hkv, H // Hkv, d, dtype="bf16")
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype="bf16", n_sink=2, n_recent=20, max_prompt=T)
    st = run_prompt(oracle, kv, Q, K, V, T, block, steps)
    print(f"smoke: prompt ok, {st['decisions']} block evictions, {st['flagged']} near-ties, "
          f"max token score rel err {st['tok_err']:.2e}, then {st['decode']['decisions']} decode evictions")


def smoke_rerank(oracle, binding):
    """A prefill chunk and decode steps with positions re-assigned to cache ranks, against the oracle."""
    from paper_2501_04987_amd import inputs

    T, B, H, Hkv, d, budget = 120, 1, 4, 2, 128, 40
    Q, K, V = inputs.batch_streams("lowrank", 3, T, B, Hkv, H // Hkv, d, dtype="bf16")
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype="bf16", n_sink=2, n_recent=10, max_chunk=64,
                        flags=binding.TREEKV_POSITION_RERANK)
    st = run_schedule(oracle, kv, Q, K, V, [50] + [0] * 30 + [40], dtype="bf16")
    print(f"smoke: re-assigned positions ok, {st['decisions']} evictions, {st['flagged']} near-ties, "
          f"max |out err| {st['max_err']:.2e}")


def smoke_wavelet(oracle, binding):
    """The Haar analysis of a small random signal, against the oracle."""
    import torch

    rng = np.random.default_rng(4)
    heads, t, d, levels = 3, 96, 128, 5
    a = rng.random((heads, t)).astype(np.float32)
    a /= a.sum(-1, keepdims=True)
    V = torch.from_numpy(rng.standard_normal((heads, t, d)).astype(np.float32)).to(torch.bfloat16)
    per_head, mean = binding.wavelet_components(torch.from_numpy(a).cuda(), V.cuda(), levels)
    torch.cuda.synchronize()
    Vf = V.float().numpy().astype(np.float64)
    want = np.stack([oracle.wavelet_components(a[h].astype(np.float64), Vf[h], levels) for h in range(heads)])
    bound = 2e-6 * float(np.abs(a[:, :, None] * Vf).max())
    np.testing.assert_allclose(per_head.cpu().numpy(), want, rtol=1e-5, atol=bound)
    np.testing.assert_allclose(mean.cpu().numpy(), want.mean(0), rtol=1e-5, atol=bound)
    print(f"smoke: wavelet analysis ok, max magnitude {want.max():.3e}")


# --------------------------------------------------------------------------- #
# inputs without near-ties: the oracle runs first and queries behind a near-tie are drawn again
# --------------------------------------------------------------------------- #
def near_ties(margins, thresh=FOLLOW_THRESH) -> int:
    """Decisions whose relative margin is below `thresh` (-1 marks a call without an eviction)."""
    m = np.asarray(margins)
    return int(np.count_nonzero((m >= 0) & (m < thresh)))


def settle_schedule(oracle, ocfg, q, k, v, schedule, redraw, t_start=0, stream=None, progress=None,
                    thresh=FOLLOW_THRESH):
    """Run the oracle alone through `schedule` (chunk lengths, 0 = one decode step) on one stream and make every
    decision's margin at least `thresh`: when a call meets a smaller one, the call is taken back, the queries of
    its tokens are drawn again (`redraw(t, n, attempt) -> [n, G, d]`; written into `q` in place) and the call repeated.
    Runs of decode steps go through the oracle's stream call, 512 steps at a time.

    q [T, G, d], k/v [T, d] float arrays.  Returns dict(out [tokens, G, d], evicted [tokens], margins [tokens],
    redraws, stream).
    """
    s = stream or oracle.OracleStream(ocfg["budget"], ocfg["G"], ocfg["d"], n_sink=ocfg["n_sink"], n_recent=ocfg["n_recent"],
                                      scale=ocfg["scale"], flags=ocfg["flags"], rope_base=ocfg.get("rope_base", 10000.0))
    n_tok = sum(max(L, 1) for L in schedule)
    out = np.empty((n_tok, s.G, s.d), np.float64)
    ev = np.empty(n_tok, np.int64)
    mg = np.empty(n_tok, np.float64)
    redraws = 0
    t, i = t_start, 0
    calls = list(schedule)
    c = 0
    while c < len(calls):
        if calls[c] == 0:                                   # a run of decode steps
            run = 1
            while c + run < len(calls) and calls[c + run] == 0 and run < 512:
                run += 1
            keep = s.clone()
            res = s.decode_stream(q[t:t + run], k[t:t + run], v[t:t + run])
            low = np.flatnonzero((res["margins"] >= 0) & (res["margins"] < thresh))
            if len(low):                                    # take the run back, redo it up to the near-tie, settle that step
                s = keep
                ok = int(low[0])
                if ok:
                    res = s.decode_stream(q[t:t + ok], k[t:t + ok], v[t:t + ok])
                    out[i:i + ok], ev[i:i + ok], mg[i:i + ok] = res["out"], res["evicted"], res["margins"]
                    t, i = t + ok, i + ok
                attempt = 0
                while True:
                    o1, e1, m1, _, _ = s.decode_step(q[t], k[t], v[t], commit=False)
                    if e1 < 0 or m1 >= thresh:
                        break
                    attempt += 1
                    redraws += 1
                    q[t] = redraw(t, 1, attempt)[0]
                o1, e1, m1, _, _ = s.decode_step(q[t], k[t], v[t])
                out[i], ev[i], mg[i] = o1, e1, m1
                t, i, c = t + 1, i + 1, c + ok + 1
            else:
                out[i:i + run], ev[i:i + run], mg[i:i + run] = res["out"], res["evicted"], res["margins"]
                t, i, c = t + run, i + run, c + run
        else:
            L = calls[c]
            attempt = 0
            while True:
                keep = s.clone()
                res = s.prefill_chunk(q[t:t + L], k[t:t + L], v[t:t + L])
                if near_ties(res["margins"], thresh) == 0:
                    break
                s = keep
                attempt += 1
                redraws += 1
                q[t:t + L] = redraw(t, L, attempt)
            out[i:i + L], ev[i:i + L], mg[i:i + L] = res["out"], res["evicted"], res["margins"]
            t, i, c = t + L, i + L, c + 1
        if progress:
            progress(t)
    return dict(out=out, evicted=ev, margins=mg, redraws=redraws, stream=s)


def check_against(ref, out_g, ev_g, tol, where):
    """One stream's GPU outputs [tokens, G, d] and evicted positions [tokens] against an oracle run that met no
    near-tie: the positions must be identical, the outputs within `tol`.  Returns the largest output error."""
    assert near_ties(ref["margins"]) == 0
    np.testing.assert_array_equal(ev_g, ref["evicted"], err_msg=f"{where}: evicted positions")
    err = float(np.abs(ref["out"] - out_g).max())
    assert err <= tol, f"{where}: attention output differs by {err} > {tol}"
    return err
