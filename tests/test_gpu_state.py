"""GPU: snapshots of a context (treekv_export_state / treekv_import_state), through the C ABI.

A snapshot is Algorithm 1's state (S, C, K, V, idx) in position order.  Restoring one must make the calls
that follow repeat bit for bit what followed the export; a snapshot built from the oracle's state must let the GPU
continue in parity with the oracle; a snapshot that describes no reachable state must be refused unit by unit.
"""
import numpy as np
import pytest

from paper_2501_04987_amd import inputs
from tests import parity_harness as ph

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2501_04987_amd import binding as b

    b.load()
    return b


def _steps(kv, Qd, Kd, Vd, t0, t1):
    """Decode steps t0 .. t1-1; returns (out, evicted, retained) stacked over the steps, on the host."""
    import torch

    outs, evs, rets = [], [], []
    for t in range(t0, t1):
        out, ret, nret, ev = kv.new_outputs()
        kv.decode_step(Qd[t], Kd[t], Vd[t], out, ret, nret, ev)
        outs.append(out); evs.append(ev); rets.append(ret)
    torch.cuda.synchronize()
    return tuple(torch.stack(x).cpu().numpy() for x in (outs, evs, rets))


@pytest.mark.parametrize("dtype,splits,G,layout", [("bf16", 1, 1, (3, 20)), ("bf16", 3, 4, (2, 11)), ("f32", 2, 1, (0, 0)),
                                                   ("bf16", 1, 2, (0, 9))])
def test_restore_repeats_bit_for_bit(binding, dtype, splits, G, layout):
    """Snapshot mid-stream (in the middle of a sweep of idx), keep decoding, restore into the same context and into
    a second one, decode the same tokens again: outputs, evicted positions and retained lists repeat bit for bit."""
    import torch

    budget, B, Hkv, d, T0, N = 57, 2, 2, 128, 150, 70
    T = T0 + N
    kind = "lowrank" if dtype == "bf16" else "iid"
    Q, K, V = inputs.batch_streams(kind, 40, T, B, Hkv, G, d, dtype=dtype)
    Qd, Kd, Vd = (ph.to_device(x, dtype) for x in (Q, K, V))
    mk = lambda: binding.TreeKV(budget, Hkv * G, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=layout[0],
                                n_recent=layout[1], kv_splits=splits)
    a, b = mk(), mk()
    _steps(a, Qd, Kd, Vd, 0, T0)
    snap = a.export_state()
    want = _steps(a, Qd, Kd, Vd, T0, T)
    assert (want[1] >= 0).all()                       # every one of these steps evicted
    status = torch.full((B, Hkv), 7, dtype=torch.int32, device="cuda")
    for kv in (a, b):
        kv.import_state(snap, status)
        got = _steps(kv, Qd, Kd, Vd, T0, T)
        assert (status.cpu().numpy() == 0).all()
        for w, g, name in zip(want, got, ("out", "evicted", "retained")):
            assert np.array_equal(w, g), name
    # the snapshot of the restored context is the snapshot it was restored from
    b.import_state(snap)
    assert torch.equal(b.export_state(), snap)


@pytest.mark.parametrize("splits,G", [(1, 1), (3, 2)])
def test_restore_with_reassigned_positions(binding, splits, G):
    """With positions re-assigned to cache ranks the steps after a restore depend on the order arrays the import
    rebuilds (a slot's rank is read off them): they must repeat bit for bit too, in the context the snapshot came
    from and in a fresh one."""
    import torch

    budget, B, Hkv, d, T0, N = 45, 2, 2, 128, 130, 60
    T = T0 + N
    Q, K, V = inputs.batch_streams("lowrank", 41, T, B, Hkv, G, d, dtype="bf16")
    Qd, Kd, Vd = (ph.to_device(x, "bf16") for x in (Q, K, V))
    mk = lambda: binding.TreeKV(budget, Hkv * G, d, kv_heads=Hkv, batch=B, dtype="bf16", n_sink=2, n_recent=13,
                                kv_splits=splits, flags=binding.TREEKV_POSITION_RERANK, rope_base=200.0)
    a, b = mk(), mk()
    _steps(a, Qd, Kd, Vd, 0, T0)
    snap = a.export_state()
    want = _steps(a, Qd, Kd, Vd, T0, T)
    assert (want[1] >= 0).all()
    for kv in (a, b):
        kv.import_state(snap)
        got = _steps(kv, Qd, Kd, Vd, T0, T)
        for w, g, name in zip(want, got, ("out", "evicted", "retained")):
            assert np.array_equal(w, g), name


def test_snapshot_while_filling_and_after_chunks(binding):
    """A snapshot taken before the cache is full, and one taken after prefill chunks, restore exactly."""
    import torch

    budget, B, H, d = 64, 1, 2, 128
    sched_T = 40 + 100 + 30
    Q, K, V = inputs.batch_streams("lowrank", 41, sched_T + 20, B, H, 1, d, dtype="bf16")
    Qd, Kd, Vd = (ph.to_device(x, "bf16") for x in (Q, K, V))
    a = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, n_sink=2, n_recent=10, max_chunk=128)
    b = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, n_sink=2, n_recent=10, max_chunk=128)

    def chunk(kv, t0, L):
        out, ret, nret, ev = kv.new_outputs(L)
        cut = lambda X: X[t0:t0 + L].permute(1, 0, 2, 3).contiguous()
        kv.prefill_chunk(cut(Qd), cut(Kd), cut(Vd), L, out, ret, nret, ev)
        torch.cuda.synchronize()
        return out.cpu().numpy(), ev.cpu().numpy(), ret.cpu().numpy()

    chunk(a, 0, 40)
    snap_fill = a.export_state()
    lay = a.state_layout()
    hdr = snap_fill[lay.header:lay.header + 16 * H].view(torch.int32).cpu().numpy().reshape(H, 4)
    assert (hdr[:, 0] == 40).all() and (hdr[:, 1] == 40).all() and (hdr[:, 2] == 1).all()
    want1 = chunk(a, 40, 100)
    snap_full = a.export_state()
    want2 = chunk(a, 140, 30)
    want3 = _steps(a, Qd, Kd, Vd, 170, 190)
    b.import_state(snap_fill)
    got1 = chunk(b, 40, 100)
    for w, g in zip(want1, got1):
        assert np.array_equal(w, g)
    b.reset()
    b.import_state(snap_full)
    got2 = chunk(b, 140, 30)
    got3 = _steps(b, Qd, Kd, Vd, 170, 190)
    for w, g in zip(want2 + want3, got2 + got3):
        assert np.array_equal(w, g)


def _snapshot_from_oracle(kv, streams, dtype):
    """A snapshot assembled on the host from the oracle's state (positions, S, idx, t and the cached rows)."""
    import torch

    c = kv.cfg
    lay = kv.state_layout()
    buf = np.zeros(lay.bytes, np.uint8)
    U, bud, d = c.batch * c.kv_heads, c.budget, c.head_dim
    hdr = buf[lay.header:lay.header + U * 16].view(np.int32).reshape(U, 4)
    pos = buf[lay.positions:lay.positions + U * bud * 4].view(np.int32).reshape(U, bud)
    slots = buf[lay.slots:lay.slots + U * bud * 4].view(np.int32).reshape(U, bud)
    S = buf[lay.S:lay.S + U * bud * 4].view(np.float32).reshape(U, bud)
    esz = 2 if dtype == "bf16" else 4
    Kb = buf[lay.K:lay.K + U * bud * d * esz]
    Vb = buf[lay.V:lay.V + U * bud * d * esz]
    pos[:] = -1
    slots[:] = -1                                   # unset: token i takes row i
    Kf = np.zeros((U, bud, d), np.float32)
    Vf = np.zeros((U, bud, d), np.float32)
    for (b, h), s in streams.items():
        u = b * c.kv_heads + h
        p, So, _ = s.state()
        n = len(p)
        hdr[u] = (n, s.t, s.idx, 0)
        pos[u, :n] = p
        S[u, :n] = So.astype(np.float32)
        Ko, Vo = s.kv()
        Kf[u, :n], Vf[u, :n] = Ko, Vo
    if dtype == "bf16":
        Kb.view(np.uint16)[:] = inputs.bf16_bits(Kf).reshape(-1)
        Vb.view(np.uint16)[:] = inputs.bf16_bits(Vf).reshape(-1)
    else:
        Kb.view(np.float32)[:] = Kf.reshape(-1)
        Vb.view(np.float32)[:] = Vf.reshape(-1)
    return torch.from_numpy(buf).cuda()


@pytest.mark.parametrize("T0", [30, 64, 64 + 17, 64 + 3 * 41 + 5])
def test_import_a_state_built_from_the_oracle(binding, oracle, T0):
    """The oracle runs T0 tokens alone; its state (while filling, just full, mid-sweep, several sweeps in) is written
    into a snapshot by hand; the GPU imports it and both continue, call by call, in parity."""
    import torch

    budget, B, Hkv, G, d, n_sink, n_recent = 64, 2, 2, 2, 128, 3, 20       # tree region: 41 slots
    sched = [0] * 30 + [50, 0, 0, 64, 0]
    T = T0 + sum(max(L, 1) for L in sched)
    Q, K, V = inputs.batch_streams("lowrank", 42, T, B, Hkv, G, d, dtype="bf16")
    kv = binding.TreeKV(budget, Hkv * G, d, kv_heads=Hkv, batch=B, n_sink=n_sink, n_recent=n_recent, max_chunk=64)
    cfg = ph.oracle_cfg(kv)
    streams = {}
    for b in range(B):
        for h in range(Hkv):
            res = oracle.run_decode_stream(cfg, Q[:T0, b, h * G:(h + 1) * G], K[:T0, b, h], V[:T0, b, h], keep_outputs=False)
            streams[(b, h)] = res["stream"]
    snap = _snapshot_from_oracle(kv, streams, "bf16")
    status = torch.full((B, Hkv), 7, dtype=torch.int32, device="cuda")
    kv.import_state(snap, status)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == 0).all()
    err0 = ph.compare_scores(kv, {u: dict(stream=s) for u, s in streams.items()}, "bf16")
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="bf16", streams=streams, t_start=T0)
    err = ph.compare_scores(kv, st["results"], "bf16")
    print(f"  T0={T0}: flagged={st['flagged']}/{st['decisions']} max_err={st['max_err']:.2e} score_err={err0:.1e}/{err:.1e}")
    assert st["flagged"] <= 2


def test_unreachable_snapshots_are_refused_per_unit(binding):
    """Each planted defect makes exactly its own unit fail the device-side check; that unit is left empty, the
    others are restored."""
    import torch

    budget, B, H, d, T0 = 24, 1, 8, 64, 60
    Q, K, V = inputs.batch_streams("iid", 43, T0 + 5, B, H, 1, d, dtype="f32")
    Qd, Kd, Vd = (ph.to_device(x, "f32") for x in (Q, K, V))
    a = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="f32", n_sink=2, n_recent=6)
    _steps(a, Qd, Kd, Vd, 0, T0)
    snap = a.export_state()
    lay = a.state_layout()
    bad = snap.clone()
    hdr = bad[lay.header:lay.header + H * 16].view(torch.int32).view(H, 4)
    pos = bad[lay.positions:lay.positions + H * budget * 4].view(torch.int32).view(H, budget)
    slots = bad[lay.slots:lay.slots + H * budget * 4].view(torch.int32).view(H, budget)
    hdr[1, 0] = budget + 1                 # more tokens than the budget
    hdr[2, 2] = 17                         # idx beyond the tree region (16 slots)
    pos[3, 5], pos[3, 6] = pos[3, 6].item(), pos[3, 5].item()      # positions out of order
    slots[4, 7] = slots[4, 8]              # two tokens in one slot
    slots[5, 3] = budget + 1               # a slot that does not exist
    pos[6, budget - 1] = T0 - 2            # the newest token missing from the recent window
    status = torch.full((B, H), 7, dtype=torch.int32, device="cuda")
    b = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="f32", n_sink=2, n_recent=6)
    b.import_state(bad, status)
    torch.cuda.synchronize()
    assert status.cpu().numpy().ravel().tolist() == [0, -1, -1, -1, -1, -1, -1, 0]
    want = _steps(a, Qd, Kd, Vd, T0, T0 + 5)
    got = _steps(b, Qd, Kd, Vd, T0, T0 + 5)
    for u in (0, 7):
        for w, g in zip(want, got):
            assert np.array_equal(w[:, 0, u], g[:, 0, u])
    # a refused unit starts over: it holds exactly the five tokens decoded since
    assert (got[2][-1, 0, 1:7, :5] == np.arange(5)).all() and (got[2][-1, 0, 1:7, 5:] == -1).all()


def test_snapshot_argument_errors(binding):
    import torch

    kv = binding.TreeKV(32, 2, 128)
    n = kv._lib.treekv_state_bytes(kv._h)
    assert n == kv.state_layout().bytes and n > 2 * 2 * 32 * 128 * 2
    small = torch.empty(n - 1, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.TreeKVError):
        kv.export_state(small)
    with pytest.raises(binding.TreeKVError):
        kv.import_state(small)
    buf = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.TreeKVError):
        kv.export_state(buf[16:])              # not 256-byte aligned
