"""GPU parity: the HIP decode step (through the C ABI) against the CPU oracle, element by element."""
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

    b.load()     # raises if the HIP library is not built: there is no fallback
    return b


def _run(binding, oracle, *, kind, T, B, H, Hkv, d, dtype, budget, n_sink, n_recent, seed=0, flags=0,
         kv_splits=0, scale=0.0, k_scale=1.0, every_step=True, units=None, sample=None):
    G = H // Hkv
    kw = dict(k_scale=k_scale) if kind == "iid" else {}
    Q, K, V = inputs.batch_streams(kind, seed, T, B, Hkv, G, d, dtype=dtype, **kw)
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=n_sink, n_recent=n_recent,
                        softmax_scale=scale, flags=flags, kv_splits=kv_splits)
    steps = range(T) if every_step else (sample or [T - 1])
    gpu = ph.gpu_decode_run(kv, ph.to_device(Q, dtype), ph.to_device(K, dtype), ph.to_device(V, dtype), steps)
    rep = ph.compare_decode(oracle, kv, Q, K, V, gpu, units=units, dtype=dtype)
    rep["score_err"] = ph.compare_scores(kv, rep["results"], dtype)
    # flagged near-ties are rare by construction of the inputs
    assert rep["flagged"] <= max(2, rep["decisions"] // 500), rep["flagged"]
    print(f"  flagged={rep['flagged']}/{rep['decisions']} max_err={rep['max_err']:.2e} score_err={rep['score_err']:.2e}")
    return kv, gpu, rep


@pytest.mark.parametrize("layout", [(4, 28), (0, 0)])
def test_tiny_decode_config(binding, oracle, layout):
    """2 heads, head_dim 64, fp32, budget 64, 512-token stream; K carries the 1/sqrt(64), scale 1."""
    _run(binding, oracle, kind="iid", T=512, B=1, H=2, Hkv=2, d=64, dtype="f32", budget=64,
         n_sink=layout[0], n_recent=layout[1], scale=1.0, k_scale=0.125)


@pytest.mark.parametrize("splits", [1, 2, 3, 5])
def test_bf16_ragged_budget_splits(binding, oracle, splits):
    """Budget 203 (cap 204 is not a multiple of any tile), several split counts, incl. empty splits."""
    _run(binding, oracle, kind="lowrank", T=650, B=1, H=3, Hkv=3, d=128, dtype="bf16", budget=203,
         n_sink=4, n_recent=98, kv_splits=splits, seed=3)


def test_bf16_pure_algorithm1(binding, oracle):
    """No sinks, no recent window: Algorithm 1 verbatim; the new token itself can be in the scope."""
    _run(binding, oracle, kind="lowrank", T=700, B=2, H=2, Hkv=2, d=128, dtype="bf16", budget=160,
         n_sink=0, n_recent=0, kv_splits=4, seed=5)


@pytest.mark.parametrize("G,d,dtype", [(4, 128, "bf16"), (2, 64, "bf16"), (8, 64, "f32"), (1, 128, "f32")])
def test_grouped_queries_and_types(binding, oracle, G, d, dtype):
    # the low-rank streams (values up to ~15) go with bf16; fp32 is checked to 1e-5 on unit-variance streams
    _run(binding, oracle, kind="lowrank" if dtype == "bf16" else "iid", T=400, B=2, H=2 * G, Hkv=2, d=d, dtype=dtype, budget=96,
         n_sink=2, n_recent=30, kv_splits=2, seed=7)


@pytest.mark.parametrize("budget,n_sink,n_recent", [(1, 0, 0), (2, 0, 0), (3, 1, 1), (5, 0, 4), (5, 4, 0)])
def test_degenerate_budgets(binding, oracle, budget, n_sink, n_recent):
    _run(binding, oracle, kind="iid", T=40, B=1, H=1, Hkv=1, d=64, dtype="f32", budget=budget,
         n_sink=n_sink, n_recent=n_recent)


def test_keep_left_ablation(binding, oracle):
    kv, gpu, rep = _run(binding, oracle, kind="lowrank", T=300, B=1, H=2, Hkv=2, d=128, dtype="bf16", budget=64,
                        n_sink=0, n_recent=0, flags=binding.TREEKV_KEEP_LEFT, seed=9)
    from tests.span_sim import SpanSim

    sim = SpanSim(64)
    for _ in range(300):
        sim.step()
    assert list(gpu["retained"][299][0, 0]) == [lo for lo, _ in sim.spans]


def test_default_init_layout(binding):
    """treekv_init(budget, heads, head_dim): 4 sinks + budget/2 tree slots + the rest recent."""
    kv = binding.TreeKV(1024, 32, 128)
    c = kv.cfg
    assert (c.n_sink, c.n_recent, c.budget - c.n_sink - c.n_recent) == (4, 508, 512)
    assert (c.batch, c.kv_heads, c.dtype) == (1, 32, binding.TREEKV_BF16)
    assert abs(c.softmax_scale - 128 ** -0.5) < 1e-7


def test_gather_kv_matches_retained(binding, oracle):
    import torch

    T, B, H, d, budget = 300, 1, 2, 128, 50
    Q, K, V = inputs.batch_streams("lowrank", 11, T, B, H, 1, d, dtype="bf16")
    kv = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=10)
    gpu = ph.gpu_decode_run(kv, ph.to_device(Q, "bf16"), ph.to_device(K, "bf16"), ph.to_device(V, "bf16"), [T - 1])
    Kc, Vc = kv.gather_kv()
    torch.cuda.synchronize()
    ret = gpu["retained"][T - 1]
    for h in range(H):
        np.testing.assert_array_equal(Kc[0, h].float().cpu().numpy(), K[ret[0, h], 0, h])
        np.testing.assert_array_equal(Vc[0, h].float().cpu().numpy(), V[ret[0, h], 0, h])


def test_reset_restarts_the_stream(binding, oracle):
    import torch

    T, H, d, budget = 120, 2, 64, 32
    Q, K, V = inputs.batch_streams("iid", 2, T, 1, H, 1, d, dtype="f32")
    kv = binding.TreeKV(budget, H, d, kv_heads=H, dtype="f32", n_sink=0, n_recent=0)
    Qd, Kd, Vd = (ph.to_device(x, "f32") for x in (Q, K, V))
    a = ph.gpu_decode_run(kv, Qd, Kd, Vd, [T - 1])
    kv.reset()
    b = ph.gpu_decode_run(kv, Qd, Kd, Vd, [T - 1])
    np.testing.assert_array_equal(a["out"], b["out"])          # same launches, same order: deterministic
    np.testing.assert_array_equal(a["evicted"], b["evicted"])
    np.testing.assert_array_equal(a["retained"][T - 1], b["retained"][T - 1])


def test_benchmark_launch_configuration_sampled(binding, oracle):
    """The shape bench.py times: batch 8 x 32 heads x 128, bf16, budget 2048 (4 + 1024 + 1020), one workgroup per
    unit (256 units).  Caches are filled with four 512-token prefill chunks as in the benchmark, then 300 decode
    steps run with evictions; the oracle audits 6 of the 256 streams call by call, every stream is checked for the
    properties that hold at any size."""
    B, H, d, budget, steps = 8, 32, 128, 2048, 300
    T = budget + steps
    Q, K, V = inputs.batch_streams("lowrank", 1, T, B, H, 1, d, dtype="bf16", seed_per_batch=True)
    kv = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=4, n_recent=1020)
    assert kv.cfg.kv_splits == 1
    units = [(0, 0), (1, 7), (3, 31), (4, 16), (6, 9), (7, 30)]
    st = ph.run_schedule(oracle, kv, Q, K, V, [512] * 4 + [0] * steps, dtype="bf16", units=units)
    err = ph.compare_scores(kv, st["results"], "bf16")
    print(f"  flagged={st['flagged']}/{st['decisions']} max_err={st['max_err']:.2e} score_err={err:.2e}")
    assert st["decisions"] == len(units) * steps and st["flagged"] <= 2
    import torch

    out, ret, nret, ev = kv.new_outputs()
    kv.decode_step(ph.to_device(Q[T - 1], "bf16"), ph.to_device(K[T - 1], "bf16"), ph.to_device(V[T - 1], "bf16"),
                   out, ret, nret, ev)                    # one more step for all 256 units (inputs reused)
    torch.cuda.synchronize()
    ret, nret, ev = ret.cpu().numpy(), nret.cpu().numpy(), ev.cpu().numpy()
    assert np.all(nret == budget) and np.all(np.diff(ret, axis=-1) > 0)
    assert np.all(ret[..., :4] == np.arange(4)) and np.all(ret[..., -1020:] == np.arange(T + 1 - 1020, T + 1))
    assert np.all((ev >= 4) & (ev < T + 1 - 1020)) and np.all(np.isfinite(out.cpu().numpy()))


def test_gqa_long_budget_split_path_sampled(binding, oracle):
    """32 query heads on 8 KV heads, head_dim 128, bf16, budget 4096, batch 16: 128 units, so the slots of a unit
    are split over several workgroups and merged by the second kernel; scores add up the group's 4 query heads."""
    B, H, Hkv, d, budget = 16, 32, 8, 128, 4096
    sched = [512] * 9 + [0] * 40
    T = 512 * 9 + 40
    Q, K, V = inputs.batch_streams("lowrank", 2, T, B, Hkv, H // Hkv, d, dtype="bf16", seed_per_batch=True)
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype="bf16", n_sink=4, n_recent=2044)
    assert kv.cfg.kv_splits > 1
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="bf16", units=[(0, 0), (9, 5), (15, 7)])
    err = ph.compare_scores(kv, st["results"], "bf16")
    print(f"  flagged={st['flagged']}/{st['decisions']} max_err={st['max_err']:.2e} score_err={err:.2e}")
    assert st["decisions"] == 3 * (T - budget)


def test_decode_steps_replay_from_a_hip_graph(binding):
    """No host-side state changes between steps, so a captured step can be replayed: replays with fresh inputs
    (and eager work in between) must give exactly what eager launches give."""
    import torch

    T, B, H, d, budget = 80, 2, 4, 128, 24
    Q, K, V = inputs.batch_streams("lowrank", 21, T, B, H, 1, d, dtype="bf16")
    Qd, Kd, Vd = (ph.to_device(x, "bf16") for x in (Q, K, V))
    eager = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=6, kv_splits=1)
    graph = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=6, kv_splits=1)
    want = ph.gpu_decode_run(eager, Qd, Kd, Vd, range(T))
    q_s, k_s, v_s = Qd[0].clone(), Kd[0].clone(), Vd[0].clone()          # static input buffers of the graph
    out, ret, nret, ev = graph.new_outputs()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graph.decode_step(q_s, k_s, v_s, out, ret, nret, ev)
    graph.reset()                                                        # capture does not execute; start clean
    torch.cuda.synchronize()
    for t in range(T):
        q_s.copy_(Qd[t]); k_s.copy_(Kd[t]); v_s.copy_(Vd[t])
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want["out"][t]), t
        assert np.array_equal(ev.cpu().numpy(), want["evicted"][t]), t
        assert np.array_equal(ret.cpu().numpy(), want["retained"][t]), t
        _ = (Qd[t].float() * 2).sum().item()                             # unrelated eager work between replays


def test_accumulated_weight_criterion(binding, oracle):
    """TREEKV_SCORE_ACCUMULATED: the scope compares S, not S / C (Section 4.1's other criterion); fused and split shapes."""
    for splits, G in [(1, 1), (3, 4)]:
        _run(binding, oracle, kind="lowrank", T=500, B=2, H=2 * G, Hkv=2, d=128, dtype="bf16", budget=96,
             n_sink=3, n_recent=30, flags=binding.TREEKV_SCORE_ACCUMULATED, kv_splits=splits, seed=21)
    _run(binding, oracle, kind="iid", T=300, B=1, H=2, Hkv=2, d=64, dtype="f32", budget=40, n_sink=0, n_recent=0,
         flags=binding.TREEKV_SCORE_ACCUMULATED, seed=22)
