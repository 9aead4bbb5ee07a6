"""GPU parity: decode steps, prefill chunks and the one-shot prompt compression with positions re-assigned to cache
ranks (Section 4.1, "Position Encoding") through the C ABI against the CPU oracle: q and k arrive without positional
encoding, the rotary encoding of the in-cache ranks is applied inside the call."""
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


def _run(binding, oracle, *, T, B, H, Hkv, d, dtype, budget, n_sink, n_recent, seed, kv_splits=0, rope_base=0.0,
         flags=0, kind=None, every_step=True, units=None, sample=None):
    G = H // Hkv
    kind = kind or ("lowrank" if dtype == "bf16" else "iid")
    Q, K, V = inputs.batch_streams(kind, seed, T, B, Hkv, G, d, dtype=dtype)
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=n_sink, n_recent=n_recent,
                        flags=flags | binding.TREEKV_POSITION_RERANK, kv_splits=kv_splits, rope_base=rope_base)
    steps = range(T) if every_step else (sample or [T - 1])
    gpu = ph.gpu_decode_run(kv, ph.to_device(Q, dtype), ph.to_device(K, dtype), ph.to_device(V, dtype), steps)
    rep = ph.compare_decode(oracle, kv, Q, K, V, gpu, units=units, dtype=dtype)
    rep["score_err"] = ph.compare_scores(kv, rep["results"], dtype)
    assert rep["flagged"] <= max(2, rep["decisions"] // 500), rep["flagged"]
    print(f"  flagged={rep['flagged']}/{rep['decisions']} max_err={rep['max_err']:.2e} score_err={rep['score_err']:.2e}")
    return kv, gpu, rep


@pytest.mark.parametrize("splits", [1, 3])
def test_rerank_bf16_ragged_budget(binding, oracle, splits):
    """Budget 203 with sinks and a recent ring that wraps several times; one workgroup per unit and three."""
    _run(binding, oracle, T=650, B=1, H=3, Hkv=3, d=128, dtype="bf16", budget=203, n_sink=4, n_recent=98,
         kv_splits=splits, seed=31)


def test_rerank_pure_algorithm1(binding, oracle):
    """No sinks, no recent window: the new token itself enters the tree region; a short rotary period (base 50)."""
    _run(binding, oracle, T=700, B=2, H=2, Hkv=2, d=128, dtype="bf16", budget=160, n_sink=0, n_recent=0, kv_splits=4,
         seed=32, rope_base=50.0)


@pytest.mark.parametrize("G,d,dtype,splits", [(4, 64, "bf16", 2), (2, 128, "f32", 1), (8, 64, "f32", 2),
                                              (8, 128, "bf16", 1), (1, 64, "f32", 1)])
def test_rerank_grouped_queries_and_types(binding, oracle, G, d, dtype, splits):
    _run(binding, oracle, T=400, B=2, H=2 * G, Hkv=2, d=d, dtype=dtype, budget=96, n_sink=2, n_recent=30,
         kv_splits=splits, seed=33)


def test_rerank_differs_from_plain_and_from_original_positions(binding, oracle):
    """The same stream with and without the flag: identical while nothing could differ (one token), different after;
    and once tokens have been evicted the outputs differ from rotary attention at the ORIGINAL positions (computed
    here from the retained positions the step returns)."""
    import torch

    T, H, d, budget = 80, 2, 64, 24
    Q, K, V = inputs.batch_streams("iid", 34, T, 1, H, 1, d, dtype="f32")
    Qd, Kd, Vd = (ph.to_device(x, "f32") for x in (Q, K, V))
    a = binding.TreeKV(budget, H, d, kv_heads=H, dtype="f32", n_sink=2, n_recent=6)
    b = binding.TreeKV(budget, H, d, kv_heads=H, dtype="f32", n_sink=2, n_recent=6, flags=binding.TREEKV_POSITION_RERANK)
    ga, gb = ph.gpu_decode_run(a, Qd, Kd, Vd, range(T)), ph.gpu_decode_run(b, Qd, Kd, Vd, range(T))
    assert np.array_equal(ga["out"][0], gb["out"][0])
    assert np.abs(ga["out"][5] - gb["out"][5]).max() > 1e-3
    t = T - 1
    kept = list(gb["retained"][t - 1][0, 0]) + [t]            # what step t attends: the cache after step t-1, and t
    theta = 10000.0 ** (-2.0 * np.arange(d // 2) / d)

    def rot(x, pos):
        z = (x[..., 0::2] + 1j * x[..., 1::2]) * np.exp(1j * np.multiply.outer(pos, theta))
        return z

    def attend(pos_k, pos_q):
        kz, qz = rot(K[kept, 0, 0], np.array(pos_k, dtype=np.float64)), rot(Q[t, 0, 0], float(pos_q))
        lg = np.real(kz.conj() @ qz) / np.sqrt(d)
        w = np.exp(lg - lg.max())
        return (w / w.sum()) @ V[kept, 0, 0]

    got = gb["out"][t][0, 0]
    assert np.abs(got - attend(np.arange(len(kept)), len(kept) - 1)).max() < 1e-5
    assert np.abs(got - attend(kept, t)).max() > 1e-3


def _chunks(binding, oracle, schedule, *, B, H, Hkv, d, budget, n_sink, n_recent, seed, max_chunk=0, flags=0,
            rope_base=0.0, units=None, dtype="bf16"):
    """Prefill chunks (and decode steps, 0) with re-assigned positions: the n0 cached tokens sit at ranks 0..n0-1, chunk
    token i at n0 + i; compared call by call."""
    T = sum(max(L, 1) for L in schedule)
    Q, K, V = inputs.batch_streams("lowrank" if dtype == "bf16" else "iid", seed, T, B, Hkv, H // Hkv, d, dtype=dtype)
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=n_sink, n_recent=n_recent,
                        max_chunk=max_chunk, flags=flags | binding.TREEKV_POSITION_RERANK, rope_base=rope_base)
    st = ph.run_schedule(oracle, kv, Q, K, V, schedule, dtype=dtype, units=units)
    st["score_err"] = ph.compare_scores(kv, st["results"], dtype)
    assert st["flagged"] <= max(2, st["decisions"] // 500), st["flagged"]
    print(f"  flagged={st['flagged']}/{st['decisions']} max_err={st['max_err']:.2e} score_err={st['score_err']:.2e}")
    return kv, st


def test_rerank_chunks_fill_then_evict(binding, oracle):
    """Chunks that fill the cache, cross the budget and span several sweeps of the scope index; ragged lengths."""
    _chunks(binding, oracle, [40, 17, 64, 1, 100, 33, 128, 7], B=1, H=2, Hkv=2, d=128, budget=96, n_sink=2, n_recent=30,
            max_chunk=128, seed=61)


def test_rerank_chunks_interleaved_with_decode(binding, oracle):
    _chunks(binding, oracle, [0, 0, 20, 0, 64, 0, 0, 0, 70, 0, 5, 0], B=2, H=2, Hkv=2, d=128, budget=48, n_sink=1,
            n_recent=15, max_chunk=128, seed=62, rope_base=50.0)


@pytest.mark.parametrize("G,d", [(4, 128), (2, 64), (8, 64)])
def test_rerank_chunks_grouped_queries(binding, oracle, G, d):
    _chunks(binding, oracle, [50, 90, 0, 128, 13], B=2, H=2 * G, Hkv=2, d=d, budget=72, n_sink=3, n_recent=20,
            max_chunk=128, seed=63)


@pytest.mark.parametrize("G,d", [(1, 128), (2, 64), (4, 128)])
def test_rerank_chunks_fp32_storage(binding, oracle, G, d):
    """fp32 storage: keys and queries turned to their ranks in fp32, the vector-ALU attention, held to 1e-5; chunks
    that fill the cache, cross the budget, interleave with decode steps."""
    _chunks(binding, oracle, [30, 0, 64, 9, 0, 0, 100, 1, 47], B=2, H=2 * G, Hkv=2, d=d, budget=56, n_sink=2,
            n_recent=17, max_chunk=100, seed=66, dtype="f32", rope_base=300.0)


def test_rerank_budget_beyond_the_lds_angle_tables(binding, oracle):
    """6500 slots: the decode step's two small angle tables no longer fit beside the logits and the pairs come from
    the context's full table; filled by chunks, then decode steps that evict."""
    _chunks(binding, oracle, [512] * 13 + [0] * 120, B=1, H=1, Hkv=1, d=64, budget=6500, n_sink=4, n_recent=1000,
            max_chunk=512, seed=67)


def test_rerank_chunks_pure_algorithm1_many_tiles(binding, oracle):
    """No protected tokens; 300-token chunks over a 400-slot cache: several column tiles of cache and of chunk, the
    causal diagonal crossing tiles, up to 2 sweeps per chunk."""
    _chunks(binding, oracle, [300, 300, 7, 256, 300], B=1, H=2, Hkv=2, d=128, budget=400, n_sink=0, n_recent=0,
            max_chunk=300, seed=64)


def test_rerank_chunk_of_one_token_equals_decode(binding, oracle):
    """A one-token chunk is a decode step with re-assigned positions: same evictions and retained list, outputs and
    scores equal to rounding."""
    import torch

    T, B, H, d, budget = 150, 1, 4, 128, 32
    Q, K, V = inputs.batch_streams("lowrank", 65, T, B, H, 1, d, dtype="bf16")
    mk = lambda: binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=6, max_chunk=16,
                                flags=binding.TREEKV_POSITION_RERANK)
    a, b = mk(), mk()
    Qd, Kd, Vd = (ph.to_device(x, "bf16") for x in (Q, K, V))
    oa, ra, na, ea = a.new_outputs()
    ob, rb, nb, eb = b.new_outputs(1)
    for t in range(T):
        a.decode_step(Qd[t], Kd[t], Vd[t], oa, ra, na, ea)
        cut = lambda X: X[t:t + 1].permute(1, 0, 2, 3).contiguous()
        b.prefill_chunk(cut(Qd), cut(Kd), cut(Vd), 1, ob, rb, nb, eb)
        torch.cuda.synchronize()
        assert torch.equal(ea.flatten(), eb.flatten()) and torch.equal(ra, rb) and torch.equal(na, nb), t
        assert (oa - ob[:, 0]).abs().max().item() < 2e-4
    assert (a.scores() - b.scores()).abs().max().item() < 1e-3


def test_rerank_chunks_llama_shaped_sampled(binding, oracle):
    """32 heads x 128, budget 2048 (4 + 1024 + 1020): 2560 tokens in chunks of 512, then decode steps; the oracle
    audits 4 heads call by call."""
    sched = [512] * 5 + [0] * 8
    kv, st = _chunks(binding, oracle, sched, B=1, H=32, Hkv=32, d=128, budget=2048, n_sink=4, n_recent=1020,
                     units=[(0, 0), (0, 11), (0, 22), (0, 31)], seed=66)
    assert st["decisions"] == 4 * (2560 + 8 - 2048)


def _prompt(binding, oracle, *, T, block, steps, B, H, Hkv, d, budget, n_sink, n_recent, seed, rope_base=0.0, flags=0,
            dtype="bf16"):
    Q, K, V = inputs.batch_streams("lowrank" if dtype == "bf16" else "iid", seed, T + steps, B, Hkv, H // Hkv, d, dtype=dtype)
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=n_sink, n_recent=n_recent,
                        flags=flags | binding.TREEKV_POSITION_RERANK, max_prompt=T, rope_base=rope_base)
    st = ph.run_prompt(oracle, kv, Q, K, V, T, block, steps, dtype=dtype)
    assert st["flagged"] <= max(1, st["decisions"] // 200), st["flagged"]
    print(f"  blocks evicted={st['decisions']} flagged={st['flagged']} token score rel err={st['tok_err']:.2e}")
    return st


def test_rerank_prompt_ragged_slices_then_decode(binding, oracle):
    """One-shot compression of a prompt without positional encoding (rotary encoding of the original positions
    applied while the window scores it), 37 blocks of 16 into 8 block slots, then 40 decode steps at cache ranks."""
    _prompt(binding, oracle, T=592, block=16, steps=40, B=1, H=2, Hkv=2, d=128, budget=128, n_sink=4, n_recent=20, seed=51)


@pytest.mark.parametrize("G,d,block", [(4, 64, 8), (2, 128, 16), (8, 64, 16), (1, 128, 128), (1, 64, 64)])
def test_rerank_prompt_shapes(binding, oracle, G, d, block):
    _prompt(binding, oracle, T=block * 41, block=block, steps=8, B=2, H=2 * G, Hkv=2, d=d, budget=block * 12, n_sink=3,
            n_recent=block + 5, seed=52, rope_base=500.0)


@pytest.mark.parametrize("G,d,block", [(1, 128, 16), (4, 64, 8)])
def test_rerank_prompt_fp32_storage(binding, oracle, G, d, block):
    """fp32 storage: the window's queries and every key turned to the original positions while the prompt is scored,
    then decode steps at cache ranks; held to 1e-5."""
    _prompt(binding, oracle, T=block * 37, block=block, steps=12, B=2, H=2 * G, Hkv=2, d=d, budget=block * 10, n_sink=3,
            n_recent=block + 5, seed=54, rope_base=1000.0, dtype="f32")


def test_rerank_prompt_long(binding, oracle):
    """8192 tokens in blocks of 64 into 1024 slots: several slices per head, angles far around the circle."""
    _prompt(binding, oracle, T=8192, block=64, steps=4, B=1, H=4, Hkv=4, d=128, budget=1024, n_sink=4, n_recent=508, seed=53)


def test_rerank_llama7b_shaped_layer_sampled(binding, oracle):
    """32 heads x 128, budget 1024 (4 + 512 + 508), 3000 steps; four heads checked at every step against the oracle."""
    _run(binding, oracle, T=3000, B=1, H=32, Hkv=32, d=128, dtype="bf16", budget=1024, n_sink=4, n_recent=508,
         seed=35, units=[(0, 0), (0, 9), (0, 21), (0, 31)], every_step=False, sample=[1500, 2999])


def test_rerank_benchmark_launch_configuration_sampled(binding, oracle):
    """The shape `bench.py --rerank` times: batch 8 x 32 heads x 128, bf16, budget 2048 (4 + 1024 + 1020), one
    workgroup per unit.  A 4096-token prompt is compressed in one shot (blocks of 64), then 120 decode steps run
    with evictions, all with re-assigned positions; the oracle audits 5 of the 256 streams, every stream is checked
    for the properties that hold at any size."""
    import torch

    B, H, d, budget, T, block, steps = 8, 32, 128, 2048, 4096, 64, 120
    Q, K, V = inputs.batch_streams("lowrank", 61, T + steps, B, H, 1, d, dtype="bf16", seed_per_batch=True)
    kv = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=4, n_recent=1020,
                        flags=binding.TREEKV_POSITION_RERANK, max_prompt=T)
    assert kv.cfg.kv_splits == 1
    units = [(0, 0), (2, 13), (4, 31), (5, 8), (7, 21)]
    st = ph.run_prompt(oracle, kv, Q, K, V, T, block, steps, units=units)
    print(f"  prompt: flagged={st['flagged']}/{st['decisions']} tok_err={st['tok_err']:.2e}; decode: "
          f"flagged={st['decode']['flagged']}/{st['decode']['decisions']} max_err={st['decode']['max_err']:.2e}")
    assert st["decode"]["decisions"] == len(units) * steps and st["decode"]["flagged"] <= 2
    out, ret, nret, ev = kv.new_outputs()
    t = T + steps - 1
    kv.decode_step(ph.to_device(Q[t], "bf16"), ph.to_device(K[t], "bf16"), ph.to_device(V[t], "bf16"), out, ret, nret, ev)
    torch.cuda.synchronize()
    ret, nret, ev = ret.cpu().numpy(), nret.cpu().numpy(), ev.cpu().numpy()
    assert np.all(nret == budget) and np.all(np.diff(ret, axis=-1) > 0)
    assert np.all(ret[..., :4] == np.arange(4)) and np.all(ret[..., -1020:] == np.arange(t + 2 - 1020, t + 2))
    assert np.all((ev >= 4) & (ev < t + 2 - 1020)) and np.all(np.isfinite(out.cpu().numpy()))


@pytest.mark.parametrize("splits", [1, 2])
def test_rerank_decode_steps_replay_from_a_hip_graph(binding, splits):
    """The ranks are rebuilt from the order arrays inside every step (no host-side state), so a captured step with
    re-assigned positions replays like a plain one: exactly what eager launches give, with eager work in between."""
    import torch

    T, B, H, d, budget = 70, 2, 4, 128, 24
    Q, K, V = inputs.batch_streams("lowrank", 71, T, B, H, 1, d, dtype="bf16")
    Qd, Kd, Vd = (ph.to_device(x, "bf16") for x in (Q, K, V))
    mk = lambda: binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=6, kv_splits=splits,
                                flags=binding.TREEKV_POSITION_RERANK)
    eager, graph = mk(), mk()
    want = ph.gpu_decode_run(eager, Qd, Kd, Vd, range(T))
    q_s, k_s, v_s = Qd[0].clone(), Kd[0].clone(), Vd[0].clone()
    out, ret, nret, ev = graph.new_outputs()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graph.decode_step(q_s, k_s, v_s, out, ret, nret, ev)
    graph.reset()
    torch.cuda.synchronize()
    for t in range(T):
        q_s.copy_(Qd[t]); k_s.copy_(Kd[t]); v_s.copy_(Vd[t])
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want["out"][t]), t
        assert np.array_equal(ev.cpu().numpy(), want["evicted"][t]), t
        assert np.array_equal(ret.cpu().numpy(), want["retained"][t]), t
        _ = (Qd[t].float() * 2).sum().item()
