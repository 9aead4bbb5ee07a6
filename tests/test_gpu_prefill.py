"""GPU parity: chunked prefill (through the C ABI) against the CPU oracle, mixed with decode steps."""
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


def _run(binding, oracle, schedule, *, B, H, Hkv, d, budget, n_sink, n_recent, seed=0, max_chunk=0, flags=0,
         units=None, kind="lowrank", dtype="bf16", scale=0.0, **gen_kw):
    T = sum(max(L, 1) for L in schedule)
    Q, K, V = inputs.batch_streams(kind, seed, T, B, Hkv, H // Hkv, d, dtype=dtype, **gen_kw)
    kv = binding.TreeKV(budget, H, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=n_sink, n_recent=n_recent,
                        max_chunk=max_chunk, flags=flags, softmax_scale=scale)
    st = ph.run_schedule(oracle, kv, Q, K, V, schedule, dtype=dtype, units=units)
    st["score_err"] = ph.compare_scores(kv, st["results"], dtype)
    assert st["flagged"] <= max(2, st["decisions"] // 500), st["flagged"]
    print(f"  flagged={st['flagged']}/{st['decisions']} max_err={st['max_err']:.2e} score_err={st['score_err']:.2e}")
    return kv, st


def test_prefill_fill_then_evict_with_layout(binding, oracle):
    """Chunks that fill the cache, cross the budget, and span several sweeps of the scope index."""
    _run(binding, oracle, [40, 17, 64, 1, 100, 33, 128, 7], B=1, H=2, Hkv=2, d=128, budget=96, n_sink=2, n_recent=30,
         max_chunk=128)


def test_prefill_pure_algorithm1_many_sweeps(binding, oracle):
    """No protected tokens, tree region of 50 slots, chunks of up to 200 tokens: up to 5 sweeps per chunk."""
    _run(binding, oracle, [30, 200, 3, 150, 200, 49, 51], B=1, H=2, Hkv=2, d=128, budget=50, n_sink=0, n_recent=0,
         max_chunk=256, seed=4)


def test_prefill_interleaved_with_decode(binding, oracle):
    _run(binding, oracle, [0, 0, 20, 0, 64, 0, 0, 0, 70, 0, 5, 0], B=2, H=2, Hkv=2, d=128, budget=48, n_sink=1,
         n_recent=15, max_chunk=128, seed=6)


@pytest.mark.parametrize("G,d", [(4, 128), (2, 64), (8, 64)])
def test_prefill_grouped_queries(binding, oracle, G, d):
    _run(binding, oracle, [50, 90, 0, 128, 13], B=2, H=2 * G, Hkv=2, d=d, budget=72, n_sink=3, n_recent=20,
         max_chunk=128, seed=8)


@pytest.mark.parametrize("budget,n_sink,n_recent", [(1, 0, 0), (2, 0, 0), (3, 1, 1), (6, 0, 5), (6, 5, 0)])
def test_prefill_degenerate_budgets(binding, oracle, budget, n_sink, n_recent):
    _run(binding, oracle, [5, 1, 16, 0, 33], B=1, H=1, Hkv=1, d=64, budget=budget, n_sink=n_sink, n_recent=n_recent,
         max_chunk=64, seed=9, kind="iid")


def test_prefill_keep_left(binding, oracle):
    _run(binding, oracle, [64, 64, 10, 64], B=1, H=2, Hkv=2, d=128, budget=40, n_sink=0, n_recent=8, max_chunk=64,
         flags=binding.TREEKV_KEEP_LEFT, seed=10)


def test_prefill_large_budget_runs_in_place(binding, oracle):
    """A budget whose order arrays do not fit in LDS takes the replay kernel's in-place variant."""
    _run(binding, oracle, [1024] * 9 + [700, 0, 0], B=1, H=1, Hkv=1, d=64, budget=9000, n_sink=0, n_recent=0,
         max_chunk=1024, seed=13)


def test_prefill_len1_equals_decode(binding, oracle):
    """A one-token chunk is a decode step: same evictions, same retained list, outputs within tolerance."""
    import torch

    T, B, H, d, budget = 150, 1, 4, 128, 32
    Q, K, V = inputs.batch_streams("lowrank", 12, T, B, H, 1, d, dtype="bf16")
    a = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=6, max_chunk=16)
    b = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=2, n_recent=6, max_chunk=16)
    Qd, Kd, Vd = (ph.to_device(x, "bf16") for x in (Q, K, V))
    oa, ra, na, ea = a.new_outputs()
    ob, rb, nb, eb = b.new_outputs(1)
    for t in range(T):
        a.decode_step(Qd[t], Kd[t], Vd[t], oa, ra, na, ea)
        b.prefill_chunk(Qd[t:t + 1].permute(1, 0, 2, 3).contiguous(), Kd[t:t + 1].permute(1, 0, 2, 3).contiguous(),
                        Vd[t:t + 1].permute(1, 0, 2, 3).contiguous(), 1, ob, rb, nb, eb)
        torch.cuda.synchronize()
        assert torch.equal(ea.flatten(), eb.flatten()) and torch.equal(ra, rb) and torch.equal(na, nb), t
        assert (oa - ob[:, 0]).abs().max().item() < 1e-4
    assert (a.scores() - b.scores()).abs().max().item() < 1e-3


def test_prefill_argument_errors(binding):
    import torch

    kv = binding.TreeKV(32, 2, 128, max_chunk=64)
    out, ret, nret, ev = kv.new_outputs(8)
    x = torch.zeros(1, 80, 2, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.TreeKVError):
        kv.prefill_chunk(x, x, x, 65, out, ret, nret, ev)          # longer than max_chunk
    with pytest.raises(binding.TreeKVError):
        kv.prefill_chunk(x, x, x, 0, out, ret, nret, ev)
    big = binding.TreeKV(10000, 2, 64, kv_heads=2, dtype="f32", n_sink=0, n_recent=0, max_chunk=512)
    xf = torch.zeros(1, 512, 2, 64, dtype=torch.float32, device="cuda")
    outf, retf, nretf, evf = big.new_outputs(512)
    with pytest.raises(binding.TreeKVError) as e:
        big.prefill_chunk(xf, xf, xf, 512, outf, retf, nretf, evf)  # fp32 storage: more columns than a thread's sums cover
    assert e.value.status == binding.TREEKV_EUNSUPPORTED


def test_prefill_gather_kv_matches_retained(binding, oracle):
    """After chunks and decode steps the compacted cache (treekv_gather_kv) holds exactly the rows of the retained
    positions: surviving chunk rows were scattered into the right freed slots."""
    import torch

    sched = [40, 100, 0, 64, 0, 0, 90]
    T = sum(max(L, 1) for L in sched)
    B, H, d, budget = 2, 2, 128, 56
    Q, K, V = inputs.batch_streams("lowrank", 31, T, B, H, 1, d, dtype="bf16")
    kv = binding.TreeKV(budget, H, d, kv_heads=H, batch=B, dtype="bf16", n_sink=3, n_recent=13, max_chunk=128)
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="bf16")     # retained lists compared call by call
    Kc, Vc = kv.gather_kv()
    torch.cuda.synchronize()
    for (b, h), res in st["results"].items():
        pos = res["stream"].retained()
        np.testing.assert_array_equal(Kc[b, h, :len(pos)].float().cpu().numpy(), K[pos, b, h])
        np.testing.assert_array_equal(Vc[b, h, :len(pos)].float().cpu().numpy(), V[pos, b, h])


def test_prefill_accumulated_weight_criterion(binding, oracle):
    _run(binding, oracle, [40, 64, 0, 128, 0, 0, 77, 5], B=1, H=4, Hkv=2, d=128, budget=72, n_sink=2, n_recent=20,
         max_chunk=128, flags=binding.TREEKV_SCORE_ACCUMULATED, seed=23)


@pytest.mark.parametrize("G,d", [(1, 64), (2, 128), (4, 64)])
def test_prefill_fp32_storage(binding, oracle, G, d):
    """fp32 storage: the chunk's attention runs on the vector ALUs (the matrix pipe takes bf16) and is held to 1e-5;
    chunks that fill, cross the budget and span sweeps, decode steps in between, ragged lengths."""
    _run(binding, oracle, [40, 17, 64, 1, 0, 100, 33, 0, 0, 128, 7], B=2, H=2 * G, Hkv=2, d=d, budget=96, n_sink=2,
         n_recent=30, max_chunk=128, seed=14, kind="iid", dtype="f32")


def test_prefill_fp32_tiny_configuration_in_chunks(binding, oracle):
    """The tiny fp32 configuration (2 heads x 64, budget 64, 512 tokens, K carrying the 1/sqrt(64)) fed as chunks."""
    _run(binding, oracle, [64] * 7 + [63, 1], B=1, H=2, Hkv=2, d=64, budget=64, n_sink=4, n_recent=28, max_chunk=64,
         seed=0, kind="iid", dtype="f32", scale=1.0, k_scale=0.125)


def test_prefill_fp32_degenerate_and_keep_left(binding, oracle):
    _run(binding, oracle, [5, 1, 16, 0, 33], B=1, H=1, Hkv=1, d=64, budget=3, n_sink=1, n_recent=1, max_chunk=64,
         seed=15, kind="iid", dtype="f32")
    _run(binding, oracle, [30, 30, 10, 30], B=1, H=2, Hkv=2, d=128, budget=40, n_sink=0, n_recent=8, max_chunk=32,
         flags=binding.TREEKV_KEEP_LEFT | binding.TREEKV_SCORE_ACCUMULATED, seed=16, kind="iid", dtype="f32")
