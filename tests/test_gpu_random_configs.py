"""GPU parity on randomly drawn configurations: budgets, layouts, group sizes, head dims, split counts and call
schedules that no hand-written case names, each driven call by call against the CPU oracle.  Seeds are fixed."""
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


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 1, 2, 4, 8]))
    Hkv = int(rng.integers(1, 4))
    B = int(rng.integers(1, 3))
    budget = int(rng.choice([int(rng.integers(1, 12)), int(rng.integers(12, 80)), int(rng.integers(80, 400))]))
    n_sink = int(rng.integers(0, max(1, budget // 3)))
    n_recent = int(rng.integers(0, max(1, budget - n_sink)))
    if budget - n_sink - n_recent < 1:
        n_sink, n_recent = 0, 0
    splits = int(rng.choice([0, 1, 2, 3, 7]))
    return rng, dict(d=d, G=G, Hkv=Hkv, B=B, budget=budget, n_sink=n_sink, n_recent=n_recent, splits=splits)


@pytest.mark.parametrize("seed", range(40))
def test_random_schedule_of_chunks_and_steps(binding, oracle, seed):
    """bf16: chunks of random lengths (0 = one decode step) from an empty cache well past the budget."""
    rng, c = _draw(seed)
    max_chunk = int(rng.choice([16, 64, 200]))
    sched, total = [], 0
    while total < 2 * c["budget"] + 60:
        L = 0 if rng.random() < 0.45 else int(rng.integers(1, max_chunk + 1))
        sched.append(L)
        total += max(L, 1)
    Q, K, V = inputs.batch_streams("lowrank", seed, total, c["B"], c["Hkv"], c["G"], c["d"], dtype="bf16")
    kv = binding.TreeKV(c["budget"], c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="bf16",
                        n_sink=c["n_sink"], n_recent=c["n_recent"], max_chunk=max_chunk, kv_splits=c["splits"])
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="bf16")
    ph.compare_scores(kv, st["results"], "bf16")
    assert st["flagged"] <= max(2, st["decisions"] // 200), (c, st["flagged"])


@pytest.mark.parametrize("seed", range(40, 56))
def test_random_fp32_decode_streams(binding, oracle, seed):
    """fp32 storage (decode only): the vector-ALU stream for every group size."""
    rng, c = _draw(seed)
    T = 2 * c["budget"] + 50
    Q, K, V = inputs.batch_streams("iid", seed, T, c["B"], c["Hkv"], c["G"], c["d"], dtype="f32")
    kv = binding.TreeKV(c["budget"], c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="f32",
                        n_sink=c["n_sink"], n_recent=c["n_recent"], kv_splits=c["splits"])
    st = ph.run_schedule(oracle, kv, Q, K, V, [0] * T, dtype="f32")
    ph.compare_scores(kv, st["results"], "f32")


@pytest.mark.parametrize("seed", range(56, 80))
def test_random_prompt_then_chunks_and_steps(binding, oracle, seed):
    """bf16: a prompt compressed in one shot (random block size and length), then chunks and decode steps."""
    rng, c = _draw(seed)
    block = int(rng.choice([1, 2, 4, 8, 16, 32]))
    block = min(block, 128 // c["G"])
    cb = int(rng.integers(3, 14))
    budget = cb * block
    n_sink = int(rng.integers(0, block + 2))
    n_recent = int(rng.integers(0, block + 2))
    if cb - (-(-n_sink // block)) - (-(-n_recent // block)) < 1 or budget - n_sink - n_recent < 1:
        n_sink = n_recent = 0
    T = block * int(rng.integers(1, 4 * cb))
    sched = [int(x) for x in rng.choice([0, 0, 5, 33], size=8)]
    extra = sum(max(L, 1) for L in sched)
    Q, K, V = inputs.batch_streams("lowrank", seed, T + extra, c["B"], c["Hkv"], c["G"], c["d"], dtype="bf16")
    kv = binding.TreeKV(budget, c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="bf16",
                        n_sink=n_sink, n_recent=n_recent, max_chunk=64, max_prompt=T, kv_splits=c["splits"])
    st = ph.run_prompt(oracle, kv, Q, K, V, T, block, 0)
    st2 = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="bf16", streams=st["streams"], t_start=T)
    ph.compare_scores(kv, st2["results"], "bf16")


@pytest.mark.parametrize("seed", range(80, 104))
def test_random_decode_streams_with_reassigned_positions(binding, oracle, seed):
    """Decode streams with positions re-assigned to cache ranks: both storage types, every group size, random
    layouts, split counts and rotary bases; every step compared."""
    rng, c = _draw(seed)
    dtype = "bf16" if seed % 2 == 0 else "f32"
    base = float(rng.choice([0.0, 30.0, 500000.0]))
    flags = binding.TREEKV_POSITION_RERANK | (binding.TREEKV_SCORE_ACCUMULATED if seed % 5 == 0 else 0)
    T = 2 * c["budget"] + 50
    Q, K, V = inputs.batch_streams("lowrank" if dtype == "bf16" else "iid", seed, T, c["B"], c["Hkv"], c["G"], c["d"],
                                   dtype=dtype)
    kv = binding.TreeKV(c["budget"], c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype=dtype,
                        n_sink=c["n_sink"], n_recent=c["n_recent"], kv_splits=c["splits"], flags=flags, rope_base=base)
    st = ph.run_schedule(oracle, kv, Q, K, V, [0] * T, dtype=dtype)
    ph.compare_scores(kv, st["results"], dtype)
    assert st["flagged"] <= max(2, st["decisions"] // 200), (c, st["flagged"])


@pytest.mark.parametrize("seed", range(104, 120))
def test_random_prompt_then_steps_with_reassigned_positions(binding, oracle, seed):
    """bf16, positions re-assigned: a prompt compressed in one shot (random block size, length, layout, rotary
    base), then decode steps at cache ranks."""
    rng, c = _draw(seed)
    block = int(rng.choice([1, 2, 4, 8, 16, 32]))
    block = min(block, 128 // c["G"])
    cb = int(rng.integers(3, 14))
    budget = cb * block
    n_sink = int(rng.integers(0, block + 2))
    n_recent = int(rng.integers(0, block + 2))
    if cb - (-(-n_sink // block)) - (-(-n_recent // block)) < 1 or budget - n_sink - n_recent < 1:
        n_sink = n_recent = 0
    T = block * int(rng.integers(1, 4 * cb))
    steps = int(rng.integers(3, 20))
    base = float(rng.choice([0.0, 100.0]))
    Q, K, V = inputs.batch_streams("lowrank", seed, T + steps, c["B"], c["Hkv"], c["G"], c["d"], dtype="bf16")
    kv = binding.TreeKV(budget, c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="bf16",
                        n_sink=n_sink, n_recent=n_recent, max_prompt=T, kv_splits=c["splits"],
                        flags=binding.TREEKV_POSITION_RERANK, rope_base=base)
    st = ph.run_prompt(oracle, kv, Q, K, V, T, block, steps)
    assert st["flagged"] <= max(2, st["decisions"] // 100), (c, st["flagged"])


def _random_schedule(rng, budget, max_chunk):
    sched, total = [], 0
    while total < 2 * budget + 60:
        L = 0 if rng.random() < 0.45 else int(rng.integers(1, max_chunk + 1))
        sched.append(L)
        total += max(L, 1)
    return sched, total


@pytest.mark.parametrize("seed", range(80, 96))
def test_random_fp32_schedule_of_chunks_and_steps(binding, oracle, seed):
    """fp32 storage: chunks (vector-ALU attention) and decode steps mixed, held to 1e-5."""
    rng, c = _draw(seed)
    max_chunk = int(rng.choice([16, 64, 200]))
    sched, total = _random_schedule(rng, c["budget"], max_chunk)
    Q, K, V = inputs.batch_streams("iid", seed, total, c["B"], c["Hkv"], c["G"], c["d"], dtype="f32")
    kv = binding.TreeKV(c["budget"], c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="f32",
                        n_sink=c["n_sink"], n_recent=c["n_recent"], max_chunk=max_chunk, kv_splits=c["splits"])
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="f32")
    ph.compare_scores(kv, st["results"], "f32")
    assert st["flagged"] <= max(2, st["decisions"] // 200), (c, st["flagged"])


@pytest.mark.parametrize("seed", range(96, 116))
def test_random_rerank_schedule_of_chunks_and_steps(binding, oracle, seed):
    """bf16 with positions re-assigned to cache ranks: chunks and decode steps mixed, random rotary base."""
    rng, c = _draw(seed)
    max_chunk = int(rng.choice([16, 64, 200]))
    sched, total = _random_schedule(rng, c["budget"], max_chunk)
    Q, K, V = inputs.batch_streams("lowrank", seed, total, c["B"], c["Hkv"], c["G"], c["d"], dtype="bf16")
    kv = binding.TreeKV(c["budget"], c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="bf16",
                        n_sink=c["n_sink"], n_recent=c["n_recent"], max_chunk=max_chunk, kv_splits=c["splits"],
                        flags=binding.TREEKV_POSITION_RERANK, rope_base=float(rng.choice([0.0, 50.0, 500000.0])))
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="bf16")
    ph.compare_scores(kv, st["results"], "bf16")
    assert st["flagged"] <= max(2, st["decisions"] // 200), (c, st["flagged"])


@pytest.mark.parametrize("seed", range(116, 128))
def test_random_fp32_rerank_schedule_of_chunks_and_steps(binding, oracle, seed):
    """fp32 storage with positions re-assigned to cache ranks: chunks and decode steps mixed, held to 1e-5."""
    rng, c = _draw(seed)
    max_chunk = int(rng.choice([16, 64, 200]))
    sched, total = _random_schedule(rng, c["budget"], max_chunk)
    Q, K, V = inputs.batch_streams("iid", seed, total, c["B"], c["Hkv"], c["G"], c["d"], dtype="f32")
    kv = binding.TreeKV(c["budget"], c["Hkv"] * c["G"], c["d"], kv_heads=c["Hkv"], batch=c["B"], dtype="f32",
                        n_sink=c["n_sink"], n_recent=c["n_recent"], max_chunk=max_chunk, kv_splits=c["splits"],
                        flags=binding.TREEKV_POSITION_RERANK, rope_base=float(rng.choice([0.0, 50.0, 500000.0])))
    st = ph.run_schedule(oracle, kv, Q, K, V, sched, dtype="f32")
    ph.compare_scores(kv, st["results"], "f32")
    assert st["flagged"] <= max(2, st["decisions"] // 200), (c, st["flagged"])

