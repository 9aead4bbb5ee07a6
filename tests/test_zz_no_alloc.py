"""GPU: treekv_decode_step_static (the decode step whose scratch is the library's own fixed device array) against
treekv_decode_step, through the C ABI: same kernels, so outputs, evicted positions and retained lists must be
identical bit for bit -- on calls in a row that share the one array, a large context followed by a smaller one."""
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


def _pair(binding, *, budget, B, Hkv, G, d, splits, seed, T, dtype="bf16"):
    kind = "lowrank" if dtype == "bf16" else "iid"
    Q, K, V = inputs.batch_streams(kind, seed, T, B, Hkv, G, d, dtype=dtype)
    mk = lambda: binding.TreeKV(budget, Hkv * G, d, kv_heads=Hkv, batch=B, dtype=dtype, n_sink=2, n_recent=budget // 3,
                                kv_splits=splits)
    a, b = mk(), mk()
    assert a.cfg.kv_splits == splits
    return dict(ws=a, st=b, dev=[ph.to_device(x, dtype) for x in (Q, K, V)], outs=(a.new_outputs(), b.new_outputs()))


def _step_both(p, t):
    Qd, Kd, Vd = p["dev"]
    (o1, r1, n1, e1), (o2, r2, n2, e2) = p["outs"]
    p["ws"].decode_step(Qd[t], Kd[t], Vd[t], o1, r1, n1, e1)
    p["st"].decode_step_static(Qd[t], Kd[t], Vd[t], o2, r2, n2, e2)


def _same(p, t, what):
    import torch

    (o1, r1, n1, e1), (o2, r2, n2, e2) = p["outs"]
    assert torch.equal(e1, e2) and torch.equal(r1, r2) and torch.equal(n1, n2), (what, t)
    assert torch.equal(o1, o2), (what, t)             # identical kernels and inputs: identical bits


def test_static_scratch_matches_workspace_scratch_on_calls_in_a_row(binding):
    import torch

    T = 400
    big = _pair(binding, budget=300, B=3, Hkv=4, G=4, d=128, splits=3, seed=50, T=T)
    small = _pair(binding, budget=40, B=1, Hkv=2, G=1, d=64, splits=2, seed=51, T=T, dtype="f32")
    fused = _pair(binding, budget=64, B=2, Hkv=2, G=2, d=128, splits=1, seed=52, T=T)       # uses no scratch at all
    for t in range(T):
        _step_both(big, t)          # a call on the large context ...
        _step_both(small, t)        # ... then, in a row, one on the smaller: it finds the large one's words in the array
        _step_both(fused, t)
        torch.cuda.synchronize()
        for p, what in ((big, "large"), (small, "small"), (fused, "one-kernel shape")):
            _same(p, t, what)
    assert int(big["outs"][1][3].min()) >= 0 and int(small["outs"][1][3].min()) >= 0       # both were evicting
    assert torch.equal(big["ws"].scores(), big["st"].scores()) and torch.equal(small["ws"].scores(), small["st"].scores())


def test_static_scratch_refuses_what_does_not_fit(binding):
    """128 units x 8 query heads x 4097 slots of logits exceed the 16 MiB array: refused, nothing enqueued."""
    import torch

    kv = binding.TreeKV(4096, 64, 128, kv_heads=8, batch=16, n_sink=4, n_recent=2044)
    assert kv.cfg.kv_splits > 1
    out, ret, nret, ev = kv.new_outputs()
    q = torch.zeros(16, 64, 128, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(16, 8, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.TreeKVError) as e:
        kv.decode_step_static(q, k, k, out, ret, nret, ev)
    assert e.value.status == binding.TREEKV_ESCRATCH
    kv.decode_step(q, k, k, out, ret, nret, ev)           # the workspace variant still serves it
    torch.cuda.synchronize()
    assert int(nret.min()) == 1
