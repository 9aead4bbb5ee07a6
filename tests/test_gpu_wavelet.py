"""GPU parity: the Haar wavelet analysis of Sections 3.2-3.3 (treekv_wavelet_components) through the C ABI
against the CPU oracle.  The signal is a[n] * v[n] with a the attention of one decode query over the sequence.

Tolerance: both sides start from the same fp32 a and bf16/fp32 V; the GPU forms the products and at most 31 sums
per block in fp32, so a magnitude is off by at most about 32 * 2^-24 * max|a v| before the 2^-l factor: the
tests allow 2e-6 * max|a v| absolute plus 1e-5 relative."""
import numpy as np
import pytest

from paper_2501_04987_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2501_04987_amd import binding as b

    b.load()
    return b


def _signal(seed, heads, t, d, dtype):
    """Attention of the last token's query over the whole sequence, and the values, as the GPU consumes them."""
    Q, K, V = inputs.batch_streams("lowrank" if dtype == "bf16" else "iid", seed, t, 1, heads, 1, d, dtype=dtype)
    lg = np.einsum("hd,thd->ht", Q[t - 1, 0], K[:, 0]) / np.sqrt(d)
    a = np.exp(lg - lg.max(-1, keepdims=True))
    a = np.ascontiguousarray((a / a.sum(-1, keepdims=True)).astype(np.float32))
    return a, np.ascontiguousarray(V[:, 0].transpose(1, 0, 2))        # [heads, t], [heads, t, d]


def _check(binding, oracle, seed, heads, t, d, dtype, levels):
    import torch

    a, V = _signal(seed, heads, t, d, dtype)
    ad = torch.from_numpy(a).cuda()
    Vd = torch.from_numpy(V).to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda()
    per_head, mean = binding.wavelet_components(ad, Vd, levels)
    torch.cuda.synchronize()
    got, got_mean = per_head.cpu().numpy(), mean.cpu().numpy()
    want = np.stack([oracle.wavelet_components(a[h].astype(np.float64), V[h], levels) for h in range(heads)])
    bound = 2e-6 * np.abs(a[:, :, None] * V).max()
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=bound)
    np.testing.assert_allclose(got_mean, want.mean(0), rtol=1e-5, atol=bound)
    return want


@pytest.mark.parametrize("d,dtype", [(128, "bf16"), (64, "bf16"), (128, "f32"), (64, "f32")])
def test_wavelet_paper_setup(binding, oracle, d, dtype):
    """The figure's setting: 5 levels at the 512th generation step; all four lane layouts."""
    want = _check(binding, oracle, 41, 6, 512, d, dtype, 5)
    assert want.max() > 0


@pytest.mark.parametrize("t,levels", [(32, 5), (8, 3), (2, 1), (96, 5), (1000, 3), (4128, 5)])
def test_wavelet_lengths_and_levels(binding, oracle, t, levels):
    """Lengths that end inside a wave's 32 rows and inside a workgroup's 128, fewer levels than five."""
    _check(binding, oracle, 42 + t, 3, t, 128, "bf16", levels)


def test_wavelet_refuses_what_does_not_fit(binding):
    import torch

    a = torch.zeros(2, 48, device="cuda")
    V = torch.zeros(2, 48, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.TreeKVError) as e:
        binding.wavelet_components(a, V, 5)                         # 32 does not divide 48
    assert e.value.status == binding.TREEKV_EINVAL
    V96 = torch.zeros(2, 48, 96, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.TreeKVError) as e:
        binding.wavelet_components(a, V96, 4)
    assert e.value.status == binding.TREEKV_EUNSUPPORTED


def test_wavelet_benchmark_size_sampled(binding, oracle):
    """The size `bench.py` times: 8192 heads x 512 positions x 128, 5 levels.  Eight heads are checked against the
    oracle; the mean over all heads against the per-head output itself (summed in fp64), and it must repeat bit for
    bit."""
    import torch

    heads, t, d, levels = 8192, 512, 128, 5
    g = torch.Generator(device="cuda").manual_seed(9)
    a = torch.softmax(3.0 * torch.randn(heads, t, device="cuda", generator=g), dim=-1).contiguous()
    V = torch.randn(heads, t, d, device="cuda", generator=g).to(torch.bfloat16)
    per_head, mean = binding.wavelet_components(a, V, levels)
    per_head2, mean2 = binding.wavelet_components(a, V, levels)
    torch.cuda.synchronize()
    assert torch.equal(mean, mean2) and torch.equal(per_head, per_head2)
    want_mean = per_head.double().mean(0)
    assert torch.allclose(mean.double(), want_mean, rtol=1e-5, atol=0.0)
    for h in [0, 1, 777, 4095, 4096, 6001, 8190, 8191]:
        ah, Vh = a[h].cpu().numpy(), V[h].float().cpu().numpy().astype(np.float64)
        want = oracle.wavelet_components(ah.astype(np.float64), Vh, levels)
        bound = 2e-6 * float(np.abs(ah[:, None] * Vh).max())
        np.testing.assert_allclose(per_head[h].cpu().numpy(), want, rtol=1e-5, atol=bound)
