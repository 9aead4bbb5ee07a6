"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared
symbol, validates configurations and sizes the workspace."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2501_04987_amd import binding as b
    from paper_2501_04987_amd import build

    if not os.path.exists(b.LIB_PATH):
        build.build()
    b.load()
    return b


def _declared(header="treekv.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(treekv_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(binding):
    lib = binding.load()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/treekv.h but not exported"
    assert sorted(binding.EXPORTS) == names
    probes = _declared("treekv_probe.h")
    assert sorted(binding.PROBE_EXPORTS) == probes and all(hasattr(lib, n) for n in probes)
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["treekv.h", "treekv_probe.h"]


def _init(binding, **kw):
    base = dict(budget=64, q_heads=4, kv_heads=4, head_dim=128, batch=1, dtype=binding.TREEKV_BF16, n_sink=0,
                n_recent=0, softmax_scale=0.0, flags=0, max_chunk=0, kv_splits=0)
    base.update(kw)
    cfg = binding.treekv_config(**base)
    h = C.c_void_p()
    rc = binding.load().treekv_init_ex(C.byref(h), C.byref(cfg))
    return rc, h


def test_config_validation(binding):
    lib = binding.load()
    bad = [dict(budget=0), dict(q_heads=6, kv_heads=4), dict(n_sink=40, n_recent=24), dict(dtype=7),
           dict(flags=16), dict(n_sink=-1), dict(softmax_scale=float("nan")), dict(kv_splits=100)]
    for kw in bad:
        rc, h = _init(binding, **kw)
        assert rc == binding.TREEKV_EINVAL and not h.value, kw
    for kw in [dict(head_dim=96), dict(q_heads=12, kv_heads=4), dict(max_chunk=100000)]:
        rc, h = _init(binding, **kw)
        assert rc == binding.TREEKV_EUNSUPPORTED, kw
    h = C.c_void_p()
    assert lib.treekv_init(C.byref(h), 8, 4, 128) == binding.TREEKV_EINVAL     # default layout needs budget >= 16
    assert lib.treekv_init(None, 64, 4, 128) == binding.TREEKV_EINVAL
    assert lib.treekv_strerror(binding.TREEKV_ENOWS).decode().startswith("workspace")


def test_defaults_and_workspace_size(binding):
    lib = binding.load()
    h = C.c_void_p()
    assert lib.treekv_init(C.byref(h), 2048, 32, 128) == 0
    cfg = binding.treekv_config()
    assert lib.treekv_get_config(h, C.byref(cfg)) == 0
    assert (cfg.n_sink, cfg.n_recent, cfg.batch, cfg.kv_heads, cfg.max_chunk) == (4, 1020, 1, 32, 512)
    assert abs(cfg.softmax_scale - 128 ** -0.5) < 1e-7 and cfg.kv_splits >= 1
    nbytes = lib.treekv_workspace_bytes(h)
    kv_bytes = 2 * 32 * 2049 * 128 * 2
    assert kv_bytes < nbytes < kv_bytes * 1.25       # the cache rows dominate the workspace
    # unbound context: every call that needs the workspace refuses, nothing is launched
    assert lib.treekv_reset(h, None) == binding.TREEKV_ENOWS
    assert lib.treekv_bind_workspace(h, None, nbytes) == binding.TREEKV_EINVAL
    assert lib.treekv_bind_workspace(h, C.c_void_p(0x1001), nbytes) == binding.TREEKV_ENOWS
    assert lib.treekv_bind_workspace(h, C.c_void_p(0x1000), nbytes - 1) == binding.TREEKV_ENOWS
    one = C.c_void_p(0x1000)
    assert lib.treekv_decode_step(h, one, one, one, one, one, None, None, None) == binding.TREEKV_ENOWS
    assert lib.treekv_decode_step(h, None, one, one, one, one, None, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_decode_step(h, C.c_void_p(0x1004), one, one, one, one, None, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_prefill_chunk(h, one, one, one, 0, one, one, None, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_prefill_chunk(h, one, one, one, 513, one, one, None, None, None) == binding.TREEKV_EINVAL
    lib.treekv_destroy(h)
    assert lib.treekv_workspace_bytes(None) == 0


def test_missing_library_is_loud(binding, monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libtreekv.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_splits_follow_lds_capacity(binding):
    """A configuration whose per-unit logits do not fit one workgroup's LDS is split over more workgroups at init."""
    rc, h = _init(binding, budget=16384, q_heads=32, kv_heads=8, head_dim=128, batch=64, kv_splits=0)
    assert rc == 0
    cfg = binding.treekv_config()
    binding.load().treekv_get_config(h, C.byref(cfg))
    assert cfg.kv_splits >= 2          # 512 units would run fused, but 4 x 16385 logits are 262 KB
    binding.load().treekv_destroy(h)
    rc, h = _init(binding, budget=2048, q_heads=32, kv_heads=32, head_dim=128, batch=8)
    binding.load().treekv_get_config(h, C.byref(cfg))
    assert rc == 0 and cfg.kv_splits == 1
    binding.load().treekv_destroy(h)


def test_prompt_compression_host_checks(binding):
    """treekv_prefill_prompt refuses what does not fit before anything is enqueued, and its scratch is part of the
    workspace only when max_prompt asks for it."""
    lib = binding.load()
    rc, h0 = _init(binding, budget=256, n_sink=4, n_recent=60)
    rc1, h1 = _init(binding, budget=256, n_sink=4, n_recent=60, max_prompt=4096)
    assert rc == 0 and rc1 == 0
    extra = lib.treekv_workspace_bytes(h1) - lib.treekv_workspace_bytes(h0)
    assert 2 * 4 * 4096 * 4 <= extra <= 2 * 4 * 4096 * 4 + 4 * (64 * 128 * 2 * 4 + 256 * 4) + 4096
    one = C.c_void_p(0x1000)
    call = lambda h, T, b: lib.treekv_prefill_prompt(h, one, one, one, T, b, one, None, None, None, None)
    assert call(h0, 1024, 32) == binding.TREEKV_EINVAL            # max_prompt = 0: the call is not available
    for T, b in [(1000, 32), (8192, 32), (1024, 48), (1024, 0), (16, 32), (1024, 128)]:
        assert call(h1, T, b) == binding.TREEKV_EINVAL, (T, b)    # (the last: 2 blocks, 1 sink, 1 recent, no tree block)
    assert lib.treekv_prefill_prompt(h1, None, one, one, 1024, 32, one, None, None, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_prefill_prompt(h1, C.c_void_p(0x1008), one, one, 1024, 32, one, None, None, None, None) == binding.TREEKV_EINVAL
    assert call(h1, 1024, 32) == binding.TREEKV_ENOWS             # valid arguments, but no workspace bound
    for bad_flags in (2, 16, 32):
        assert _init(binding, flags=bad_flags)[0] == binding.TREEKV_EINVAL
    rc, h2 = _init(binding, flags=binding.TREEKV_KEEP_LEFT | binding.TREEKV_SCORE_ACCUMULATED)
    assert rc == 0
    for h in (h0, h1, h2):
        lib.treekv_destroy(h)


def test_position_rerank_host_checks(binding):
    """TREEKV_POSITION_RERANK: the rotary table (one row per distance in the cache or prompt position) and the turned
    window queries are part of the workspace, as are the turned keys and queries of a prefill chunk (two bf16 parts of
    every cache row and chunk token), and the base defaults to 10000."""
    lib = binding.load()
    rc0, h0 = _init(binding, budget=256, n_sink=4, n_recent=60, max_prompt=1024)
    rc1, h1 = _init(binding, budget=256, n_sink=4, n_recent=60, max_prompt=1024, flags=binding.TREEKV_POSITION_RERANK)
    assert rc0 == 0 and rc1 == 0
    extra = lib.treekv_workspace_bytes(h1) - lib.treekv_workspace_bytes(h0)
    assert extra >= 1024 * 64 * 8 + 4 * 2 * 128 * 128 * 2   # (cos, sin) per prompt position and plane; queries hi + lo
    assert extra >= 4 * 2 * (257 + 512) * 128 * 2 + 2 * 512 * 4 * 128 * 2      # a chunk's turned keys and queries
    cfg = binding.treekv_config()
    lib.treekv_get_config(h1, C.byref(cfg))
    assert cfg.rope_base == 10000.0 and cfg.flags == binding.TREEKV_POSITION_RERANK
    one = C.c_void_p(0x1000)
    assert lib.treekv_prefill_prompt(h1, one, one, one, 1024, 32, one, None, None, None, None) == binding.TREEKV_ENOWS
    assert lib.treekv_prefill_chunk(h1, one, one, one, 16, one, one, None, None, None) == binding.TREEKV_ENOWS
    assert _init(binding, flags=binding.TREEKV_POSITION_RERANK, rope_base=-1.0)[0] == binding.TREEKV_EINVAL
    assert _init(binding, flags=binding.TREEKV_POSITION_RERANK, rope_base=float("nan"))[0] == binding.TREEKV_EINVAL
    for h in (h0, h1):
        lib.treekv_destroy(h)


def test_wavelet_host_checks(binding):
    lib = binding.load()
    one = C.c_void_p(0x1000)
    call = lambda a, V, dtype, heads, t, d, levels, out: lib.treekv_wavelet_components(a, V, dtype, heads, t, d, levels,
                                                                                      out, None, None)
    assert call(None, one, 0, 1, 64, 128, 5, one) == binding.TREEKV_EINVAL
    assert call(one, one, 0, 1, 64, 128, 5, None) == binding.TREEKV_EINVAL
    assert call(one, one, 5, 1, 64, 128, 5, one) == binding.TREEKV_EINVAL       # unknown storage type
    assert call(one, one, 0, 0, 64, 128, 5, one) == binding.TREEKV_EINVAL
    assert call(one, one, 0, 1, 48, 128, 5, one) == binding.TREEKV_EINVAL       # 32 does not divide 48
    assert call(one, one, 0, 1, 64, 128, 0, one) == binding.TREEKV_EINVAL
    assert call(one, C.c_void_p(0x1004), 0, 1, 64, 128, 5, one) == binding.TREEKV_EINVAL
    assert call(one, one, 0, 1, 64, 128, 6, one) == binding.TREEKV_EUNSUPPORTED
    assert call(one, one, 0, 1, 64, 96, 5, one) == binding.TREEKV_EUNSUPPORTED
    assert call(one, one, 0, 70000, 64, 128, 5, one) == binding.TREEKV_EUNSUPPORTED


def test_default_layout_through_the_config(binding):
    """n_sink = n_recent = TREEKV_DEFAULT_LAYOUT selects the layout treekv_init chooses; one of them alone is an error."""
    lib = binding.load()
    d = binding.TREEKV_DEFAULT_LAYOUT
    rc, h = _init(binding, budget=1024, n_sink=d, n_recent=d, batch=3)
    assert rc == 0
    cfg = binding.treekv_config()
    lib.treekv_get_config(h, C.byref(cfg))
    assert (cfg.n_sink, cfg.budget - cfg.n_sink - cfg.n_recent, cfg.n_recent, cfg.batch) == (4, 512, 508, 3)
    lib.treekv_destroy(h)
    assert _init(binding, budget=8, n_sink=d, n_recent=d)[0] == binding.TREEKV_EINVAL
    assert _init(binding, budget=64, n_sink=d, n_recent=3)[0] == binding.TREEKV_EINVAL


def test_snapshot_sizes_and_argument_checks(binding):
    """The snapshot's arrays are laid out back to back on 256-byte boundaries; bad arguments are refused before
    anything is enqueued (so these calls need no GPU)."""
    lib = binding.load()
    rc, h = _init(binding, budget=100, q_heads=8, kv_heads=2, batch=3, n_sink=1, n_recent=9)
    assert rc == 0
    lay = binding.treekv_state_layout()
    assert lib.treekv_get_state_layout(h, C.byref(lay)) == 0
    U, c, d = 6, 100, 128
    up = lambda x: (x + 255) // 256 * 256
    want = [0]
    for b in (U * 16, U * c * 4, U * c * 4, U * c * 4, U * c * d * 2, U * c * d * 2):
        want.append(want[-1] + up(b))
    assert [lay.header, lay.positions, lay.slots, lay.S, lay.K, lay.V, lay.bytes] == want
    assert lib.treekv_state_bytes(h) == lay.bytes and lib.treekv_state_bytes(None) == 0
    buf = C.c_void_p(0x10000)
    assert lib.treekv_export_state(h, None, lay.bytes, None) == binding.TREEKV_EINVAL
    assert lib.treekv_export_state(h, buf, lay.bytes - 1, None) == binding.TREEKV_EINVAL
    assert lib.treekv_export_state(h, C.c_void_p(0x10010), lay.bytes, None) == binding.TREEKV_EINVAL
    assert lib.treekv_import_state(h, None, lay.bytes, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_import_state(h, buf, 5, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_export_state(h, buf, lay.bytes, None) == binding.TREEKV_ENOWS        # no workspace bound
    assert lib.treekv_import_state(h, buf, lay.bytes, None, None) == binding.TREEKV_ENOWS
    assert lib.treekv_get_state_layout(None, C.byref(lay)) == binding.TREEKV_EINVAL
    lib.treekv_destroy(h)


def test_probe_argument_checks(binding):
    lib = binding.load()
    buf = C.c_void_p(0x100000)
    assert lib.treekv_probe_read(buf, (1 << 20) + 16, 1024, 4, buf, None) == binding.TREEKV_EINVAL      # not whole MiB
    assert lib.treekv_probe_read(None, 1 << 20, 1024, 4, buf, None) == binding.TREEKV_EINVAL
    assert lib.treekv_probe_read(buf, 1 << 20, 48, 4, buf, None) == binding.TREEKV_EINVAL               # not a power of two
    assert lib.treekv_probe_read(buf, 1 << 20, 1024, 3, buf, None) == binding.TREEKV_EINVAL
    assert lib.treekv_probe_copy(buf, C.c_void_p(0x100008), 1 << 20, None) == binding.TREEKV_EINVAL
    assert lib.treekv_probe_mfma(buf, 256, 3, 10, None, None) == binding.TREEKV_EINVAL
    assert lib.treekv_probe_mfma(None, 256, 1, 10, None, None) == binding.TREEKV_EINVAL
