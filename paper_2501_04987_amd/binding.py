"""ctypes binding of the TreeKV C ABI (see include/treekv.h), same names, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if `libtreekv.so` has not been
built, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtreekv.so")

TREEKV_OK = 0
TREEKV_EINVAL = -1
TREEKV_ENOWS = -2
TREEKV_EHIP = -3
TREEKV_EUNSUPPORTED = -4
TREEKV_ESCRATCH = -5
TREEKV_BF16 = 0
TREEKV_F32 = 1
TREEKV_KEEP_LEFT = 1
TREEKV_SCORE_ACCUMULATED = 4
TREEKV_POSITION_RERANK = 8
TREEKV_DEFAULT_LAYOUT = -1

EXPORTS = [
    "treekv_init", "treekv_init_ex", "treekv_destroy", "treekv_get_config", "treekv_workspace_bytes",
    "treekv_bind_workspace", "treekv_reset", "treekv_decode_step", "treekv_decode_step_static", "treekv_prefill_chunk", "treekv_prefill_prompt",
    "treekv_scores", "treekv_state_bytes", "treekv_get_state_layout", "treekv_export_state", "treekv_import_state",
    "treekv_gather_kv", "treekv_wavelet_components", "treekv_strerror", "treekv_last_hip_error",
]
PROBE_EXPORTS = ["treekv_probe_read", "treekv_probe_copy", "treekv_probe_mfma"]       # include/treekv_probe.h


class treekv_config(C.Structure):
    _fields_ = [
        ("budget", C.c_int32), ("q_heads", C.c_int32), ("kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("batch", C.c_int32), ("dtype", C.c_int32), ("n_sink", C.c_int32), ("n_recent", C.c_int32),
        ("softmax_scale", C.c_float), ("flags", C.c_int32), ("max_chunk", C.c_int32), ("kv_splits", C.c_int32),
        ("max_prompt", C.c_int32), ("rope_base", C.c_float),
    ]


class treekv_state_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("header", "positions", "slots", "S", "K", "V", "bytes")]


_lib = None


def load() -> C.CDLL:
    """Load the built HIP library; raise if it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2501_04987_amd.build` "
                           "(or __graft_entry__.build()) first")
    import torch  # noqa: F401  (first, so that this process has one HIP runtime: the one torch brings)

    lib = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.c_void_p
    lib.treekv_init.argtypes = [C.POINTER(vp), C.c_int, C.c_int, C.c_int]
    lib.treekv_init_ex.argtypes = [C.POINTER(vp), C.POINTER(treekv_config)]
    lib.treekv_destroy.argtypes = [vp]
    lib.treekv_destroy.restype = None
    lib.treekv_get_config.argtypes = [vp, C.POINTER(treekv_config)]
    lib.treekv_workspace_bytes.argtypes = [vp]
    lib.treekv_workspace_bytes.restype = C.c_size_t
    lib.treekv_bind_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.treekv_reset.argtypes = [vp, vp]
    lib.treekv_decode_step.argtypes = [vp, vp, vp, vp, vp, i32p, i32p, i32p, vp]
    lib.treekv_decode_step_static.argtypes = [vp, vp, vp, vp, vp, i32p, i32p, i32p, vp]
    lib.treekv_prefill_chunk.argtypes = [vp, vp, vp, vp, C.c_int, vp, i32p, i32p, i32p, vp]
    lib.treekv_prefill_prompt.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, i32p, i32p, i32p, vp, vp]
    lib.treekv_scores.argtypes = [vp, vp, vp]
    lib.treekv_gather_kv.argtypes = [vp, vp, vp, vp]
    lib.treekv_state_bytes.argtypes = [vp]
    lib.treekv_state_bytes.restype = C.c_size_t
    lib.treekv_get_state_layout.argtypes = [vp, C.POINTER(treekv_state_layout)]
    lib.treekv_export_state.argtypes = [vp, vp, C.c_size_t, vp]
    lib.treekv_import_state.argtypes = [vp, vp, C.c_size_t, i32p, vp]
    lib.treekv_wavelet_components.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp]
    lib.treekv_probe_read.argtypes = [vp, C.c_size_t, C.c_int, C.c_int, vp, vp]
    lib.treekv_probe_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.treekv_probe_mfma.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), vp]
    lib.treekv_strerror.argtypes = [C.c_int]
    lib.treekv_strerror.restype = C.c_char_p
    lib.treekv_last_hip_error.argtypes = [vp]
    lib.treekv_last_hip_error.restype = C.c_char_p
    _lib = lib
    return lib


class TreeKVError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str = ""):
        self.status = status
        msg = f"{what}: {load().treekv_strerror(status).decode()} ({status})"
        super().__init__(msg + (f": {detail}" if detail else ""))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def wavelet_components(a, V, levels: int, per_head=None, mean=None):
    """treekv_wavelet_components on torch tensors: a [heads, t] float32, V [heads, t, d] bf16 or float32 ->
    (per_head [heads, levels, t], mean [levels, t]), float32, on V's device and the current stream."""
    import torch

    lib = load()
    heads, t, d = V.shape
    dtype = {torch.bfloat16: TREEKV_BF16, torch.float32: TREEKV_F32}[V.dtype]
    if per_head is None:
        per_head = torch.empty(heads, levels, t, dtype=torch.float32, device=V.device)
    if mean is None:
        mean = torch.empty(levels, t, dtype=torch.float32, device=V.device)
    assert a.dtype == torch.float32 and a.shape == (heads, t) and a.is_contiguous() and V.is_contiguous()
    rc = lib.treekv_wavelet_components(_ptr(a), _ptr(V), dtype, heads, t, d, int(levels), _ptr(per_head), _ptr(mean),
                                       C.c_void_p(torch.cuda.current_stream(V.device).cuda_stream))
    if rc != TREEKV_OK:
        raise TreeKVError(rc, "treekv_wavelet_components")
    return per_head, mean


class TreeKV:
    """One attention layer's TreeKV state on the GPU.  Thin wrapper: one method per ABI call."""

    def __init__(self, budget: int, heads: int, head_dim: int, *, kv_heads: int | None = None, batch: int = 1,
                 dtype: str = "bf16", n_sink: int | None = None, n_recent: int | None = None,
                 softmax_scale: float = 0.0, flags: int = 0, max_chunk: int = 0, kv_splits: int = 0,
                 max_prompt: int = 0, rope_base: float = 0.0, device="cuda", workspace=None):
        import torch

        self._torch = torch
        self._lib = load()
        self._h = C.c_void_p()
        self.device = torch.device(device)
        if kv_heads is None and batch == 1 and dtype == "bf16" and n_sink is None and n_recent is None \
                and softmax_scale == 0.0 and flags == 0 and max_chunk == 0 and kv_splits == 0 and max_prompt == 0 \
                and rope_base == 0.0:
            rc = self._lib.treekv_init(C.byref(self._h), budget, heads, head_dim)
        else:
            if n_sink is None and n_recent is None:      # the library's default layout, as treekv_init takes it
                n_sink = n_recent = TREEKV_DEFAULT_LAYOUT
            cfg = treekv_config(budget, heads, kv_heads or heads, head_dim, batch,
                                {"bf16": TREEKV_BF16, "f32": TREEKV_F32}[dtype], n_sink or 0, n_recent or 0,
                                softmax_scale, flags, max_chunk, kv_splits, max_prompt, rope_base)
            rc = self._lib.treekv_init_ex(C.byref(self._h), C.byref(cfg))
        if rc != TREEKV_OK:
            self._h = C.c_void_p()
            raise TreeKVError(rc, "treekv_init")
        self.cfg = treekv_config()
        self._lib.treekv_get_config(self._h, C.byref(self.cfg))
        self.storage_dtype = torch.bfloat16 if self.cfg.dtype == TREEKV_BF16 else torch.float32
        nbytes = self._lib.treekv_workspace_bytes(self._h)
        if workspace is None:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.workspace = workspace
        self._check(self._lib.treekv_bind_workspace(self._h, _ptr(workspace), workspace.numel()), "treekv_bind_workspace")
        self.reset()

    # -- plumbing ----------------------------------------------------------------
    def _check(self, rc: int, what: str):
        if rc != TREEKV_OK:
            raise TreeKVError(rc, what, self._lib.treekv_last_hip_error(self._h).decode() if self._h else "")

    def _stream(self):
        return C.c_void_p(self._torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.treekv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def units(self):
        return self.cfg.batch * self.cfg.kv_heads

    def new_outputs(self, length: int | None = None):
        """Allocate (out, retained, n_retained, evicted) for a decode step (length None) or a chunk."""
        t, c = self._torch, self.cfg
        if length is None:
            out = t.empty(c.batch, c.q_heads, c.head_dim, dtype=t.float32, device=self.device)
            ev = t.empty(c.batch, c.kv_heads, dtype=t.int32, device=self.device)
        else:
            out = t.empty(c.batch, length, c.q_heads, c.head_dim, dtype=t.float32, device=self.device)
            ev = t.empty(c.batch, c.kv_heads, length, dtype=t.int32, device=self.device)
        ret = t.empty(c.batch, c.kv_heads, c.budget, dtype=t.int32, device=self.device)
        nret = t.empty(c.batch, c.kv_heads, dtype=t.int32, device=self.device)
        return out, ret, nret, ev

    # -- the ABI calls -------------------------------------------------------------
    def reset(self):
        self._check(self._lib.treekv_reset(self._h, self._stream()), "treekv_reset")

    def decode_step(self, q, k, v, out, retained, n_retained=None, evicted=None):
        self._check(self._lib.treekv_decode_step(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(retained),
                                                 _ptr(n_retained), _ptr(evicted), self._stream()),
                    "treekv_decode_step")

    def decode_step_static(self, q, k, v, out, retained, n_retained=None, evicted=None):
        self._check(self._lib.treekv_decode_step_static(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(retained),
                                                        _ptr(n_retained), _ptr(evicted), self._stream()),
                    "treekv_decode_step_static")

    def prefill_chunk(self, Q, K, V, length, out, retained, n_retained=None, evicted=None):
        self._check(self._lib.treekv_prefill_chunk(self._h, _ptr(Q), _ptr(K), _ptr(V), int(length), _ptr(out),
                                                   _ptr(retained), _ptr(n_retained), _ptr(evicted), self._stream()),
                    "treekv_prefill_chunk")

    def prefill_prompt(self, Qw, K, V, length, block, retained, n_retained=None, evicted_blocks=None,
                       token_scores=None):
        self._check(self._lib.treekv_prefill_prompt(self._h, _ptr(Qw), _ptr(K), _ptr(V), int(length), int(block),
                                                    _ptr(retained), _ptr(n_retained), _ptr(evicted_blocks),
                                                    _ptr(token_scores), self._stream()),
                    "treekv_prefill_prompt")

    def scores(self, scores=None):
        c = self.cfg
        if scores is None:
            scores = self._torch.empty(c.batch, c.kv_heads, c.budget, dtype=self._torch.float32, device=self.device)
        self._check(self._lib.treekv_scores(self._h, _ptr(scores), self._stream()), "treekv_scores")
        return scores

    def state_layout(self) -> treekv_state_layout:
        lay = treekv_state_layout()
        self._check(self._lib.treekv_get_state_layout(self._h, C.byref(lay)), "treekv_get_state_layout")
        return lay

    def export_state(self, dst=None):
        """Snapshot of the context into `dst` (uint8 device tensor of treekv_state_bytes; allocated if None)."""
        if dst is None:
            dst = self._torch.zeros(self._lib.treekv_state_bytes(self._h), dtype=self._torch.uint8, device=self.device)
        self._check(self._lib.treekv_export_state(self._h, _ptr(dst), dst.numel(), self._stream()), "treekv_export_state")
        return dst

    def import_state(self, src, status=None):
        self._check(self._lib.treekv_import_state(self._h, _ptr(src), src.numel(), _ptr(status), self._stream()),
                    "treekv_import_state")

    def gather_kv(self, K_out=None, V_out=None):
        c = self.cfg
        shape = (c.batch, c.kv_heads, c.budget, c.head_dim)
        if K_out is None:
            K_out = self._torch.empty(shape, dtype=self.storage_dtype, device=self.device)
        if V_out is None:
            V_out = self._torch.empty(shape, dtype=self.storage_dtype, device=self.device)
        self._check(self._lib.treekv_gather_kv(self._h, _ptr(K_out), _ptr(V_out), self._stream()), "treekv_gather_kv")
        return K_out, V_out
