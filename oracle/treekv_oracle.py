"""ctypes wrapper around the fp64 CPU oracle (TEST INFRASTRUCTURE, NOT THE PRODUCT).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It builds `treekv_oracle.cpp` with g++ on first use and never touches
the HIP library or the package's binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "treekv_oracle.cpp")
_LIB = os.path.join(_HERE, "libtreekv_oracle.so")
_lock = threading.Lock()
_lib = None

KEEP_LEFT = 1
IDX_LITERAL = 2
SCORE_ACCUMULATED = 4
POSITION_RERANK = 8


def build(force: bool = False) -> str:
    """Compile the oracle (plain g++ -O2, no SIMD intrinsics, no fast-math)."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + f".{os.getpid()}.tmp"
            subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", tmp, _SRC])
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        dp = C.POINTER(C.c_double)
        lp = C.POINTER(C.c_longlong)
        ip = C.POINTER(C.c_int)
        lib.tko_new.restype = C.c_void_p
        lib.tko_new.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int]
        lib.tko_free.argtypes = [C.c_void_p]
        lib.tko_clone.restype = C.c_void_p
        lib.tko_clone.argtypes = [C.c_void_p]
        lib.tko_len.argtypes = [C.c_void_p]
        lib.tko_len.restype = C.c_int
        lib.tko_t.argtypes = [C.c_void_p]
        lib.tko_t.restype = C.c_longlong
        lib.tko_idx.argtypes = [C.c_void_p]
        lib.tko_idx.restype = C.c_int
        lib.tko_state.argtypes = [C.c_void_p, lp, dp, lp]
        lib.tko_kv.argtypes = [C.c_void_p, dp, dp]
        lib.tko_decode_step.argtypes = [C.c_void_p, dp, dp, dp, dp, C.c_longlong, C.c_double, C.c_int, lp, dp]
        lib.tko_decode_stream.argtypes = [C.c_void_p, dp, dp, dp, C.c_int, dp, lp, C.c_double, lp, dp, lp]
        lib.tko_set_rope_base.argtypes = [C.c_void_p, C.c_double]
        lib.tko_prefill_chunk.restype = C.c_int
        lib.tko_prefill_chunk.argtypes = [C.c_void_p, dp, dp, dp, C.c_int, dp, lp, C.c_double, lp, dp, ip, ip]
        lib.tko_prefill_prompt.restype = C.c_int
        lib.tko_prefill_prompt.argtypes = [C.c_void_p, dp, dp, dp, C.c_int, C.c_int, lp, C.c_double, lp, dp, lp, dp, dp]
        lib.tko_wavelet_components.restype = C.c_int
        lib.tko_wavelet_components.argtypes = [dp, dp, C.c_int, C.c_int, C.c_int, dp, dp, dp]
        _lib = lib
    return _lib


def _dptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _lptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_longlong))


def _iptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_int))


class OracleStream:
    """TreeKV state of one (batch, kv-head) stream, fp64 (Algorithm 1 with the layout reading)."""

    def __init__(self, budget: int, G: int, d: int, *, n_sink: int = 0, n_recent: int = 0,
                 scale: float | None = None, flags: int = 0, rope_base: float = 10000.0):
        self._lib = _load()
        self.budget, self.G, self.d = budget, G, d
        self.n_sink, self.n_recent = n_sink, n_recent
        self.scale = float(1.0 / np.sqrt(d)) if scale is None else float(scale)
        self._h = self._lib.tko_new(budget, n_sink, n_recent, G, d, self.scale, flags)
        if not self._h:
            raise ValueError("invalid oracle configuration")
        self.rope_base = float(rope_base)
        self._lib.tko_set_rope_base(self._h, self.rope_base)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._lib.tko_free(h)

    def __len__(self):
        return self._lib.tko_len(self._h)

    def clone(self) -> "OracleStream":
        """An independent copy of the whole state."""
        other = object.__new__(OracleStream)
        other.__dict__.update({k: v for k, v in self.__dict__.items() if k != "_h"})
        other._h = self._lib.tko_clone(self._h)
        return other

    @property
    def t(self) -> int:
        return self._lib.tko_t(self._h)

    @property
    def idx(self) -> int:
        """The paper's 1-based idx."""
        return self._lib.tko_idx(self._h)

    def state(self):
        """(positions, S, C) of the cached tokens, in cache order."""
        n = len(self)
        pos = np.empty(n, np.int64)
        S = np.empty(n, np.float64)
        Cn = np.empty(n, np.int64)
        self._lib.tko_state(self._h, _lptr(pos), _dptr(S), _lptr(Cn))
        return pos, S, Cn

    def retained(self) -> np.ndarray:
        return self.state()[0]

    def kv(self):
        n = len(self)
        K = np.empty((n, self.d), np.float64)
        V = np.empty((n, self.d), np.float64)
        self._lib.tko_kv(self._h, _dptr(K), _dptr(V))
        return K, V

    def decode_step(self, q, k, v, *, forced_pos: int = -1, follow_thresh: float = 0.0,
                    commit: bool = True):
        """Returns (out [G, d], evicted position or -1, margin or -1, adopted, disagreed)."""
        q = np.ascontiguousarray(q, np.float64).reshape(self.G, self.d)
        k = np.ascontiguousarray(k, np.float64).reshape(self.d)
        v = np.ascontiguousarray(v, np.float64).reshape(self.d)
        out = np.empty((self.G, self.d), np.float64)
        res = np.zeros(3, np.int64)
        margin = C.c_double(-1.0)
        self._lib.tko_decode_step(self._h, _dptr(q), _dptr(k), _dptr(v), _dptr(out), int(forced_pos),
                                  float(follow_thresh), int(commit), _lptr(res), C.byref(margin))
        return out, int(res[0]), float(margin.value), int(res[1]), int(res[2])

    def decode_stream(self, q, k, v, *, forced=None, follow_thresh: float = 0.0, keep_outputs: bool = True):
        """T decode steps in a row from the current state: q [T, G, d], k/v [T, d]; forced: optional [T] evicted
        positions of another implementation.  Returns dict(out [T, G, d] or None, evicted [T], margins [T],
        adopted, disagreed)."""
        T = q.shape[0]
        q = np.ascontiguousarray(q, np.float64).reshape(T, self.G, self.d)
        k = np.ascontiguousarray(k, np.float64).reshape(T, self.d)
        v = np.ascontiguousarray(v, np.float64).reshape(T, self.d)
        out = np.empty((T, self.G, self.d), np.float64) if keep_outputs else None
        ev = np.empty(T, np.int64)
        mg = np.empty(T, np.float64)
        counts = np.zeros(2, np.int64)
        fp = None if forced is None else np.ascontiguousarray(forced, np.int64).reshape(T)
        self._lib.tko_decode_stream(self._h, _dptr(q), _dptr(k), _dptr(v), T, _dptr(out) if keep_outputs else None,
                                    _lptr(fp) if fp is not None else None, float(follow_thresh), _lptr(ev),
                                    _dptr(mg), _lptr(counts))
        return dict(out=out, evicted=ev, margins=mg, adopted=int(counts[0]), disagreed=int(counts[1]))

    def prefill_chunk(self, Q, K, V, *, forced_pos=None, follow_thresh: float = 0.0):
        """Q [L, G, d], K [L, d], V [L, d] -> dict(out, evicted, margins, adopted, disagreed)."""
        Q = np.ascontiguousarray(Q, np.float64)
        L = Q.shape[0]
        Q = Q.reshape(L, self.G, self.d)
        K = np.ascontiguousarray(K, np.float64).reshape(L, self.d)
        V = np.ascontiguousarray(V, np.float64).reshape(L, self.d)
        out = np.empty((L, self.G, self.d), np.float64)
        ev = np.empty(L, np.int64)
        mg = np.empty(L, np.float64)
        ad = np.zeros(L, np.int32)
        dis = np.zeros(L, np.int32)
        fp = None
        if forced_pos is not None:
            fp = np.ascontiguousarray(forced_pos, np.int64).reshape(L)
        rc = self._lib.tko_prefill_chunk(self._h, _dptr(Q), _dptr(K), _dptr(V), L, _dptr(out),
                                         _lptr(fp) if fp is not None else None, float(follow_thresh),
                                         _lptr(ev), _dptr(mg), _iptr(ad), _iptr(dis))
        if rc != 0:
            raise ValueError("prefill_chunk failed")
        return dict(out=out, evicted=ev, margins=mg, adopted=ad, disagreed=dis)

    def prefill_prompt(self, Qw, K, V, block: int, *, forced_blocks=None, follow_thresh: float = 0.0):
        """One-shot block-level compression of a whole prompt (Section 4.2); the stream must be empty.

        Qw [block, G, d] (queries of the last block), K/V [T, d] -> dict(evicted_blocks [T/block],
        margins, adopted, disagreed, token_scores [T], block_scores [T/block]).
        """
        K = np.ascontiguousarray(K, np.float64)
        T = K.shape[0]
        K = K.reshape(T, self.d)
        V = np.ascontiguousarray(V, np.float64).reshape(T, self.d)
        Qw = np.ascontiguousarray(Qw, np.float64).reshape(block, self.G, self.d)
        N = T // block if block > 0 else 0
        ev = np.full(max(N, 1), -1, np.int64)
        mg = np.full(max(N, 1), -1.0, np.float64)
        counts = np.zeros(2, np.int64)
        tok = np.empty(T, np.float64)
        blk = np.empty(max(N, 1), np.float64)
        fb = None if forced_blocks is None else np.ascontiguousarray(forced_blocks, np.int64).reshape(N)
        rc = self._lib.tko_prefill_prompt(self._h, _dptr(Qw), _dptr(K), _dptr(V), T, int(block),
                                          _lptr(fb) if fb is not None else None, float(follow_thresh),
                                          _lptr(ev), _dptr(mg), _lptr(counts), _dptr(tok), _dptr(blk))
        if rc != 0:
            raise ValueError("prefill_prompt: arguments do not fit this stream")
        return dict(evicted_blocks=ev[:N], margins=mg[:N], adopted=int(counts[0]), disagreed=int(counts[1]),
                    token_scores=tok, block_scores=blk[:N])


def run_decode_stream(cfg: dict, q, k, v, *, forced=None, follow_thresh: float = 0.0,
                      keep_outputs: bool = True):
    """Run a whole decode stream through one OracleStream.

    cfg: dict(budget, G, d, n_sink, n_recent, scale, flags); q [T, G, d], k/v [T, d].
    forced: optional [T] evicted positions of another implementation.
    Returns dict(out [T, G, d] or None, evicted [T], margins [T], adopted, disagreed, stream).
    """
    s = OracleStream(cfg["budget"], cfg["G"], cfg["d"], n_sink=cfg.get("n_sink", 0),
                     n_recent=cfg.get("n_recent", 0), scale=cfg.get("scale"), flags=cfg.get("flags", 0),
                     rope_base=cfg.get("rope_base", 10000.0))
    res = s.decode_stream(q, k, v, forced=forced, follow_thresh=follow_thresh, keep_outputs=keep_outputs)
    res["stream"] = s
    return res


def wavelet_components(a, V, levels: int, *, want_coeffs: bool = False):
    """Sections 3.2-3.3 for one head at one step: a [t], V [t, d] -> magnitude [levels, t] of Rec(D_l), averaged
    over the d columns; with want_coeffs also (coeffs [d, t] = [A_L, D_L, .., D_1] per column, rec_sum [d, t])."""
    a = np.ascontiguousarray(a, np.float64)
    V = np.ascontiguousarray(V, np.float64)
    t, d = V.shape
    mag = np.empty((levels, t), np.float64)
    co = np.empty((d, t), np.float64) if want_coeffs else None
    rs = np.empty((d, t), np.float64) if want_coeffs else None
    rc = _load().tko_wavelet_components(_dptr(a.reshape(t)), _dptr(V), t, d, int(levels), _dptr(mag),
                                        _dptr(co) if want_coeffs else None, _dptr(rs) if want_coeffs else None)
    if rc != 0:
        raise ValueError("wavelet_components: the length must be a multiple of 2**levels")
    return (mag, co, rs) if want_coeffs else mag


def run_many(fn, jobs, workers: int | None = None):
    """Run `fn(job)` for every job on a thread pool (the C calls release the GIL)."""
    workers = workers or min(len(jobs), os.cpu_count() or 1)
    if workers <= 1:
        return [fn(j) for j in jobs]
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(fn, jobs))
