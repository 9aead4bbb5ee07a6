"""Seeded synthetic q/k/v streams for the TreeKV hot path.

This module is shared by the GPU path's tests, the CPU oracle's tests and the
benchmark.  It holds no attention, softmax, score or eviction arithmetic: it
only draws random numbers, mixes in a low-rank component, and rounds to the
storage type.  Every stream is keyed by (seed, layer, batch, kv_head) so that a
subset of streams can be regenerated on the CPU without generating the rest.

The paper evaluates on language-model activations (Llama-2-7B on PG19 and
OpenWebText2, Llama-3.2-1B-Instruct on LongBench; Section 5.1).  Those weights
and corpora are not available here, so Gaussian streams of the same shapes
stand in for them; the low-rank component makes attention concentrate on a few
slots, as it does in a trained model.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits", "bf16_to_f32", "round_to_storage", "unit_rng",
    "stream_iid", "stream_lowrank", "batch_streams", "device_lowrank", "redrawn_queries",
]


# --------------------------------------------------------------------------- #
# storage-type helpers
# --------------------------------------------------------------------------- #
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Return float32 values exactly representable in `dtype` ("bf16" or "f32")."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(x))
    raise ValueError(f"unknown storage dtype {dtype!r}")


# --------------------------------------------------------------------------- #
# CPU generators (numpy, counter-based Philox keyed per stream)
# --------------------------------------------------------------------------- #
def unit_rng(seed: int, layer: int, batch: int, kv_head: int, sub: int = 0) -> np.random.Generator:
    key = np.array([np.uint64(seed) & np.uint64(0xFFFFFFFFFFFFFFFF),
                    (np.uint64(layer) << np.uint64(48)) | (np.uint64(batch) << np.uint64(32))
                    | (np.uint64(kv_head) << np.uint64(16)) | np.uint64(sub)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def stream_iid(seed: int, T: int, G: int, d: int, *, layer: int = 0, batch: int = 0,
               kv_head: int = 0, k_scale: float = 1.0, dtype: str = "f32"):
    """iid N(0,1) q, k, v for one (layer, batch, kv_head) stream.

    Returns q [T, G, d], k [T, d], v [T, d] as float32 holding values that are
    exact in `dtype`.  `k_scale` multiplies K before rounding (the tiny decode
    configuration folds 1/sqrt(d) into K).
    """
    rng = unit_rng(seed, layer, batch, kv_head)
    q = rng.standard_normal((T, G, d), dtype=np.float32)
    k = rng.standard_normal((T, d), dtype=np.float32) * np.float32(k_scale)
    v = rng.standard_normal((T, d), dtype=np.float32)
    return round_to_storage(q, dtype), round_to_storage(k, dtype), round_to_storage(v, dtype)


def _lowrank_basis(layer: int, kv_head: int, d: int, rank: int):
    basis = unit_rng(0x5EED, layer, 0, kv_head, sub=1)  # the basis depends on (layer, kv_head) only
    U = basis.standard_normal((d, rank), dtype=np.float32) / np.float32(np.sqrt(d))
    Uv = basis.standard_normal((d, rank), dtype=np.float32) / np.float32(np.sqrt(d))
    return U, Uv


def redrawn_queries(kind: str, seed: int, t: int, n: int, attempt: int, G: int, d: int, *, layer: int = 0,
                    batch: int = 0, kv_head: int = 0, rank: int = 8, beta: float = 4.0, dtype: str = "bf16"):
    """Fresh queries for tokens t .. t+n-1 of one stream: the same distribution as `stream_iid` / `stream_lowrank`
    draw q from, from a generator keyed by (stream, t, attempt) with attempt >= 1.  Returns [n, G, d] float32.

    A parity run may not want decisions whose score margin is below what two precisions can resolve; whoever
    builds its inputs (with whatever reference it has) replaces the queries of such a step or chunk by these.
    """
    assert attempt >= 1
    key = np.array([(np.uint64(seed) ^ np.uint64(0x7E57ED0000000000)) + np.uint64(attempt),
                    (np.uint64(layer) << np.uint64(48)) | (np.uint64(batch) << np.uint64(32))
                    | (np.uint64(kv_head) << np.uint64(16)) | np.uint64(2)], dtype=np.uint64)
    rng = np.random.Generator(np.random.Philox(key=key, counter=np.array([0, 0, 0, t], dtype=np.uint64)))
    q = rng.standard_normal((n, G, d), dtype=np.float32)
    if kind == "lowrank":
        U, _ = _lowrank_basis(layer, kv_head, d, rank)
        q = q + np.float32(beta) * (rng.standard_normal((n, G, rank), dtype=np.float32) @ U.T)
    elif kind != "iid":
        raise ValueError(kind)
    return round_to_storage(q, dtype)


def stream_lowrank(seed: int, T: int, G: int, d: int, *, layer: int = 0, batch: int = 0,
                   kv_head: int = 0, rank: int = 8, beta: float = 4.0, dtype: str = "bf16"):
    """N(0,1) plus a per-head rank-`rank` component of strength `beta`.

    q = g_q + beta * z_q U^T, k = g_k + beta * z_k U^T, v = g_v + beta * z_v U'^T
    with U, U' in R^{d x rank}, entries N(0,1)/sqrt(d), fixed per (layer,
    kv_head) and shared by the G query heads of the group and by all batch
    elements.  The shared basis makes q.k have a heavy-tailed component, so a
    handful of slots carry most of the softmax mass.
    """
    U, Uv = _lowrank_basis(layer, kv_head, d, rank)
    rng = unit_rng(seed, layer, batch, kv_head)
    q = rng.standard_normal((T, G, d), dtype=np.float32)
    k = rng.standard_normal((T, d), dtype=np.float32)
    v = rng.standard_normal((T, d), dtype=np.float32)
    zq = rng.standard_normal((T, G, rank), dtype=np.float32)
    zk = rng.standard_normal((T, rank), dtype=np.float32)
    zv = rng.standard_normal((T, rank), dtype=np.float32)
    b = np.float32(beta)
    q = q + b * (zq @ U.T)
    k = k + b * (zk @ U.T)
    v = v + b * (zv @ Uv.T)
    return round_to_storage(q, dtype), round_to_storage(k, dtype), round_to_storage(v, dtype)


def batch_streams(kind: str, seed: int, T: int, B: int, Hkv: int, G: int, d: int, *,
                  layer: int = 0, dtype: str = "bf16", seed_per_batch: bool = False, **kw):
    """Stack per-stream generators into step-major arrays.

    Returns Q [T, B, Hkv*G, d], K [T, B, Hkv, d], V [T, B, Hkv, d] float32
    (values exact in `dtype`).  Query head h belongs to KV head h // G.
    With `seed_per_batch` sequence b uses seed `seed + b`.
    """
    gen = {"iid": stream_iid, "lowrank": stream_lowrank}[kind]
    Q = np.empty((T, B, Hkv * G, d), np.float32)
    K = np.empty((T, B, Hkv, d), np.float32)
    V = np.empty((T, B, Hkv, d), np.float32)
    for b in range(B):
        for h in range(Hkv):
            s = seed + b if seed_per_batch else seed
            q, k, v = gen(s, T, G, d, layer=layer, batch=b, kv_head=h, dtype=dtype, **kw)
            Q[:, b, h * G:(h + 1) * G, :] = q
            K[:, b, h, :] = k
            V[:, b, h, :] = v
    return Q, K, V


# --------------------------------------------------------------------------- #
# device generator for workloads too large to pre-generate on the host
# --------------------------------------------------------------------------- #
def device_lowrank(seed: int, T: int, B: int, Hkv: int, G: int, d: int, *, device="cuda",
                   rank: int = 8, beta: float = 4.0, dtype: str = "bf16", slab: int | None = None):
    """Same recipe as `stream_lowrank`, drawn on the device with torch's generator.

    Returns torch tensors Q [T, B, Hkv*G, d], K [T, B, Hkv, d], V [T, B, Hkv, d]
    in the storage dtype.  The random stream differs from the numpy one; tests
    that audit such a run copy the audited streams' inputs back from the device,
    so the device buffers are the single source of truth.  With `slab` the tokens
    are drawn `slab` at a time into preallocated tensors (the float32 intermediates
    of a long stream would otherwise be several times the result's size); the
    values then depend on `slab` too.
    """
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    tdt = {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)

    U = randn(Hkv, d, rank) / (d ** 0.5)
    Uv = randn(Hkv, d, rank) / (d ** 0.5)

    def draw(n):
        q = randn(n, B, Hkv, G, d) + beta * torch.einsum("tbhgr,hdr->tbhgd", randn(n, B, Hkv, G, rank), U)
        k = randn(n, B, Hkv, d) + beta * torch.einsum("tbhr,hdr->tbhd", randn(n, B, Hkv, rank), U)
        v = randn(n, B, Hkv, d) + beta * torch.einsum("tbhr,hdr->tbhd", randn(n, B, Hkv, rank), Uv)
        return q.reshape(n, B, Hkv * G, d).to(tdt), k.to(tdt), v.to(tdt)

    if slab is None:
        q, k, v = draw(T)
        return q.contiguous(), k.contiguous(), v.contiguous()
    Q = torch.empty(T, B, Hkv * G, d, dtype=tdt, device=device)
    K = torch.empty(T, B, Hkv, d, dtype=tdt, device=device)
    V = torch.empty(T, B, Hkv, d, dtype=tdt, device=device)
    for lo in range(0, T, slab):
        n = min(slab, T - lo)
        Q[lo:lo + n], K[lo:lo + n], V[lo:lo + n] = draw(n)
    return Q, K, V
