"""Seeded synthetic inputs for the five benchmark configurations of the LoLA layer.

This module is shared by the CPU oracle's tests and by the HIP path's tests and benchmark; it
holds no arithmetic of the method itself (no feature map, no attention, no scoring) - only the
random draws, the storage-type rounding of the drawn values, and the shape tables.

Every array is returned as float32 whose values are exactly representable in the
configuration's storage type (bf16 or fp32), so the oracle and the GPU receive the same bits.
Draw order per configuration: W_q, W_k, then q, k, v.  The generator is numpy's counter-based
Philox, keyed by (seed, sub-stream), so a sub-stream (e.g. one sequence of the decode batch) can
be regenerated on its own.

The inputs are stand-ins for the activations of the Llama-shaped models the paper evaluates
(Sec. 4: Llama-3.2-1B / Llama-3.1-8B head shapes); none of the paper's datasets is involved.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Shape:
    name: str
    dtype: str          # "f32" | "bf16": storage type of q, k, v, W, out and cached K, V
    B: int
    Hq: int
    Hkv: int
    d: int              # head_dim (= d_k = d_v)
    D: int              # feature dimension of phi (W is [d, D/2])
    T: int              # prefill length
    eta: int            # sliding-window size
    lam: int            # sparse-cache budget
    C: int              # prefill chunk
    seed: int
    n_decode: int = 0   # decode steps after the prefill
    n_clusters: int = 0  # >0: keys from a Gaussian mixture
    n_planted: int = 0   # >0: planted (k*, v*) pairs re-queried at the end

    @property
    def m(self):
        return self.D // 2

    @property
    def g(self):
        return self.Hq // self.Hkv


CONFIGS = {
    1: Shape("tiny_f32", "f32", 1, 1, 1, 64, 64, 256, 16, 16, 16, seed=0, n_decode=32),
    2: Shape("1b_prefill", "bf16", 1, 32, 8, 64, 128, 4096, 64, 64, 64, seed=1),
    3: Shape("8b_prefill", "bf16", 4, 32, 8, 128, 128, 4096, 64, 128, 64, seed=2, n_clusters=16),
    4: Shape("8b_decode", "bf16", 64, 32, 8, 128, 128, 32768, 64, 128, 64, seed=3, n_decode=1024),
    5: Shape("8b_recall_64k", "bf16", 1, 32, 8, 128, 128, 65536, 64, 256, 64, seed=4, n_clusters=64, n_planted=32),
}


def scaled(cfg_id: int, **kw) -> Shape:
    """A configuration with some sizes overridden (small parity cases keep the value recipe)."""
    return replace(CONFIGS[cfg_id], **kw)


def rng(seed: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(sub)]))


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32. In place."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    flat = x.reshape(-1)
    step = 1 << 24
    for a in range(0, flat.size, step):
        b = flat[a:a + step].view(np.uint32)
        b += np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
        b &= np.uint32(0xFFFF0000)
    return x


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    return bf16_round(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _normal(g: np.random.Generator, shape) -> np.ndarray:
    return g.standard_normal(size=shape, dtype=np.float32)


def weights(sh: Shape):
    """W_q [Hq, d, m], W_k [Hkv, d, m], entries N(0, 1/d), from sub-stream 0 of the seed."""
    g = rng(sh.seed, 0)
    s = np.float32(1.0 / np.sqrt(sh.d))
    Wq = _normal(g, (sh.Hq, sh.d, sh.m)) * s
    Wk = _normal(g, (sh.Hkv, sh.d, sh.m)) * s
    return store(Wq, sh.dtype), store(Wk, sh.dtype)


def _mixture_keys(g, sh: Shape, n_tok: int):
    """k = mu_c + 0.3 eps per (batch, kv head): centres ~ N(0, I), c uniform."""
    centres = _normal(g, (sh.B, sh.Hkv, sh.n_clusters, sh.d))
    assign = g.integers(0, sh.n_clusters, size=(sh.B, sh.Hkv, n_tok))
    k = np.take_along_axis(centres, assign[..., None], axis=2)
    k = k + np.float32(0.3) * _normal(g, (sh.B, sh.Hkv, n_tok, sh.d))
    return k.astype(np.float32), centres


def sequence_inputs(sh: Shape, n_tok: int | None = None):
    """q [B,Hq,N,d], k, v [B,Hkv,N,d] for N = T + n_decode tokens (or n_tok), plus a dict of extras.

    Recipe by configuration family:
      plain N(0,1) (configs 1, 4); N(0,1) then divided by the vector's RMS (config 2);
      mixture keys (configs 3, 5); config 5 additionally plants n_planted pairs and re-queries
      them with the last n_planted queries.
    """
    N = sh.T + sh.n_decode if n_tok is None else n_tok
    g = rng(sh.seed, 1)
    extras = {}
    q = _normal(g, (sh.B, sh.Hq, N, sh.d))
    if sh.n_clusters > 0:
        k, centres = _mixture_keys(g, sh, N)
    else:
        k = _normal(g, (sh.B, sh.Hkv, N, sh.d))
    v = _normal(g, (sh.B, sh.Hkv, N, sh.d))
    if sh.name == "1b_prefill":
        for a in (q, k, v):
            a /= np.sqrt(np.mean(a * a, axis=-1, keepdims=True))
    if sh.n_planted > 0:
        P = sh.n_planted
        lo, hi = sh.eta + sh.lam, max(sh.eta + sh.lam + P, N - min(4096, N // 4))
        pos = np.sort(g.choice(np.arange(lo, hi), size=P, replace=False))
        kstar = _normal(g, (sh.B, sh.Hkv, P, sh.d))
        # remove the component inside the span of the cluster centres (if it is not the whole space)
        if sh.n_clusters < sh.d:
            for b in range(sh.B):
                for h in range(sh.Hkv):
                    Qb, _ = np.linalg.qr(centres[b, h].astype(np.float64).T)   # [d, n_clusters]
                    ks = kstar[b, h].astype(np.float64)
                    kstar[b, h] = (ks - (ks @ Qb) @ Qb.T).astype(np.float32)
        vstar = np.float32(3.0) * _normal(g, (sh.B, sh.Hkv, P, sh.d))
        k[:, :, pos, :] = kstar
        v[:, :, pos, :] = vstar
        noise = np.float32(0.05) * _normal(g, (sh.B, sh.Hq, P, sh.d))
        q[:, :, N - P:, :] = np.repeat(kstar, sh.g, axis=1) + noise
        extras["planted_pos"] = pos
    return store(q, sh.dtype), store(k, sh.dtype), store(v, sh.dtype), extras


def decode_batch_sequence(sh: Shape, b: int, n_prefill: int | None = None):
    """Config-4 style inputs of ONE sequence b (its own Philox sub-stream, so any subset of the
    batch can be produced without the rest): k, v [Hkv, n_prefill, d] for the prefill and
    q [n_decode, Hq, d], k, v [n_decode, Hkv, d] for the decode steps; all N(0,1)."""
    T = sh.T if n_prefill is None else n_prefill
    g = rng(sh.seed, 1000 + b)
    kp = store(_normal(g, (sh.Hkv, T, sh.d)), sh.dtype)
    vp = store(_normal(g, (sh.Hkv, T, sh.d)), sh.dtype)
    qd = store(_normal(g, (sh.n_decode, sh.Hq, sh.d)), sh.dtype)
    kd = store(_normal(g, (sh.n_decode, sh.Hkv, sh.d)), sh.dtype)
    vd = store(_normal(g, (sh.n_decode, sh.Hkv, sh.d)), sh.dtype)
    return kp, vp, qd, kd, vd
