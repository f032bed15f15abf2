"""ctypes front end of the CPU oracle (``lola_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
CPU-baseline leg, never by the HIP product path.  Builds the C file with gcc on first use
(``build()``), in fp64 (the oracle proper) and optionally in fp32 (a drift probe).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# The checks of the oracle itself (a sanitizer build, planted mistakes) run the pin suite against
# another build of it: LOLA_ORACLE_SRC names the C file, LOLA_ORACLE_LIBDIR the folder that takes the
# libraries, LOLA_ORACLE_CFLAGS extra compiler flags.  Unset, the oracle proper is built in place.
_SRC = os.environ.get("LOLA_ORACLE_SRC") or os.path.join(_HERE, "lola_oracle.c")
_LIBDIR = os.environ.get("LOLA_ORACLE_LIBDIR") or _HERE
_EXTRA_CFLAGS = os.environ.get("LOLA_ORACLE_CFLAGS", "").split()

PHI_SOFTMAX, PHI_EXP = 0, 1
HIDE_STATE, HIDE_SPARSE = 1, 2   # restricted-query ablation: what the query does not read
# what ranks the eligible pairs: self-recall error, or one of the query-dependent sums of the scoring ablation
SCORE_SRE, SCORE_WERR_SQ, SCORE_WERR_ABS, SCORE_OVEREST, SCORE_ATTN = 0, 1, 2, 3, 4


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "d", "D", "eta", "lam", "C", "phi_kind")] + [
        ("scale", C.c_double), ("hide", C.c_int32), ("score_kind", C.c_int32)
    ]


def _lib_path(real: str) -> str:
    return os.path.join(_LIBDIR, f"liblola_oracle_{real}.so")


def build(force: bool = False) -> None:
    """Compile the oracle (fp64 and fp32 arithmetic variants) with gcc."""
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = _lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", f"-DORC_REAL={ctype}",
               "-Wall", "-Wextra", *_EXTRA_CFLAGS, "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


_libs: dict[str, C.CDLL] = {}


def _lib(real: str) -> C.CDLL:
    if real not in _libs:
        build()
        L = C.CDLL(_lib_path(real))
        vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L.orc_state_new.restype = vp
        L.orc_state_new.argtypes = [C.POINTER(_Cfg)]
        L.orc_state_free.argtypes = [vp]
        L.orc_decode_step.restype = C.c_int
        L.orc_decode_step.argtypes = [vp] * 7 + [vp, dbl, vp]
        L.orc_prefill.restype = C.c_int
        L.orc_prefill.argtypes = [vp] * 6 + [C.c_int, vp, vp, dbl, vp, vp]
        for n in ("orc_get_H", "orc_get_s", "orc_get_sparse_idx", "orc_get_window_idx"):
            getattr(L, n).argtypes = [vp, vp]
        L.orc_get_pairs.restype = C.c_int
        L.orc_get_pairs.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp]
        L.orc_get_scores.restype = C.c_int
        L.orc_get_scores.argtypes = [vp, C.c_int, C.c_int, vp]
        L.orc_get_folded.restype = i64
        L.orc_get_folded.argtypes = [vp, C.c_int, vp, i64]
        L.orc_get_n_tokens.restype = i64
        L.orc_get_n_tokens.argtypes = [vp, C.c_int]
        L.orc_get_stats.restype = dbl
        L.orc_get_stats.argtypes = [vp, vp]
        L.orc_set_stream.restype = C.c_int
        L.orc_set_stream.argtypes = [vp, C.c_int] + [vp] * 5 + [C.c_int] + [vp] * 3 + [C.c_int]
        L.orc_set_n_tokens.argtypes = [vp, C.c_int, i64]
        L.orc_phi.argtypes = [C.POINTER(_Cfg), vp, vp, vp]
        L.orc_sre_probe.restype = dbl
        L.orc_sre_probe.argtypes = [vp, C.c_int, vp, vp, vp]
        L.orc_cache_elems.restype = i64
        L.orc_cache_elems.argtypes = [i64] * 6 + [C.c_int]
        L.orc_real_bytes.restype = C.c_int
        L.orc_num_threads.restype = C.c_int
        _libs[real] = L
    return _libs[real]


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(_lib("f64").orc_num_threads())


def cache_elems(t, eta, lam, dk, dv, D, two_chunks=True) -> int:
    return int(_lib("f64").orc_cache_elems(t, eta, lam, dk, dv, D, int(two_chunks)))


def phi(W, x, kind=PHI_SOFTMAX, real="f64") -> np.ndarray:
    """phi(x) for a single vector; W is [d, D/2]."""
    W = _f32(W)
    d, m = W.shape
    cfg = _Cfg(1, 1, 1, d, 2 * m, 0, 0, 1, kind, 0.0, 0, 0)
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(2 * m, dtype=np.float64)
    _lib(real).orc_phi(C.byref(cfg), _ptr(W), _ptr(x), _ptr(out))
    return out


class Oracle:
    """State of one LoLA layer (all sequences and kv heads) plus the two update/attend calls."""

    def __init__(self, B, Hq, Hkv, d, D, eta, lam, C_, phi_kind=PHI_SOFTMAX, scale=0.0, real="f64", query_hide=0,
                 score_kind=SCORE_SRE):
        self.L = _lib(real)
        self.B, self.Hq, self.Hkv, self.d, self.D = B, Hq, Hkv, d, D
        self.eta, self.lam, self.C, self.m = eta, lam, C_, D // 2
        self.cfg = _Cfg(B, Hq, Hkv, d, D, eta, lam, C_, phi_kind, float(scale), int(query_hide), int(score_kind))
        self.h = self.L.orc_state_new(C.byref(self.cfg))
        if not self.h:
            raise ValueError("invalid oracle configuration")

    def __del__(self):
        if getattr(self, "h", None):
            self.L.orc_state_free(self.h)
            self.h = None

    # -- the layer ---------------------------------------------------------------------------
    def prefill(self, q, k, v, Wq, Wk, force_sel=None, tie_eps=1e-4, want_log=False):
        """q [B,Hq,T,d] or None (update only); k, v [B,Hkv,T,d].  Returns out (or None) and,
        with want_log, (out, sel_log [B,Hkv,n_chunks,lam], margins [B,Hkv,n_chunks])."""
        k = _f32(k)
        T = k.shape[2]
        k = _f32(k, (self.B, self.Hkv, T, self.d))
        v = _f32(v, (self.B, self.Hkv, T, self.d))
        Wk = _f32(Wk, (self.Hkv, self.d, self.m))
        out = None
        if q is not None:
            q = _f32(q, (self.B, self.Hq, T, self.d))
            Wq = _f32(Wq, (self.Hq, self.d, self.m))
            out = np.empty((self.B, self.Hq, T, self.d), dtype=np.float64)
        nch = (T + self.C - 1) // self.C
        if force_sel is not None:
            force_sel = np.ascontiguousarray(force_sel, dtype=np.int32)
            assert force_sel.shape == (self.B, self.Hkv, nch, self.lam)
        sel = np.empty((self.B, self.Hkv, nch, self.lam), dtype=np.int32) if want_log else None
        mar = np.empty((self.B, self.Hkv, nch), dtype=np.float64) if want_log else None
        rc = self.L.orc_prefill(self.h, _ptr(q), _ptr(k), _ptr(v), _ptr(Wq) if q is not None else None, _ptr(Wk),
                                T, _ptr(out), _ptr(force_sel), float(tie_eps), _ptr(sel), _ptr(mar))
        if rc != 0:
            raise RuntimeError(f"orc_prefill failed ({rc})")
        return (out, sel, mar) if want_log else out

    def decode_step(self, q, k, v, Wq, Wk, force_sel=None, tie_eps=1e-4, want_margin=False):
        """q [B,Hq,d]; k, v [B,Hkv,d].  Returns out [B,Hq,d] (and margins [B,Hkv])."""
        q = _f32(q, (self.B, self.Hq, self.d))
        k = _f32(k, (self.B, self.Hkv, self.d))
        v = _f32(v, (self.B, self.Hkv, self.d))
        Wq = _f32(Wq, (self.Hq, self.d, self.m))
        Wk = _f32(Wk, (self.Hkv, self.d, self.m))
        out = np.empty((self.B, self.Hq, self.d), dtype=np.float64)
        if force_sel is not None:
            force_sel = np.ascontiguousarray(force_sel, dtype=np.int32)
            assert force_sel.shape == (self.B, self.Hkv, self.lam)
        mar = np.empty((self.B, self.Hkv), dtype=np.float64) if want_margin else None
        rc = self.L.orc_decode_step(self.h, _ptr(q), _ptr(k), _ptr(v), _ptr(Wq), _ptr(Wk), _ptr(out),
                                    _ptr(force_sel), float(tie_eps), _ptr(mar))
        if rc != 0:
            raise RuntimeError(f"orc_decode_step failed ({rc})")
        return (out, mar) if want_margin else out

    # -- state access ------------------------------------------------------------------------
    @property
    def H(self):
        out = np.empty((self.B, self.Hkv, self.D, self.d), dtype=np.float64)
        self.L.orc_get_H(self.h, _ptr(out))
        return out

    @property
    def s(self):
        out = np.empty((self.B, self.Hkv, self.D), dtype=np.float64)
        self.L.orc_get_s(self.h, _ptr(out))
        return out

    @property
    def sparse_idx(self):
        out = np.empty((self.B, self.Hkv, self.lam), dtype=np.int32)
        self.L.orc_get_sparse_idx(self.h, _ptr(out))
        return out

    @property
    def window_idx(self):
        out = np.empty((self.B, self.Hkv, self.eta), dtype=np.int32)
        self.L.orc_get_window_idx(self.h, _ptr(out))
        return out

    def pairs(self, stream, which):
        """(k, v, idx) of the sparse cache (which=0) or the window (which=1) of one stream."""
        cap = (self.lam if which == 0 else self.eta) + 1
        k = np.empty((cap, self.d)); v = np.empty((cap, self.d)); idx = np.empty(cap, dtype=np.int64)
        n = self.L.orc_get_pairs(self.h, stream, which, _ptr(k), _ptr(v), _ptr(idx))
        return k[:n].copy(), v[:n].copy(), idx[:n].copy()

    def scores(self, stream, which):
        """Query-dependent scores gathered so far by the pairs of `pairs(stream, which)`, same order."""
        out = np.empty((self.lam if which == 0 else self.eta) + 1)
        n = self.L.orc_get_scores(self.h, stream, which, _ptr(out))
        return out[:n].copy()

    def folded(self, stream):
        n = self.L.orc_get_folded(self.h, stream, None, 0)
        out = np.empty(max(n, 1), dtype=np.int64)
        self.L.orc_get_folded(self.h, stream, _ptr(out), n)
        return out[:n].copy()

    def n_tokens(self, b=0):
        return int(self.L.orc_get_n_tokens(self.h, b))

    def stats(self):
        """dict(scored, adopted, mismatch, min_margin) summed over streams."""
        a = np.zeros(3, dtype=np.int64)
        mm = self.L.orc_get_stats(self.h, _ptr(a))
        return {"scored": int(a[0]), "adopted": int(a[1]), "mismatch": int(a[2]), "min_margin": float(mm)}

    def set_stream(self, stream, H, s, spk, spv, spidx, wk, wv, widx):
        H = np.ascontiguousarray(H, dtype=np.float64); s = np.ascontiguousarray(s, dtype=np.float64)
        spk = _f32(spk).reshape(-1, self.d); spv = _f32(spv).reshape(-1, self.d)
        wk = _f32(wk).reshape(-1, self.d); wv = _f32(wv).reshape(-1, self.d)
        spidx = np.ascontiguousarray(spidx, dtype=np.int64); widx = np.ascontiguousarray(widx, dtype=np.int64)
        rc = self.L.orc_set_stream(self.h, stream, _ptr(H), _ptr(s), _ptr(spk), _ptr(spv), _ptr(spidx), len(spidx),
                                   _ptr(wk), _ptr(wv), _ptr(widx), len(widx))
        if rc != 0:
            raise RuntimeError("orc_set_stream failed")

    def set_n_tokens(self, b, n):
        self.L.orc_set_n_tokens(self.h, b, int(n))

    def sre_probe(self, stream, Wk_h, k, v):
        Wk_h = _f32(Wk_h, (self.d, self.m))
        k = np.ascontiguousarray(k, dtype=np.float64); v = np.ascontiguousarray(v, dtype=np.float64)
        return float(self.L.orc_sre_probe(self.h, stream, _ptr(Wk_h), _ptr(k), _ptr(v)))
