"""Thin ctypes binding of ``include/lola.h``: argument marshalling only.

Every step of the layer runs in the HIP library; torch is used for device memory and for the
stream handle.  There is no CPU fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # loads the HIP runtime the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblola.so")

LOLA_F32, LOLA_BF16 = 0, 1
LOLA_PHI_SOFTMAX, LOLA_PHI_EXP = 0, 1
LOLA_HIDE_STATE, LOLA_HIDE_SPARSE = 1, 2
LOLA_SCORE_SRE, LOLA_SCORE_WERR_SQ, LOLA_SCORE_WERR_ABS, LOLA_SCORE_OVEREST, LOLA_SCORE_ATTN = 0, 1, 2, 3, 4
EXPORTS = ("lola_state_bytes", "lola_prefill_workspace_bytes", "lola_state_init", "lola_state_flush", "lola_prefill",
           "lola_decode_step", "lola_status_str", "lola_kernel_path", "lola_release_streams", "lola_prefill_noalloc",
           "lola_noalloc_scratch_bytes", "lola_step_scratch_bytes")


class LolaConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "feat_dim", "window", "sparse_budget", "chunk",
        "dtype", "out_dtype", "phi_kind")] + [("softmax_scale", C.c_float), ("fold_defer", C.c_int32), ("query_hide", C.c_int32),
                                        ("score_kind", C.c_int32), ("prefill_overlap", C.c_int32)]


class LolaState(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens",
        "pend_phi", "pend_v", "pend_count", "win_score", "sp_score")]


class LolaError(RuntimeError):
    pass


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LolaError(f"{LIB_PATH} is missing: run `python -m paper_2505_23666_amd.build` first")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        cfgp, stp = C.POINTER(LolaConfig), C.POINTER(LolaState)
        L.lola_state_bytes.restype = sz
        L.lola_state_bytes.argtypes = [cfgp, C.POINTER(sz)]
        L.lola_step_scratch_bytes.restype = sz
        L.lola_step_scratch_bytes.argtypes = [cfgp]
        L.lola_prefill_workspace_bytes.restype = sz
        L.lola_prefill_workspace_bytes.argtypes = [cfgp, i32, i32, C.POINTER(sz)]
        L.lola_state_init.restype = C.c_int
        L.lola_state_init.argtypes = [cfgp, stp, vp]
        L.lola_state_flush.restype = C.c_int
        L.lola_state_flush.argtypes = [cfgp, stp, vp]
        L.lola_prefill.restype = C.c_int
        L.lola_prefill.argtypes = [cfgp, stp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.lola_decode_step.restype = C.c_int
        L.lola_decode_step.argtypes = [cfgp, stp, vp, vp, vp, vp, vp, vp, vp]
        L.lola_status_str.restype = C.c_char_p
        L.lola_status_str.argtypes = [C.c_int]
        L.lola_kernel_path.restype = C.c_char_p
        L.lola_kernel_path.argtypes = [cfgp, i32]
        L.lola_prefill_noalloc.restype = C.c_int
        L.lola_prefill_noalloc.argtypes = [cfgp, stp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
        L.lola_noalloc_scratch_bytes.restype = sz
        L.lola_noalloc_scratch_bytes.argtypes = []
        L.lola_release_streams.restype = None
        L.lola_release_streams.argtypes = []
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise LolaError(f"{what}: {lib().lola_status_str(rc).decode()} ({rc})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def lola_state_bytes(cfg: LolaConfig):
    fb = (C.c_size_t * 14)()
    tot = lib().lola_state_bytes(C.byref(cfg), fb)
    return int(tot), [int(x) for x in fb]


def lola_step_scratch_bytes(cfg: LolaConfig) -> int:
    return int(lib().lola_step_scratch_bytes(C.byref(cfg)))


def lola_prefill_workspace_bytes(cfg: LolaConfig, T: int, with_outputs: bool = True):
    mn = C.c_size_t(0)
    full = lib().lola_prefill_workspace_bytes(C.byref(cfg), T, int(with_outputs), C.byref(mn))
    return int(full), int(mn.value)


def lola_state_init(cfg: LolaConfig, st: LolaState) -> None:
    _check(lib().lola_state_init(C.byref(cfg), C.byref(st), _stream()), "lola_state_init")


def lola_state_flush(cfg: LolaConfig, st: LolaState) -> None:
    _check(lib().lola_state_flush(C.byref(cfg), C.byref(st), _stream()), "lola_state_flush")


def lola_prefill(cfg, st, q, k, v, Wq, Wk, T, out, sel_trace, workspace) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lola_prefill(C.byref(cfg), C.byref(st), _ptr(q), _ptr(k), _ptr(v), _ptr(Wq), _ptr(Wk), int(T),
                              _ptr(out), _ptr(sel_trace), _ptr(workspace), nbytes, _stream()), "lola_prefill")


def lola_prefill_noalloc(cfg, st, q, k, v, Wq, Wk, T, out, sel_trace) -> None:
    _check(lib().lola_prefill_noalloc(C.byref(cfg), C.byref(st), _ptr(q), _ptr(k), _ptr(v), _ptr(Wq), _ptr(Wk), int(T),
                                      _ptr(out), _ptr(sel_trace), _stream()), "lola_prefill_noalloc")


def lola_decode_step(cfg, st, q, k, v, Wq, Wk, out) -> None:
    _check(lib().lola_decode_step(C.byref(cfg), C.byref(st), _ptr(q), _ptr(k), _ptr(v), _ptr(Wq), _ptr(Wk),
                                  _ptr(out), _stream()), "lola_decode_step")


def lola_release_streams() -> None:
    lib().lola_release_streams()


def lola_kernel_path(cfg: LolaConfig, which: int) -> str:
    return lib().lola_kernel_path(C.byref(cfg), which).decode()


_TORCH_DT = {LOLA_F32: torch.float32, LOLA_BF16: torch.bfloat16}


class LolaLayer:
    """Device buffers of one layer's memories plus the three calls, for tests and benchmarks."""

    def __init__(self, B, Hq, Hkv, d, D, eta, lam, C_, dtype="bf16", out_dtype="f32",
                 phi_kind=LOLA_PHI_SOFTMAX, scale=0.0, fold_defer=0, query_hide=0, score_kind=0,
                 prefill_overlap=0, step_scratch=True, device="cuda:0"):
        self.device = torch.device(device)
        self.dt = LOLA_BF16 if dtype == "bf16" else LOLA_F32
        self.odt = LOLA_BF16 if out_dtype == "bf16" else LOLA_F32
        self.cfg = LolaConfig(B, Hq, Hkv, d, D, eta, lam, C_, self.dt, self.odt, phi_kind, float(scale), int(fold_defer),
                              int(query_hide), int(score_kind), int(prefill_overlap))
        self.score_kind = int(score_kind)
        self.fold_defer = R = int(fold_defer)
        self.B, self.Hq, self.Hkv, self.d, self.D, self.eta, self.lam, self.C = B, Hq, Hkv, d, D, eta, lam, C_
        tot, fb = lola_state_bytes(self.cfg)
        if tot == 0:
            raise LolaError("invalid configuration")
        tdt, dev = _TORCH_DT[self.dt], self.device
        self.H = torch.empty((B, Hkv, d, D), dtype=torch.float32, device=dev)   # H^T, see lola.h
        self.s = torch.empty((B, Hkv, D), dtype=torch.float32, device=dev)
        self.win_k = torch.empty((B, Hkv, eta, d), dtype=tdt, device=dev)
        self.win_v = torch.empty((B, Hkv, eta, d), dtype=tdt, device=dev)
        self.sp_k = torch.empty((B, Hkv, lam, d), dtype=tdt, device=dev)
        self.sp_v = torch.empty((B, Hkv, lam, d), dtype=tdt, device=dev)
        self.sp_idx = torch.empty((B, Hkv, lam), dtype=torch.int32, device=dev)
        self.sp_count = torch.empty((B, Hkv), dtype=torch.int32, device=dev)
        self.n_tokens = torch.empty((B, Hkv), dtype=torch.int64, device=dev)
        self.pend_phi = torch.empty((B, Hkv, R, D), dtype=torch.float32, device=dev)
        self.pend_v = torch.empty((B, Hkv, R, d), dtype=torch.float32, device=dev)
        self.pend_count = torch.empty((B, Hkv) if R else (0,), dtype=torch.int32, device=dev)
        sk = 1 if self.score_kind else 0
        self.win_score = torch.empty((B, Hkv, eta) if sk else (0,), dtype=torch.float32, device=dev)
        self.sp_score = torch.empty((B, Hkv, lam) if sk else (0,), dtype=torch.float32, device=dev)
        fields = [self.H, self.s, self.win_k, self.win_v, self.sp_k, self.sp_v, self.sp_idx, self.sp_count, self.n_tokens,
                  self.pend_phi, self.pend_v, self.pend_count, self.win_score, self.sp_score]
        assert [t.numel() * t.element_size() for t in fields] == fb
        self.st = LolaState(*[t.data_ptr() if t.numel() else None for t in fields])
        # optional scratch of the generation step when the scores are self-recall errors (see lola.h, sp_score)
        self.step_scratch = None
        nscr = lola_step_scratch_bytes(self.cfg)
        if step_scratch and nscr:
            self.step_scratch = torch.empty((nscr // 4,), dtype=torch.float32, device=dev)
            self.st.sp_score = self.step_scratch.data_ptr()
        self.workspace = None
        with torch.cuda.device(self.device):
            lola_state_init(self.cfg, self.st)

    @property
    def lola_path(self):
        """Kernel families (prefill, generation step) this configuration runs on."""
        return lola_kernel_path(self.cfg, 0), lola_kernel_path(self.cfg, 1)

    def reset(self):
        with torch.cuda.device(self.device):
            lola_state_init(self.cfg, self.st)

    def flush(self):
        """Apply the listed (deferred) folds to H and s in memory."""
        with torch.cuda.device(self.device):
            lola_state_flush(self.cfg, self.st)

    def _ws(self, T, with_out, limit_bytes=None):
        full, mn = lola_prefill_workspace_bytes(self.cfg, T, with_out)
        want = full if limit_bytes is None else max(mn, min(full, limit_bytes))
        if self.workspace is None or self.workspace.numel() < want:
            self.workspace = torch.empty(want, dtype=torch.uint8, device=self.device)
        return self.workspace[:want] if limit_bytes is not None else self.workspace

    def prefill(self, q, k, v, Wq, Wk, out=None, trace=False, workspace_limit=None, noalloc=False):
        """q [B,Hq,T,d] or None; k, v [B,Hkv,T,d].  Returns out (or None), plus the selection
        trace [B,Hkv,n_chunks,lam] when trace=True.  noalloc=True calls lola_prefill_noalloc (`out` must be given:
        this wrapper then allocates nothing either, unless a trace is asked for)."""
        T = k.shape[2]
        assert k.shape == (self.B, self.Hkv, T, self.d) and v.shape == k.shape and k.is_contiguous() and v.is_contiguous()
        if q is not None:
            assert q.shape == (self.B, self.Hq, T, self.d) and q.is_contiguous()
            if out is None:
                out = torch.empty((self.B, self.Hq, T, self.d), dtype=_TORCH_DT[self.odt], device=self.device)
        tr = None
        if trace:
            nch = (T + self.C - 1) // self.C
            tr = torch.empty((self.B, self.Hkv, nch, self.lam), dtype=torch.int32, device=self.device)
        trp = tr if (tr is not None and tr.numel()) else None
        with torch.cuda.device(self.device):
            if noalloc:
                lola_prefill_noalloc(self.cfg, self.st, q, k, v, Wq, Wk, T, out, trp)
            else:
                lola_prefill(self.cfg, self.st, q, k, v, Wq, Wk, T, out, trp, self._ws(T, q is not None, workspace_limit))
        return (out, tr) if trace else out

    def decode_step(self, q, k, v, Wq, Wk, out=None):
        assert q.shape == (self.B, self.Hq, self.d) and k.shape == (self.B, self.Hkv, self.d) and v.shape == k.shape
        assert q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
        if out is None:
            out = torch.empty((self.B, self.Hq, self.d), dtype=_TORCH_DT[self.odt], device=self.device)
        with torch.cuda.device(self.device):
            lola_decode_step(self.cfg, self.st, q, k, v, Wq, Wk, out)
        return out
