"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes the state and workspace as documented, and rejects bad arguments before
anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2505_23666_amd import binding as lb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(lb.LIB_PATH):
        from paper_2505_23666_amd import build
        build.build_library()
    return lb.lib()


def cfg(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, feat_dim=128, window=64, sparse_budget=128,
                chunk=64, dtype=lb.LOLA_BF16, out_dtype=lb.LOLA_F32, phi_kind=0, softmax_scale=0.0)
    base.update(kw)
    return lb.LolaConfig(**base)


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "lola.h")).read()
    declared = set(re.findall(r"\b(lola_[a-z_]+)\s*\(", header))
    assert declared == set(lb.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_step_scratch_bytes(L):
    """The generation step's optional scratch: none at the compile-time shapes (one fused kernel) or with
    query-dependent scores (sp_score holds the sums then); at the run-time shapes room for the cached pairs' scores and
    for sixteen shares of the outputs per stream."""
    assert lb.lola_step_scratch_bytes(cfg()) == 0
    assert lb.lola_step_scratch_bytes(cfg(feat_dim=256, window=256, sparse_budget=256, score_kind=1)) == 0
    assert lb.lola_step_scratch_bytes(cfg(feat_dim=256, window=256, sparse_budget=256)) == 4 * 16 * (4 * 128 + 8) * 4
    assert lb.lola_step_scratch_bytes(cfg(head_dim=64, window=128, sparse_budget=2048)) == 4 * 16 * (4 * 64 + 8) * 4
    assert lb.lola_step_scratch_bytes(cfg(head_dim=64, window=64, sparse_budget=2560 + 1920)) == 0   # more keys than the output kernel takes
    assert lb.lola_step_scratch_bytes(cfg(head_dim=100)) == 0


def test_state_bytes(L):
    tot, fb = lb.lola_state_bytes(cfg())
    ns = 4
    assert fb == [ns * 128 * 128 * 4, ns * 128 * 4, ns * 64 * 128 * 2, ns * 64 * 128 * 2, ns * 128 * 128 * 2,
                  ns * 128 * 128 * 2, ns * 128 * 4, ns * 4, ns * 8, 0, 0, 0, 0, 0]
    assert tot == sum(fb)
    # deferred folds: a list of 8 (phi, v) rows in fp32 and its length per stream
    tot8, fb8 = lb.lola_state_bytes(cfg(fold_defer=8))
    assert fb8[:9] == fb[:9] and fb8[9:] == [ns * 8 * 128 * 4, ns * 8 * 128 * 4, ns * 4, 0, 0] and tot8 == sum(fb8)
    # query-dependent scores: one sum per ring slot and per sparse slot; they exclude deferred folds
    tots, fbs = lb.lola_state_bytes(cfg(score_kind=lb.LOLA_SCORE_ATTN))
    assert fbs[:12] == fb[:12] and fbs[12:] == [ns * 64 * 4, ns * 128 * 4] and tots == sum(fbs)
    assert lb.lola_state_bytes(cfg(score_kind=2, fold_defer=8))[0] == 0
    assert lb.lola_state_bytes(cfg(score_kind=5))[0] == 0
    assert lb.lola_state_bytes(cfg(fold_defer=3))[0] == 0                 # not a supported list length
    assert lb.lola_state_bytes(cfg(fold_defer=8, head_dim=32))[0] == 0    # no kernel with deferred folds for this shape
    assert lb.lola_state_bytes(cfg(fold_defer=8, head_dim=64))[0] > 0     # the 1B head shape has one
    assert lb.lola_state_bytes(cfg(head_dim=100))[0] == 0
    assert lb.lola_state_bytes(cfg(feat_dim=127))[0] == 0
    assert lb.lola_state_bytes(cfg(n_q_heads=7))[0] == 0


def test_workspace_bytes_monotone(L):
    full, mn = lb.lola_prefill_workspace_bytes(cfg(), 4096, True)
    full2, mn2 = lb.lola_prefill_workspace_bytes(cfg(), 8192, True)
    assert mn == mn2 and full2 > full > mn > 0
    # an update-only call keeps no snapshots; on the MFMA path it still has per-chunk scratch (features of the keys),
    # recommended for at most 64 chunks per pass
    upd, mnu = lb.lola_prefill_workspace_bytes(cfg(), 4096, False)
    upd2, _ = lb.lola_prefill_workspace_bytes(cfg(), 1 << 20, False)
    assert mnu < mn and mnu <= upd == upd2 < full
    gen = cfg(window=32)        # generic kernels: nothing per chunk
    updg, mnug = lb.lola_prefill_workspace_bytes(gen, 4096, False)
    assert updg == mnug > 0


def test_status_strings(L):
    for code in range(-7, 1):
        assert L.lola_status_str(code)
    assert lb.lola_kernel_path(cfg(), 0) in ("generic", "mfma")


def test_arguments_rejected_before_launch(L):
    """Every call below must return an error from host-side validation (no GPU is present here)."""
    c = cfg()
    fake = 0x1000  # aligned, never dereferenced on the host
    st = lb.LolaState(*([fake] * 9 + [None] * 5))
    bad_st = lb.LolaState(*([fake] * 8 + [None] * 6))
    f = lambda *a: L.lola_decode_step(*a)
    vp = C.c_void_p
    assert f(C.byref(c), C.byref(bad_st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -1
    assert f(C.byref(c), C.byref(st), None, vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -1
    assert f(C.byref(c), C.byref(st), vp(fake + 4), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -4
    assert f(C.byref(cfg(dtype=7)), C.byref(st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -3
    assert f(C.byref(cfg(window=-1)), C.byref(st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -2
    p = lambda cc, s, q, k, out, T, ws, wsb: L.lola_prefill(C.byref(cc), C.byref(s), q, k, vp(fake), vp(fake), vp(fake), T, out,
                                                           None, ws, wsb, None)
    assert p(c, st, vp(fake), vp(fake), None, 64, vp(fake), 1 << 40) == -1          # q without out
    assert p(c, st, vp(fake), None, vp(fake), 64, vp(fake), 1 << 40) == -1          # k missing
    assert p(c, st, vp(fake), vp(fake), vp(fake), -1, vp(fake), 1 << 40) == -2      # negative T
    assert p(c, st, vp(fake), vp(fake), vp(fake), 64, None, 0) == -6                 # no workspace
    assert p(c, st, vp(fake), vp(fake), vp(fake), 64, vp(fake), 1024) == -6          # workspace too small
    assert p(c, st, None, None, None, 0, None, 0) == 0                                # T = 0: nothing is touched
    assert L.lola_state_init(C.byref(c), C.byref(bad_st), None) == -1
    # deferred folds: the list pointers become required; shapes without the fused generation step are refused
    c8 = cfg(fold_defer=8)
    assert f(C.byref(c8), C.byref(st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -1
    assert L.lola_state_flush(C.byref(c8), C.byref(st), None) == -1
    assert L.lola_state_flush(C.byref(cfg(fold_defer=8, sparse_budget=256)), C.byref(st), None) == -5
    assert L.lola_state_flush(C.byref(cfg(fold_defer=5)), C.byref(st), None) == -2
    cs = cfg(score_kind=lb.LOLA_SCORE_WERR_SQ)
    assert f(C.byref(cs), C.byref(st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -1   # score fields missing
    sts = lb.LolaState(*([fake] * 9 + [None] * 3 + [fake] * 2))
    assert p(cs, sts, None, vp(fake), None, 64, vp(fake), 1 << 40) == -5    # update-only call: these scores need queries
    assert lb.lola_kernel_path(cs, 0) == "mfma" and lb.lola_kernel_path(cs, 1) == "mfma"    # the run-time-parameter kernels
    assert lb.lola_kernel_path(cfg(feat_dim=256, window=256, sparse_budget=256), 0) == "mfma"    # run-time window / budget kernels
    assert lb.lola_kernel_path(cfg(feat_dim=256, window=256, sparse_budget=200), 0) == "mixed"   # budget not a multiple of 64
    assert lb.lola_kernel_path(cfg(feat_dim=256, window=256, sparse_budget=256, chunk=128), 0) == "generic"
    assert lb.lola_kernel_path(cfg(sparse_budget=0), 0) == "mfma"
    # which kernel family serves what (prefill, generation step)
    path = lambda **kw: (lb.lola_kernel_path(cfg(**kw), 0), lb.lola_kernel_path(cfg(**kw), 1))
    assert path() == ("mfma", "mfma")                                            # the 8B shape: compile-time kernels
    assert path(sparse_budget=256) == ("mfma", "mfma")                           # fused step only for budgets 64 / 128: run-time step kernels
    assert path(sparse_budget=0) == ("mfma", "mixed")                            # no cache: row-split evolution; step: generic update, MFMA outputs
    assert path(sparse_budget=0, window=192) == ("mfma", "mixed")
    assert path(window=128, sparse_budget=1024, feat_dim=256) == ("mfma", "mfma")
    assert path(window=128, sparse_budget=2048, feat_dim=256) == ("generic", "mfma")   # prefill kernels stop at budget 1024
    assert path(window=100, sparse_budget=128) == ("mixed", "mfma")              # window not a multiple of 64: generic evolution
    assert path(n_q_heads=16) == ("mfma", "mfma")                                # 8 query heads per kv head (cfg has 2 kv heads)
    assert path(n_q_heads=32) == ("mfma", "generic")                             # 16: the step kernels take at most 8
    assert path(dtype=lb.LOLA_F32) == ("generic", "generic")
    assert path(head_dim=256, feat_dim=256) == ("generic", "generic")
    assert f(C.byref(cfg(query_hide=4)), C.byref(st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None) == -2


def test_unsupported_tilings_are_refused_before_anything_is_enqueued(L):
    """A configuration that passes the range checks but that no kernel can tile into LDS must come back as
    LOLA_ERR_UNSUPPORTED from the host-side checks.  No GPU is present here, so anything that reached a
    launch (the flush of deferred folds, the first prefill kernel) would come back as LOLA_ERR_HIP instead."""
    vp = C.c_void_p
    fake = 0x1000
    st = lb.LolaState(*([fake] * 9 + [None] * 5))
    big = cfg(dtype=lb.LOLA_F32, head_dim=256, feat_dim=512, window=4096, sparse_budget=4096, chunk=1024)
    assert lb.lola_state_bytes(big)[0] > 0                      # a valid configuration
    full, mn = lb.lola_prefill_workspace_bytes(big, 1024, True)
    assert mn > 0
    rc = L.lola_prefill(C.byref(big), C.byref(st), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), 1024, vp(fake), None,
                        vp(fake), 1 << 50, None)
    assert rc == -5
    # the generation step of this shape fits (it would be launched); with a query-dependent score it does not
    bigs = cfg(dtype=lb.LOLA_F32, head_dim=256, feat_dim=512, window=4096, sparse_budget=4096, chunk=1024, score_kind=1)
    sts = lb.LolaState(*([fake] * 9 + [None] * 3 + [fake] * 2))
    rc = L.lola_decode_step(C.byref(bigs), C.byref(sts), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), vp(fake), None)
    assert rc == -5
    # streams, query heads and sequences must fit the launch grids' y / z limits
    assert lb.lola_state_bytes(cfg(batch=40000, n_q_heads=2, n_kv_heads=2))[0] == 0
    assert lb.lola_state_bytes(cfg(batch=1, n_q_heads=131072, n_kv_heads=2))[0] == 0
    assert lb.lola_state_bytes(cfg(prefill_overlap=2))[0] == 0
    L.lola_release_streams()    # nothing was created: a no-op


def test_benchmark_work_counts_match_the_documented_figures():
    """The algorithmic bytes / flops bench.py divides by are the ones the design notes derive from the
    layer's definition (8B shape: 235 524 B per stream and step, 121.24 MB per launch at batch 64;
    57.7 MFLOP per chunk and stream, 118.1 GFLOP per configuration-3 call)."""
    import bench
    import workloads as wl
    per_stream, per_launch = bench.decode_alg_bytes(wl.CONFIGS[4], 4)
    assert per_stream == 235524 and per_launch == 235524 * 512 + 40 * 128 * 64 * 2 == 121243648
    per_chunk, per_call = bench.prefill_alg_flops(wl.CONFIGS[3])
    assert per_chunk == 57671680 and per_call == per_chunk * 64 * 32
    assert abs(per_call / 1e9 - 118.1) < 0.05
