"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.

Small cases compare every output element, every state element and every selection; the
full-size configurations compare every element on all streams the oracle can finish in
reasonable time (stated per test) and the whole state of those streams.
"""
import os
import sys
import time

import numpy as np
import pytest
import torch

import workloads as wl
import parity as P
from oracle import lola_oracle as orc

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rand_case(seed, B, Hq, Hkv, d, D, N, dtype, wscale=1.0):
    g = wl.rng(seed, 5)
    q = wl.store(g.standard_normal((B, Hq, N, d), dtype=np.float32), dtype)
    k = wl.store(g.standard_normal((B, Hkv, N, d), dtype=np.float32), dtype)
    v = wl.store(g.standard_normal((B, Hkv, N, d), dtype=np.float32), dtype)
    Wq = wl.store((wscale * g.standard_normal((Hq, d, D // 2), dtype=np.float32) / np.sqrt(d)).astype(np.float32), dtype)
    Wk = wl.store((wscale * g.standard_normal((Hkv, d, D // 2), dtype=np.float32) / np.sqrt(d)).astype(np.float32), dtype)
    return q, k, v, Wq, Wk


def steps(q, k, v, t0, n):
    tr = lambda a: np.ascontiguousarray(a[:, :, t0:t0 + n].transpose(2, 0, 1, 3))
    return tr(q), tr(k), tr(v)


# ---------------------------------------------------------------------------------------------
# configuration 1 in full: fp32, prefill of 256 tokens then 32 generation steps
# ---------------------------------------------------------------------------------------------
def test_config1_tiny_fp32_prefill_then_decode():
    sh = wl.CONFIGS[1]
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    T = sh.T
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk)
    say("config1 prefill", rep)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, T, sh.n_decode), Wq, Wk)
    say("config1 decode", rep)
    assert rep["scored"] > 0


# ---------------------------------------------------------------------------------------------
# edge cases: ragged tails, empty memories, degenerate sizes, both storage types, both phi kinds
# ---------------------------------------------------------------------------------------------
EDGE = [
    # name            dtype  B Hq Hkv  d    D  eta lam  C    T  nd
    ("ragged_tail",   "f32", 2, 4, 2, 32,  16,  8,  6,  8,  77, 5),
    ("chunk_lt_win",  "f32", 1, 2, 1, 32,  24, 12,  5,  4,  50, 4),
    ("chunk_gt_win",  "bf16", 1, 2, 2, 64, 32,  5,  7, 16,  70, 9),
    ("no_window",     "f32", 1, 2, 1, 32,  16,  0,  4,  8,  40, 6),
    ("no_sparse",     "bf16", 2, 2, 2, 64, 64,  8,  0,  8,  64, 6),
    ("no_caches",     "f32", 1, 1, 1, 32,   8,  0,  0,  4,  19, 5),
    ("short_T",       "bf16", 1, 4, 1, 128, 64, 64, 32, 64,  9, 70),
    ("warmup_partial", "f32", 1, 1, 1, 32,  16,  4, 10,  8,  64, 3),
    ("head256",       "bf16", 1, 2, 1, 256, 128, 16, 16, 16, 96, 4),
    ("wide_features", "f32", 1, 1, 1, 64, 256, 16,  8, 16,  80, 3),
    ("gqa8",          "bf16", 1, 8, 1, 64, 128, 16, 24, 16, 128, 4),
]


@pytest.mark.parametrize("case", EDGE, ids=[c[0] for c in EDGE])
def test_edge_cases(case):
    name, dtype, B, Hq, Hkv, d, D, eta, lam, C, T, nd = case
    say("edge", case)
    sh = wl.Shape(name, dtype, B, Hq, Hkv, d, D, T, eta, lam, C, seed=0)
    q, k, v, Wq, Wk = rand_case(100 + len(name), B, Hq, Hkv, d, D, T + nd, dtype)
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, nd), Wq, Wk)
    say("  ", rep, rep2)


def test_decode_from_empty_state():
    sh = wl.Shape("cold", "bf16", 2, 4, 2, 64, 32, T=0, eta=6, lam=5, C=8, seed=0)
    q, k, v, Wq, Wk = rand_case(7, 2, 4, 2, 64, 32, 40, "bf16")
    layer, o = P.make_layer(sh), P.make_oracle(sh)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, 0, 40), Wq, Wk)
    say("cold decode", rep)


@pytest.mark.parametrize("lam,phi_kind", [(128, 0), (64, 0), (128, 1)])
def test_8b_shape_decode_from_cold_start(lam, phi_kind):
    """The fused generation kernel through all its regimes: window filling, cache warm-up (pairs
    appended unscored), then steady state with scoring, fold and in-place slot replacement."""
    sh = wl.Shape("cold8b", "bf16", 2, 8, 2, 128, 128, T=0, eta=64, lam=lam, C=64, seed=0)
    n = 64 + lam + 60
    q, k, v, Wq, Wk = rand_case(31 + lam, 2, 8, 2, 128, 128, n, "bf16", wscale=0.5 if phi_kind else 1.0)
    kw = dict(phi_kind=phi_kind)
    layer = P.make_layer(sh, **kw)
    o = P.make_oracle(sh, **kw)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, 0, n), Wq, Wk)
    say("8B-shape cold decode", lam, phi_kind, rep)
    assert rep["scored"] == 4 * 60


@pytest.mark.parametrize("lam,phi_kind,defer,hide,g", [(64, 0, 0, 0, 4), (128, 1, 8, 0, 4), (64, 0, 8, 2, 2), (128, 0, 0, 1, 1)])
def test_1b_head_shape_generation_step(lam, phi_kind, defer, hide, g):
    """The fused generation kernel at head_dim 64 (a wavefront owns 16 rows of the state instead of 32):
    cold start through warm-up into steady state, with and without deferred folds, restricted queries,
    smaller groups; then a prefill call (MFMA kernels too) and more steps."""
    sh = wl.Shape("dec1b", "bf16", 2, 2 * g, 2, 64, 128, T=0, eta=64, lam=lam, C=64, seed=0)
    n1, n_pre, n2 = 64 + lam + 29, 64 * 2 + 11, 13
    q, k, v, Wq, Wk = rand_case(140 + lam + g, 2, 2 * g, 2, 64, 128, n1 + n_pre + n2, "bf16", wscale=0.5 if phi_kind else 1.0)
    kw = dict(phi_kind=phi_kind, fold_defer=defer, query_hide=hide)
    okw = dict(phi_kind=phi_kind, query_hide=hide)
    layer = P.make_layer(sh, **kw)
    assert layer.lola_path == ("mfma", "mfma")
    o = P.make_oracle(sh, **okw)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, 0, n1), Wq, Wk)
    assert rep["scored"] == 4 * 29
    layer, o, rep2 = P.prefill_parity(sh, q[:, :, n1:n1 + n_pre], k[:, :, n1:n1 + n_pre], v[:, :, n1:n1 + n_pre], Wq, Wk,
                                      layer=layer, oracle=o, layer_kw=kw)
    rep3 = P.decode_parity(sh, layer, o, *steps(q, k, v, n1 + n_pre, n2), Wq, Wk)
    say("1B head shape generation step", lam, phi_kind, defer, hide, g, rep, rep2, rep3)


@pytest.mark.parametrize("lam,phi_kind", [(128, 0), (64, 1)])
def test_deferred_folds(lam, phi_kind):
    """fold_defer = 8 on the fused generation kernel: the folded pair of a step is listed instead of
    being applied to H in memory; memory + list must equal the oracle's state at every list length,
    outputs every step, through cold start, a prefill call in between (which applies the list),
    more steps, and an explicit flush."""
    R = 8
    listed = lambda n: n if n <= R else 1 + (n - 1) % R    # pairs listed after n steady steps: the step that finds R listed
                                                           # writes them back and starts a new list with its own pair
    sh = wl.Shape("defer8b", "bf16", 2, 8, 2, 128, 128, T=0, eta=64, lam=lam, C=64, seed=0)
    n_pre = 64 * 2 + 17
    blocks = [64 + lam + 5, 3, 8, 6]           # steady steps so far: 5, 8, 16, 22
    n = sum(blocks) + n_pre + 11
    q, k, v, Wq, Wk = rand_case(77 + lam, 2, 8, 2, 128, 128, n, "bf16", wscale=0.5 if phi_kind else 1.0)
    kw = dict(phi_kind=phi_kind)
    layer = P.make_layer(sh, fold_defer=R, **kw)
    assert layer.lola_path[1] == "mfma"
    o = P.make_oracle(sh, **kw)
    t0, steady = 0, 0
    for nb in blocks:
        rep = P.decode_parity(sh, layer, o, *steps(q, k, v, t0, nb), Wq, Wk)   # ends with a state check (memory + list)
        t0 += nb
        steady = t0 - 64 - lam
        cnt = layer.pend_count.cpu().numpy()
        say("deferred folds", lam, phi_kind, "steps", t0, "listed", cnt.ravel().tolist(), rep)
        assert (cnt == listed(steady)).all()
    # a prefill call starts by applying the list; its own folds go to H directly
    layer, o, rep = P.prefill_parity(sh, q[:, :, t0:t0 + n_pre], k[:, :, t0:t0 + n_pre], v[:, :, t0:t0 + n_pre], Wq, Wk,
                                     layer=layer, oracle=o, layer_kw=kw)
    t0 += n_pre
    assert (layer.pend_count.cpu().numpy() == 0).all()
    say("deferred folds: prefill in between", rep)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, t0, 11), Wq, Wk)
    assert (layer.pend_count.cpu().numpy() == listed(11)).all()
    # explicit flush: memory alone is the state
    layer.flush()
    torch.cuda.synchronize()
    assert (layer.pend_count.cpu().numpy() == 0).all()
    g = P.gpu_state_np(layer)
    P.check_state(g, o, P.TOL["bf16"])
    layer.flush()     # idempotent
    torch.cuda.synchronize()
    g2 = P.gpu_state_np(layer)
    assert np.array_equal(g["H"], g2["H"]) and np.array_equal(g["s"], g2["s"])
    say("deferred folds: after flush", rep)


def test_deferred_folds_refused_elsewhere():
    """Shapes without the fused generation kernel do not take fold_defer."""
    from paper_2505_23666_amd import binding as lb
    with pytest.raises(lb.LolaError):
        lb.LolaLayer(1, 4, 1, 32, 128, 64, 64, 64, fold_defer=8)
    with pytest.raises(lb.LolaError):
        lb.LolaLayer(1, 4, 1, 128, 128, 64, 128, 64, fold_defer=4)


@pytest.mark.parametrize("hide", [1, 2, 3])
def test_restricted_query_generic_kernels(hide):
    """Queries that do not read the hidden state (1), the sparse cache (2) or both (3); the
    memories evolve as usual.  fp32, generic kernels, prefill with a ragged tail then decode."""
    sh = wl.Shape("hide", "f32", 2, 4, 2, 32, 16, T=0, eta=8, lam=6, C=8, seed=0)
    T = 8 * 9 + 5
    q, k, v, Wq, Wk = rand_case(50 + hide, 2, 4, 2, 32, 16, T + 12, "f32")
    kw = dict(query_hide=hide)
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk, layer_kw=kw)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, 12), Wq, Wk)
    say("restricted query (generic)", hide, rep, rep2)
    assert rep["scored"] > 0 and rep2["scored"] > 0


@pytest.mark.parametrize("hide,defer", [(1, 0), (2, 8), (3, 0), (3, 8)])
def test_restricted_query_mfma_kernels(hide, defer):
    """The same on the MFMA prefill kernels and the fused generation step (8B head shape), with
    and without deferred folds."""
    sh = wl.scaled(3, B=1, T=64 * 6 + 10 + 20)
    T = 64 * 6 + 10
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    kw = dict(query_hide=hide, fold_defer=defer)
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk, layer_kw=kw)
    assert layer.lola_path == ("mfma", "mfma")
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, 20), Wq, Wk)
    say("restricted query (mfma)", hide, defer, rep, rep2)
    assert rep2["scored"] - rep["scored"] == 8 * 20


@pytest.mark.parametrize("kind", [1, 2, 3, 4])
def test_query_dependent_scores(kind):
    """The importance scores of the scoring ablation instead of the self-recall error: sums over the
    queries that see a key inside the sliding window, gathered by the generation step and by the
    prefill (ragged calls that resume mid-chunk, several workspace passes), cache decided by them."""
    sh = wl.Shape("qscore", "bf16", 2, 4, 2, 64, 32, T=0, eta=12, lam=9, C=16, seed=0)
    q, k, v, Wq, Wk = rand_case(90 + kind, 2, 4, 2, 64, 32, 16 * 9 + 5 + 30, "bf16")
    kw = dict(score_kind=kind)
    cuts = [0, 7, 16 * 4 + 3, 16 * 9 + 5]
    layer, o = None, None
    for i in range(3):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o,
                                         workspace_limit=0 if i == 2 else None, layer_kw=kw)
        say("query-dependent scores, prefill part", kind, i, rep)
    assert layer.lola_path == ("generic", "generic")
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, cuts[3], 18), Wq, Wk)
    a = cuts[3] + 18
    layer, o, rep2 = P.prefill_parity(sh, q[:, :, a:a + 12], k[:, :, a:a + 12], v[:, :, a:a + 12], Wq, Wk, layer=layer, oracle=o,
                                      layer_kw=kw)
    say("query-dependent scores, decode + short prefill", kind, rep, rep2)
    assert rep2["scored"] > 40


def test_query_dependent_scores_fp32_cold_decode_and_8b_shape():
    """fp32 storage from an empty state through warm-up; and the 8B head shape (generic kernels there)."""
    sh = wl.Shape("qscore32", "f32", 1, 2, 1, 32, 16, T=0, eta=5, lam=4, C=4, seed=0)
    q, k, v, Wq, Wk = rand_case(95, 1, 2, 1, 32, 16, 40, "f32")
    kw = dict(score_kind=3)
    layer, o = P.make_layer(sh, **kw), P.make_oracle(sh, **kw)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, 0, 40), Wq, Wk)
    say("query-dependent scores, fp32 cold decode", rep)
    sh = wl.scaled(3, B=1, T=64 * 4 + 9 + 6, lam=64)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    kw = dict(score_kind=1)
    T = 64 * 4 + 9
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk, layer_kw=kw)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, 6), Wq, Wk)
    say("query-dependent scores, 8B head shape", rep, rep2)


@pytest.mark.parametrize("kind,d,D,eta,lam", [(1, 128, 128, 64, 128), (2, 64, 128, 64, 64), (3, 128, 256, 128, 64), (4, 128, 128, 192, 256)])
def test_query_dependent_scores_on_the_mfma_prefill_kernels(kind, d, D, eta, lam):
    """The four query-dependent scores (Sec. 4 / appendix "scoring ablation") where the selection, fold and outputs of
    the prefill run on the MFMA kernels (the sums are given to the selection): three calls on one state (ragged tail,
    resumed mid-chunk, several workspace passes), every selection, output, state element and per-slot sum against the
    oracle; then generation steps."""
    sh = wl.Shape("qscore_mfma", "bf16", 2, 4, 2, d, D, T=0, eta=eta, lam=lam, C=64, seed=0)
    n_fill = (eta + lam) // 64
    cuts = [0, 64 * (n_fill + 3) + 23]
    cuts.append(cuts[-1] + 64 * 3)
    cuts.append(cuts[-1] + 64 * 5 + 7)
    nd = 4
    q, k, v, Wq, Wk = rand_case(900 + kind + d + D, 2, 4, 2, d, D, cuts[-1] + nd, "bf16")
    kw = dict(score_kind=kind)
    layer, o = None, None
    for i in range(3):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o, layer_kw=kw,
                                         workspace_limit=0 if i == 2 else None)
        say("query-dependent scores on the MFMA prefill kernels, call", kind, i, layer.lola_path, rep)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, cuts[3], nd), Wq, Wk)
    say("query-dependent scores on the MFMA prefill kernels, generation steps", rep2)


@pytest.mark.parametrize("g", [1, 2, 3])
def test_mfma_kernels_with_other_group_sizes(g):
    """Multi-head attention (one query head per kv head) and small groups on the MFMA kernels: the
    generation step is built for up to four query rows per stream, the prefill kernels take any."""
    sh = wl.Shape("group", "bf16", 1, 2 * g, 2, 128, 128, T=0, eta=64, lam=64, C=64, seed=0)
    T = 64 * 4 + 21
    q, k, v, Wq, Wk = rand_case(120 + g, 1, 2 * g, 2, 128, 128, T + 16, "bf16")
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk)
    assert layer.lola_path == ("mfma", "mfma")
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, 16), Wq, Wk)
    say("group size", g, rep, rep2)


def test_exp_feature_map():
    sh = wl.Shape("expphi", "f32", 1, 2, 1, 32, 16, T=64, eta=8, lam=6, C=8, seed=0)
    q, k, v, Wq, Wk = rand_case(8, 1, 2, 1, 32, 16, 70, "f32", wscale=0.5)
    kw = dict(phi_kind=orc.PHI_EXP)
    layer, o, rep = P.prefill_parity(sh, q[:, :, :64], k[:, :, :64], v[:, :, :64], Wq, Wk, layer_kw=kw)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, 64, 6), Wq, Wk)
    say("exp phi", rep, rep2)


def test_resume_and_multipass_workspace():
    """prefill(T1); prefill(T2) == prefill(T1+T2) on the GPU too, with a workspace that forces
    several passes, and an update-only call in between matches the oracle's."""
    sh = wl.Shape("resume", "bf16", 2, 4, 2, 64, 64, T=0, eta=16, lam=12, C=16, seed=0)
    q, k, v, Wq, Wk = rand_case(9, 2, 4, 2, 64, 64, 16 * 11 + 5, "bf16")
    cuts = [0, 48, 48 + 64, 16 * 11 + 5]
    layer, o = None, None
    for i in range(3):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o,
                                         with_outputs=(i != 1), workspace_limit=0 if i == 2 else None)
        say("resume part", i, rep)
    # one call over everything gives the same memories
    one = P.make_layer(sh)
    one.prefill(P.to_dev(q, "bf16"), P.to_dev(k, "bf16"), P.to_dev(v, "bf16"), P.w_to_dev(Wq, "bf16"), P.w_to_dev(Wk, "bf16"))
    torch.cuda.synchronize()
    assert torch.equal(P.torch.sort(one.sp_idx, -1).values, torch.sort(layer.sp_idx, -1).values)
    assert torch.allclose(one.H, layer.H, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("lam,phi_kind", [(64, 0), (128, 1), (256, 0)])
def test_8b_shape_resume_ragged_multipass(lam, phi_kind):
    """The MFMA prefill kernels (8B head shape) across call boundaries that are not chunk-aligned:
    the second call starts mid-chunk (its chunks are regular again but offset), the third is
    update-only with a ragged tail, the last runs in several workspace passes."""
    sh = wl.scaled(3, B=1, T=64 * 14 + 29, lam=lam)
    Wq, Wk = wl.weights(sh)
    if phi_kind:     # keep exp(+-z) in a moderate range
        Wq, Wk = wl.store(0.5 * Wq, sh.dtype), wl.store(0.5 * Wk, sh.dtype)
    q, k, v, _ = wl.sequence_inputs(sh)
    cuts = [0, 64 * 5 + 3, 64 * 8 + 3, 64 * 10 + 40, sh.T]
    layer, o = None, None
    for i in range(4):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o,
                                         with_outputs=(i != 2), workspace_limit=0 if i == 3 else None,
                                         layer_kw=dict(phi_kind=phi_kind))
        say("8b resume part", i, rep)


def test_run_time_window_kernels_outputs_on_the_second_stream():
    """The same at a run-time-parameter shape (window 128, budget 192, 256 features, batch 4): the pass is cut into pieces,
    each piece runs the shape-generic leg (window and cache are still filling when the second piece would start at a larger
    budget), the feature kernel and the MFMA evolution, the outputs of a piece on the second stream; against the oracle,
    and bit for bit against a call that stays on one stream."""
    sh = wl.Shape("wide2s", "bf16", 4, 32, 8, 128, 256, T=64 * 40 + 21, eta=128, lam=192, C=64, seed=0)
    q, k, v, Wq, Wk = rand_case(4321, 4, 32, 8, 128, 256, sh.T, "bf16")
    kw = dict(prefill_overlap=1)
    layer, o, rep = P.prefill_parity(sh, q, k, v, Wq, Wk, layer_kw=kw)
    say("two-stream call, run-time window / budget", layer.lola_path, rep)
    dq, dk, dv = P.to_dev(q, "bf16"), P.to_dev(k, "bf16"), P.to_dev(v, "bf16")
    dWq, dWk = P.w_to_dev(Wq, "bf16"), P.w_to_dev(Wk, "bf16")
    ref_layer = P.make_layer(sh)
    ref = ref_layer.prefill(dq, dk, dv, dWq, dWk).clone()
    one = P.make_layer(sh, **kw)
    out = one.prefill(dq, dk, dv, dWq, dWk)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    for name in ("H", "s", "sp_idx", "sp_k", "win_k", "n_tokens"):
        assert torch.equal(getattr(one, name), getattr(ref_layer, name)), name
    P.lb.lola_release_streams()


def test_8b_shape_outputs_on_the_second_stream():
    """A call large enough that the MFMA prefill cuts its pass into pieces and runs the outputs of a
    piece on the library's second stream beside the evolution of the next one (batch 4, 33 chunks
    with a ragged tail: two pieces); every output and all memories against the oracle; then a second
    call on the same state, and work on the caller's stream right behind the call (a copy of the
    outputs) must see all of them."""
    sh = wl.scaled(3, T=64 * 32 + 37 + 64 * 33)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    cut = 64 * 32 + 37
    kw = dict(prefill_overlap=1)
    layer, o, rep = P.prefill_parity(sh, q[:, :, :cut], k[:, :, :cut], v[:, :, :cut], Wq, Wk, layer_kw=kw)
    say("two-stream call 1", rep)
    layer, o, rep = P.prefill_parity(sh, q[:, :, cut:], k[:, :, cut:], v[:, :, cut:], Wq, Wk, layer=layer, oracle=o, layer_kw=kw)
    say("two-stream call 2", rep)
    # the same tokens in one call: the copy enqueued right behind the call holds the finished outputs, and they are
    # bit for bit those of a call that stays on one stream (prefill_overlap = 0)
    dq, dk, dv = P.to_dev(q[:, :, :cut], "bf16"), P.to_dev(k[:, :, :cut], "bf16"), P.to_dev(v[:, :, :cut], "bf16")
    dWq, dWk = P.w_to_dev(Wq, "bf16"), P.w_to_dev(Wk, "bf16")
    ref = P.make_layer(sh).prefill(dq, dk, dv, dWq, dWk).clone()
    one = P.make_layer(sh, **kw)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    for _ in range(3):
        one.reset()
        with torch.cuda.stream(side):
            out = one.prefill(dq, dk, dv, dWq, dWk)
            snap = out.clone()
            out.zero_()
        side.synchronize()
        assert torch.equal(snap, ref)
    # the library's second stream can be destroyed and comes back on the next call that wants it
    from paper_2505_23666_amd import binding as lb
    lb.lola_release_streams()
    one.reset()
    assert torch.equal(one.prefill(dq, dk, dv, dWq, dWk), ref)
    torch.cuda.synchronize()
    lb.lola_release_streams()


def test_8b_shape_budget_256_outputs_on_the_second_stream():
    """Sparse budget 256 at the 8B head shape with the outputs on the second stream: the candidates' features stream
    through LDS in batches requested one ahead, and every piece of the pass starts with a launch of the feature kernel
    of the run-time shapes (the pairs that leave the window in its chunks, the cache slots as it finds them).  Two calls
    with a ragged boundary against the oracle, then the first call again on one stream: bit for bit the same outputs."""
    sh = wl.scaled(3, lam=256, T=64 * 32 + 37 + 64 * 17)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    cut = 64 * 32 + 37
    kw = dict(prefill_overlap=1)
    layer, o, rep = P.prefill_parity(sh, q[:, :, :cut], k[:, :, :cut], v[:, :, :cut], Wq, Wk, layer_kw=kw)
    say("budget 256, two-stream call 1", rep)
    assert layer.lola_path[0] == "mfma"
    layer, o, rep = P.prefill_parity(sh, q[:, :, cut:], k[:, :, cut:], v[:, :, cut:], Wq, Wk, layer=layer, oracle=o, layer_kw=kw)
    say("budget 256, two-stream call 2", rep)
    dq, dk, dv = P.to_dev(q[:, :, :cut], "bf16"), P.to_dev(k[:, :, :cut], "bf16"), P.to_dev(v[:, :, :cut], "bf16")
    dWq, dWk = P.w_to_dev(Wq, "bf16"), P.w_to_dev(Wk, "bf16")
    ref = P.make_layer(sh).prefill(dq, dk, dv, dWq, dWk).clone()
    two = P.make_layer(sh, **kw)
    for _ in range(2):
        two.reset()
        assert torch.equal(two.prefill(dq, dk, dv, dWq, dWk), ref)
    torch.cuda.synchronize()


def test_two_stream_prefill_from_two_host_threads():
    """Two host threads, each with a layer and a stream of its own, call the prefill at the same time; both calls use
    the library's one second stream and its events.  Each result must equal the one the same call gives alone."""
    import threading
    sh = wl.scaled(3, T=64 * 33 + 11)
    Wq, Wk = wl.weights(sh)
    dWq, dWk = P.w_to_dev(Wq, "bf16"), P.w_to_dev(Wk, "bf16")
    cases = []
    for seed in (11, 12):
        q, k, v, _ = wl.sequence_inputs(wl.scaled(3, T=sh.T, seed=seed))
        lay = P.make_layer(sh, prefill_overlap=1)
        dq, dk, dv = P.to_dev(q, "bf16"), P.to_dev(k, "bf16"), P.to_dev(v, "bf16")
        ref = lay.prefill(dq, dk, dv, dWq, dWk).clone()
        torch.cuda.synchronize()
        ref_state = [t.clone() for t in (lay.H, lay.s, lay.sp_idx, lay.win_k)]
        cases.append((lay, dq, dk, dv, ref, ref_state))
    outs, errs = [None, None], []

    def run(i):
        try:
            lay, dq, dk, dv, _, _ = cases[i]
            st = torch.cuda.Stream()
            for _ in range(4):
                lay.reset()
                with torch.cuda.stream(st):
                    outs[i] = lay.prefill(dq, dk, dv, dWq, dWk)
                st.synchronize()
        except Exception as e:   # surfaced in the main thread
            errs.append(e)

    torch.cuda.synchronize()
    th = [threading.Thread(target=run, args=(i,)) for i in range(2)]
    for t in th:
        t.start()
    for t in th:
        t.join()
    assert not errs, errs
    torch.cuda.synchronize()
    for i, (lay, _, _, _, ref, ref_state) in enumerate(cases):
        assert torch.equal(outs[i], ref)
        for got, want in zip((lay.H, lay.s, lay.sp_idx, lay.win_k), ref_state):
            assert torch.equal(got, want)


@pytest.mark.parametrize("lam", [64, 128, 256])
def test_1b_shape_resume_ragged_multipass(lam):
    """The MFMA prefill kernels at the 1B head shape (head_dim 64, 128 features) across call boundaries that are
    not chunk-aligned, an update-only call and a multi-pass workspace; then generation steps (generic kernel)."""
    sh = wl.scaled(2, T=64 * 12 + 21, lam=lam, n_decode=3)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    cuts = [0, 64 * 4 + 5, 64 * 7 + 5, 64 * 9 + 33, sh.T]
    layer, o = None, None
    for i in range(4):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o,
                                         with_outputs=(i != 2), workspace_limit=0 if i == 3 else None)
        say("1b resume part", i, rep)
    assert layer.lola_path[0] == "mfma"
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, sh.T, sh.n_decode), Wq, Wk)
    say("1b decode after prefill", rep2)


def test_bf16_outputs():
    sh = wl.scaled(2, T=256)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    _, _, rep = P.prefill_parity(sh, q, k, v, Wq, Wk, out_dtype="bf16")
    say("bf16 out", rep)


def test_bf16_outputs_on_the_mfma_kernels():
    """bf16 output storage through the MFMA prefill and generation-step kernels (8B head shape)."""
    sh = wl.scaled(3, B=1, T=64 * 5, n_decode=6)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    T = sh.T
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk, out_dtype="bf16")
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, sh.n_decode), Wq, Wk, out_dtype="bf16")
    say("bf16 out, mfma kernels", rep, rep2)
    assert layer.lola_path == ("mfma", "mfma")


def test_empty_prefill_call_changes_nothing():
    """T = 0 is accepted and leaves the memories as they were (checked bit for bit)."""
    sh = wl.scaled(3, B=1, T=64 * 4)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    layer, o, _ = P.prefill_parity(sh, q, k, v, Wq, Wk)
    before = [getattr(layer, n).clone() for n in ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens")]
    e = torch.empty((sh.B, sh.Hkv, 0, sh.d), dtype=torch.bfloat16, device=layer.device)
    eq = torch.empty((sh.B, sh.Hq, 0, sh.d), dtype=torch.bfloat16, device=layer.device)
    out = layer.prefill(eq, e, e.clone(), P.w_to_dev(Wq, sh.dtype), P.w_to_dev(Wk, sh.dtype))
    torch.cuda.synchronize()
    assert out.shape == (sh.B, sh.Hq, 0, sh.d)
    for a, n in zip(before, ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens")):
        assert torch.equal(a, getattr(layer, n)), n


def test_maximum_sizes_generic_family():
    """Largest head and feature dimensions the interface admits (d = 256, D = 512), with a cache larger than the
    window and a chunk that is not a divisor of anything."""
    sh = wl.Shape("maxdims", "bf16", 1, 2, 1, 256, 512, T=75, eta=12, lam=20, C=10, seed=0)
    q, k, v, Wq, Wk = rand_case(77, 1, 2, 1, 256, 512, 75 + 4, "bf16")
    layer, o, rep = P.prefill_parity(sh, q[:, :, :75], k[:, :, :75], v[:, :, :75], Wq, Wk)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, 75, 4), Wq, Wk)
    say("max dims", rep, rep2)


@pytest.mark.parametrize("eta,lam,chunk", [(256, 256, 64), (512, 512, 64), (128, 768, 64), (512, 1024, 128), (512, 1024, 64), (100, 200, 64)],
                         ids=["eta256_lam256", "eta512_lam512", "eta128_lam768", "eta512_lam1024_chunk128", "eta512_lam1024", "eta100_lam200"])
def test_paper_scale_cache_parameters(eta, lam, chunk):
    """Cache parameters of the paper's long-context runs (Sec. 4: the S-NIAH table's window = sparse budget = 256 and
    512, the RULER setting window 128 / budget 768, the LongBench setting window 512 / budget 1024; feature dimension
    2 d = 256, head_dim 128): a prefill with a ragged tail that runs well past the point where the cache is full,
    then generation steps; every output, state element and selection against the oracle."""
    n_full = (eta + lam) // chunk + 5              # chunks until the cache is full, then five scored selections
    T = chunk * n_full + 9
    sh = wl.Shape("paperscale", "bf16", 1, 4, 1, 128, 256, T=T, eta=eta, lam=lam, C=chunk, seed=0)
    q, k, v, Wq, Wk = rand_case(211 + eta + lam, 1, 4, 1, 128, 256, T + 3, "bf16")
    layer, o, rep = P.prefill_parity(sh, q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, 3), Wq, Wk)
    say("paper-scale cache", eta, lam, chunk, layer.lola_path, rep, rep2)
    # chunk 64: the run-time-parameter MFMA kernels; window / budget not in multiples of 64: only the outputs on MFMA
    assert layer.lola_path[0] == ("generic" if chunk != 64 else "mfma" if eta % 64 == 0 and lam % 64 == 0 else "mixed")
    assert rep["scored"] >= 5 and rep2["scored"] - rep["scored"] == 3


def test_run_time_shape_decode_from_cold_start_with_the_work_in_shares():
    """Generation steps from empty memories at a run-time shape with few streams and the optional scratch: the output
    kernel takes the keys in shares from the first step on (one key, then ragged shares, most of them empty at first),
    the update's split forms leave the streams alone while window and cache fill (the shape-generic step takes them),
    then score in shares once the cache is full; every step against the oracle."""
    eta, lam = 64, 512
    sh = wl.Shape("coldwide", "bf16", 1, 4, 2, 128, 256, T=0, eta=eta, lam=lam, C=64, seed=0)
    n = eta + lam + 12
    q, k, v, Wq, Wk = rand_case(77, 1, 4, 2, 128, 256, n, "bf16")
    layer = P.make_layer(sh)
    assert layer.step_scratch is not None
    o = P.make_oracle(sh)
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, 0, n), Wq, Wk)
    say("run-time shape cold decode, work in shares", rep)
    assert rep["scored"] == 2 * 12


@pytest.mark.parametrize("d,D,eta,lam,B,Hkv", [(128, 256, 128, 768, 2, 2), (64, 256, 64, 512, 2, 2), (128, 128, 64, 1024, 2, 2),
                                               (64, 128, 128, 512, 2, 2), (128, 128, 64, 768, 16, 4), (128, 256, 64, 512, 8, 8)])
def test_generation_step_scoring_split_over_workgroups(d, D, eta, lam, B, Hkv):
    """With few streams and a sparse budget of 512 or more the generation step at the run-time shapes scores a stream's
    cached pairs on several workgroups (the scores pass through the optional scratch in the state) and a second launch
    selects and folds; the output kernel likewise takes the keys in shares on several workgroups and a small launch adds
    the shares up.  Same prefill, then generation steps on a layer with the scratch and on one without it (one
    workgroup per stream does everything): every memory equal bit for bit at every step, the outputs equal up to the
    order of the fp32 sums.  (The split form
    is the one the paper-scale cases compare with the oracle.)  With 4 streams every wavefront of the score part takes
    single tiles of 16 pairs; with 64 streams there are not enough compute units for that and it takes pairs of tiles."""
    Hq = 2 * Hkv
    sh = wl.Shape("split", "bf16", B, Hq, Hkv, d, D, T=64 * ((eta + lam) // 64 + 2) + 5, eta=eta, lam=lam, C=64, seed=0)
    nd = 5
    q, k, v, Wq, Wk = rand_case(900 + d + D + eta + lam, B, Hq, Hkv, d, D, sh.T + nd, "bf16")
    dWq, dWk = P.w_to_dev(Wq, "bf16"), P.w_to_dev(Wk, "bf16")
    T = sh.T
    dq, dk, dv = P.to_dev(q[:, :, :T], "bf16"), P.to_dev(k[:, :, :T], "bf16"), P.to_dev(v[:, :, :T], "bf16")
    lays = [P.make_layer(sh, step_scratch=True), P.make_layer(sh, step_scratch=False)]
    assert lays[0].step_scratch is not None and lays[1].step_scratch is None
    for lay in lays:
        lay.prefill(dq, dk, dv, dWq, dWk)
    for i in range(nd):
        sq, sk_, sv = (P.to_dev(np.ascontiguousarray(x[:, :, T + i]), "bf16") for x in (q, k, v))
        outs = [lay.decode_step(sq, sk_, sv, dWq, dWk) for lay in lays]
        torch.cuda.synchronize()
        # (the outputs' sums over the keys are taken in shares with the scratch: same result up to the order of the fp32 sums)
        assert torch.allclose(outs[0], outs[1], rtol=1e-5, atol=2e-6), (i, float((outs[0] - outs[1]).abs().max()))
        for name in ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens"):
            assert torch.equal(getattr(lays[0], name), getattr(lays[1], name)), (i, name)
    say("generation step, scoring split over workgroups", d, D, eta, lam, "equal over", nd, "steps")


@pytest.mark.parametrize("d,D,eta,lam,phi_kind", [(128, 256, 128, 192, 0), (128, 128, 128, 64, 1), (64, 128, 192, 320, 0),
                                                  (64, 256, 64, 128, 1), (128, 128, 64, 512, 0), (128, 128, 192, 0, 0), (64, 256, 128, 0, 1)])
def test_run_time_window_and_budget_on_the_mfma_prefill_kernels(d, D, eta, lam, phi_kind):
    """The MFMA state-evolution and output kernels with run-time window and sparse budget (multiples of 64) at every
    head / feature dimension they are built for, both feature maps.  Three calls on one state: from empty memories with
    a ragged tail, a resumed call that starts mid-chunk (the generic kernel takes the irregular chunks) and one
    processed in several workspace passes; the selection of every chunk is compared; then generation steps."""
    sh = wl.Shape("wide", "bf16", 2, 4, 2, d, D, T=0, eta=eta, lam=lam, C=64, seed=0)
    n_fill = (eta + lam) // 64
    cuts = [0, 64 * (n_fill + 3) + 23]
    cuts.append(cuts[-1] + 64 * 3)
    cuts.append(cuts[-1] + 64 * 6 + 7)
    nd = 3
    q, k, v, Wq, Wk = rand_case(700 + d + D + eta + lam, 2, 4, 2, d, D, cuts[-1] + nd, "bf16", wscale=0.5 if phi_kind else 1.0)
    kw = dict(phi_kind=phi_kind)
    layer, o = None, None
    for i in range(3):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o, layer_kw=kw,
                                         workspace_limit=0 if i == 2 else None)
        assert layer.lola_path[0] == "mfma"
        say("run-time window / budget, call", i, rep)
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, cuts[3], nd), Wq, Wk)
    say("run-time window / budget, generation steps", rep2)


@pytest.mark.parametrize("d,g,phi_kind", [(128, 4, 0), (64, 4, 0), (128, 2, 1)])
def test_no_sparse_cache_on_the_mfma_prefill_kernels(d, g, phi_kind):
    """Sparse budget 0 (the sliding-window + linear-attention base model, appendix "Efficiency Analysis") at the MFMA
    shapes: the state evolution runs split over the value columns of H (scan_nocache_kernel).  Three calls on one
    state: from empty memories with a ragged tail, a resumed call that starts mid-chunk (generic kernels take the
    irregular chunks) and a long one processed in several workspace passes; then generation steps (generic kernel)."""
    sh = wl.Shape("nocache", "bf16", 2, 2 * g, 2, d, 128, T=0, eta=64, lam=0, C=64, seed=0)
    cuts = [0, 64 * 5 + 23, 64 * 5 + 23 + 64 * 3, 64 * 5 + 23 + 64 * 3 + 64 * 11 + 7]
    nd = 5
    q, k, v, Wq, Wk = rand_case(300 + d + g, 2, 2 * g, 2, d, 128, cuts[-1] + nd, "bf16", wscale=0.5 if phi_kind else 1.0)
    kw = dict(phi_kind=phi_kind)
    layer, o = None, None
    for i in range(3):
        a, b = cuts[i], cuts[i + 1]
        layer, o, rep = P.prefill_parity(sh, q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], Wq, Wk, layer=layer, oracle=o, layer_kw=kw,
                                         workspace_limit=0 if i == 2 else None)
        assert layer.lola_path[0] == "mfma"
        say("no sparse cache, call", i, rep)
    # an update-only call, then generation steps
    a = cuts[3]
    rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, a, nd), Wq, Wk)
    say("no sparse cache, generation steps", rep2)


def test_random_small_shapes():
    """Twenty seeded random shapes (both storage types, both feature maps, odd chunk / window / budget
    combinations, ragged lengths, GQA groups 1..4): prefill in two calls, then generation steps."""
    g = wl.rng(424242, 0)
    for case in range(20):
        dtype = "bf16" if case % 2 else "f32"
        d = int(g.choice([32, 64, 128]))
        D = int(g.choice([8, 16, 32, 64, 128]))
        Hkv = int(g.integers(1, 3)); grp = int(g.integers(1, 5)); Hq = Hkv * grp
        B = int(g.integers(1, 3))
        eta = int(g.integers(0, 20)); lam = int(g.integers(0, 20)); C_ = int(g.integers(1, 24))
        T = int(g.integers(1, 90)); nd = int(g.integers(1, 6))
        kind = int(case % 5 == 0)
        say("random shape", case, dict(dtype=dtype, B=B, Hq=Hq, Hkv=Hkv, d=d, D=D, eta=eta, lam=lam, C=C_, T=T, nd=nd, kind=kind))
        sh = wl.Shape(f"rnd{case}", dtype, B, Hq, Hkv, d, D, T, eta, lam, C_, seed=0)
        q, k, v, Wq, Wk = rand_case(5000 + case, B, Hq, Hkv, d, D, T + nd, dtype, wscale=0.5 if kind else 1.0)
        kw = dict(phi_kind=kind)
        cut = T // 2
        layer, o = None, None
        for a_, b_ in ((0, cut), (cut, T)):
            if b_ > a_:
                layer, o, rep = P.prefill_parity(sh, q[:, :, a_:b_], k[:, :, a_:b_], v[:, :, a_:b_], Wq, Wk, layer=layer,
                                                 oracle=o, layer_kw=kw)
        if layer is None:
            layer, o = P.make_layer(sh, **kw), P.make_oracle(sh, **kw)
        rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, nd), Wq, Wk)
        say("   ", rep2)


def test_random_small_shapes_with_options():
    """Sixteen more seeded random shapes with the options switched on at random: restricted queries and
    the query-dependent scores, including windows and budgets of zero."""
    g = wl.rng(777, 0)
    for case in range(16):
        dtype = "bf16" if case % 2 else "f32"
        d = int(g.choice([32, 64])); D = int(g.choice([8, 16, 32, 64]))
        Hkv = int(g.integers(1, 3)); grp = int(g.integers(1, 4)); Hq = Hkv * grp
        B = int(g.integers(1, 3))
        eta = int(g.integers(0, 14)); lam = int(g.integers(0, 14)); C_ = int(g.integers(1, 18))
        T = int(g.integers(2, 70)); nd = int(g.integers(1, 6))
        hide = int(g.integers(0, 4)); sk = int(g.integers(0, 5))
        say("random shape with options", case, dict(dtype=dtype, B=B, Hq=Hq, Hkv=Hkv, d=d, D=D, eta=eta, lam=lam, C=C_, T=T, nd=nd,
                                                   hide=hide, score_kind=sk))
        sh = wl.Shape(f"rndo{case}", dtype, B, Hq, Hkv, d, D, T, eta, lam, C_, seed=0)
        q, k, v, Wq, Wk = rand_case(6000 + case, B, Hq, Hkv, d, D, T + nd, dtype)
        kw = dict(query_hide=hide, score_kind=sk)
        cut = T // 2
        layer, o = None, None
        for a_, b_ in ((0, cut), (cut, T)):
            layer, o, rep = P.prefill_parity(sh, q[:, :, a_:b_], k[:, :, a_:b_], v[:, :, a_:b_], Wq, Wk, layer=layer,
                                             oracle=o, layer_kw=kw)
        rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T, nd), Wq, Wk)
        say("   ", rep2)


def test_random_shapes_of_the_run_time_parameter_kernels():
    """Fourteen seeded random configurations inside the range of the MFMA kernels with run-time window and budget
    (head_dim 64 / 128, 128 / 256 features, window and budget in multiples of 64 including budget 0 and the largest
    budget, groups 1..4, both feature maps, restricted queries and query-dependent scores at random, with and without
    the second stream): prefill in two calls (the second resumes mid-chunk past the full cache), then generation steps."""
    g = wl.rng(31337, 0)
    for case in range(14):
        d = int(g.choice([64, 128])); D = int(g.choice([128, 256]))
        Hkv = int(g.integers(1, 3)); grp = int(g.integers(1, 5)); Hq = Hkv * grp
        B = int(g.integers(1, 3))
        eta = 64 * int(g.integers(1, 5)); lam = 64 * int(g.choice([0, 1, 2, 3, 5, 16]))
        kind = int(g.integers(0, 2)); hide = int(g.choice([0, 0, 1, 2, 3])); sk = int(g.choice([0, 0, 0, 1, 2, 3, 4]))
        if lam == 0 and eta == 64 and D == 128 and sk:   # (that corner stays on the shape-generic evolution: covered elsewhere)
            sk = 0
        n_fill = (eta + lam) // 64
        T1 = 64 * (n_fill + 2) + int(g.integers(1, 64)); T2 = 64 * int(g.integers(1, 4)) + int(g.integers(0, 64)); nd = int(g.integers(2, 5))
        over = int(g.integers(0, 2))
        say("random run-time shape", case, dict(B=B, Hq=Hq, Hkv=Hkv, d=d, D=D, eta=eta, lam=lam, T1=T1, T2=T2, nd=nd, phi=kind,
                                               hide=hide, score_kind=sk, overlap=over))
        sh = wl.Shape(f"rndw{case}", "bf16", B, Hq, Hkv, d, D, 0, eta, lam, 64, seed=0)
        q, k, v, Wq, Wk = rand_case(7000 + case, B, Hq, Hkv, d, D, T1 + T2 + nd, "bf16", wscale=0.5 if kind else 1.0)
        kw = dict(phi_kind=kind, query_hide=hide, score_kind=sk, prefill_overlap=over)
        layer, o = None, None
        for a_, b_ in ((0, T1), (T1, T1 + T2)):
            layer, o, rep = P.prefill_parity(sh, q[:, :, a_:b_], k[:, :, a_:b_], v[:, :, a_:b_], Wq, Wk, layer=layer,
                                             oracle=o, layer_kw=kw)
        rep2 = P.decode_parity(sh, layer, o, *steps(q, k, v, T1 + T2, nd), Wq, Wk)
        say("   ", layer.lola_path, rep, rep2)
    P.lb.lola_release_streams()


def test_generation_steps_replayed_from_a_hip_graph():
    """The library only enqueues kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a generation step can be captured into a HIP graph.  Every replay is
    checked against an eager layer fed the same tokens, with eager work between the replays."""
    sh = wl.scaled(3, B=2, T=64 * 4 + 24)
    T = 64 * 4
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    dWq, dWk = P.w_to_dev(Wq, sh.dtype), P.w_to_dev(Wk, sh.dtype)
    dq, dk, dv = (P.to_dev(x, sh.dtype) for x in steps(q, k, v, T, 24))
    for defer in (0, 8):
        eager, graphed = P.make_layer(sh, fold_defer=defer), P.make_layer(sh, fold_defer=defer)
        for lay in (eager, graphed):
            lay.prefill(None, P.to_dev(k[:, :, :T], sh.dtype), P.to_dev(v[:, :, :T], sh.dtype), None, dWk)
        sq, sk_, sv = torch.empty_like(dq[0]), torch.empty_like(dk[0]), torch.empty_like(dv[0])
        out_g = torch.empty((sh.B, sh.Hq, sh.d), dtype=torch.float32, device=P.DEV)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):       # warm-up outside capture, on the capture stream
            sq.copy_(dq[0]); sk_.copy_(dk[0]); sv.copy_(dv[0])
            graphed.decode_step(sq, sk_, sv, dWq, dWk, out=out_g)
        torch.cuda.current_stream().wait_stream(side)
        ref = eager.decode_step(dq[0], dk[0], dv[0], dWq, dWk)
        torch.cuda.synchronize()
        assert torch.equal(ref, out_g)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            graphed.decode_step(sq, sk_, sv, dWq, dWk, out=out_g)
        for i in range(1, 24):
            sq.copy_(dq[i]); sk_.copy_(dk[i]); sv.copy_(dv[i])
            gr.replay()
            ref = eager.decode_step(dq[i], dk[i], dv[i], dWq, dWk)
            torch.cuda.synchronize()
            assert torch.equal(ref, out_g), f"replay {i} (fold_defer={defer}) differs from the eager step"
        for name in ("H", "s", "sp_idx", "sp_k", "win_k", "n_tokens"):
            assert torch.equal(getattr(eager, name), getattr(graphed, name)), name
        say("graph replays match eager steps, fold_defer", defer)


@pytest.mark.parametrize("g,d,D,eta,lam,sk", [(8, 128, 128, 64, 128, 0), (6, 64, 256, 128, 64, 0), (8, 128, 128, 64, 64, 2), (5, 64, 128, 64, 0, 0)])
def test_generation_step_with_more_than_four_query_heads_per_kv_head(g, d, D, eta, lam, sk):
    """Groups of 5 to 8 query heads per kv head (the fused generation step takes at most 4): update and output kernels with
    run-time window and budget, the output kernel in its 8-row form.  Cold start through window filling, cache filling and
    steady state, a prefill call in between, more steps."""
    sh = wl.Shape("g8", "bf16", 2, 2 * g, 2, d, D, T=0, eta=eta, lam=lam, C=64, seed=0)
    n1, n_pre, n2 = eta + lam + 21, 64 * 2 + 11, 9
    q, k, v, Wq, Wk = rand_case(1500 + g + d, 2, 2 * g, 2, d, D, n1 + n_pre + n2, "bf16")
    kw = dict(score_kind=sk)
    layer, o = P.make_layer(sh, **kw), P.make_oracle(sh, **kw)
    assert layer.lola_path[1] == ("mfma" if lam else "mixed")
    rep = P.decode_parity(sh, layer, o, *steps(q, k, v, 0, n1), Wq, Wk)
    layer, o, rep2 = P.prefill_parity(sh, q[:, :, n1:n1 + n_pre], k[:, :, n1:n1 + n_pre], v[:, :, n1:n1 + n_pre], Wq, Wk,
                                      layer=layer, oracle=o, layer_kw=kw)
    rep3 = P.decode_parity(sh, layer, o, *steps(q, k, v, n1 + n_pre, n2), Wq, Wk)
    say("generation step, group size", g, d, D, eta, lam, sk, rep, rep2, rep3)


def test_three_launch_generation_step_replayed_from_a_hip_graph():
    """The generation step at a run-time-parameter shape (update kernel, shape-generic kernel for streams still filling,
    output kernel) captured into a HIP graph from an empty state: the replays take the streams through window filling,
    cache filling and steady state, each checked against an eager layer fed the same tokens."""
    sh = wl.Shape("graphwide", "bf16", 2, 4, 2, 128, 256, T=0, eta=64, lam=64, C=64, seed=0)
    n = 64 + 64 + 20
    q, k, v, Wq, Wk = rand_case(1234, 2, 4, 2, 128, 256, n, "bf16")
    dWq, dWk = P.w_to_dev(Wq, sh.dtype), P.w_to_dev(Wk, sh.dtype)
    dq, dk, dv = (P.to_dev(x, sh.dtype) for x in steps(q, k, v, 0, n))
    eager, graphed = P.make_layer(sh), P.make_layer(sh)
    assert eager.lola_path[1] == "mfma"
    sq, sk_, sv = torch.empty_like(dq[0]), torch.empty_like(dk[0]), torch.empty_like(dv[0])
    out_g = torch.empty((sh.B, sh.Hq, sh.d), dtype=torch.float32, device=P.DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up outside capture, on the capture stream
        sq.copy_(dq[0]); sk_.copy_(dk[0]); sv.copy_(dv[0])
        graphed.decode_step(sq, sk_, sv, dWq, dWk, out=out_g)
    torch.cuda.current_stream().wait_stream(side)
    ref = eager.decode_step(dq[0], dk[0], dv[0], dWq, dWk)
    torch.cuda.synchronize()
    assert torch.equal(ref, out_g)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        graphed.decode_step(sq, sk_, sv, dWq, dWk, out=out_g)
    for i in range(1, n):
        sq.copy_(dq[i]); sk_.copy_(dk[i]); sv.copy_(dv[i])
        gr.replay()
        ref = eager.decode_step(dq[i], dk[i], dv[i], dWq, dWk)
        torch.cuda.synchronize()
        assert torch.equal(ref, out_g), f"replay {i} differs from the eager step"
    for name in ("H", "s", "sp_idx", "sp_k", "win_k", "n_tokens"):
        assert torch.equal(getattr(eager, name), getattr(graphed, name)), name


def test_prefill_replayed_from_a_hip_graph():
    """A prefill call large enough for the two-stream path, captured into a HIP graph: under capture the library keeps
    everything on the caller's stream.  Every replay (each continues the sequence with the same tokens) is checked
    against an eager layer, which runs the same calls on two streams: the results do not depend on the way a call ran."""
    sh = wl.scaled(3, T=64 * 33)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    dWq, dWk = P.w_to_dev(Wq, sh.dtype), P.w_to_dev(Wk, sh.dtype)
    dq, dk, dv = P.to_dev(q, sh.dtype), P.to_dev(k, sh.dtype), P.to_dev(v, sh.dtype)
    eager, graphed = P.make_layer(sh), P.make_layer(sh)
    out_g = torch.empty((sh.B, sh.Hq, sh.T, sh.d), dtype=torch.float32, device=P.DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up outside capture, on the capture stream (allocates the workspace)
        graphed.prefill(dq, dk, dv, dWq, dWk, out=out_g)
    torch.cuda.current_stream().wait_stream(side)
    ref = eager.prefill(dq, dk, dv, dWq, dWk)
    torch.cuda.synchronize()
    assert torch.equal(ref, out_g)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        graphed.prefill(dq, dk, dv, dWq, dWk, out=out_g)
    for i in range(3):
        out_g.zero_()
        gr.replay()
        ref = eager.prefill(dq, dk, dv, dWq, dWk)
        torch.cuda.synchronize()
        assert torch.equal(ref, out_g), f"replay {i} differs from the eager call"
    for name in ("H", "s", "sp_idx", "sp_k", "win_k", "n_tokens"):
        assert torch.equal(getattr(eager, name), getattr(graphed, name)), name


def test_run_to_run_determinism():
    sh = wl.scaled(3, B=1, T=512)
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    outs = []
    for _ in range(2):
        layer = P.make_layer(sh)
        out = layer.prefill(P.to_dev(q, sh.dtype), P.to_dev(k, sh.dtype), P.to_dev(v, sh.dtype), P.w_to_dev(Wq, sh.dtype), P.w_to_dev(Wk, sh.dtype))
        torch.cuda.synchronize()
        outs.append((out.clone(), layer.H.clone(), layer.sp_idx.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# ---------------------------------------------------------------------------------------------
# the benchmark configurations at full size
# ---------------------------------------------------------------------------------------------
def test_config2_1b_prefill_full():
    sh = wl.CONFIGS[2]
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    t = time.time()
    _, _, rep = P.prefill_parity(sh, q, k, v, Wq, Wk, layer_kw=dict(prefill_overlap=1))
    say("config2 full (all 8 streams, all 4096 x 32 output rows)", rep, f"{time.time() - t:.1f}s")
    assert rep["scored"] == 8 * (4096 // 64 - 2)


def test_config3_8b_prefill_full():
    sh = wl.CONFIGS[3]
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    t = time.time()
    _, _, rep = P.prefill_parity(sh, q, k, v, Wq, Wk, layer_kw=dict(prefill_overlap=1))
    say("config3 full (all 32 streams, all outputs)", rep, f"{time.time() - t:.1f}s")


def test_config5_recall_64k_full():
    """T = 65536 on the GPU for all 8 kv heads; the oracle follows 3 of them (all their outputs)."""
    sh = wl.CONFIGS[5]
    Wq, Wk = wl.weights(sh)
    q, k, v, ex = wl.sequence_inputs(sh)
    t = time.time()
    layer, o, rep = P.prefill_parity(sh, q, k, v, Wq, Wk, hsel=[0, 3, 7], layer_kw=dict(prefill_overlap=1))
    pos = set(int(p) for p in ex["planted_pos"])
    g_frac = np.mean([len(pos & set(layer.sp_idx[0, h].cpu().numpy().tolist())) / len(pos) for h in range(sh.Hkv)])
    o_frac = np.mean([len(pos & set(o.sparse_idx[0, h].tolist())) / len(pos) for h in range(3)])
    say("config5 full", rep, f"planted kept: gpu {g_frac:.3f} (8 heads) oracle {o_frac:.3f} (3 heads)", f"{time.time() - t:.1f}s")


def test_config4_decode_batch64_full():
    """Batch 64, each sequence prefilled with 32768 tokens (update-only call), then generation
    steps.  The oracle follows sequences 0, 21, 42, 63 end to end (prefill + every step)."""
    sh = wl.CONFIGS[4]
    n_steps = int(os.environ.get("LOLA_TEST_DECODE_STEPS", "1024"))
    bsel = [0, 21, 42, 63]
    Wq, Wk = wl.weights(sh)
    layer = P.make_layer(sh)
    o = orc.Oracle(len(bsel), sh.Hq, sh.Hkv, sh.d, sh.D, sh.eta, sh.lam, sh.C)
    dWk = P.w_to_dev(Wk, sh.dtype)
    qd = np.empty((n_steps, sh.B, sh.Hq, sh.d), np.float32)
    kd = np.empty((n_steps, sh.B, sh.Hkv, sh.d), np.float32)
    vd = np.empty((n_steps, sh.B, sh.Hkv, sh.d), np.float32)
    # the GPU prefills the batch in groups of 8 sequences (bounds host memory); the state tensors of
    # a group are views into the batch-64 layer
    t = time.time()
    from concurrent.futures import ThreadPoolExecutor
    grp = 8
    sub = P.make_layer(sh, B=grp)
    ok_, ov_ = {}, {}
    for g0 in range(0, sh.B, grp):
        with ThreadPoolExecutor(8) as ex:
            seqs = list(ex.map(lambda b: wl.decode_batch_sequence(sh, b), range(g0, g0 + grp)))
        kp = np.stack([s[0] for s in seqs]); vp = np.stack([s[1] for s in seqs])
        for i, s in enumerate(seqs):
            qd[:, g0 + i], kd[:, g0 + i], vd[:, g0 + i] = s[2][:n_steps], s[3][:n_steps], s[4][:n_steps]
            if g0 + i in bsel:
                ok_[g0 + i], ov_[g0 + i] = s[0], s[1]
        sub.reset()
        _, trace = sub.prefill(None, P.to_dev(kp, sh.dtype), P.to_dev(vp, sh.dtype), None, dWk, trace=True)
        torch.cuda.synchronize()
        for name in ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens"):
            getattr(layer, name)[g0:g0 + grp].copy_(getattr(sub, name))
        for b in bsel:
            if g0 <= b < g0 + grp:
                ok_[b] = (ok_[b], trace[b - g0].cpu().numpy())
        say(f"  prefilled sequences {g0}..{g0 + grp - 1}  {time.time() - t:.1f}s")
    # oracle prefill of the followed sequences, adopting near-ties from the GPU trace
    kp = np.stack([ok_[b][0] for b in bsel]); vp = np.stack([ov_[b] for b in bsel])
    tr = np.stack([ok_[b][1] for b in bsel])
    o.prefill(None, kp, vp, None, Wk, force_sel=tr, tie_eps=P.TIE_EPS)
    st = o.stats()
    say("config4 oracle prefill", st, f"{time.time() - t:.1f}s")
    assert st["mismatch"] == 0
    P.check_state(P.gpu_state_np(layer, bsel), o, P.TOL[sh.dtype])
    # a second layer in the same state runs the same steps with deferred folds (the mode the benchmark times)
    shadow = P.make_layer(sh, fold_defer=8)
    for name in ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens"):
        getattr(shadow, name).copy_(getattr(layer, name))
    rep = P.decode_parity(sh, layer, o, qd, kd, vd, Wq, Wk, bsel=bsel, shadow=shadow)
    say(f"config4 decode x{n_steps} (sequences {bsel}, every step)", rep, f"{time.time() - t:.1f}s")
