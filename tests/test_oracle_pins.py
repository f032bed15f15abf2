"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU involved).

Each test names the passage it pins.  The references below are closed forms, brute force or
library routines (numpy / scipy), never the oracle's own code.
"""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.special import softmax

import workloads as wl
from oracle import lola_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------------------------
# helpers: library-routine statements of the definitions
# ---------------------------------------------------------------------------------------------
def np_phi(W, X, kind=orc.PHI_SOFTMAX):
    """Sec. 2.3 eq. (feature_map) for rows of X; W [d, m]."""
    z = np.asarray(X, np.float64) @ np.asarray(W, np.float64)
    if kind == orc.PHI_EXP:
        return np.concatenate([np.exp(z), np.exp(-z)], axis=-1)
    return np.concatenate([softmax(z, axis=-1), softmax(-z, axis=-1)], axis=-1)


def brute_causal_softmax(q, k, v, g):
    """Sec. 2.1: y_t = sum_{i<=t} alpha_ti v_i, alpha = softmax(q.k / sqrt(d)); q [B,Hq,T,d]."""
    B, Hq, T, d = q.shape
    out = np.zeros((B, Hq, T, d))
    for b in range(B):
        for h in range(Hq):
            kk, vv = k[b, h // g].astype(np.float64), v[b, h // g].astype(np.float64)
            logits = q[b, h].astype(np.float64) @ kk.T / np.sqrt(d)
            logits = np.where(np.tril(np.ones((T, T), bool)), logits, -np.inf)
            out[b, h] = softmax(logits, axis=-1) @ vv
    return out


def rand_inputs(seed, B, Hq, Hkv, d, D, N, wscale=1.0):
    g = wl.rng(seed, 77)
    q = g.standard_normal((B, Hq, N, d)).astype(np.float32)
    k = g.standard_normal((B, Hkv, N, d)).astype(np.float32)
    v = g.standard_normal((B, Hkv, N, d)).astype(np.float32)
    Wq = (wscale * g.standard_normal((Hq, d, D // 2)) / np.sqrt(d)).astype(np.float32)
    Wk = (wscale * g.standard_normal((Hkv, d, D // 2)) / np.sqrt(d)).astype(np.float32)
    return q, k, v, Wq, Wk


def run_decode(o, q, k, v, Wq, Wk, t0, n):
    outs = [o.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], Wq, Wk) for t in range(t0, t0 + n)]
    return np.stack(outs, axis=2)


# ---------------------------------------------------------------------------------------------
# feature map
# ---------------------------------------------------------------------------------------------
def test_phi_hand_values():
    """Sec. 2.3 eq. (feature_map), softmax kind: one non-zero entry W[2][1] = ln 3 of a 3x4 W and
    x = e_2 give z = (0, ln3, 0, 0): softmax(z) = (1,3,1,1)/6, softmax(-z) = (3,1,3,3)/10.
    A transposed W, a swapped half or a wrong sign fails this."""
    W = np.zeros((3, 4), np.float32)
    W[2, 1] = np.log(3.0)
    p = orc.phi(W, [0.0, 0.0, 1.0])
    np.testing.assert_allclose(p, [1 / 6, 3 / 6, 1 / 6, 1 / 6, 0.3, 0.1, 0.3, 0.3], rtol=0, atol=1e-7)
    # x = e_0 sees only zeros of W: uniform
    np.testing.assert_allclose(orc.phi(W, [1.0, 0.0, 0.0]), [0.25] * 8, atol=1e-15)
    # exponential kind of the paper: [exp(z), exp(-z)], z = (0, ln3 * 2, 0, 0) for x = 2 e_2
    p = orc.phi(W, [0.0, 5.0, 2.0], kind=orc.PHI_EXP)
    np.testing.assert_allclose(p, [1, 9, 1, 1, 1, 1 / 9, 1, 1], rtol=1e-6)


@pytest.mark.parametrize("kind", [orc.PHI_SOFTMAX, orc.PHI_EXP])
def test_phi_matches_library_softmax(kind):
    g = wl.rng(5, 1)
    W = (g.standard_normal((7, 5)) / 3).astype(np.float32)
    X = g.standard_normal((4, 7))
    ref = np_phi(W, X, kind)
    for i in range(4):
        np.testing.assert_allclose(orc.phi(W, X[i], kind), ref[i], rtol=1e-12)
    if kind == orc.PHI_SOFTMAX:  # each half is a probability vector
        assert abs(ref[:, :5].sum(-1) - 1).max() < 1e-12 and abs(ref[:, 5:].sum(-1) - 1).max() < 1e-12


# ---------------------------------------------------------------------------------------------
# pin 1: the window covers everything -> plain causal softmax attention (Sec. 2.1)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("C", [1, 5, 64])
def test_full_window_is_causal_softmax_prefill(C):
    B, Hq, Hkv, d, D, T = 2, 4, 2, 8, 8, 37
    q, k, v, Wq, Wk = rand_inputs(11, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=64, lam=3, C_=C)
    out = o.prefill(q, k, v, Wq, Wk)
    np.testing.assert_allclose(out, brute_causal_softmax(q, k, v, Hq // Hkv), rtol=1e-11, atol=1e-13)
    assert np.all(o.H == 0) and np.all(o.s == 0) and np.all(o.sparse_idx == -1)


def test_full_window_is_causal_softmax_decode():
    B, Hq, Hkv, d, D, T = 1, 6, 2, 8, 4, 29
    q, k, v, Wq, Wk = rand_inputs(12, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=T, lam=2, C_=4)
    out = run_decode(o, q, k, v, Wq, Wk, 0, T)
    np.testing.assert_allclose(out, brute_causal_softmax(q, k, v, Hq // Hkv), rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------------------------------------
# restricted-query ablation (appendix "Sparse Cache & Linear Attention Ablation"): the memories
# are updated as usual, the query reads only some of them
# ---------------------------------------------------------------------------------------------
def brute_window_softmax(q, k, v, g, first_visible):
    """softmax attention of query t over tokens first_visible[t] .. t (library softmax)."""
    B, Hq, T, d = q.shape
    out = np.zeros((B, Hq, T, d))
    for b in range(B):
        for h in range(Hq):
            kk, vv = k[b, h // g].astype(np.float64), v[b, h // g].astype(np.float64)
            for t in range(T):
                lo = first_visible[t]
                w = softmax(q[b, h, t].astype(np.float64) @ kk[lo:t + 1].T / np.sqrt(d))
                out[b, h, t] = w @ vv[lo:t + 1]
    return out


@pytest.mark.parametrize("eta,lam,C", [(6, 4, 6), (5, 3, 8), (7, 0, 3), (4, 5, 1)])
def test_hide_state_and_sparse_is_sliding_window_attention(eta, lam, C):
    """With both hidden only the window (and the chunk's causal part) is read: decode sees the last
    eta tokens, a prefill query sees from eta tokens before its chunk's start."""
    B, Hq, Hkv, d, D, T = 1, 4, 2, 8, 6, 41
    q, k, v, Wq, Wk = rand_inputs(41, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C, query_hide=orc.HIDE_STATE | orc.HIDE_SPARSE)
    out = run_decode(o, q, k, v, Wq, Wk, 0, T)
    ref = brute_window_softmax(q, k, v, Hq // Hkv, [max(0, t - eta + 1) for t in range(T)])
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)
    o2 = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C, query_hide=3)
    out2 = o2.prefill(q, k, v, Wq, Wk)
    ref2 = brute_window_softmax(q, k, v, Hq // Hkv, [max(0, (t // C) * C - eta) for t in range(T)])
    np.testing.assert_allclose(out2, ref2, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("hide", [1, 2, 3])
def test_hidden_memories_are_still_updated(hide):
    """Hiding changes what the query reads, never the memories."""
    B, Hq, Hkv, d, D, T, eta, lam, C = 2, 4, 2, 8, 6, 50, 5, 4, 7
    q, k, v, Wq, Wk = rand_inputs(42, B, Hq, Hkv, d, D, T + 9)
    a = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C)
    b = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C, query_hide=hide)
    ya, yb = a.prefill(q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk), b.prefill(q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk)
    ya2, yb2 = run_decode(a, q, k, v, Wq, Wk, T, 9), run_decode(b, q, k, v, Wq, Wk, T, 9)
    assert np.array_equal(a.H, b.H) and np.array_equal(a.s, b.s)
    assert np.array_equal(a.sparse_idx, b.sparse_idx) and np.array_equal(a.window_idx, b.window_idx)
    assert not np.allclose(ya[:, :, eta + lam + 3:], yb[:, :, eta + lam + 3:]) and not np.allclose(ya2, yb2)


@pytest.mark.parametrize("hide", [0, 1, 2])
def test_hide_matches_sum_over_the_visible_memories(hide):
    """Decode output rebuilt from the state the oracle reports after the step: the hidden state
    through the library feature map, the listed sparse and window tokens through exp."""
    B, Hq, Hkv, d, D, T, eta, lam, C = 1, 4, 2, 8, 6, 40, 5, 4, 4
    g = Hq // Hkv
    q, k, v, Wq, Wk = rand_inputs(43, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C, query_hide=hide)
    for t in range(T):
        y = o.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], Wq, Wk)
        H, s, sp, wi = o.H, o.s, o.sparse_idx, o.window_idx
        for hq in range(Hq):
            h = hq // g
            qq = q[0, hq, t].astype(np.float64)
            num, den = np.zeros(d), 0.0
            if not hide & 1:
                ph = np_phi(Wq[hq], qq[None])[0]
                num, den = num + ph @ H[0, h], den + ph @ s[0, h]
            toks = [int(i) for i in wi[0, h] if i >= 0] + ([] if hide & 2 else [int(i) for i in sp[0, h] if i >= 0])
            for i in toks:
                w = np.exp(qq @ k[0, h, i].astype(np.float64) / np.sqrt(d))
                num, den = num + w * v[0, h, i].astype(np.float64), den + w
            np.testing.assert_allclose(y[0, hq], num / den, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# query-dependent scores of the scoring ablation (Sec. 4 / appendix "scoring ablation"): every
# token's score written out from the definition, the cache must hold the lambda best tokens that
# have left the window, everything else that left must have been folded
# ---------------------------------------------------------------------------------------------
def brute_query_scores(kind, q, k, Wq, Wk, g, eta, n_seen):
    """Score(k_i) = sum_{t=i}^{i+eta-1} sum_{heads of the group} term(q_t, k_i), over queries t < n_seen."""
    B, Hq, T, d = q.shape
    Hkv = Hq // g
    sc = np.zeros((B, Hkv, T))
    for b in range(B):
        for h in range(Hkv):
            phk = np_phi(Wk[h], k[b, h])
            for r in range(g):
                hq = h * g + r
                phq = np_phi(Wq[hq], q[b, hq])
                w = np.exp(q[b, hq].astype(np.float64) @ k[b, h].astype(np.float64).T / np.sqrt(d))   # [t, i]
                a = phq @ phk.T
                term = {1: (w - a) ** 2, 2: np.abs(w - a), 3: a / w, 4: w}[kind]
                for i in range(T):
                    hi = min(i + eta, n_seen)
                    if hi > i:
                        sc[b, h, i] += term[i:hi, i].sum()
    return sc


@pytest.mark.parametrize("kind", [1, 2, 3, 4])
@pytest.mark.parametrize("mode", ["decode", "prefill", "mixed"])
def test_query_dependent_scores_from_the_definition(kind, mode):
    B, Hq, Hkv, d, D, T, eta, lam, C = 1, 4, 2, 8, 6, 45, 5, 4, 7
    g = Hq // Hkv
    q, k, v, Wq, Wk = rand_inputs(60 + kind, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C, score_kind=kind)
    if mode == "decode":
        run_decode(o, q, k, v, Wq, Wk, 0, T)
    elif mode == "prefill":
        o.prefill(q, k, v, Wq, Wk)
    else:   # chunk boundaries that do not line up with C, then generation steps, then a chunked call again
        o.prefill(q[:, :, :17], k[:, :, :17], v[:, :, :17], Wq, Wk)
        run_decode(o, q, k, v, Wq, Wk, 17, 9)
        o.prefill(q[:, :, 26:], k[:, :, 26:], v[:, :, 26:], Wq, Wk)
    sc = brute_query_scores(kind, q, k, Wq, Wk, g, eta, T)
    left = T - eta                                     # tokens 0 .. left-1 have left the window, their scores are final
    for h in range(Hkv):
        order = sorted(range(left), key=lambda i: (-sc[0, h, i], i))
        keep = sorted(order[:lam])
        assert [int(x) for x in o.sparse_idx[0, h] if x >= 0] == keep
        assert sorted(o.folded(h).tolist()) == sorted(order[lam:])
        _, _, idx = o.pairs(h, 0)
        np.testing.assert_allclose(o.scores(h, 0), sc[0, h, idx], rtol=1e-11)
        _, _, widx = o.pairs(h, 1)                     # window pairs: partial sums over the queries seen so far
        np.testing.assert_allclose(o.scores(h, 1), sc[0, h, widx], rtol=1e-11)
        # the hidden state is the sum over the folded tokens (Sec. 2.2, eq. recurrent_update)
        ph = np_phi(Wk[h], k[0, h])
        fl = order[lam:]
        np.testing.assert_allclose(o.H[0, h], ph[fl].T @ v[0, h, fl].astype(np.float64), rtol=1e-10, atol=1e-12)


def test_query_dependent_scores_need_queries():
    o = orc.Oracle(1, 2, 1, 8, 4, 3, 2, 4, score_kind=orc.SCORE_ATTN)
    q, k, v, Wq, Wk = rand_inputs(70, 1, 2, 1, 8, 4, 8)
    with pytest.raises(Exception):
        o.prefill(None, k, v, None, Wk)


# ---------------------------------------------------------------------------------------------
# pin 2: no window, no sparse cache -> normalised linear attention (Sec. 2.2 eq. lin_attn_forward)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [orc.PHI_SOFTMAX, orc.PHI_EXP])
def test_empty_caches_is_linear_attention(kind):
    B, Hq, Hkv, d, D, T = 2, 4, 2, 6, 10, 23
    q, k, v, Wq, Wk = rand_inputs(13, B, Hq, Hkv, d, D, T, wscale=0.7)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=0, lam=0, C_=1, phi_kind=kind)
    out = run_decode(o, q, k, v, Wq, Wk, 0, T)
    g = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            pk = np_phi(Wk[h // g], k[b, h // g], kind)          # [T, D]
            pq = np_phi(Wq[h], q[b, h], kind)
            Hc = np.cumsum(pk[:, :, None] * v[b, h // g].astype(np.float64)[:, None, :], axis=0)  # [T, D, d]
            sc = np.cumsum(pk, axis=0)
            ref = np.einsum("tf,tfj->tj", pq, Hc) / np.einsum("tf,tf->t", pq, sc)[:, None]
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(o.H[0, 0], np_phi(Wk[0], k[0, 0], kind).T @ v[0, 0].astype(np.float64), rtol=1e-11)


# ---------------------------------------------------------------------------------------------
# pin 3: lambda = 0 -> sliding window + linear attention base model, closed form
# (appendix "Efficiency Analysis", the lambda = 0 case)
# ---------------------------------------------------------------------------------------------
def swa_la_reference(q, k, v, Wq, Wk, eta, first_visible, g):
    """first_visible(t) = index of the oldest token query t reads by softmax; older ones are folded."""
    B, Hq, T, d = q.shape
    out = np.zeros((B, Hq, T, d))
    for b in range(B):
        for h in range(Hq):
            kk, vv = k[b, h // g].astype(np.float64), v[b, h // g].astype(np.float64)
            pk, pq = np_phi(Wk[h // g], kk), np_phi(Wq[h], q[b, h])
            for t in range(T):
                lo = first_visible(t)
                Hs = pk[:lo].T @ vv[:lo]
                ss = pk[:lo].sum(0)
                w = np.exp(kk[lo:t + 1] @ q[b, h, t].astype(np.float64) / np.sqrt(d))
                out[b, h, t] = (pq[t] @ Hs + w @ vv[lo:t + 1]) / (pq[t] @ ss + w.sum())
    return out


@pytest.mark.parametrize("eta,C", [(4, 4), (6, 4), (3, 5), (8, 8)])
def test_lambda0_prefill_closed_form(eta, C):
    B, Hq, Hkv, d, D, T = 1, 2, 1, 6, 8, 31
    q, k, v, Wq, Wk = rand_inputs(14, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=0, C_=C)
    out = o.prefill(q, k, v, Wq, Wk)
    ref = swa_la_reference(q, k, v, Wq, Wk, eta, lambda t: max(0, (t // C) * C - eta), Hq // Hkv)
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)
    nf = max(0, T - eta)
    pk = np_phi(Wk[0], k[0, 0])
    np.testing.assert_allclose(o.H[0, 0], pk[:nf].T @ v[0, 0, :nf].astype(np.float64), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(o.s[0, 0], pk[:nf].sum(0), rtol=1e-12)


def test_lambda0_decode_closed_form():
    B, Hq, Hkv, d, D, T, eta = 1, 2, 2, 6, 8, 25, 5
    q, k, v, Wq, Wk = rand_inputs(15, B, Hq, Hkv, d, D, T)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=0, C_=4)
    out = run_decode(o, q, k, v, Wq, Wk, 0, T)
    ref = swa_la_reference(q, k, v, Wq, Wk, eta, lambda t: max(0, t - eta + 1), 1)
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# pin 4: the three memories partition the past; H is the sum over exactly the folded pairs
# (abstract / Sec. 3 "Method Overview"; folded pairs stay "indefinitely")
# ---------------------------------------------------------------------------------------------
def check_partition(o, k, v, Wk, n):
    for si in range(o.B * o.Hkv):
        b, h = divmod(si, o.Hkv)
        win = [i for i in o.window_idx[b, h] if i >= 0]
        sp = [i for i in o.sparse_idx[b, h] if i >= 0]
        fo = list(o.folded(si))
        assert sorted(win + sp + fo) == list(range(n)), "lost or duplicated token"
        assert win == list(range(max(0, n - o.eta), n))
        assert len(sp) <= o.lam
        pk = np_phi(Wk[h], k[b, h, fo]) if fo else np.zeros((0, o.D))
        np.testing.assert_allclose(o.H[b, h], pk.T @ v[b, h, fo].astype(np.float64), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(o.s[b, h], pk.sum(0), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("eta,lam,C,T", [(4, 3, 4, 40), (5, 2, 3, 41), (2, 6, 7, 45), (0, 3, 2, 17), (8, 8, 8, 64)])
def test_partition_invariant(eta, lam, C, T):
    B, Hq, Hkv, d, D = 2, 4, 2, 6, 8
    nd = 9
    q, k, v, Wq, Wk = rand_inputs(16, B, Hq, Hkv, d, D, T + nd)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=lam, C_=C)
    o.prefill(q[:, :, :T], k[:, :, :T], v[:, :, :T], Wq, Wk)
    check_partition(o, k, v, Wk, T)
    for t in range(T, T + nd):
        o.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], Wq, Wk)
        check_partition(o, k, v, Wk, t + 1)


# ---------------------------------------------------------------------------------------------
# pin 5: cache-size accounting reproduces the printed compression rates
# ---------------------------------------------------------------------------------------------
def test_cache_size_matches_printed_rates():
    fx = json.load(open(os.path.join(GOLDEN, "cache_compression_rates.json")))
    dk, dv, D = fx["d_k"], fx["d_v"], fx["D"]
    for row in fx["rows"]:
        for t, key in ((2048, "rate_2k"), (4096, "rate_4k")):
            rate = t * (dk + dv) / orc.cache_elems(t, row["eta"], row["lambda"], dk, dv, D)
            assert abs(rate / row[key] - 1) <= fx["rel_tol"], (row, t, rate)
    assert orc.cache_elems(4096, 256, 256, 128, 128, 256) == 229632
    # short contexts: never more than the plain KV cache
    assert orc.cache_elems(100, 256, 256, 128, 128, 256) == 100 * 256


# ---------------------------------------------------------------------------------------------
# pin 6: one selection step maximises the summed SRE over subsets of size lambda (Sec. 3, G_t)
# ---------------------------------------------------------------------------------------------
def test_selection_is_best_subset_decode():
    B, Hq, Hkv, d, D, eta, lam = 1, 1, 1, 5, 6, 3, 4
    N = 40
    q, k, v, Wq, Wk = rand_inputs(17, B, Hq, Hkv, d, D, N)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=lam, C_=2)
    checked = 0
    for t in range(N):
        E = [i for i in o.sparse_idx[0, 0] if i >= 0] + ([t - eta] if t >= eta else [])
        expect = None
        if len(E) > lam:
            sc = {i: o.sre_probe(0, Wk[0], k[0, 0, i], v[0, 0, i]) for i in E}
            best = max(itertools.combinations(E, lam), key=lambda S: sum(sc[i] for i in S))
            expect = sorted(best)
        o.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], Wq, Wk)
        if expect is not None:
            assert [i for i in o.sparse_idx[0, 0] if i >= 0] == expect
            checked += 1
    assert checked > 20


def test_selection_is_best_subset_chunk():
    B, Hq, Hkv, d, D, eta, lam, C = 1, 1, 1, 5, 6, 4, 3, 4
    N = 48
    q, k, v, Wq, Wk = rand_inputs(18, B, Hq, Hkv, d, D, N)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=lam, C_=C)
    for a in range(0, N, C):
        E = [i for i in o.sparse_idx[0, 0] if i >= 0] + list(range(max(0, a - eta), a + C - eta))
        expect = sorted(E)
        if len(E) > lam:
            sc = {i: o.sre_probe(0, Wk[0], k[0, 0, i], v[0, 0, i]) for i in E}
            expect = sorted(max(itertools.combinations(E, lam), key=lambda S: sum(sc[i] for i in S)))
        o.prefill(q[:, :, a:a + C], k[:, :, a:a + C], v[:, :, a:a + C], Wq, Wk)
        assert [i for i in o.sparse_idx[0, 0] if i >= 0] == expect


# ---------------------------------------------------------------------------------------------
# pin 7: constant feature map (W = 0, D = 4) and q = 0: every stored token has weight 1 wherever
# it lives, so the output is the running mean of the values for every eta, lambda, C
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("eta,lam,C", [(0, 0, 1), (3, 0, 3), (3, 2, 3), (4, 5, 2), (1, 1, 1), (5, 3, 7)])
def test_constant_features_running_mean(eta, lam, C):
    B, Hq, Hkv, d, D, T = 1, 2, 1, 3, 4, 26
    g = wl.rng(19, 0)
    v = g.integers(-4, 5, size=(B, Hkv, T, d)).astype(np.float32)
    k = g.standard_normal((B, Hkv, T, d)).astype(np.float32)
    q = np.zeros((B, Hq, T, d), np.float32)
    W0q, W0k = np.zeros((Hq, d, 2), np.float32), np.zeros((Hkv, d, 2), np.float32)
    mean = np.cumsum(v[0, 0].astype(np.float64), 0) / np.arange(1, T + 1)[:, None]
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=lam, C_=C)
    out = run_decode(o, q, k, v, W0q, W0k, 0, T)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], mean, rtol=1e-12, atol=1e-12)
    o = orc.Oracle(B, Hq, Hkv, d, D, eta=eta, lam=lam, C_=C)
    out = o.prefill(q, k, v, W0q, W0k)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], mean, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# pin 8: after exactly one fold the state recalls that pair's value for every key (eq. property
# with a single pair), so SRE(k_f, v_f) = 0 and SRE(k', v') = |v_f - v'|
# ---------------------------------------------------------------------------------------------
def test_single_pair_recall():
    d, D = 5, 6
    q, k, v, Wq, Wk = rand_inputs(20, 1, 1, 1, d, D, 3)
    o = orc.Oracle(1, 1, 1, d, D, eta=0, lam=0, C_=1)
    # empty state: recall is defined as 0, SRE = |v|
    assert abs(o.sre_probe(0, Wk[0], k[0, 0, 1], v[0, 0, 1]) - np.linalg.norm(v[0, 0, 1].astype(np.float64))) < 1e-12
    o.decode_step(q[:, :, 0], k[:, :, 0], v[:, :, 0], Wq, Wk)
    assert list(o.folded(0)) == [0]
    assert o.sre_probe(0, Wk[0], k[0, 0, 0], v[0, 0, 0]) < 1e-12
    want = np.linalg.norm(v[0, 0, 0].astype(np.float64) - v[0, 0, 1].astype(np.float64))
    assert abs(o.sre_probe(0, Wk[0], k[0, 0, 1], v[0, 0, 1]) - want) < 1e-12


# ---------------------------------------------------------------------------------------------
# pin 9: resume invariance; prefill + decode hand-off; fp32 arithmetic stays within 1e-5 of fp64
# ---------------------------------------------------------------------------------------------
def test_resume_invariance():
    B, Hq, Hkv, d, D, eta, lam, C = 2, 4, 2, 6, 8, 4, 3, 4
    T1, T2 = 20, 17
    q, k, v, Wq, Wk = rand_inputs(21, B, Hq, Hkv, d, D, T1 + T2)
    a = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C)
    full = a.prefill(q, k, v, Wq, Wk)
    b = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C)
    o1 = b.prefill(q[:, :, :T1], k[:, :, :T1], v[:, :, :T1], Wq, Wk)
    o2 = b.prefill(q[:, :, T1:], k[:, :, T1:], v[:, :, T1:], Wq, Wk)
    np.testing.assert_array_equal(np.concatenate([o1, o2], 2), full)
    np.testing.assert_array_equal(a.H, b.H)
    np.testing.assert_array_equal(a.sparse_idx, b.sparse_idx)


def test_update_only_prefill_equals_full_prefill_state():
    B, Hq, Hkv, d, D, eta, lam, C, T = 1, 2, 1, 6, 8, 4, 3, 4, 33
    q, k, v, Wq, Wk = rand_inputs(22, B, Hq, Hkv, d, D, T)
    a = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C)
    a.prefill(q, k, v, Wq, Wk)
    b = orc.Oracle(B, Hq, Hkv, d, D, eta, lam, C)
    assert b.prefill(None, k, v, None, Wk) is None
    np.testing.assert_array_equal(a.H, b.H)
    np.testing.assert_array_equal(a.sparse_idx, b.sparse_idx)
    np.testing.assert_array_equal(a.window_idx, b.window_idx)


def test_fp32_arithmetic_within_tolerance_on_config1():
    sh = wl.CONFIGS[1]
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    outs = {}
    for real in ("f64", "f32"):
        o = orc.Oracle(sh.B, sh.Hq, sh.Hkv, sh.d, sh.D, sh.eta, sh.lam, sh.C, real=real)
        y = o.prefill(q[:, :, :sh.T], k[:, :, :sh.T], v[:, :, :sh.T], Wq, Wk)
        yd = run_decode(o, q, k, v, Wq, Wk, sh.T, sh.n_decode)
        outs[real] = (np.concatenate([y, yd], 2), o.sparse_idx.copy(), o.H.copy())
    y64, y32 = outs["f64"][0], outs["f32"][0]
    rel = np.abs(y64 - y32).max(-1) / np.maximum(np.abs(y64).max(-1), 1e-6)
    assert rel.max() < 1e-5
    np.testing.assert_array_equal(outs["f64"][1], outs["f32"][1])


# ---------------------------------------------------------------------------------------------
# pin 10: the hand-worked five-token example
# ---------------------------------------------------------------------------------------------
def _handworked():
    fx = json.load(open(os.path.join(GOLDEN, "handworked_tiny.json")))
    w, v = np.array(fx["w"], np.float64), np.array(fx["v"], np.float32)
    T = len(w)
    k = np.zeros((1, 1, T, 2), np.float32)
    k[0, 0, :, 0] = np.log(w)
    k[0, 0, :, 1] = [0.3, -1.0, 2.0, 0.7, -0.2]    # ignored: q has a zero second component
    q = np.zeros((1, 1, T, 2), np.float32)
    q[..., 0] = 1.0
    W = np.full((1, 2, 1), 0.37, np.float32)          # irrelevant: a single projection gives phi = [1, 1]
    return fx, q, k, v[None, None], W


def test_handworked_decode():
    fx, q, k, v, W = _handworked()
    o = orc.Oracle(1, 1, 1, 2, 2, eta=1, lam=1, C_=1, scale=1.0)
    for t in range(5):
        y = o.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], W, W)
        want = np.array(fx["decode"]["y_num"][t], np.float64) / fx["decode"]["y_den"][t]
        np.testing.assert_allclose(y[0, 0], want, rtol=2e-7)   # ln(w) is stored in float32
        assert [i for i in o.sparse_idx[0, 0] if i >= 0] == fx["decode"]["sparse_after"][t]
        assert list(o.folded(0)) == fx["decode"]["folded_after"][t]


def test_handworked_prefill():
    fx, q, k, v, W = _handworked()
    o = orc.Oracle(1, 1, 1, 2, 2, eta=1, lam=1, C_=1, scale=1.0)
    y = o.prefill(q, k, v, W, W)
    want = np.array(fx["prefill"]["y_num"], np.float64) / np.array(fx["prefill"]["y_den"], np.float64)[:, None]
    np.testing.assert_allclose(y[0, 0], want, rtol=2e-7)
    assert [i for i in o.sparse_idx[0, 0] if i >= 0] == fx["prefill"]["sparse_final"]
    assert [i for i in o.window_idx[0, 0] if i >= 0] == fx["prefill"]["window_final"]
    assert list(o.folded(0)) == fx["prefill"]["folded_final"]
    np.testing.assert_array_equal(o.H[0, 0], [fx["prefill"]["H_row_final"]] * 2)
    np.testing.assert_array_equal(o.s[0, 0], fx["prefill"]["s_final"])


# ---------------------------------------------------------------------------------------------
# the harness feature: adopting another implementation's choice inside a near-tie only
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("gap,adopt", [(1e-6, True), (1e-2, False)])
def test_forced_selection_only_inside_tie_band(gap, adopt):
    # W = 0: SRE = distance to the mean of the folded values.  eta = 0, lambda = 1.
    d = 2
    W0 = np.zeros((1, d, 2), np.float32)
    vals = np.array([[0, 0], [1, 0], [1 + gap, 0], [5, 5]], np.float32)   # token 1 vs 2 differ by `gap`
    k = np.zeros((1, 1, 4, d), np.float32)
    q = np.zeros((1, 1, 4, d), np.float32)
    o = orc.Oracle(1, 1, 1, d, 4, eta=0, lam=1, C_=1)
    o.decode_step(q[:, :, 0], k[:, :, 0], vals[None, None, 0], W0, W0)            # cached (|E| <= lambda)
    o.decode_step(q[:, :, 1], k[:, :, 1], vals[None, None, 1], W0, W0)            # H empty: keep |v| larger = 1, fold 0
    assert list(o.folded(0)) == [0] and o.sparse_idx[0, 0, 0] == 1
    # E = {1, 2}: scores 1 and 1+gap -> the oracle keeps 2.  Another implementation kept 1:
    force = np.array([[[1]]], np.int32)
    o.decode_step(q[:, :, 2], k[:, :, 2], vals[None, None, 2], W0, W0, force_sel=force, tie_eps=1e-4)
    st = o.stats()
    if adopt:
        assert o.sparse_idx[0, 0, 0] == 1 and st["adopted"] == 1 and st["mismatch"] == 0
    else:
        assert o.sparse_idx[0, 0, 0] == 2 and st["adopted"] == 0 and st["mismatch"] == 1


@pytest.mark.parametrize("delta,adopt", [(5e-5, True), (1e-3, False)])
def test_forced_selection_band_is_relative_for_query_dependent_scores(delta, adopt):
    # Attention-weight score (appendix "scoring ablation"), eta = lambda = 1, one query head, scale 1:
    # a key is seen in the window by the query of its own position only, so Score(k_i) = exp(q_i . k_i).
    # Tokens 1 and 2 score e^6 and e^(6 + delta): about 403 apart by 403 * delta.  delta = 5e-5 gives a
    # difference of 0.02: far outside an absolute band of 1e-4, inside the relative band 1e-4 * 403.
    d = 2
    W = np.zeros((1, d, 1), np.float32)
    qx = np.array([0.0, 6.0, 6.0 + delta, 0.0], np.float32)
    q = np.zeros((1, 1, 4, d), np.float32); q[0, 0, :, 0] = qx
    k = np.zeros((1, 1, 4, d), np.float32); k[0, 0, :, 0] = 1.0
    v = np.arange(8, dtype=np.float32).reshape(1, 1, 4, d)
    o = orc.Oracle(1, 1, 1, d, 2, eta=1, lam=1, C_=1, scale=1.0, score_kind=orc.SCORE_ATTN)
    for t in range(2):
        o.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], W, W)
    assert o.sparse_idx[0, 0, 0] == 0                       # token 0 left the window into an empty cache
    o.decode_step(q[:, :, 2], k[:, :, 2], v[:, :, 2], W, W)   # token 1 leaves: e^6 beats e^0
    assert o.sparse_idx[0, 0, 0] == 1 and list(o.folded(0)) == [0]
    # token 2 leaves: the oracle would keep it (larger score); another implementation kept token 1
    force = np.array([[[1]]], np.int32)
    o.decode_step(q[:, :, 3], k[:, :, 3], v[:, :, 3], W, W, force_sel=force, tie_eps=1e-4)
    st = o.stats()
    gap = float(np.exp(np.float64(qx[2])) - np.exp(6.0))
    assert gap > 1e-4                                        # an absolute band would refuse both cases
    if adopt:
        assert o.sparse_idx[0, 0, 0] == 1 and st["adopted"] == 1 and st["mismatch"] == 0
    else:
        assert o.sparse_idx[0, 0, 0] == 2 and st["adopted"] == 0 and st["mismatch"] == 1
