"""lola_prefill_noalloc (the entry point that allocates nothing: its scratch is a static array in the
library's device data) against lola_prefill on the same inputs, through the C ABI: two calls in a
row on one state, the second with a smaller input, on the MFMA kernels and on the generic ones; and a
request beyond the static scratch must be refused before anything is enqueued."""
import numpy as np
import pytest
import torch

import workloads as wl
import parity as P
from paper_2505_23666_amd import binding as lb

pytestmark = pytest.mark.gpu

FIELDS = ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens")


def _rel(a, b):
    a, b = a.double(), b.double()
    return float((a - b).abs().max() / b.abs().max().clamp_min(1e-6))


def _compare(sh, layer_ref, layer_new, out_ref, out_new, tr_ref, tr_new, what):
    _, reg = P.bounds(sh.dtype)
    # same kernels, possibly another split of the chunks into passes: selections and cached rows are exact,
    # floating-point results are held to the regression bound of the parity tests
    assert torch.equal(tr_ref, tr_new), f"{what}: selections differ"
    for name in ("win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens"):
        assert torch.equal(getattr(layer_ref, name), getattr(layer_new, name)), f"{what}: {name}"
    rows = (out_new.double() - out_ref.double()).abs().amax(-1) / out_ref.double().abs().amax(-1).clamp_min(1e-6)
    assert float(rows.max()) <= reg, f"{what}: outputs differ by {float(rows.max()):.3e}"
    assert _rel(layer_new.H, layer_ref.H) <= reg and _rel(layer_new.s, layer_ref.s) <= reg, what
    return float(rows.max())


@pytest.mark.parametrize("name,sh,T1,T2", [
    ("mfma 8B shape", wl.scaled(3, B=2, T=64 * 21 + 23 + 64 * 3 + 9), 64 * 21 + 23, 64 * 3 + 9),
    ("generic fp32", wl.Shape("noalloc32", "f32", 2, 4, 2, 32, 16, T=8 * 9 + 5 + 21, eta=8, lam=6, C=8, seed=0), 8 * 9 + 5, 21),
])
def test_noalloc_prefill_matches_prefill_two_calls_in_a_row(name, sh, T1, T2):
    Wq, Wk = wl.weights(sh)
    q, k, v, _ = wl.sequence_inputs(sh)
    dWq, dWk = P.w_to_dev(Wq, sh.dtype), P.w_to_dev(Wk, sh.dtype)
    ref, new = P.make_layer(sh), P.make_layer(sh)
    assert lb.lib().lola_noalloc_scratch_bytes() == 64 << 20
    for a, b in ((0, T1), (T1, T1 + T2)):     # the second call is the smaller one
        dq, dk, dv = (P.to_dev(np.ascontiguousarray(x[:, :, a:b]), sh.dtype) for x in (q, k, v))
        out_ref, tr_ref = ref.prefill(dq, dk, dv, dWq, dWk, trace=True)
        out_new = torch.empty_like(out_ref)
        _, tr_new = new.prefill(dq, dk, dv, dWq, dWk, out=out_new, trace=True, noalloc=True)
        torch.cuda.synchronize()
        err = _compare(sh, ref, new, out_ref, out_new, tr_ref, tr_new, f"{name}, tokens [{a}, {b})")
        print(f"noalloc {name}: tokens [{a}, {b}) largest output difference {err:.2e}", flush=True)
    # the first call's outputs against the oracle as well (the new entry point on its own, end to end)
    fresh = P.make_layer(sh)
    fresh_out = torch.empty((sh.B, sh.Hq, T1, sh.d), dtype=torch.float32, device=P.DEV)
    dq, dk, dv = (P.to_dev(np.ascontiguousarray(x[:, :, :T1]), sh.dtype) for x in (q, k, v))
    fresh.prefill(dq, dk, dv, dWq, dWk, out=fresh_out, noalloc=True)
    torch.cuda.synchronize()
    o = P.make_oracle(sh)
    y = o.prefill(np.ascontiguousarray(q[:, :, :T1]), np.ascontiguousarray(k[:, :, :T1]), np.ascontiguousarray(v[:, :, :T1]), Wq, Wk)
    tol, reg = P.bounds(sh.dtype)
    err = P.row_rel_err(fresh_out.cpu().numpy(), y).max()
    assert err <= reg, err


def test_noalloc_prefill_refuses_what_does_not_fit():
    sh = wl.scaled(4, T=64)    # batch 64: the copies of 512 streams' caches alone exceed 64 MiB
    layer = P.make_layer(sh)
    full, mn = lb.lola_prefill_workspace_bytes(layer.cfg, 64, False)
    assert mn > 64 << 20
    k = torch.zeros((sh.B, sh.Hkv, 64, sh.d), dtype=torch.bfloat16, device=P.DEV)
    Wk = torch.zeros((sh.Hkv, sh.D // 2, sh.d), dtype=torch.bfloat16, device=P.DEV)
    before = layer.n_tokens.clone()
    with pytest.raises(lb.LolaError, match="static scratch"):
        layer.prefill(None, k, k, None, Wk, noalloc=True)
    torch.cuda.synchronize()
    assert torch.equal(layer.n_tokens, before)     # nothing was enqueued
