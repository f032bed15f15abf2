#!/usr/bin/env python3
"""Benchmark of the LoLA layer on one MI355X.

Headline figure (the JSON line's `value`): tokens/s per layer of the 8B-shaped generation step,
batch 64, every sequence's memories initialised by prefilling 32768 seeded N(0,1) tokens; one
"step" is one `lola_decode_step` call over the whole batch (window eviction, self-recall scoring,
top-lambda reselection, state fold, outputs).  The calls cycle over `--layers` independent copies
of the layer state so that the working set (about 80 MiB per layer) is streamed from HBM rather
than served from the 256 MB last-level cache, as it would be in a 32-layer model.

Also reported in the same line: `roofline` (algorithmic bytes of one decode launch over its
measured duration, against 8 TB/s), `prefill` (8B-shaped chunked prefill, B=4 x 4096 tokens:
tokens/s per layer and algorithmic TFLOP/s against the bf16 MFMA peak) and `cpu_baseline` (the
CPU oracle timed on a bounded sample of the same decode workload on this machine's cores).

Everything is synthetic and seeded (see workloads.py); inputs are resident in HBM before the
timed region starts.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def decode_alg_bytes(sh, out_bytes):
    """Bytes one generation step must move per (sequence, kv head), from the layer's definition:
    read window and sparse K,V and the slot indices, read and write H, read and write s, read the
    new pair, write it to its ring slot, write one sparse slot (pair + index), read the group's
    queries, write their outputs."""
    e = 2  # bf16
    d, D, eta, lam, g = sh.d, sh.D, sh.eta, sh.lam, sh.g
    per_stream = (2 * eta * d * e + 2 * lam * d * e + lam * 4 + 2 * D * d * 4 + 2 * D * 4 + 2 * d * e + 2 * d * e
                  + (2 * d * e + 4) + g * d * e + g * d * out_bytes)
    weights = (sh.Hq + sh.Hkv) * d * sh.m * e
    return per_stream, per_stream * sh.B * sh.Hkv + weights


def decode_deferred_bytes(sh, out_bytes, R=8):
    """Bytes per launch of the step as timed with deferred folds (fold_defer = R): H and s are written on one step in R,
    the list of folded pairs (phi and v in fp32) is read every step (R / 2 + 1/2 pairs on average) and one pair is
    appended; everything else as in decode_alg_bytes."""
    per_stream, _ = decode_alg_bytes(sh, out_bytes)
    d, D = sh.d, sh.D
    pair = (D + d) * 4
    per_stream += -(D * d * 4 + D * 4) + (D * d * 4 + D * 4) // R + pair * (R + 1) // 2 + pair
    weights = (sh.Hq + sh.Hkv) * d * sh.m * 2
    return per_stream, per_stream * sh.B * sh.Hkv + weights


def prefill_alg_flops(sh):
    """Multiply-adds x 2 of one chunk of one stream in steady state, from the equations."""
    g, C_, d, D, m, lam, eta = sh.g, sh.C, sh.d, sh.D, sh.m, sh.lam, sh.eta
    nq, nE, nk = g * C_, lam + C_, lam + eta + C_
    per_chunk = 2 * (nq * d * m + nE * d * m + 2 * nq * nk * d + nq * D * d + nE * D * d + C_ * D * d)
    return per_chunk, per_chunk * (sh.T // C_) * sh.B * sh.Hkv


def extras(torch, wl, lb, dev, only=None):
    """Side measurements: one prefill call with outputs and a run of generation steps per mode, bf16, seeded N(0,1)
    inputs; tokens/s per layer from HIP events.  Not the headline metric: context for the rows built beside it."""
    def to_dev(x):
        return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).to(dev).view(torch.bfloat16)

    def run(label, B, Hq, Hkv, d, D, eta, lam, Cc, T, n_dec, **kw):
        if only and only not in label:
            return None
        g = wl.rng(11, 3)
        mk = lambda *shape: to_dev(wl.store(g.standard_normal(shape, dtype=np.float32), "bf16"))
        q, k, v = mk(B, Hq, T, d), mk(B, Hkv, T, d), mk(B, Hkv, T, d)
        Wq = to_dev(wl.store((g.standard_normal((Hq, D // 2, d), dtype=np.float32) / np.sqrt(d)).astype(np.float32), "bf16"))
        Wk = to_dev(wl.store((g.standard_normal((Hkv, D // 2, d), dtype=np.float32) / np.sqrt(d)).astype(np.float32), "bf16"))
        qd, kd, vd = mk(n_dec, B, Hq, d), mk(n_dec, B, Hkv, d), mk(n_dec, B, Hkv, d)
        lay = lb.LolaLayer(B, Hq, Hkv, d, D, eta, lam, Cc, dtype="bf16", out_dtype="f32", device=dev, **kw)
        out = torch.empty((B, Hq, T, d), dtype=torch.float32, device=dev)
        res = {"mode": label, "shape": f"B{B} Hq{Hq} Hkv{Hkv} d{d} D{D} eta{eta} lambda{lam} C{Cc}", "kernels": lay.lola_path}
        times = []
        for r in range(3):
            lay.reset()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); lay.prefill(q, k, v, Wq, Wk, out=out); e1.record()
            torch.cuda.synchronize()
            if r:
                times.append(e0.elapsed_time(e1))
        ms = float(np.mean(times))
        res["prefill_tokens"] = B * T
        res["prefill_ms"] = round(ms, 3)
        res["prefill_tokens_per_s_per_layer"] = round(B * T / (ms * 1e-3), 1)
        o1 = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
        for i in range(4):
            lay.decode_step(qd[i], kd[i], vd[i], Wq, Wk, out=o1)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(4, n_dec):
            lay.decode_step(qd[i], kd[i], vd[i], Wq, Wk, out=o1)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (n_dec - 4)
        res["decode_us_per_step"] = round(us, 2)
        res["decode_tokens_per_s_per_layer"] = round(B / (us * 1e-6), 1)
        log(f"[extras] {label}: {res['shape']} {res['kernels']}: prefill {res['prefill_tokens_per_s_per_layer'] / 1e6:.3f} M tokens/s/layer "
            f"({ms:.2f} ms), decode {us:.1f} us/step = {res['decode_tokens_per_s_per_layer'] / 1e6:.4f} M tokens/s/layer")
        return res

    def per_chunk(label, eta, lam, D, B=4, Hq=32, Hkv=8, d=128):
        """Update-only prefill calls of 4 096 and of 8 192 tokens: the difference over the 64 extra chunks is the state
        evolution's time per regular chunk with nothing else on the chip."""
        if only and only not in label:
            return None
        g = wl.rng(11, 3)
        mk = lambda *shape: to_dev(wl.store(g.standard_normal(shape, dtype=np.float32), "bf16"))
        Wk = to_dev(wl.store((g.standard_normal((Hkv, D // 2, d), dtype=np.float32) / np.sqrt(d)).astype(np.float32), "bf16"))
        lay = lb.LolaLayer(B, Hq, Hkv, d, D, eta, lam, 64, dtype="bf16", out_dtype="f32", device=dev)
        ms = []
        for T in (4096, 8192):
            k, v = mk(B, Hkv, T, d), mk(B, Hkv, T, d)
            ts = []
            for r in range(3):
                lay.reset()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); lay.prefill(None, k, v, None, Wk); e1.record()
                torch.cuda.synchronize()
                if r:
                    ts.append(e0.elapsed_time(e1))
            ms.append(float(np.mean(ts)))
        us = (ms[1] - ms[0]) * 1e3 / 64
        res = {"mode": label, "shape": f"B{B} Hq{Hq} Hkv{Hkv} d{d} D{D} eta{eta} lambda{lam} C64", "kernels": lay.lola_path,
               "update_only_ms_T4096": round(ms[0], 3), "update_only_ms_T8192": round(ms[1], 3), "evolution_us_per_chunk": round(us, 2)}
        log(f"[extras] {label}: {res['shape']} {res['kernels']}: update-only prefill {ms[0]:.2f} ms at T 4096, {ms[1]:.2f} ms at T 8192 "
            f"-> {us:.1f} us per regular chunk")
        return res

    rows = []
    s8 = dict(B=4, Hq=32, Hkv=8, d=128, D=128, eta=64, lam=128, Cc=64, T=2048, n_dec=68)
    rows.append(run("8B shape, self-recall error (reference point)", **s8))
    rows.append(run("1B shape (head_dim 64, lambda 64), deferred folds", B=16, Hq=32, Hkv=8, d=64, D=128, eta=64, lam=64, Cc=64, T=2048,
                    n_dec=68, fold_defer=8))
    rows.append(run("8B shape, batch 16, deferred folds", B=16, Hq=32, Hkv=8, d=128, D=128, eta=64, lam=128, Cc=64, T=2048, n_dec=68,
                    fold_defer=8))
    rows.append(run("8B shape, batch 128, deferred folds (two rounds of workgroups per launch)", B=128, Hq=32, Hkv=8, d=128, D=128, eta=64, lam=128,
                    Cc=64, T=1024, n_dec=68, fold_defer=8))
    rows.append(run("8B shape, batch 256, deferred folds (four rounds of workgroups per launch)", B=256, Hq=32, Hkv=8, d=128, D=128, eta=64, lam=128,
                    Cc=64, T=512, n_dec=68, fold_defer=8))
    rows.append(run("8B shape, queries do not read the sparse cache", **s8, query_hide=2))
    rows.append(run("8B shape, queries do not read the hidden state", **s8, query_hide=1, fold_defer=8))
    rows.append(run("8B shape, attention-weight score (kind 4)", **s8, score_kind=4))
    rows.append(run("8B shape, squared weight-error score (kind 1)", **s8, score_kind=1))
    long = dict(B=4, Hq=32, Hkv=8, d=128, D=256, Cc=64, T=2048, n_dec=36, prefill_overlap=1)
    rows.append(run("long-context cache parameters eta=lambda=256, D=2d", eta=256, lam=256, **long))
    rows.append(run("long-context cache parameters eta=lambda=512, D=2d", eta=512, lam=512, **long))
    rows.append(run("long-context cache parameters eta=128, lambda=768, D=2d", eta=128, lam=768, **long))
    rows.append(run("long-context cache parameters eta=512, lambda=1024, D=2d", eta=512, lam=1024, **long))
    rows.append(run("batch 32 at the long-context cache parameters eta = lambda = 256, D = 2d", eta=256, lam=256, **dict(long, B=32, T=1024)))
    rows.append(run("no sparse cache (sliding window + linear attention base model), window 64", B=4, Hq=32, Hkv=8, d=128, D=128, eta=64,
                    lam=0, Cc=64, T=2048, n_dec=36))
    rows.append(run("no sparse cache, window 192 (ablation: extended window)", B=4, Hq=32, Hkv=8, d=128, D=128, eta=192, lam=0, Cc=64, T=2048, n_dec=36))
    # the shape of the paper's isolated layer-latency table (Sec. 5 "Efficiency Analysis": batch 2, 32 heads without grouping,
    # head_dim 128, T = 4096, eta = 64, lambda = 128) except for the feature dimension (128 here, 2 d there)
    rows.append(run("layer-latency table shape: batch 2, 32 heads (no grouping), T 4096", B=2, Hq=32, Hkv=32, d=128, D=128, eta=64, lam=128,
                    Cc=64, T=4096, n_dec=36, fold_defer=8))
    rows.append(per_chunk("state evolution per chunk, eta=lambda=256, D=2d", 256, 256, 256))
    rows.append(per_chunk("state evolution per chunk, eta=512, lambda=1024, D=2d", 512, 1024, 256))
    rows.append(per_chunk("state evolution per chunk, eta=128, lambda=512, D=d", 128, 512, 128))
    rows.append(per_chunk("state evolution per chunk, eta=64, lambda=256, D=d", 64, 256, 128))
    rows.append(per_chunk("state evolution per chunk, eta=64, lambda=128, D=d", 64, 128, 128))
    return {"metric": "LoLA layer side modes, tokens/s/layer", "data": "synthetic", "dtype": "bf16", "rows": [r for r in rows if r]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--layers", type=int, default=32, help="independent layer-state copies cycled by the decode loop")
    ap.add_argument("--prefill-tokens", type=int, default=32768, help="tokens prefilled per sequence before decoding")
    ap.add_argument("--prefill-reps", type=int, default=5)
    ap.add_argument("--fold-defer", type=int, default=8, choices=(0, 8),
                    help="deferred folds of the generation step (include/lola.h, lola_config.fold_defer); the other mode is "
                         "timed as a side leg")
    ap.add_argument("--skip-alt", action="store_true", help="skip the side leg that times the other fold mode")
    ap.add_argument("--extras", action="store_true",
                    help="instead of the benchmark proper, time the layer's other modes (restricted queries, query-dependent "
                         "scores, the paper's long-context cache parameters) on small seeded workloads and print one JSON line")
    ap.add_argument("--extras-only", default=None, help="with --extras: run only the rows whose label contains this text")
    ap.add_argument("--skip-prefill", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB device copy (known traffic, calibrates the HBM byte counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the layer shards over (batch, kv head) with no exchange, and this "
              "build has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2505_23666_amd import binding as lb

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.extras:
        print(json.dumps(extras(torch, wl, lb, dev, args.extras_only)), flush=True)
        return
    sh = wl.scaled(4, T=args.prefill_tokens)
    K, W, L = args.steps, args.warmup, args.layers

    def to_dev(x):
        return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).to(dev).view(torch.bfloat16)

    Wq, Wk = wl.weights(sh)
    dWq, dWk = to_dev(Wq.transpose(0, 2, 1)), to_dev(Wk.transpose(0, 2, 1))   # library layout [H, m, d]

    # ---- state initialisation: update-only prefill of every sequence, 8 sequences at a time ----
    t0 = time.time()
    layers = [lb.LolaLayer(sh.B, sh.Hq, sh.Hkv, sh.d, sh.D, sh.eta, sh.lam, sh.C, dtype="bf16", out_dtype="f32", device=dev,
                           fold_defer=args.fold_defer) for _ in range(L)]
    # layer copy l takes l % 8 untimed steps first, so that the copies' lists of deferred folds have every length and
    # one launch in eight of ANY timed window writes H back (all copies in step would hide the write-backs between windows)
    stagger = 8 if args.fold_defer else 1
    n_tok = (K + W + L - 1) // L + stagger
    qd = np.empty((n_tok, sh.B, sh.Hq, sh.d), np.float32)
    kd = np.empty((n_tok, sh.B, sh.Hkv, sh.d), np.float32)
    vd = np.empty((n_tok, sh.B, sh.Hkv, sh.d), np.float32)
    grp = 8
    sub = lb.LolaLayer(grp, sh.Hq, sh.Hkv, sh.d, sh.D, sh.eta, sh.lam, sh.C, dtype="bf16", out_dtype="f32", device=dev)
    fields = ("H", "s", "win_k", "win_v", "sp_k", "sp_v", "sp_idx", "sp_count", "n_tokens")
    shd = wl.scaled(4, T=args.prefill_tokens, n_decode=n_tok)
    prefill_ms = 0.0
    for g0 in range(0, sh.B, grp):
        with ThreadPoolExecutor(8) as ex:
            seqs = list(ex.map(lambda b: wl.decode_batch_sequence(shd, b), range(g0, g0 + grp)))
        kp = to_dev(np.stack([s[0] for s in seqs]))
        vp = to_dev(np.stack([s[1] for s in seqs]))
        for i, s in enumerate(seqs):
            qd[:, g0 + i], kd[:, g0 + i], vd[:, g0 + i] = s[2], s[3], s[4]
        sub.reset()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        sub.prefill(None, kp, vp, None, dWk)
        e1.record()
        torch.cuda.synchronize()
        prefill_ms += e0.elapsed_time(e1)
        for name in fields:
            getattr(layers[0], name)[g0:g0 + grp].copy_(getattr(sub, name))
        del kp, vp
    for l in range(1, L):
        for name in fields:
            getattr(layers[l], name).copy_(getattr(layers[0], name))
    torch.cuda.synchronize()
    log(f"[setup] {sh.B} sequences x {sh.T} tokens prefilled (update-only) in {prefill_ms:.1f} ms GPU time; "
        f"{L} layer copies; {time.time() - t0:.1f}s wall")
    state0 = {name: getattr(layers[0], name).clone() for name in fields} if not args.skip_cpu else None

    dq, dk, dv = to_dev(qd), to_dev(kd), to_dev(vd)
    outs = [torch.empty((sh.B, sh.Hq, sh.d), dtype=torch.float32, device=dev) for _ in range(L)]

    # ---- decode loop: pre-marshalled calls so that the host does not gate the launches ----
    fn = lb.lib().lola_decode_step
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp_ = lambda t: C.c_void_p(t.data_ptr())
    mk_call = lambda l, t: (C.byref(layers[l].cfg), C.byref(layers[l].st), vp_(dq[t]), vp_(dk[t]), vp_(dv[t]), vp_(dWq), vp_(dWk),
                            vp_(outs[l]), stream)
    for l in range(L):
        for t in range(l % stagger):
            rc = fn(*mk_call(l, t))
            assert rc == 0, rc
    torch.cuda.synchronize()
    if args.fold_defer:
        listed = sorted(set(int(layers[l].pend_count[0, 0]) for l in range(L)))
        log(f"[setup] lists of deferred folds at the start of the decode loop hold {listed} pairs over the {L} layer copies")
    calls = [mk_call(i % L, (i % L) % stagger + i // L) for i in range(K + W)]
    def timed(cs, n_warm, n_timed):
        for i in range(n_warm):
            rc = fn(*cs[i])
            assert rc == 0, rc
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        tw = time.perf_counter()
        ev0.record()
        for i in range(n_warm, n_warm + n_timed):
            rc = fn(*cs[i])
            if rc != 0:
                raise RuntimeError(f"lola_decode_step failed: {rc}")
        ev1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - tw, ev0.elapsed_time(ev1)

    t_wall, gpu_ms = timed(calls, W, K)
    ms_per_step = t_wall * 1e3 / K
    value = sh.B * K / t_wall
    per_stream, per_launch = decode_alg_bytes(sh, 4)
    launch_us = gpu_ms * 1e3 / K      # one kernel launch per step
    achieved = per_launch / (launch_us * 1e-6) / 1e9
    log(f"[decode] {K} steps: wall {t_wall * 1e3:.1f} ms, gpu {gpu_ms:.1f} ms, {launch_us:.2f} us/launch, "
        f"{value / 1e6:.3f} M tokens/s/layer, {achieved:.0f} GB/s algorithmic")
    # ---- side leg: the same steps in the other fold mode, on copies of the states as they stand now ----
    decode_alt = None
    if not args.skip_alt:
        alt_R = 0 if args.fold_defer else 8
        Ka = min(K, 256)
        alt = [lb.LolaLayer(sh.B, sh.Hq, sh.Hkv, sh.d, sh.D, sh.eta, sh.lam, sh.C, dtype="bf16", out_dtype="f32", device=dev,
                            fold_defer=alt_R) for _ in range(L)]
        for l in range(L):
            layers[l].flush()
            for name in fields:
                getattr(alt[l], name).copy_(getattr(layers[l], name))
        acalls = [(C.byref(alt[i % L].cfg), C.byref(alt[i % L].st), vp_(dq[(i // L) % n_tok]), vp_(dk[(i // L) % n_tok]),
                   vp_(dv[(i // L) % n_tok]), vp_(dWq), vp_(dWk), vp_(outs[i % L]), stream) for i in range(Ka + W)]
        _, a_ms = timed(acalls, W, Ka)
        decode_alt = {"fold_defer": alt_R, "steps": Ka, "launch_us": round(a_ms * 1e3 / Ka, 3),
                      "tokens_per_s_per_layer": round(sh.B * Ka / (a_ms * 1e-3), 1)}
        log(f"[decode, fold_defer={alt_R}] {Ka} steps: {decode_alt['launch_us']:.2f} us/launch, "
            f"{decode_alt['tokens_per_s_per_layer'] / 1e6:.3f} M tokens/s/layer")
        del alt, acalls
    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    def stored(fname, key):
        """A figure kept in a committed rocprofv3 summary (counter runs are separate from this run)."""
        path = os.path.join(ROOT, "profiles", fname)
        if os.path.exists(path):
            for line in open(path):
                if line.startswith(key + ":"):
                    return float(line.split(":")[1])
        return None

    traffic = stored("decode_8b_b64_hbm_traffic.md", "traffic_bytes_per_launch")
    _, per_launch_timed = decode_deferred_bytes(sh, 4) if args.fold_defer else (per_stream, per_launch)
    moved = per_launch_timed / (launch_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": "profiles/decode_8b_b64_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                  "command, calibrated against a device copy; not a reading of this run)",
                "kernel": lb.lola_kernel_path(layers[0].cfg, 1) + " decode", "launch_us": round(launch_us, 3),
                "alg_bytes_per_launch": per_launch,
                "note": "achieved/frac divide the bytes of the method as written (H rewritten every step) by the measured launch time; "
                        "the timed mode (fold_defer) moves fewer bytes: see timed_mode",
                "timed_mode": {"fold_defer": args.fold_defer, "model_bytes_per_launch": per_launch_timed,
                               "achieved": round(moved, 1), "frac": round(moved / HBM_PEAK_GBS, 4),
                               "measured_traffic_frac": None if traffic is None else
                               round(traffic / (launch_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
                "target": {"frac": 0.60, "launch_us": round(per_launch / (0.6 * HBM_PEAK_GBS * 1e9) * 1e6, 2), "met": bool(achieved / HBM_PEAK_GBS >= 0.6)}}

    # ---- prefill leg (configuration 3) ----
    prefill = None
    prefill_1b = None
    prefill_64k = None
    if not args.skip_prefill:
        del layers[1:], calls
        torch.cuda.empty_cache()

        def prefill_leg(cid, label, reps=None, cpu_sample=None):
            """Times lola_prefill (with outputs) on one of the prefill configurations.  cpu_sample = (sequences, kv heads,
            tokens): the part of the same workload the oracle is timed on."""
            sc = wl.CONFIGS[cid]
            Wq_, Wk_ = wl.weights(sc)
            q_, k_, v_, extra_ = wl.sequence_inputs(sc)
            lay = lb.LolaLayer(sc.B, sc.Hq, sc.Hkv, sc.d, sc.D, sc.eta, sc.lam, sc.C, dtype="bf16", out_dtype="f32", device=dev,
                               prefill_overlap=1)
            a_ = [to_dev(x) for x in (q_, k_, v_, Wq_.transpose(0, 2, 1), Wk_.transpose(0, 2, 1))]
            out_ = torch.empty((sc.B, sc.Hq, sc.T, sc.d), dtype=torch.float32, device=dev)
            times = []
            for r in range((reps or args.prefill_reps) + 1):
                lay.reset()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                lay.prefill(*a_, out=out_)
                e1.record()
                torch.cuda.synchronize()
                if r > 0:
                    times.append(e0.elapsed_time(e1))
            ms = float(np.mean(times))
            _, flops = prefill_alg_flops(sc)
            tf = flops / (ms * 1e-3) / 1e12
            # What bounds the call is the chunk recurrence: one workgroup (one compute unit) per stream evolves the memories
            # chunk by chunk.  Beside the nominal fraction of the chip's MFMA peak: the fraction of the peak of the compute
            # units the recurrence can occupy, and the time per chunk of the serial chain.
            ns_, nch_ = sc.B * sc.Hkv, sc.T // sc.C
            cus = min(256, ns_)
            res = {"workload": label,
                   "tokens_per_s_per_layer": round(sc.B * sc.T / (ms * 1e-3), 1), "ms_per_call": round(ms, 3),
                   "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 5),
                                "traffic": stored("prefill_8b_mfma_kernel_stats.md", f"traffic_bytes_per_call_cfg{cid}"),
                                "traffic_source": "profiles/prefill_8b_mfma_kernel_stats.md (stored rocprofv3 --pmc figure, if any)",
                                "alg_flops_per_call": flops, "alg_bytes_per_call": sc.B * sc.Hq * sc.T * sc.d * (2 + 4) + 2 * sc.B * sc.Hkv * sc.T * sc.d * 2,
                                "kernel": lb.lola_kernel_path(lay.cfg, 0) + " prefill",
                                "streams": ns_, "serial_chunks": nch_, "us_per_chunk_of_the_serial_chain": round(ms * 1e3 / nch_, 2),
                                "frac_of_occupied_cus": round(tf / (MFMA_BF16_PEAK_TFLOPS * cus / 256), 5)}}
            if cpu_sample is not None and not args.skip_cpu:
                from oracle import lola_oracle as orc
                bs, hs, Ts = cpu_sample
                hq = [h_ * sc.g + r_ for h_ in hs for r_ in range(sc.g)]
                o_ = orc.Oracle(len(bs), len(hq), len(hs), sc.d, sc.D, sc.eta, sc.lam, sc.C)
                cut = lambda a, heads: np.ascontiguousarray(a[np.ix_(bs, heads)][:, :, :Ts])
                t1 = time.perf_counter()
                o_.prefill(cut(q_, hq), cut(k_, hs), cut(v_, hs), np.ascontiguousarray(Wq_[hq]), np.ascontiguousarray(Wk_[hs]))
                dt = time.perf_counter() - t1
                # tokens/s/layer of the whole layer (all kv heads): the sample's heads are this fraction of a layer
                frac_layer = len(hs) / sc.Hkv
                res["cpu_baseline"] = {"value": round(len(bs) * Ts * frac_layer / dt, 2), "unit": "tokens/s/layer",
                                       "cores": orc.num_threads(), "kind": "oracle",
                                       "sample": f"prefill with outputs of sequences {list(bs)}, kv heads {list(hs)}, first {Ts} of "
                                                 f"{sc.T} tokens; {dt:.1f}s"}
                log(f"[cpu] oracle on {label}: {res['cpu_baseline']['value']} tokens/s/layer on {res['cpu_baseline']['cores']} threads "
                    f"({res['cpu_baseline']['sample']})")
            log(f"[prefill] {label}: {ms:.2f} ms per call, {res['tokens_per_s_per_layer'] / 1e6:.3f} M tokens/s/layer, "
                f"{tf:.2f} TFLOP/s algorithmic")
            if extra_ and "planted_pos" in extra_:
                # needle-style stand-in: how many of the planted positions the sparse cache holds at the end
                torch.cuda.synchronize()
                pos = set(int(p_) for p_ in extra_["planted_pos"])
                idx = lay.sp_idx.cpu().numpy()
                res["planted_positions_kept"] = round(float(np.mean(
                    [len(pos & set(idx[b_, h_].tolist())) / len(pos) for b_ in range(sc.B) for h_ in range(sc.Hkv)])), 4)
                log(f"[prefill] {label}: fraction of the {len(pos)} planted positions in the sparse cache at the end "
                    f"{res['planted_positions_kept']:.3f} (mean over kv heads)")
            return res

        prefill = prefill_leg(3, "configs[2]: 8B-shape prefill B=4 T=4096 eta=64 lambda=128 C=64 bf16",
                              cpu_sample=([0, 1, 2, 3], list(range(8)), 4096))
        prefill_1b = prefill_leg(2, "configs[1]: 1B-shape prefill B=1 T=4096 head_dim=64 eta=64 lambda=64 C=64 bf16",
                                 cpu_sample=([0], list(range(8)), 4096))
        prefill_64k = prefill_leg(5, "configs[4]: 8B-shape prefill B=1 T=65536 eta=64 lambda=256 C=64 bf16", reps=2,
                                  cpu_sample=([0], [0, 3, 7], 65536))

    # ---- CPU baseline: the oracle on a sample of the same decode workload ----
    cpu = None
    if not args.skip_cpu:
        from oracle import lola_oracle as orc
        n_seq = 8
        o = orc.Oracle(n_seq, sh.Hq, sh.Hkv, sh.d, sh.D, sh.eta, sh.lam, sh.C)
        hs = {n: (state0[n][:n_seq].float() if state0[n].dtype == torch.bfloat16 else state0[n][:n_seq]).cpu().numpy() for n in fields}
        ntk = int(hs["n_tokens"][0, 0])
        for b in range(n_seq):
            o.set_n_tokens(b, ntk)
            for h in range(sh.Hkv):
                cnt = int(hs["sp_count"][b, h])
                wtok = np.arange(max(0, ntk - sh.eta), ntk)
                o.set_stream(b * sh.Hkv + h, hs["H"][b, h].T, hs["s"][b, h], hs["sp_k"][b, h, :cnt], hs["sp_v"][b, h, :cnt],
                             hs["sp_idx"][b, h, :cnt], hs["win_k"][b, h][wtok % sh.eta], hs["win_v"][b, h][wtok % sh.eta], wtok)
        # the sample needs more steps than the GPU loop generated: draw a longer decode tail for these sequences
        n_cpu = 2048
        shc = wl.scaled(4, T=64, n_decode=n_cpu)
        tails = [wl.decode_batch_sequence(shc, 5000 + b) for b in range(n_seq)]
        cq = np.stack([t[2] for t in tails], 1); ck = np.stack([t[3] for t in tails], 1); cv = np.stack([t[4] for t in tails], 1)
        run = lambda t: o.decode_step(cq[t], ck[t], cv[t], Wq, Wk)
        t1 = time.perf_counter(); run(0); run(1); per = (time.perf_counter() - t1) / 2
        n_steps = int(max(2, min(n_cpu - 2, args.cpu_seconds / max(per, 1e-6))))
        t1 = time.perf_counter()
        for t in range(2, 2 + n_steps):
            run(t)
        dt = time.perf_counter() - t1
        cpu = {"value": round(n_seq * n_steps / dt, 2), "unit": "tokens/s/layer", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"{n_steps} generation steps of {n_seq} of the 64 sequences ({n_seq * sh.Hkv} streams), started from the "
                         f"GPU's post-prefill state; {dt:.1f}s"}
        log(f"[cpu] oracle: {cpu['value']} tokens/s/layer on {cpu['cores']} threads")

    line = {
        "metric": "LoLA layer tokens/s (prefill & decode, 8B shape) + % HBM/MFMA peak",
        "value": round(value, 1), "unit": "tokens/s/layer", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[3]: 8B-shape decode, batch 64, 32 q / 8 kv heads, head_dim 128, feat_dim 128, "
                               f"eta 64, lambda 128, bf16 K/V + fp32 H/s, states prefilled with {sh.T} tokens, "
                               f"{L} layer-state copies cycled, fold_defer {args.fold_defer}",
                   "global_batch": sh.B, "prefill_tokens": sh.T, "layer_copies": L, "fold_defer": args.fold_defer},
        "roofline": roofline, "cpu_baseline": cpu, "decode_other_fold_mode": decode_alt, "prefill": prefill, "prefill_1b": prefill_1b,
        "prefill_64k": prefill_64k,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
