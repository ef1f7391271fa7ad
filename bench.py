#!/usr/bin/env python3
"""Benchmark of the Highway-BP backward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--k ITER]

One step = one pass of the whole hot path over one batch of synthetic input
already resident in HBM: hbp_backward(k) (the residual-path-only estimate, then k
iterations of {batched block VJP, residual-path scan}) followed by
hbp_param_grads.  Prints ONE JSON line: backward tokens/s, the roofline of the
dominant kernel class measured live with HIP events on the launch stream, the
other classes' rooflines, throughput and gradient error at k = 1..4 against
exact BP, and the CPU oracle timed on the host cores on a token sample.
The default workload is the largest of the benchmark's stacks that fits one
GPU (deep_large: 96 blocks, d = 2048, d_ff = 8192, 16384 tokens, about 100 GB).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_FP32_VECTOR_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch (read + written) measured with rocprofv3's FETCH_SIZE and WRITE_SIZE counters, scaled by
# what the same counters read for a plain 1 GiB copy: one entry per workload that has such a profile, each naming
# the summary under profiles/ it was copied from (a figure of that run, not of this one); other workloads
# report null.
MEASURED_TRAFFIC = {
    "deep_large": {"source": "profiles/bench_deep_large_hbm_traffic.txt",
                   "vjp1": 1.363e11, "vjp2": 8.394e10, "dw": 3.043e11, "scan": 1.545e10},
    "transformer_mlp": {"source": "profiles/bench_transformer_mlp_hbm_traffic.txt",
                        "vjp1": 2.347e10, "vjp2": 1.131e10, "dw": 2.446e10, "scan": 3.815e9},
    "resnet_like": {"source": "profiles/bench_resnet_like_hbm_traffic.txt",
                    "vjp1": 2.687e9, "vjp2": 1.610e9, "dw": 1.477e9, "scan": 6.481e8},
    "postnorm_mlp": {"source": "profiles/bench_postnorm_mlp_hbm_traffic.txt",
                     "vjp1": 5.608e9, "vjp2": 2.760e9, "dw": 2.832e9, "scan": 1.149e9},
    "gated_rnn": {"source": "profiles/bench_gated_rnn_hbm_traffic.txt",
                  "vjp1": 9.402e8, "vjp2": 9.398e8, "dw": 6.041e8, "scan": 6.420e8},
    "gpt2_paper": {"source": "profiles/bench_gpt2_paper_hbm_traffic.txt",
                   "vjp1": 1.771e9, "vjp2": 5.342e8, "dw": 8.928e8, "attn": 1.620e9, "scan": 1.242e9},
    "roberta_like": {"source": "profiles/bench_roberta_like_hbm_traffic.txt",
                     "vjp1": 9.146e8, "vjp2": 3.333e8, "dw": 5.587e8, "attn": 6.076e8, "scan": 5.378e8},
    "transformer_attn": {"source": "profiles/bench_transformer_attn_hbm_traffic.txt",
                         "vjp1": 5.563e9, "vjp2": 1.432e9, "dw": 2.169e9, "attn": 3.903e9, "scan": 2.458e9},
    "lstm_cell": {"source": "profiles/bench_lstm_cell_hbm_traffic.txt",
                  "vjp1": 3.491e9, "vjp2": 2.148e9, "dw": 1.838e9, "scan": 1.701e9},
}


def storage_bytes(w):
    return 2 if w.dtype == "bf16" else 4


def algorithmic_work(w, k):
    """Flops / bytes per launch class for one step (multiply-add = 2 flops).

    vjp1, vjp2: 2*rows*d*d_ff per launch over the blocks that launch covers
    (iteration `it` recomputes blocks 0 .. L-it only).  dw: the token
    contractions of hbp_param_grads.  scan: every state element is read once
    per input stream and written once."""
    if w.kind == "transformer":
        return transformer_work(w, k)
    s = storage_bytes(w)
    L, N, d, dff = w.L, w.N, w.d, w.d_ff
    per_block = 2.0 * N * d * dff
    iters = min(k, L)
    blocks = sum(L - it + 1 for it in range(1, iters + 1))
    vjp1 = per_block * (blocks + L)        # + the one in hbp_param_grads
    vjp2 = per_block * blocks
    rec = w.kind in ("rnn", "gated", "lstm", "gru")
    dw = 2.0 * per_block * L + (2.0 * N * L * dff * w.d_in if rec else 0.0)
    cellk = w.kind in ("gated", "lstm", "gru")
    hw = d // 2 if w.kind == "lstm" else d             # width the cell's weights act on
    if cellk:                              # no second weight: one parameter contraction (over the hidden part), and
        per_block = 2.0 * N * hw * dff     # the first half of step (i) is elementwise (counted in bytes below)
        dw = per_block * L + 2.0 * N * L * dff * w.d_in
        vjp1 = 0.0
        vjp2 = per_block * blocks
    S = float(L) * N * d
    # per iteration the scan reads dn (+ y with a norm; + e only when a norm sits between
    # the block and the residual path: otherwise e was added by the second contraction)
    e_in_scan = w.loss_every_state and w.norm == "rms"
    lam_tok = 1 if (w.lam == "sigmoid_full" or w.kind in ("gated", "lstm", "gru")) else 0   # coefficients per token: one more stream
    streams_in = 1 + (1 if (w.norm == "rms" or w.post == "rms") else 0) + (1 if e_in_scan else 0) + lam_tok
    mask = S / 8.0 if w.post == "relu" else 0.0       # one bit per element per scan
    scan_iter = S * s * (streams_in + 1) + mask
    scan_init = S * s * (1 + (1 if w.loss_every_state else 0) + lam_tok) + mask
    # bytes the contractions must move: each operand read once, each result written once (weights once per
    # launch when all steps share them).  They decide which roofline binds: at the published peaks the
    # chip's balance is 2500 TFLOP/s / 8 TB/s = 312 flop per byte.
    shared = rec
    aux1 = 0.0 if w.act == "identity" else float(N) * dff * s            # act' (or z) read by the first epilogue
    wbytes = float(d) * dff * s

    def b1(nb):
        return nb * (N * d * s + aux1 + N * dff * s) + (1 if shared else nb) * wbytes

    def b2(nb):
        e_aux = N * d * s if (w.loss_every_state and w.norm == "none") else 0.0
        return nb * (N * dff * s + N * d * s + e_aux) + (1 if shared else nb) * wbytes
    per_it = [L - it + 1 for it in range(1, iters + 1)]
    if w.kind == "gated":                  # reads g, x, [u | c]; writes da [N, 2H]
        def b1(nb):
            return nb * float(N) * (2 * d + 2 * dff) * s
    if w.kind == "gru":                    # elementwise: g, x, [z | r | n] in, da [N,3H] out, tmp in and out; + the H x H product
        def b1(nb):
            return nb * float(N) * (2 * d + 2 * dff + 2 * d) * s
    if w.kind == "lstm":                   # reads g, c, c', the gates (+ e's cell half); writes da [N, 4H] and v's cell half
        def b1(nb):
            return nb * float(N) * (d + 2 * hw + 2 * dff + hw + (hw if w.loss_every_state else 0)) * s

        def b2(nb):
            return nb * float(N) * (dff + hw + (hw if w.loss_every_state else 0)) * s + hw * dff * s
    vjp1_bytes = sum(b1(nb) for nb in per_it) + b1(L)
    vjp2_bytes = sum(b2(nb) for nb in per_it)
    dw_bytes = L * ((1.0 if cellk else 2.0) * N * (hw + dff) * s) \
        + (1 if shared else L) * (1.0 if cellk else 2.0) * hw * dff * 4 \
        + ((L * N * (dff + w.d_in) * s + dff * w.d_in * 4.0) if shared else 0.0)
    return {"vjp1": vjp1, "vjp2": vjp2, "dw": dw, "scan_bytes": scan_init + iters * scan_iter,
            "scan_launches": 1 + iters, "vjp1_bytes": vjp1_bytes, "vjp2_bytes": vjp2_bytes, "dw_bytes": dw_bytes}


def transformer_work(w, k):
    """The same figures for the alternating attention / MLP stack (L = 2 x layers).  An attention sub-block's step (i)
    is: do = g Wo (class vjp1), the attention's own backward (class attn: the five products S, dP, dV, dQ, dK of
    2 T^2 dh flops each per sequence and head, half of that under a causal mask; it reads q, k, v, do, o and writes
    dq, dk, dv), dn = [dq | dk | dv] Wqkv (class vjp2).  An iteration covers blocks 0 .. L-it."""
    s = storage_bytes(w)
    L, N, d, dff, T = w.L, w.N, w.d, w.d_ff, w.seq_len
    iters = min(k, L)
    his = [L - it + 1 for it in range(1, iters + 1)]
    n_attn = [(h + 1) // 2 for h in his]          # even l below l_hi
    n_mlp = [h // 2 for h in his]
    Lh = L // 2
    mlp_f, wo_f, qkv_f = 2.0 * N * d * dff, 2.0 * N * d * d, 2.0 * N * 3 * d * d
    attn_f = 5 * 2.0 * T * T * (d // w.heads) * (N // T) * w.heads * (0.5 if w.causal else 1.0)
    e_aux = N * d * s if (w.loss_every_state and w.norm == "none") else 0.0
    aux1 = 0.0 if w.act == "identity" else float(N) * dff * s
    b1m = lambda nb: nb * (N * d * s + aux1 + N * dff * s + d * dff * s)
    b1a = lambda nb: nb * (2.0 * N * d * s + d * d * s)
    b2m = lambda nb: nb * (N * dff * s + N * d * s + e_aux + d * dff * s)
    b2a = lambda nb: nb * (N * 3 * d * s + N * d * s + e_aux + 3 * d * d * s)
    S = float(L) * N * d
    streams_in = 1 + (1 if (w.norm == "rms" or w.post == "rms") else 0) + (1 if (w.loss_every_state and w.norm == "rms") else 0)
    return {
        "vjp1": mlp_f * (sum(n_mlp) + Lh) + wo_f * (sum(n_attn) + Lh),
        "vjp2": mlp_f * sum(n_mlp) + qkv_f * sum(n_attn),
        "attn": attn_f * (sum(n_attn) + Lh),
        "dw": Lh * (2 * mlp_f + wo_f + qkv_f),
        "vjp1_bytes": sum(b1m(a) for a in n_mlp) + b1m(Lh) + sum(b1a(a) for a in n_attn) + b1a(Lh),
        "vjp2_bytes": sum(b2m(a) for a in n_mlp) + sum(b2a(a) for a in n_attn),
        "attn_bytes": (sum(n_attn) + Lh) * 8.0 * N * d * s,
        "dw_bytes": Lh * (2.0 * N * (d + dff) * s + 2 * d * dff * 4.0 + 2.0 * N * d * s + 4.0 * N * d * s + 4 * d * d * 4.0),
        "scan_bytes": S * s * (1 + (1 if w.loss_every_state else 0)) + iters * S * s * (streams_in + 1),
        "scan_launches": 1 + iters,
    }


def gpu_errors(B, torch, p, ks, gamma=None):
    """Relative L2 error and cosine of the k-iteration estimate against exact BP,
    both from the GPU library, for states 0..L-1 and for all parameter gradients."""
    def sums(a_list, b_list):   # (|a-b|^2, |a|^2, |b|^2, a.b) in fp64, one tensor slab at a time
        acc = torch.zeros(4, dtype=torch.float64, device=a_list[0].device)
        for a, b in zip(a_list, b_list):
            a = a.reshape(-1).double()
            b = b.reshape(-1).double()
            acc += torch.stack([((a - b) ** 2).sum(), (a * a).sum(), (b * b).sum(), (a * b).sum()])
        return [float(v) for v in acc]

    def figures(est, ref):
        d2, a2, b2, ab = sums(est, ref)
        return (d2 / b2) ** 0.5, ab / (a2 * b2) ** 0.5

    B.hbp_exact_backward(p)
    B.hbp_param_grads(p)
    torch.cuda.synchronize()
    L = p.g.shape[0] - 1
    G = p.g[:-1].clone()
    PG = [t.clone() for t in (p.dW1, p.dW2, p.dU, p.dWqkv, p.dWo) if t is not None]
    out = {}
    for k in ks:
        B.hbp_backward(p, k, gamma=gamma)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        s_rel, s_cos = figures([p.g[l] for l in range(L)], [G[l] for l in range(L)])
        pg = [t for t in (p.dW1, p.dW2, p.dU, p.dWqkv, p.dWo) if t is not None]
        if pg[0].dim() == 3:    # per-layer slabs
            est = [t[l] for t in pg for l in range(t.shape[0])]
            ref = [t[l] for t in PG for l in range(t.shape[0])]
        else:
            est, ref = pg, PG
        p_rel, p_cos = figures(est, ref)
        out[str(k)] = {"state_rel_l2": s_rel, "state_cos": s_cos, "param_rel_l2": p_rel, "param_cos": p_cos}
    return out


def time_steps(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_graph(torch, fn, steps):
    """Seconds per replay of fn's launches recorded once into a HIP graph (the library's calls only enqueue
    kernels and device-to-device copies on the current stream, so they can be captured)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    del graph
    return dt


def cpu_baseline(w, k, budget_tokens):
    """The oracle as it stands on a token sample at the workload's full depth and
    widths (cost per token is constant: tokens are independent)."""
    from oracle import hbp_oracle as O
    from paper_2501_17086_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    n = min(budget_tokens, w.N)
    inp = synth.make_inputs(w, tokens=slice(0, n))
    if w.kind == "transformer":      # n is a whole number of sequences
        st = O.Stack(w.kind, w.act, w.norm, inp["W1"], inp["W2"], lam=inp["lam"], eps=w.eps, Wqkv=inp["Wqkv"],
                     Wo=inp["Wo"], T=w.seq_len, heads=w.heads, causal=w.causal, post=w.post)
    elif w.kind in ("gated", "lstm", "gru"):
        st = O.Stack(w.kind, w.act, w.norm, inp["W1"], None, U=inp["U"], L=w.L)
    else:
        st = O.Stack(w.kind, w.act, w.norm, inp["W1"], inp["W2"], lam=inp["lam"], U=inp["U"], eps=w.eps, L=w.L,
                     post=w.post)
    sv = O.forward(st, inp["x0"], inp["xin"])
    t0 = time.perf_counter()
    g = O.hbp_backward(st, sv, inp["e"], k, gamma=w.gamma)
    O.param_grads(st, sv, g, inp["xin"])
    dt = time.perf_counter() - t0
    toks = n * (w.L if w.kind in ("rnn", "gated", "lstm", "gru") else 1)
    return {"value": toks / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} of {w.N} token rows at full L={w.L}, d={w.d}, d_ff={w.d_ff}; "
                      f"hbp_backward(k={k}) + param_grads in {dt:.1f} s (forward untimed)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="deep_large",
                    help="default: the largest single-GPU stack (L=96, d=2048, d_ff=8192, 16384 tokens)")
    ap.add_argument("--k", type=int, default=2, help="Highway-BP iterations in the timed step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the k = 1..4 / exact table")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="token rows of the oracle sample (0 = auto)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="time torch.matmul (the vendor library) on random bf16 operands of the workload's three "
                         "contraction shapes and layouts, one block at a time, and exit: what the same hardware gives "
                         "a tuned library on these shapes (a reference for the roofline fractions, not a target)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run plain 1 GiB device copies and exit (reference for rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no collectives or sharding are built)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2501_17086_amd import binding as B, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()   # fail loudly if the HIP library is not built

    if args.copy_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        print(json.dumps({"copy_bytes_read": a.numel() * 4, "copy_bytes_written": a.numel() * 4, "copies": 10,
                          "GBps_read_plus_write": 2 * a.numel() * 4 / dt / 1e9}))
        return

    w = synth.WORKLOADS[args.workload]
    k = args.k
    if args.vendor_gemm:
        # per block: vjp1  da[N,d_ff] = g[N,d] W2[d,d_ff]; vjp2  dn[N,d] = da[N,d_ff] W1[d_ff,d]; dw  dW2[d,d_ff] = g^T[d,N] z[N,d_ff]
        # (operands as the backward pass holds them: weights untransposed, the token contraction over rows)
        gen = torch.Generator(device="cuda:0").manual_seed(1)
        rnd = lambda *shape: torch.randn(*shape, generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
        N, d, dff = w.N * (w.L if w.kind in ("rnn", "gated", "lstm", "gru") else 1), w.d, w.d_ff
        N = min(N, 32768)
        g_, da_, z_, W1_, W2_ = rnd(N, d), rnd(N, dff), rnd(N, dff), rnd(dff, d), rnd(d, dff)
        res = {}
        for name, fn, flops in (("vjp1", lambda: g_ @ W2_, 2.0 * N * d * dff), ("vjp2", lambda: da_ @ W1_, 2.0 * N * d * dff),
                                ("dw", lambda: g_.t() @ z_, 2.0 * N * d * dff),
                                ("square_8192_nt", None, 0.0)):
            if fn is None:
                a_, b_ = rnd(8192, 8192), rnd(8192, 8192)
                fn, flops = (lambda: a_ @ b_.t()), 2.0 * 8192 ** 3
            t = time_steps(torch, fn, 20, 5)
            res[name] = {"ms": t * 1e3, "TFLOP/s": flops / t / 1e12, "frac_of_2500": flops / t / 1e12 / PEAK_MFMA_BF16_TFLOPS}
        print(json.dumps({"vendor_gemm": "torch.matmul, bf16, randn operands", "workload": w.name, "rows": N, "d": d,
                          "d_ff": dff, "results": res}))
        return
    inp = synth.make_inputs(w)
    p = B.allocate(w, inp)
    B.hbp_forward(p)            # support, untimed: fills the saved forward state
    torch.cuda.synchronize()

    def step():
        B.hbp_backward(p, k)
        B.hbp_param_grads(p)

    # the headline: K steps with the library's per-launch event timing off
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    # the per-class launch durations: the same step, again, with a HIP event pair around every launch on the
    # launch stream (hbp_profile_enable); about 3 s of steps at most
    prof_steps = max(2, min(args.steps, int(3.0 / sec) + 1))
    B.profile_enable(True)
    B.profile_read()
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = B.profile_read()
    B.profile_enable(False)

    tokens = w.tokens
    work = algorithmic_work(w, k)
    ms = {c: prof[c][0] / prof_steps for c in prof}
    launches = {c: prof[c][1] // prof_steps for c in prof}
    traffic = MEASURED_TRAFFIC.get(w.name, {})

    def mfma_roof(cls):
        t = ms[cls] * 1e-3
        ach = work[cls] / t / 1e12 if t > 0 else 0.0
        peak = PEAK_MFMA_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_VECTOR_TFLOPS
        gbs = work[cls + "_bytes"] / t / 1e9 if t > 0 else 0.0
        intensity = work[cls] / work[cls + "_bytes"]
        return {"bound": "mfma" if w.dtype == "bf16" else "alu", "achieved": ach, "peak": peak,
                "unit": "TFLOP/s", "frac": ach / peak, "traffic": traffic.get(cls), "traffic_source": traffic.get("source"),
                "kernel_class": cls,
                # the same launches against the other roofline: below peak / 8 TB/s flop per byte the
                # memory roofline is the one that binds at the published peaks
                "flop_per_byte": intensity, "hbm_GBps": gbs, "hbm_frac": gbs / PEAK_HBM_GBS,
                "binding_at_peaks": "hbm" if intensity < peak * 1e3 / PEAK_HBM_GBS else "mfma",
                "ms_per_step": ms[cls], "launches_per_step": launches[cls],
                "avg_launch_ms": ms[cls] / max(launches[cls], 1)}

    roofs = {c: mfma_roof(c) for c in ("vjp1", "vjp2", "dw") + (("attn",) if w.kind == "transformer" else ())}
    if w.kind in ("gated", "lstm", "gru"):   # step (i)'s first half is elementwise there (GRU: plus an H x H product): memory roofline
        t1 = ms["vjp1"] * 1e-3
        a1 = work["vjp1_bytes"] / t1 / 1e9 if t1 > 0 else 0.0
        roofs["vjp1"] = {"bound": "hbm", "achieved": a1, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": a1 / PEAK_HBM_GBS, "traffic": None, "kernel_class": "vjp1",
                         "ms_per_step": ms["vjp1"], "launches_per_step": launches["vjp1"],
                         "avg_launch_ms": ms["vjp1"] / max(launches["vjp1"], 1)}
    t_scan = ms["scan"] * 1e-3
    ach = work["scan_bytes"] / t_scan / 1e9 if t_scan > 0 else 0.0
    roofs["scan"] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": ach / PEAK_HBM_GBS, "traffic": traffic.get("scan"), "traffic_source": traffic.get("source"),
                     "kernel_class": "scan",
                     "ms_per_step": ms["scan"], "launches_per_step": launches["scan"],
                     "avg_launch_ms": ms["scan"] / max(launches["scan"], 1)}
    dominant = max([c for c in ("vjp1", "vjp2", "dw", "scan", "attn") if c in roofs], key=lambda c: ms[c])

    out = {
        "metric": "Highway-BP backward tokens/s (hbp_backward(k) + hbp_param_grads)",
        "value": tokens / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "k": k, "L": w.L, "tokens": tokens, "d": w.d, "d_ff": w.d_ff,
                   "kind": w.kind, "norm": w.norm, "act": w.act, "gamma": w.gamma,
                   **({"seq_len": w.seq_len, "heads": w.heads, "causal": w.causal} if w.kind == "transformer" else {})},
        "roofline": roofs[dominant],
        "roofline_by_class": roofs,
        "class_ms_per_step": ms,
        # steps run before the tables below: warm-up, timed, and the ones with per-launch events
        "steps_run": {"warmup": args.warmup, "timed": args.steps, "per_launch_events": prof_steps},
    }

    reps = max(3, min(args.steps // 2, int(2.0 / sec) + 1))   # repetitions per line of the tables below
    if not args.no_sweep:
        sweep = {}
        for kk in (1, 2, 3, 4):
            def f(kk=kk):
                B.hbp_backward(p, kk)
                B.hbp_param_grads(p)
            t = time_steps(torch, f, reps, 1)
            sweep[str(kk)] = {"tokens_per_s": tokens / t, "ms": t * 1e3}

        def fe():
            B.hbp_exact_backward(p)
            B.hbp_param_grads(p)
        t = time_steps(torch, fe, reps, 1)
        sweep["exact"] = {"tokens_per_s": tokens / t, "ms": t * 1e3, "launch": "eager"}
        if w.kind in ("rnn", "gated", "lstm", "gru"):
            # Step-by-step backpropagation through time is thousands of short dependent launches: eager, it is
            # bound by the host's launch rate.  The same call sequence recorded once into a HIP graph and replayed
            # is the baseline that speed-ups are quoted against.
            tg = time_graph(torch, fe, reps)
            sweep["exact_graph"] = {"tokens_per_s": tokens / tg, "ms": tg * 1e3, "launch": "hip graph replay"}
            tg2 = time_graph(torch, step, reps)
            sweep["hbp_graph"] = {"k": k, "tokens_per_s": tokens / tg2, "ms": tg2 * 1e3, "launch": "hip graph replay"}
        errs = gpu_errors(B, torch, p, (0, 1, 2, 3, 4))
        for kk, v in errs.items():
            sweep.setdefault(kk, {}).update(v)
        out["per_k"] = sweep
        # the re-split iteration (gamma of the layer's residual connection counted with the block);
        # gamma = 1 is the fixed-point-iteration baseline
        if not ((w.norm == "rms" or w.post == "rms") and w.d > 2048) and w.post != "relu":
            gs = {}
            for gm in (0.2, 0.5, 1.0):
                def fg(gm=gm):
                    B.hbp_backward(p, k, gamma=gm)
                    B.hbp_param_grads(p)
                t = time_steps(torch, fg, reps, 1)
                e = gpu_errors(B, torch, p, (1, 2, 3, 4), gamma=gm)
                gs[str(gm)] = {"ms_at_k": t * 1e3, "k": k,
                               "param_rel_l2": {kk: v["param_rel_l2"] for kk, v in e.items()},
                               "state_rel_l2": {kk: v["state_rel_l2"] for kk, v in e.items()}}
            out["per_gamma"] = gs

    if not args.no_sweep:
        # the initial estimate w^0 by each form of the scan (the paper's Algorithm 1 among them)
        abl = {}
        S_bytes = float(w.L) * w.N * w.d * storage_bytes(w)
        alg_bytes = S_bytes * (1 + (1 if w.loss_every_state else 0)
                               + (1 if (w.lam == "sigmoid_full" or w.kind in ("gated", "lstm", "gru")) else 0))
        algos = ("auto", "sequential")
        if w.post == "none":
            algos += ("chunked",) + (("single_pass",) if w.dtype == "bf16" else ()) + ("hillis_steele",)
        for algo in algos:
            need = B.scan_workspace_size(p.desc, algo)
            if algo in ("auto", "sequential"):       # these run in the workspace of the backward calls
                t = time_steps(torch, lambda: B.hbp_initial_estimate(p, algo), reps, 1)
                abl[algo] = {"ms": t * 1e3, "algorithmic_GBps": alg_bytes / t / 1e9, "workspace_MB": need / 1e6}
                continue
            if need > 16 << 30:
                continue
            ws = torch.zeros(max(need, 16), dtype=torch.uint8, device=p.g.device)
            t = time_steps(torch, lambda: B.hbp_initial_estimate(p, algo, workspace=ws), reps, 1)
            abl[algo] = {"ms": t * 1e3, "algorithmic_GBps": alg_bytes / t / 1e9, "workspace_MB": need / 1e6}
            del ws
        out["scan_forms_w0"] = abl

    if not args.no_sweep:
        # The whole training step (conclusion of the paper: few iterations early, exact backpropagation at the end;
        # cost model T_forward + (k / L) T_backward + O(k log L)): forward, stand-in loss, backward, parameter
        # gradients, optimizer update (AdamW with clipping, fp32 master weights).  Run last: it moves the weights.
        st_o = B.allocate_optim(p, adamw=True)
        tgt = torch.zeros_like(p.e)
        opt = B.make_optim("adamw", lr=1e-4, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.1, clip_norm=1.0, step=1)
        tr = {"optimizer": "adamw, clip 1.0, fp32 master weights"}
        tr["forward_ms"] = time_steps(torch, lambda: B.hbp_forward(p), reps, 1) * 1e3
        tr["loss_ms"] = time_steps(torch, lambda: B.hbp_loss_mse(p, tgt, st_o), reps, 1) * 1e3
        B.hbp_backward(p, k)
        B.hbp_param_grads(p)
        tr["optimizer_ms"] = time_steps(torch, lambda: B.hbp_optimizer_step(p, opt, st_o), reps, 1) * 1e3
        steps_ms = {}
        for kk in (1, 2, 3, -1):
            t = time_steps(torch, lambda kk=kk: B.hbp_train_step(p, kk, tgt, opt, st_o), reps, 1)
            steps_ms["exact" if kk < 0 else str(kk)] = {"ms": t * 1e3, "tokens_per_s": tokens / t}
        tr["train_step"] = steps_ms
        tr["loss_after"] = float(st_o.loss)
        out["training_step"] = tr
        del st_o, tgt

    if not args.no_cpu_baseline:
        # about 10-20 s of oracle work on the GPU machine's host cores
        n = args.cpu_tokens or {"mlp_small_f32": 128, "resnet_like": 8192, "resnet_postact": 8192, "postnorm_mlp": 2048, "transformer_mlp": 2048,
                                "deep_large": 256, "gated_rnn": 16, "gated_rnn_contractive": 16,
                                "gated_rnn_token_gates": 16, "gru_cell": 16, "gru_std_cell": 12, "lstm_cell": 8,
                                "gpt2_paper": 16 * 256, "transformer_attn": 1024, "roberta_like": 8 * 128}.get(w.name, 64)
        out["cpu_baseline"] = cpu_baseline(w, k, n)

    def finite(o):   # JSON has no NaN/Infinity: overflowed error figures become null
        if isinstance(o, float):
            return o if np.isfinite(o) else None
        if isinstance(o, dict):
            return {k: finite(v) for k, v in o.items()}
        if isinstance(o, (list, tuple)):
            return [finite(v) for v in o]
        return o

    print(json.dumps(finite(out)))


if __name__ == "__main__":
    main()
