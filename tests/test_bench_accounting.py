"""The algorithmic flop and byte counts bench.py divides by measured times (its roofline figures), against a count made
launch by launch: every iteration's block range, every contraction's 2 M N K and operand sizes, every scan's streams.
CPU only."""
import numpy as np
import pytest

import bench
from paper_2501_17086_amd import synth

W = synth.WORKLOADS


def _count_depth(w, k):
    """An MLP depth stack: iteration `it` recomputes blocks 0 .. L - it; hbp_param_grads recomputes da for all blocks."""
    s = 2 if w.dtype == "bf16" else 4
    L, N, d, f = w.L, w.N, w.d, w.d_ff
    out = dict(vjp1=0.0, vjp2=0.0, dw=0.0, vjp1_bytes=0.0, vjp2_bytes=0.0, dw_bytes=0.0, scan_bytes=0.0)
    S = L * N * d * s
    with_norm = w.norm == "rms"
    out["scan_bytes"] += S * (1 + (1 if w.loss_every_state else 0))                  # w0: (e and) g out
    for it in range(1, min(k, L) + 1):
        for _ in range(L - it + 1):
            out["vjp1"] += 2.0 * N * d * f
            out["vjp1_bytes"] += N * d * s + d * f * s + N * f * s + N * f * s       # g, W2, act', da
            out["vjp2"] += 2.0 * N * f * d
            out["vjp2_bytes"] += N * f * s + f * d * s + N * d * s                   # da, W1, dn
        out["scan_bytes"] += S * (1 + (1 if with_norm else 0) + 1)                   # dn (, y) in, g out
    for _ in range(L):                                                                # parameter gradients
        out["vjp1"] += 2.0 * N * d * f
        out["vjp1_bytes"] += N * d * s + d * f * s + 2 * N * f * s
        out["dw"] += 2 * 2.0 * N * d * f
        out["dw_bytes"] += 2 * (N * d * s + N * f * s + d * f * 4)
    return out


@pytest.mark.parametrize("name,k", [("deep_large", 2), ("transformer_mlp", 3), ("resnet_like", 1), ("resnet_like", 40)])
def test_depth_stack_counts(name, k):
    w = W[name]
    got, want = bench.algorithmic_work(w, k), _count_depth(w, k)
    for key, v in want.items():
        assert got[key] == pytest.approx(v, rel=1e-12), key


def test_transformer_counts():
    """The alternating stack: per iteration the attention sub-blocks (even l) and MLP sub-blocks (odd l) below L - it + 1."""
    w, k = W["gpt2_paper"], 3
    s, L, N, d, f, T = 2, w.L, w.N, w.d, w.d_ff, w.seq_len
    attn_f = 5 * 2.0 * T * T * (d // w.heads) * (N // T) * w.heads * 0.5
    want = dict(vjp1=0.0, vjp2=0.0, dw=0.0, attn=0.0, attn_bytes=0.0)
    ranges = [range(0, L - it + 1) for it in range(1, k + 1)]
    for it, blocks in enumerate(ranges + [range(L)]):
        last = it == len(ranges)                      # hbp_param_grads: first halves only
        for l in blocks:
            if l % 2 == 0:
                want["vjp1"] += 2.0 * N * d * d       # do = g Wo
                want["attn"] += attn_f
                want["attn_bytes"] += 8.0 * N * d * s
                if not last:
                    want["vjp2"] += 2.0 * N * 3 * d * d
            else:
                want["vjp1"] += 2.0 * N * d * f
                if not last:
                    want["vjp2"] += 2.0 * N * f * d
    want["dw"] = (L // 2) * (2 * 2.0 * N * d * f + 2.0 * N * d * d + 2.0 * N * 3 * d * d)
    got = bench.algorithmic_work(w, k)
    for key, v in want.items():
        assert got[key] == pytest.approx(v, rel=1e-12), key


def test_recurrent_counts():
    """The RNN along time: one weight set, rows = steps x batch; iteration `it` covers steps 0 .. T - it."""
    w, k = W["gated_rnn"], 2
    L, N, d, f = w.L, w.N, w.d, w.d_ff
    vjp = sum(2.0 * N * d * f * (L - it + 1) for it in range(1, k + 1))
    got = bench.algorithmic_work(w, k)
    assert got["vjp2"] == pytest.approx(vjp)
    assert got["vjp1"] == pytest.approx(vjp + 2.0 * N * d * f * L)
    assert got["dw"] == pytest.approx(2 * 2.0 * N * L * d * f + 2.0 * N * L * f * w.d_in)


def test_published_peaks():
    assert bench.PEAK_MFMA_BF16_TFLOPS == 2500.0 and bench.PEAK_HBM_GBS == 8000.0


def test_more_than_one_gpu_is_refused_with_a_message():
    """bench.py runs on one GPU: any other --gpus exits with status 2 and says why, before anything touches a GPU."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
