"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times: the library runs the whole workload; the oracle recomputes a sample of
token rows (tokens are independent in every workload, so a row's result does
not depend on the others) element by element; the parameter gradients, which
sum over all tokens, are checked (i) element by element against the oracle on
runs with the token count cut to what the oracle finishes in seconds (full
depth and widths, the contractions over tokens still split into shares), and
(ii) at the full token count by random projections against a plain contraction
of the library's own g and saved activations."""
import json
import os

import numpy as np
import pytest

from oracle import hbp_oracle as O
from paper_2501_17086_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

W = synth.WORKLOADS


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    from paper_2501_17086_amd import binding
    binding.lib()
    return binding


def _sample_rows(n, count, seed, seq_len=0):
    """Token rows the oracle recomputes; with seq_len > 0 whole sequences (attention couples a sequence's tokens)."""
    r = np.random.default_rng(seed)
    if seq_len:
        seqs = np.unique(np.concatenate([[n // seq_len - 1], r.integers(0, n // seq_len, size=count)]))
        return (seqs[:, None] * seq_len + np.arange(seq_len)[None, :]).reshape(-1)
    rows = np.unique(np.concatenate([[0, n - 1], r.integers(0, n, size=count)]))
    return rows


def _projection_check(p, w, inp, tol):
    """Every parameter gradient of hbp_param_grads (they sum over all tokens, so no token sample can check them)
    against a plain contraction of the library's own g and saved state with a random vector u:
        dW2_l u = sum_n g_{l+1}[n] (z_l[n] . u)        dW1_l u = sum_n da_l[n] (y_l[n] . u)
        dU u    = sum_{l,n} da_l[n] (xin_l[n] . u)
    in fp64.  da is recomputed here from g: for the two-matrix blocks as (g_{l+1} W2_l) (.) act' with torch's
    matmul; for the cells by the oracle's block_preact_grad, step by step.  Per-block weights: three blocks;
    shared weights: the one sum over all steps."""
    gen = torch.Generator(device="cpu").manual_seed(7)
    dev = p.g.device
    L = w.L

    def check(name, dW, left, right):
        """dW [r, c] u  against  left^T (right u), u random in R^c."""
        u = torch.randn(dW.shape[1], generator=gen, dtype=torch.float64).to(dev)
        got, want = dW.double() @ u, left.T @ (right @ u)
        err = float((got - want).norm() / want.norm())
        assert err < tol, f"{w.name}: {name} projection {err:.3e}"

    if w.kind == "transformer":
        # three layers; the gradient of [q | k | v] by torch's autograd through torch's own attention, in fp64, on the
        # library's saved q, k, v and its do = g Wo
        Bn, T, Hn, d = w.N // w.seq_len, w.seq_len, w.heads, w.d
        ys = p.y if p.y is not None else p.x          # the blocks' input: the normed state, or the state itself
        for j in sorted({0, L // 4, L // 2 - 1}):
            gm, zl, ym = p.g[2 * j + 2].double(), p.z[j].double(), ys[2 * j + 1].double()
            da = (gm @ p.W2[j].double()) * p.dphi[j].double()
            check(f"dW2[{j}]", p.dW2[j], gm, zl)
            check(f"dW1[{j}]", p.dW1[j], da, ym)
            ga, ya = p.g[2 * j + 1].double(), ys[2 * j].double()
            check(f"dWo[{j}]", p.dWo[j], ga, p.attn_o[j].double())
            qkv = p.qkv[j].double().reshape(Bn, T, 3, Hn, d // Hn).permute(2, 0, 3, 1, 4).clone().requires_grad_(True)
            o = torch.nn.functional.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=w.causal)
            o.backward((ga @ p.Wo[j].double()).reshape(Bn, T, Hn, d // Hn).permute(0, 2, 1, 3))
            dqkv = qkv.grad.permute(1, 3, 0, 2, 4).reshape(Bn * T, 3 * d)
            check(f"dWqkv[{j}]", p.dWqkv[j], dqkv, ya)
        return
    if w.kind == "mlp":
        for l in sorted({0, L // 2, L - 1}):
            gl, zl = p.g[l + 1].double(), p.z[l].double()
            yl = (p.y if p.y is not None else p.x)[l].double()
            dphi = p.dphi[l].double() if p.dphi is not None else 1.0 - zl * zl
            da = (gl @ p.W2[l].double()) * dphi
            check(f"dW2[{l}]", p.dW2[l], gl, zl)
            check(f"dW1[{l}]", p.dW1[l], da, yl)
        return
    g1 = p.g[1:].reshape(-1, w.d).double()
    xin = p.xin.reshape(-1, w.d_in).double()
    if w.kind == "rnn":
        z = p.z.reshape(-1, w.d_ff).double()
        y = p.x[:-1].reshape(-1, w.d).double()
        da = (g1 @ p.W2.double()) * (1.0 - z * z)
        check("dW2", p.dW2, g1, z)
    else:
        # the cells: da of every step from the oracle's own definition, on the library's g and saved state
        st = H.oracle_stack(w, inp)
        Hh = w.d // 2 if w.kind == "lstm" else w.d
        zz = H.to_np(p.z)
        saved = {"x": H.to_np(p.x), "u": zz[..., :Hh], "c": zz[..., Hh:], "gates": zz, "zrn": zz}
        gg = H.to_np(p.g)
        da_np = np.stack([O.block_preact_grad(st, l, saved, gg[l + 1]) for l in range(L)])
        da = torch.from_numpy(da_np.reshape(-1, w.d_ff)).to(dev)
        y = p.x[:-1][..., w.d - Hh:].reshape(-1, Hh).double()      # the part of the state the weights act on
    if w.kind == "gru":     # the gates' rows see x, the candidate's rows r (.) x
        r = p.z[..., Hh:2 * Hh].reshape(-1, Hh).double()
        check("dW1[z, r]", p.dW1[:2 * Hh], da[:, :2 * Hh], y)
        check("dW1[n]", p.dW1[2 * Hh:], da[:, 2 * Hh:], r * y)
    else:
        check("dW1", p.dW1, da, y)
    check("dU", p.dU, da, xin)


def _subset(w, inp, rows):
    sub = {k: (v[rows] if k in ("x0",) else v[:, rows] if k in ("xin",) else v) for k, v in inp.items()
           if v is not None}
    sub["e"] = inp["e"][:, rows] if w.loss_every_state else inp["e"][rows]
    sub.setdefault("U", None); sub.setdefault("xin", None); sub.setdefault("lam", inp["lam"])
    return sub


def _run(B, w, ks, rows_count, shared_state=False, check_exact=True):
    inp = synth.make_inputs(w)
    p = B.allocate(w, inp)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    rows = _sample_rows(w.N, rows_count, 3, w.seq_len if w.kind == "transformer" else 0)
    sub = _subset(w, inp, rows)
    st = H.oracle_stack(w, sub)
    sv = O.forward(st, sub["x0"], sub["xin"])
    rows_t = torch.from_numpy(rows).to(p.x.device)
    if shared_state:
        # the oracle's forward state of the sampled rows, rounded to storage, replaces the library's
        sv = H.oracle_saved_rounded(w, sv)
        tfm = w.kind == "transformer"
        put = lambda t, a: t.__setitem__((slice(None), rows_t), torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(t.device).to(t.dtype))
        for name, t in (("x", p.x), ("y", p.y), ("z", p.z), ("dphi", p.dphi),
                        ("rpost" if w.post == "rms" else "rinv", p.rinv)):
            if t is not None:
                put(t, sv[name][1::2] if (tfm and name in ("z", "dphi")) else sv[name])
        if tfm:      # the attention sub-blocks' saved state, and their row statistics per (sequence, head, position)
            put(p.qkv, sv["qkv"][0::2])
            put(p.attn_o, sv["o"][0::2])
            seqs = torch.from_numpy(rows[::w.seq_len] // w.seq_len).to(p.x.device)
            stats = np.stack([H.attn_row_stats(st, sv["qkv"][l]) for l in range(0, w.L, 2)])
            lse = p.lse.view(w.L // 2, w.N // w.seq_len, w.heads, w.seq_len)
            lse[:, seqs] = torch.from_numpy(stats.reshape(w.L // 2, len(seqs), w.heads, w.seq_len).astype(np.float32)).to(lse.device)
        if p.mask is not None:
            bits = np.packbits(sv["mask"].astype(np.uint8), axis=-1, bitorder="little")
            p.mask[:, rows_t] = torch.from_numpy(bits).to(p.mask.device)
    tol = H.TOL[w.dtype]
    for k in ks:
        B.hbp_backward(p, k)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        want = H.as_kept(st, sv, O.hbp_backward(st, sv, sub["e"], k, gamma=w.gamma))
        got = H.to_np(p.g[:, rows_t])
        H.assert_close(got, want, tol, f"{w.name} k={k}: g on {len(rows)} sampled rows")
        _projection_check(p, w, inp, 5e-3)
    if check_exact:
        B.hbp_exact_backward(p)
        torch.cuda.synchronize()
        want = H.as_kept(st, sv, O.exact_backward(st, sv, sub["e"]))
        H.assert_close(H.to_np(p.g[:, rows_t]), want, tol, f"{w.name} exact: g on sampled rows")
    del p
    torch.cuda.empty_cache()


def _run_cut(B, w, ks):
    """The workload at full depth and widths with its token count cut: the library against the oracle on EVERY
    element of every state gradient and parameter gradient."""
    inp = synth.make_inputs(w)
    st = H.oracle_stack(w, inp)
    sv = O.forward(st, inp["x0"], inp["xin"])
    p = B.allocate(w, inp)
    B.hbp_forward(p)
    tol = H.TOL[w.dtype]
    for k in ks:
        B.hbp_backward(p, k)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        want = O.hbp_backward(st, sv, inp["e"], k, gamma=w.gamma)
        H.assert_close(H.to_np(p.g), want, tol, f"{w.name} k={k}: g")
        pg = O.param_grads(st, sv, want, inp["xin"])
        for nm, t in (("dW1", p.dW1), ("dW2", p.dW2), ("dU", p.dU), ("dWqkv", p.dWqkv), ("dWo", p.dWo)):
            if t is not None:
                H.assert_close(H.to_np(t), pg[nm], tol, f"{w.name} k={k}: {nm}", row_floor=0.5)
    del p
    torch.cuda.empty_cache()


@pytest.mark.timeout(300)
def test_resnet_like_cut_to_2048_tokens_every_element(B):
    # 32 blocks at d = 512, d_ff = 2048; 2048 tokens: the contractions over tokens run in one share
    _run_cut(B, synth.scaled(W["resnet_like"], name="resnet_like_2048", N=2048), ks=(2,))


@pytest.mark.timeout(300)
def test_gated_rnn_contractive_cut_to_2_rows_every_element(B):
    # T = 4096 steps, 2 batch rows: 8192 rows per contraction over tokens, in 4 shares (split-K); chunked scan
    _run_cut(B, synth.scaled(W["gated_rnn_contractive"], name="gated_rnn_2rows", N=2), ks=(2,))


@pytest.mark.timeout(300)
def test_gru_cell_cut_to_2_rows_every_element(B):
    _run_cut(B, synth.scaled(W["gru_cell"], name="gru_cell_2rows", N=2), ks=(2,))


@pytest.mark.timeout(300)
def test_gru_std_cell_cut_to_2_rows_every_element(B):
    _run_cut(B, synth.scaled(W["gru_std_cell"], name="gru_std_cell_2rows", N=2), ks=(2,))


@pytest.mark.timeout(300)
def test_lstm_cell_cut_to_2_rows_every_element(B):
    _run_cut(B, synth.scaled(W["lstm_cell"], name="lstm_cell_2rows", N=2), ks=(2,))


@pytest.mark.timeout(300)
def test_gpt2_paper_cut_to_8_sequences_every_element(B):
    # 12 layers = 24 sub-blocks at width 256, 4 heads, context 256, gamma = 0.2; 8 of the 128 sequences
    _run_cut(B, synth.scaled(W["gpt2_paper"], name="gpt2_paper_8seq", N=8 * 256), ks=(1, 3))


@pytest.mark.timeout(300)
def test_gpt2_paper_full(B):
    # the paper's GPT-2 configuration whole (128 sequences of 256 tokens); the oracle recomputes the last sequence and
    # three others
    _run(B, W["gpt2_paper"], ks=(1, 3), rows_count=3)


@pytest.mark.timeout(300)
def test_roberta_like_full_shared_state(B):
    # 12 post-norm layers at width 768, 12 heads, 32 sequences of 128 tokens, not causal, gamma = 0.8; the oracle
    # recomputes the last sequence and two others; as for the post-norm MLP stack the backward is compared on the
    # oracle's forward state of those sequences
    _run(B, W["roberta_like"], ks=(1, 3), rows_count=2, shared_state=True)


@pytest.mark.timeout(300)
def test_transformer_attn_full(B):
    # 12 layers = 24 sub-blocks at width 1024, 16 heads, 16 sequences of 1024 tokens; the oracle recomputes the last one
    _run(B, W["transformer_attn"], ks=(1,), rows_count=0, check_exact=False)


@pytest.mark.timeout(300)
def test_resnet_like_full(B):
    _run(B, W["resnet_like"], ks=(1, 2, 3, 4), rows_count=40)


@pytest.mark.timeout(300)
def test_resnet_postact_full_shared_state(B):
    # a ReLU after the sum: in the storage type a sum within rounding of zero can fall on either side, so the two
    # forwards' masks differ in a fraction of a percent of the elements; the backward is compared on the oracle's
    # forward state (its mask included) for the sampled rows
    _run(B, W["resnet_postact"], ks=(1, 2, 4), rows_count=40, shared_state=True)


@pytest.mark.timeout(300)
def test_postnorm_mlp_full_shared_state(B):
    # 24 post-norm layers: compared on the oracle's forward state for the sampled rows (the two forwards differ by
    # storage rounding, which the iteration without gamma amplifies with k on such a stack)
    _run(B, W["postnorm_mlp"], ks=(0, 1, 2), rows_count=16, shared_state=True)


@pytest.mark.timeout(300)
def test_transformer_mlp_full(B):
    _run(B, W["transformer_mlp"], ks=(1, 4), rows_count=24)


@pytest.mark.timeout(300)
def test_gated_rnn_contractive_full(B):
    _run(B, W["gated_rnn_contractive"], ks=(1, 4), rows_count=2, check_exact=True)


@pytest.mark.timeout(300)
def test_gru_cell_full(B):
    # T = 4096 steps of the gated cell, each side on its own forward
    _run(B, W["gru_cell"], ks=(1, 3), rows_count=2, check_exact=True)


@pytest.mark.timeout(300)
def test_gru_std_cell_full(B):
    # the standard GRU (reset gate included) at T = 4096, batch 32, H = 1024
    _run(B, W["gru_std_cell"], ks=(1, 3), rows_count=2, check_exact=True)


@pytest.mark.timeout(300)
def test_lstm_cell_full(B):
    _run(B, W["lstm_cell"], ks=(1, 3), rows_count=2, check_exact=True)


@pytest.mark.timeout(300)
def test_gated_rnn_chaotic_full_shared_state(B):
    # exact BPTT over 4096 chaotic steps overflows the storage type: only the k-iteration estimates
    _run(B, W["gated_rnn"], ks=(1, 2, 4), rows_count=2, shared_state=True, check_exact=False)


def _library_state(p, w, rows_t):
    """The forward state hbp_forward left in device memory, for the sampled rows, as the oracle's `saved`."""
    g = lambda t: H.to_np(t[:, rows_t])
    L = w.L
    n = len(rows_t)
    return {"x": g(p.x), "y": g(p.y), "z": g(p.z), "dphi": g(p.dphi), "rinv": g(p.rinv),
            "mask": np.ones((L, n, w.d)), "rpost": np.ones((L, n))}


@pytest.mark.timeout(1100)
def test_deep_large_full(B):
    """The largest stack (96 blocks, d = 2048, d_ff = 8192, 16384 tokens), on 6 sampled token rows, three ways:
      own state     the oracle's backward run from the forward state hbp_forward itself left in memory: the
                    backward kernels on exactly the inputs bench.py gives them (bar: 2e-2);
      shared state  the oracle's own forward state, rounded to storage, uploaded for the sampled rows (bar: 2e-2);
      end to end    each side on its own forward from x_0 (bar 2e-2 at k = 1).  A forward pass that stores every
                    state in bf16 accumulates that rounding over 96 blocks (x_96 differs from the fp64 forward's
                    by 1e-2), and the ill-conditioned block Jacobians amplify it: at k = 3 the ORACLE's backward
                    on its own forward run with every state rounded to storage (block by block) differs from the
                    oracle's backward on its fp64 forward by about the bar itself.  That is asserted here, beside
                    a looser bar of 3e-2 for the library at k = 3.
    The forward state itself (x, y, z, act', 1/rms) is held to the bar too.  The figures are printed, and written as
    JSON into the directory HBP_TEST_OUT names when that variable is set."""
    w = W["deep_large"]
    tol = H.TOL[w.dtype]
    inp = synth.make_inputs(w)
    p = B.allocate(w, inp)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    rows = _sample_rows(w.N, 4, 3)
    rows_t = torch.from_numpy(rows).to(p.x.device)
    sub = _subset(w, inp, rows)
    st = H.oracle_stack(w, sub)
    sv_fp64 = O.forward(st, sub["x0"], None)
    sv_round = H.oracle_saved_rounded(w, sv_fp64)
    sv_step = H.forward_rounded_stepwise(w, st, sub["x0"])
    sv_lib = _library_state(p, w, rows_t)
    fig = {"rows": [int(r) for r in rows]}
    # forward state: library against oracle
    for nm in ("x", "y", "z", "dphi", "rinv"):
        fig["forward_" + nm] = H.rel(sv_lib[nm], sv_fp64[nm])
        assert fig["forward_" + nm] < tol, f"deep_large forward {nm}: {fig['forward_' + nm]:.3e}"
    for k in (1, 3):
        B.hbp_backward(p, k)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        got = H.to_np(p.g[:, rows_t])
        want_lib = O.hbp_backward(st, sv_lib, sub["e"], k)
        want_fp64 = O.hbp_backward(st, sv_fp64, sub["e"], k)
        want_round = O.hbp_backward(st, sv_round, sub["e"], k)
        want_step = O.hbp_backward(st, sv_step, sub["e"], k)
        H.assert_close(got, want_lib, tol, f"deep_large k={k}, own state: g on sampled rows")
        fig[f"k{k}_own_state"] = H.rel(got, want_lib)
        fig[f"k{k}_end_to_end"] = H.rel(got, want_fp64)
        fig[f"k{k}_oracle_state_rounded_once_vs_fp64_state"] = H.rel(want_round, want_fp64)
        fig[f"k{k}_oracle_state_rounded_every_block_vs_fp64_state"] = H.rel(want_step, want_fp64)
        _projection_check(p, w, inp, 5e-3)
    assert fig["k1_end_to_end"] < tol, f"deep_large k=1 end to end {fig['k1_end_to_end']:.3e}"
    assert fig["k3_end_to_end"] < 1.5 * tol, f"deep_large k=3 end to end {fig['k3_end_to_end']:.3e}"
    # the oracle alone, on a forward whose states are rounded to storage block by block, moves by the same order
    fig["forward_x_oracle_rounded_every_block"] = H.rel(sv_step["x"], sv_fp64["x"])
    assert fig["k3_oracle_state_rounded_every_block_vs_fp64_state"] > 0.5 * fig["k3_end_to_end"], fig
    # shared state
    for name, t in (("x", p.x), ("y", p.y), ("z", p.z), ("dphi", p.dphi), ("rinv", p.rinv)):
        t[:, rows_t] = torch.from_numpy(sv_round[name].astype(np.float32)).to(t.device).to(t.dtype)
    for k in (1, 3):
        B.hbp_backward(p, k)
        torch.cuda.synchronize()
        want = O.hbp_backward(st, sv_round, sub["e"], k)
        H.assert_close(H.to_np(p.g[:, rows_t]), want, tol, f"deep_large k={k}, shared state: g on sampled rows")
        fig[f"k{k}_shared_state"] = H.rel(H.to_np(p.g[:, rows_t]), want)
    B.hbp_exact_backward(p)
    torch.cuda.synchronize()
    want = O.exact_backward(st, sv_round, sub["e"])
    H.assert_close(H.to_np(p.g[:, rows_t]), want, tol, "deep_large exact, shared state: g on sampled rows")
    fig["exact_shared_state"] = H.rel(H.to_np(p.g[:, rows_t]), want)
    print("deep_large parity figures:", json.dumps(fig))
    out = os.environ.get("HBP_TEST_OUT", "")
    if out and os.path.isdir(out):
        with open(os.path.join(out, "deep_large_parity.json"), "w") as f:
            json.dump(fig, f, indent=1)
    del p
    torch.cuda.empty_cache()
