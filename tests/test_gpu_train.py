"""The training step around the backward pass on the GPU against the oracle: the stand-in loss and its gradient,
gradient clipping, SGD with momentum and AdamW over several steps, and whole training steps under a schedule of
iterations that ends with exact backpropagation (the paper's conclusion), all through the C ABI."""
import numpy as np
import pytest

from oracle import hbp_oracle as O
from paper_2501_17086_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

W = synth.WORKLOADS
SMALL_F32 = synth.scaled(W["mlp_small_f32"], name="train_f32", L=4, N=64, d=64, d_ff=128, norm="rms", lam="uniform",
                         lam_lo=0.9, lam_hi=1.0)
SMALL_BF16 = synth.scaled(W["resnet_like"], name="train_bf16", L=4, N=256, d=256, d_ff=512, w2_scale=0.5)
TFM_F32 = synth.scaled(W["gpt2_paper"], name="train_tfm_f32", dtype="f32", L=4, N=48, seq_len=12, d=32, heads=2, d_ff=64,
                       w1_std=0.0, w2_std=0.0, w2_scale=0.7, gamma=0.2)
RNN_F32 = synth.scaled(W["gated_rnn_contractive"], name="train_rnn_f32", dtype="f32", L=12, N=4, d=64, d_ff=64, d_in=32)


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    from paper_2501_17086_amd import binding
    binding.lib()
    return binding


def _target(w, seed=11):
    rng = np.random.default_rng(seed)
    shape = (w.L + 1, w.N, w.d) if w.loss_every_state else (w.N, w.d)
    return synth.storage_round(w, (0.1 * rng.standard_normal(shape)).astype(np.float32))


@pytest.mark.parametrize("w", [SMALL_F32, SMALL_BF16, RNN_F32], ids=lambda w: w.name)
def test_loss_and_its_gradient(B, w):
    inp = synth.make_inputs(w)
    st = H.oracle_stack(w, inp)
    p = B.allocate(w, inp)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tgt = _target(w)
    t_dev = torch.from_numpy(tgt).to(p.x.device).to(p.x.dtype)
    p.e = torch.full_like(p.g if w.loss_every_state else p.g[0], float("nan"))
    os_ = B.allocate_optim(p, adamw=False)
    B.hbp_loss_mse(p, t_dev, os_)
    torch.cuda.synchronize()
    loss, e = O.mse_loss_and_grad(H.to_np(p.x), tgt, w.loss_every_state)      # on the library's own states
    assert float(os_.loss) == pytest.approx(loss, rel=1e-5)
    H.assert_close(H.to_np(p.e), e, 1e-6 if w.dtype == "f32" else 4e-3, f"{w.name}: e")


@pytest.mark.parametrize("kind", ["sgd", "adamw"])
@pytest.mark.parametrize("master", [True, False])
def test_optimizer_steps(B, kind, master):
    """Five updates from fixed random gradients against the oracle's fp64 steps; with clipping on."""
    w = SMALL_F32
    inp = synth.make_inputs(w)
    p = B.allocate(w, inp)
    os_ = B.allocate_optim(p, adamw=kind == "adamw", master=master)
    rng = np.random.default_rng(2)
    W1, W2 = inp["W1"].astype(np.float64), inp["W2"].astype(np.float64)
    m1, m2, v1, v2 = (np.zeros_like(a) for a in (W1, W2, W1, W2))
    hp = dict(lr=0.05, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.01, clip_norm=3.0)
    for step in range(1, 6):
        g1 = rng.standard_normal(W1.shape).astype(np.float32)
        g2 = rng.standard_normal(W2.shape).astype(np.float32)
        p.dW1.copy_(torch.from_numpy(g1)); p.dW2.copy_(torch.from_numpy(g2))
        B.hbp_optimizer_step(p, B.make_optim(kind, step=step, **hp), os_)
        torch.cuda.synchronize()
        sc = O.clip_scale([g1, g2], hp["clip_norm"])
        if kind == "sgd":
            W1, m1 = O.sgd_momentum_step(W1, g1, m1, hp["lr"], hp["beta1"], hp["weight_decay"], sc)
            W2, m2 = O.sgd_momentum_step(W2, g2, m2, hp["lr"], hp["beta1"], hp["weight_decay"], sc)
        else:
            W1, m1, v1 = O.adamw_step(W1, g1, m1, v1, step, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                                      hp["weight_decay"], sc)
            W2, m2, v2 = O.adamw_step(W2, g2, m2, v2, step, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                                      hp["weight_decay"], sc)
        H.assert_close(H.to_np(p.W1), W1, 1e-5, f"{kind} step {step}: W1")
        H.assert_close(H.to_np(p.W2), W2, 1e-5, f"{kind} step {step}: W2")
        if master:
            assert torch.equal(os_.master[0], p.W1) and torch.equal(os_.master[1], p.W2)     # fp32 storage


def _oracle_train(w, inp, tgt, ks, kind, hp):
    """The same loop in the oracle (fp64).  Returns the losses and the final weights."""
    names = ["W1", "W2", "U", "Wqkv", "Wo"]
    inp = {**{n: None for n in names}, **inp}
    Ws = {n: (None if inp[n] is None else inp[n].astype(np.float64)) for n in names}
    m = {n: (None if Ws[n] is None else np.zeros_like(Ws[n])) for n in names}
    v = {n: (None if Ws[n] is None else np.zeros_like(Ws[n])) for n in names}
    losses = []
    for step, k in enumerate(ks, start=1):
        cur = dict(inp); cur.update({n: Ws[n] for n in names})
        st = H.oracle_stack(w, cur)
        sv = O.forward(st, inp["x0"], inp["xin"])
        loss, e = O.mse_loss_and_grad(sv["x"], tgt, w.loss_every_state)
        losses.append(loss)
        g = O.exact_backward(st, sv, e) if k < 0 else O.hbp_backward(st, sv, e, k, gamma=w.gamma)
        pg = O.param_grads(st, sv, g, inp["xin"])
        have = [n for n in names if Ws[n] is not None]
        sc = O.clip_scale([pg["d" + n] for n in have], hp["clip_norm"])
        for n in have:
            if kind == "sgd":
                Ws[n], m[n] = O.sgd_momentum_step(Ws[n], pg["d" + n], m[n], hp["lr"], hp["beta1"], hp["weight_decay"], sc)
            else:
                Ws[n], m[n], v[n] = O.adamw_step(Ws[n], pg["d" + n], m[n], v[n], step, hp["lr"], hp["beta1"],
                                                 hp["beta2"], hp["eps"], hp["weight_decay"], sc)
    return losses, Ws


@pytest.mark.parametrize("w,kind", [(SMALL_F32, "sgd"), (SMALL_F32, "adamw"), (RNN_F32, "adamw"), (TFM_F32, "adamw")],
                         ids=["mlp_sgd", "mlp_adamw", "rnn_adamw", "transformer_adamw"])
def test_training_steps_under_a_schedule_of_iterations(B, w, kind):
    """Nine whole steps (forward, loss, backward, parameter gradients, update) with k = 1, 1, 1, 2, 2, 2, then exact
    backpropagation three times: losses and final weights against the same loop in the oracle (fp32 storage)."""
    inp = synth.make_inputs(w)
    tgt = _target(w)
    ks = [1, 1, 1, 2, 2, 2, -1, -1, -1]
    hp = dict(lr=0.02 if kind == "sgd" else 2e-3, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=1e-3, clip_norm=1.0)
    want_losses, want_W = _oracle_train(w, inp, tgt, ks, kind, hp)
    p = B.allocate(w, inp)
    p.e = torch.zeros_like(p.g if w.loss_every_state else p.g[0])
    os_ = B.allocate_optim(p, adamw=kind == "adamw")
    t_dev = torch.from_numpy(tgt).to(p.x.device).to(p.x.dtype)
    losses = []
    for step, k in enumerate(ks, start=1):
        B.hbp_train_step(p, k, t_dev, B.make_optim(kind, step=step, **hp), os_)
        torch.cuda.synchronize()
        losses.append(float(os_.loss))
    assert np.allclose(losses, want_losses, rtol=2e-4), (losses, want_losses)
    assert losses[-1] < losses[0]
    for n, t in (("W1", p.W1), ("W2", p.W2), ("U", p.U), ("Wqkv", p.Wqkv), ("Wo", p.Wo)):
        if t is not None:
            # the update itself (what training moved), not the weights it is small against
            H.assert_close(H.to_np(t) - inp[n], want_W[n] - inp[n], 2e-3, f"{w.name} {kind}: change of {n}", row_floor=0.5)


def test_one_training_step_in_bf16(B):
    """bf16 storage with fp32 master weights: the first step's update of the master weights against the oracle."""
    w = SMALL_BF16
    inp = synth.make_inputs(w)
    tgt = _target(w)
    hp = dict(lr=0.05, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.0, clip_norm=0.0)
    want_losses, want_W = _oracle_train(w, inp, tgt, [2], "sgd", hp)
    p = B.allocate(w, inp)
    p.e = torch.zeros_like(p.g[0])
    os_ = B.allocate_optim(p, adamw=False)
    t_dev = torch.from_numpy(tgt).to(p.x.device).to(p.x.dtype)
    B.hbp_train_step(p, 2, t_dev, B.make_optim("sgd", **hp), os_)
    torch.cuda.synchronize()
    assert float(os_.loss) == pytest.approx(want_losses[0], rel=2e-2)
    for i, n in enumerate(("W1", "W2")):
        H.assert_close(H.to_np(os_.master[i]) - inp[n], want_W[n] - inp[n], 2e-2, f"bf16 step: change of {n}", row_floor=0.5)
        # the stored weights are the master weights rounded to storage
        assert torch.equal(getattr(p, n), os_.master[i].to(torch.bfloat16))


def test_optimizer_rejects_bad_arguments(B):
    w = SMALL_F32
    p = B.allocate(w, synth.make_inputs(w))
    os_ = B.allocate_optim(p, adamw=False)
    for bad in (dict(lr=-1.0), dict(lr=0.1, beta1=1.0), dict(lr=0.1, weight_decay=-0.1)):
        with pytest.raises(B.HbpError) as ei:
            B.hbp_optimizer_step(p, B.make_optim("sgd", **bad), os_)
        assert ei.value.status == 1
    with pytest.raises(B.HbpError) as ei:       # AdamW without second moments
        B.hbp_optimizer_step(p, B.make_optim("adamw", lr=0.1), os_)
    assert ei.value.status == 4
    with pytest.raises(B.HbpError) as ei:       # AdamW counts its steps from 1
        B.hbp_optimizer_step(p, B.make_optim("adamw", lr=0.1, step=0), B.allocate_optim(p, adamw=True))
    assert ei.value.status == 1
