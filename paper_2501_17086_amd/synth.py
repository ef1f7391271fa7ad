"""Seeded synthetic inputs for the Highway-BP workloads.

This module only draws random tensors (and rounds them to the storage type).
It holds none of the method's arithmetic and serves both the GPU library's
callers (tests, bench) and the CPU oracle's callers, so that both sides see
the same bits.

Generator: numpy's counter-based Philox, keyed by (seed, tensor id, block
index), so any block's tensor can be regenerated on its own and in any order.

Workloads follow the five stacks the benchmark names: a small fp32 residual
MLP stack, a ResNet-like and two Transformer-depth pre-RMSNorm MLP stacks in
bf16, and a gated RNN along time with shared weights.  Conventions: N(0, 1/fan_in)
gives the variance; N(0, 0.02) gives the standard deviation (the usual
transformer initialisation); lambda is per (block, channel) and shared by all
tokens; in the RNN lambda_t = sigmoid(N(3, 0.5^2)) is constant data.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

# tensor ids for the Philox key
_T_W1, _T_W2, _T_U, _T_LAM, _T_X0, _T_XIN, _T_E, _T_WQKV, _T_WO = 1, 2, 3, 4, 5, 6, 7, 8, 9


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str            # 'mlp' | 'rnn' | 'gated' (recurrent cell x' = (1-u) x + u c; d_ff = 2 d) | 'lstm' (state
                         # [c | h], d = 2H, d_ff = 4H) | 'gru' (the standard GRU, gates [z | r | n]; d_ff = 3 d)
                         # | 'transformer' (L = 2 x layers: attention sub-blocks at even l, MLP sub-blocks at odd l;
                         # the N tokens are N / seq_len sequences of seq_len consecutive rows)
    dtype: str           # 'f32' | 'bf16'   (storage; accumulation is fp32 on the GPU)
    act: str             # 'gelu' | 'tanh' | 'identity'
    norm: str            # 'none' | 'rms'
    L: int               # blocks (depth) or time steps T
    N: int               # tokens (rnn: batch rows per step)
    d: int               # state width (rnn: hidden H)
    d_ff: int            # block inner width (rnn: H)
    d_in: int = 0        # rnn input width
    lam: str = "one"     # 'one' | 'uniform' | 'sigmoid' ([L,d]) | 'sigmoid_full' ([L,N,d]: per token as well)
    lam_lo: float = 1.0
    lam_hi: float = 1.0
    w1_std: float = 0.0  # 0 -> 1/sqrt(fan_in)
    w2_std: float = 0.0
    w2_scale: float = 1.0
    rec_scale: float = 1.0   # extra factor on W_h and W_o (rnn variants)
    loss_every_state: bool = False
    post: str = "none"   # 'none' | 'relu' | 'rms': what the residual function applies after the sum
    gate_bias: float = 0.0   # 'gated': constant added to the update gate's pre-activation (see make_inputs)
    eps: float = 1e-6
    ks: tuple = (1, 2, 3, 4)
    seed: int = 0
    heads: int = 0       # 'transformer': attention heads, sequence length, causal mask
    seq_len: int = 0
    causal: bool = True
    gamma: float = 0.0   # the share of the residual connection counted with the block that the workload is run with

    @property
    def tokens(self) -> int:
        return self.N * self.L if self.kind in ("rnn", "gated", "lstm", "gru") else self.N


WORKLOADS: Dict[str, Workload] = {
    # small fp32 residual MLP stack, lambda = 1, no norm
    "mlp_small_f32": Workload("mlp_small_f32", "mlp", "f32", "gelu", "none", L=8, N=128, d=64, d_ff=256,
                              ks=(0, 1, 2, 8)),
    # ResNet-like: per-channel lambda ~ U(0.9,1), W2 scaled by 1/sqrt(L)
    "resnet_like": Workload("resnet_like", "mlp", "bf16", "gelu", "rms", L=32, N=8192, d=512, d_ff=2048,
                            lam="uniform", lam_lo=0.9, lam_hi=1.0, w2_scale=1.0 / np.sqrt(32.0)),
    # Transformer-depth MLP stack, lambda = 1
    "transformer_mlp": Workload("transformer_mlp", "mlp", "bf16", "gelu", "rms", L=48, N=16384, d=1024,
                                d_ff=4096, w1_std=0.02, w2_std=0.02, w2_scale=1.0 / np.sqrt(96.0)),
    # gated RNN along time, shared weights, a loss at every step
    "gated_rnn": Workload("gated_rnn", "rnn", "bf16", "tanh", "none", L=4096, N=32, d=1024, d_ff=1024,
                          d_in=1024, lam="sigmoid", lam_lo=3.0, lam_hi=0.5, loss_every_state=True),
    # the same stack with the original ResNet's residual function: a ReLU after the sum
    "resnet_postact": Workload("resnet_postact", "mlp", "bf16", "gelu", "rms", L=32, N=8192, d=512, d_ff=2048,
                               lam="uniform", lam_lo=0.9, lam_hi=1.0, w2_scale=1.0 / np.sqrt(32.0), post="relu"),
    # a post-norm stack (the norm after the sum instead of inside the block), transformer widths
    "postnorm_mlp": Workload("postnorm_mlp", "mlp", "bf16", "gelu", "none", L=24, N=8192, d=1024, d_ff=4096,
                             w1_std=0.02, w2_std=0.02, post="rms"),
    # large deep stack
    "deep_large": Workload("deep_large", "mlp", "bf16", "gelu", "rms", L=96, N=16384, d=2048, d_ff=8192,
                           lam="uniform", lam_lo=0.8, lam_hi=1.0, w1_std=0.02, w2_std=0.02,
                           w2_scale=1.0 / np.sqrt(192.0), ks=(1, 2, 3)),
}
# The paper's GPT-2 configuration (appendix, hyperparameter table: 12 layers, hidden 256, context 256, batch 128;
# every layer split into attention and feed-forward sub-layers, L = 24; run with gamma = 0.2), with RMS norm and no
# biases, and a larger stack of the same kind (12 layers of width 1024, 16 heads, 16 sequences of 1024 tokens).
WORKLOADS["gpt2_paper"] = Workload("gpt2_paper", "transformer", "bf16", "gelu", "rms", L=24, N=128 * 256, d=256,
                                   d_ff=1024, w1_std=0.02, w2_std=0.02, w2_scale=1.0 / np.sqrt(24.0), heads=4,
                                   seq_len=256, causal=True, gamma=0.2, ks=(1, 2, 3))
WORKLOADS["transformer_attn"] = Workload("transformer_attn", "transformer", "bf16", "gelu", "rms", L=24, N=16 * 1024,
                                         d=1024, d_ff=4096, w1_std=0.02, w2_std=0.02, w2_scale=1.0 / np.sqrt(24.0),
                                         heads=16, seq_len=1024, causal=True, gamma=0.2, ks=(1, 2, 3))
# The paper's RoBERTa configuration (12 post-norm layers, hidden 768, 12 heads, inputs of 128 tokens, batch 32; run with
# gamma = 0.8), random weights, RMS norm after each residual sum, no biases
WORKLOADS["roberta_like"] = Workload("roberta_like", "transformer", "bf16", "gelu", "none", L=24, N=32 * 128, d=768,
                                     d_ff=3072, w1_std=0.02, w2_std=0.02, heads=12, seq_len=128, causal=False,
                                     post="rms", gamma=0.8, ks=(1, 2, 3))
# contractive variant of the RNN (recurrent weights x 0.25): the stack as
# specified is chaotic, so exact BPTT gradients overflow over 4096 steps.
WORKLOADS["gated_rnn_contractive"] = replace(WORKLOADS["gated_rnn"], name="gated_rnn_contractive",
                                             rec_scale=0.25)
# a recurrent cell whose residual coefficient is its own update gate (the GRU row of the paper's table of layer
# decompositions): T = 4096, batch 32, H = 1024, gates biased towards closed (1 - u around 0.95)
WORKLOADS["gru_cell"] = Workload("gru_cell", "gated", "bf16", "tanh", "none", L=4096, N=32, d=1024, d_ff=2048,
                                 d_in=1024, loss_every_state=True, gate_bias=-3.0, rec_scale=0.5)
# the standard GRU (reset gate included), the cell of the paper's GRU experiments, at the same sizes
WORKLOADS["gru_std_cell"] = Workload("gru_std_cell", "gru", "bf16", "tanh", "none", L=4096, N=32, d=1024, d_ff=3072,
                                     d_in=1024, loss_every_state=True, gate_bias=-3.0, rec_scale=0.5)
# an LSTM cell (the LSTM row of the same table): state [c | h] of 2 x 1024, forget gates around 0.95
WORKLOADS["lstm_cell"] = Workload("lstm_cell", "lstm", "bf16", "tanh", "none", L=4096, N=32, d=2048, d_ff=4096,
                                  d_in=1024, loss_every_state=True, gate_bias=3.0, rec_scale=0.5)
# the contractive RNN with a gate per (step, batch row, channel): a diagonal K that depends on the data
WORKLOADS["gated_rnn_token_gates"] = replace(WORKLOADS["gated_rnn_contractive"], name="gated_rnn_token_gates",
                                             lam="sigmoid_full")


def scaled(w: Workload, **kw) -> Workload:
    """The same recipe at other sizes (for parity tests)."""
    return replace(w, **kw)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def storage_round(w: Workload, a: np.ndarray) -> np.ndarray:
    return round_bf16(a) if w.dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


def _rng(w: Workload, tid: int, idx: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(w.seed << 8) | tid, idx]))


def _normal(w: Workload, tid: int, idx: int, shape, std: float) -> np.ndarray:
    return _rng(w, tid, idx).standard_normal(shape, dtype=np.float32) * np.float32(std)


def weights_block(w: Workload, l: int):
    """(W1_l [d_ff,d], W2_l [d,d_ff]) for block l (rnn: l is ignored)."""
    idx = 0 if w.kind in ("rnn", "gated", "lstm", "gru") else l
    if w.kind == "lstm":       # W1 = [W_i; W_f; W_o; W_g] acts on the hidden half of the state
        H = w.d // 2
        return storage_round(w, _normal(w, _T_W1, idx, (w.d_ff, H), w.rec_scale / np.sqrt(H))), None
    s1 = w.w1_std if w.w1_std > 0 else 1.0 / np.sqrt(w.d)
    s2 = (w.w2_std if w.w2_std > 0 else 1.0 / np.sqrt(w.d_ff)) * w.w2_scale
    W1 = _normal(w, _T_W1, idx, (w.d_ff, w.d), s1 * w.rec_scale)
    W2 = _normal(w, _T_W2, idx, (w.d, w.d_ff), s2 * w.rec_scale)
    return storage_round(w, W1), storage_round(w, W2)


def attention_weights_block(w: Workload, j: int):
    """(Wqkv_j [3d,d], Wo_j [d,d]) of layer j of a 'transformer' stack; Wo scaled like W2."""
    s1 = w.w1_std if w.w1_std > 0 else 1.0 / np.sqrt(w.d)
    s2 = (w.w2_std if w.w2_std > 0 else 1.0 / np.sqrt(w.d)) * w.w2_scale
    return (storage_round(w, _normal(w, _T_WQKV, j, (3 * w.d, w.d), s1)),
            storage_round(w, _normal(w, _T_WO, j, (w.d, w.d), s2)))


def make_lambda(w: Workload, tokens=None) -> Optional[np.ndarray]:
    """lambda [L,d] fp32, or None when lambda = 1; 'sigmoid_full': [L,N,d] in the
    storage type (gates that depend on the token, e.g. computed from a cell's input)."""
    if w.lam == "one":
        return None
    g = _rng(w, _T_LAM)
    if w.lam == "sigmoid_full":
        sl = tokens if tokens is not None else slice(None)
        out = np.empty((w.L, len(np.arange(w.N)[sl]), w.d), np.float32)
        for l in range(w.L):   # drawn layer by layer in the full token range, then cut
            a = g.standard_normal((w.N, w.d), dtype=np.float32) * np.float32(w.lam_hi) + np.float32(w.lam_lo)
            out[l] = (1.0 / (1.0 + np.exp(-a.astype(np.float64)))).astype(np.float32)[sl]
        return storage_round(w, out)
    if w.lam == "uniform":
        return g.uniform(w.lam_lo, w.lam_hi, (w.L, w.d)).astype(np.float32)
    a = g.standard_normal((w.L, w.d), dtype=np.float32) * np.float32(w.lam_hi) + np.float32(w.lam_lo)
    return (1.0 / (1.0 + np.exp(-a.astype(np.float64)))).astype(np.float32)


def make_inputs(w: Workload, tokens=None) -> Dict[str, Optional[np.ndarray]]:
    """All tensors of a workload as fp32 numpy arrays holding storage-representable
    values.  `tokens` restricts the token axis (rnn: the batch axis) to a slice
    or an index array; the full tensors are drawn and then cut, so a subset sees
    the same values as the full run.

    Keys: W1, W2 (mlp: [L,...]; rnn: shared), U (rnn), lam, x0 [N,d],
    xin [L,N,d_in] (rnn), e ([N,d], or [L+1,N,d] with e[0] = 0 when every state
    has a loss).
    """
    sl = tokens if tokens is not None else slice(None)
    out: Dict[str, Optional[np.ndarray]] = {}
    if w.kind in ("mlp", "transformer"):
        nb = w.L // 2 if w.kind == "transformer" else w.L
        W1 = np.empty((nb, w.d_ff, w.d), np.float32)
        W2 = np.empty((nb, w.d, w.d_ff), np.float32)
        if w.kind == "transformer":
            out["Wqkv"] = np.empty((nb, 3 * w.d, w.d), np.float32)
            out["Wo"] = np.empty((nb, w.d, w.d), np.float32)

        def fill(l):   # every block has its own generator key: order of evaluation is free
            W1[l], W2[l] = weights_block(w, l)
            if w.kind == "transformer":
                out["Wqkv"][l], out["Wo"][l] = attention_weights_block(w, l)
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(nb)))
        out["U"] = None
        out["xin"] = None
    else:
        W1, W2 = weights_block(w, 0)
        out["U"] = storage_round(w, _normal(w, _T_U, 0, (w.d_ff, w.d_in), 1.0 / np.sqrt(w.d_in)))
        out["xin"] = storage_round(w, _normal(w, _T_XIN, 0, (w.L, w.N, w.d_in), 1.0)[:, sl])
    out["W1"], out["W2"] = W1, W2
    if w.kind == "gru":
        # W1 = [W_z; W_r; W_n]; as for the gated cell below, a constant bias of the update gate z through input channel 0
        out["W2"] = None
        H = w.d
        out["xin"][..., 0] = 1.0
        out["U"][:H, 0] = np.float32(w.gate_bias)
        out["U"][H:, 0] = 0.0
        out["U"] = storage_round(w, out["U"])
    if w.kind == "gated":
        # W1 = [W_u; W_c].  The cell has no bias term: a constant update-gate bias (gates that are mostly closed,
        # i.e. a long memory, as in a trained GRU) is realised through the input: channel 0 of xin is 1 and its
        # column of U holds the bias for the gate rows and 0 for the candidate rows.
        out["W2"] = None
        H = w.d
        out["xin"][..., 0] = 1.0
        out["U"][:H, 0] = np.float32(w.gate_bias)
        out["U"][H:, 0] = 0.0
        out["U"] = storage_round(w, out["U"])
    if w.kind == "lstm":
        # as for the gated cell: a constant forget-gate bias (gates mostly open: a long-lived cell state) through
        # input channel 0, which is 1; rows H..2H of U are the forget gate's
        H = w.d // 2
        out["xin"][..., 0] = 1.0
        out["U"][:, 0] = 0.0
        out["U"][H:2 * H, 0] = np.float32(w.gate_bias)
        out["U"] = storage_round(w, out["U"])
    out["lam"] = make_lambda(w, tokens)
    if w.kind in ("rnn", "gated", "lstm", "gru"):
        out["x0"] = np.zeros((w.N, w.d), np.float32)[sl]
    else:
        out["x0"] = storage_round(w, _normal(w, _T_X0, 0, (w.N, w.d), 1.0)[sl])
    if w.loss_every_state:
        e = _normal(w, _T_E, 0, (w.L + 1, w.N, w.d), 1.0)
        e[0] = 0.0
        out["e"] = storage_round(w, e[:, sl])
    else:
        out["e"] = storage_round(w, _normal(w, _T_E, 0, (w.N, w.d), 1.0)[sl])
    return out
