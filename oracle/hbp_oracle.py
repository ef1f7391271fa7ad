"""CPU oracle for the Highway-BP backward pass (arXiv 2501.17086).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, fp64 definition that
the GPU library is checked against.  Nothing in the product path may import it;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.  It
shares no code with the HIP path and never receives values computed by it.

Every function is written from the paper's definitions (numpy fp64; a matmul
and erf are the only library steps; no blocking, fusion or reordering):

  model      Section "Notations and assumptions": h_i = f_i(h_{i-1}),
             f_i(x) = r_i(x, g_i(x)), Jacobian J_i + K_i.  Here the residual
             function is r(x, z) = lam (.) x + z, so K = diag(lam), and the
             block is  g(x) = W2 . act(W1 . norm(x) [+ U . xin]).  With
             post = 'relu' the residual function is the one of the original
             ResNet in the table of layer decompositions, r(x, z) =
             ReLU(lam (.) x + z): with m = 1[lam (.) x + z > 0],
             K = dr/dx = diag(m (.) lam) and J = dr/dz . dg/dx = diag(m) . dg/dx.
             post = 'rms' is the post-norm row of the table (f = Norm(x + Layer(x)) written as
             a(x) (.) x + b(x) with r(x, z) = z1 (.) x + z2), for the RMS norm without gain: with
             s = lam (.) x + g(x) and rho = 1/sqrt(mean(s^2) + eps):  a = lam rho (rho one number per token),
             b = g(x) rho.  K = dr/dx = diag(lam rho), held as data like any z1; J = F - K with F the layer's
             whole Jacobian, whose VJP is  G -> lam (.) P(G) + P(G) . dg/dx,  P(G) = rho (G - x' mean(G (.) x'))
             the norm's backward at the new state x'.
             kind = 'gated' is the GRU row of the same table, f(x) = a(x) (.) x + b(x)
             with g = [a, b] and r(x, z) = z1 (.) x + z2, for the cell  u = sigmoid(W_u x + U_u xin),
             c = tanh(W_c x + U_c xin),  a = 1 - u,  b = u (.) c  (a GRU without its reset gate):
             K = dr/dx = diag(a), a function of the state, and J = diag(x) . da/dx + db/dx.
             kind = 'gru' is the same row for the standard cell with its reset gate:  z = sigmoid(W_z x + U_z xin),
             r = sigmoid(W_r x + U_r xin),  n = tanh(W_n (r (.) x) + U_n xin),  a = 1 - z,  b = z (.) n  (the
             candidate sees the state through the reset gate: two dependent products per step).  K = diag(1 - z).
             kind = 'lstm' is the LSTM row: the state is x = [c | h] (cell and hidden part),
             f(x) = [a(x) (.) c + b(x), c3(x)] and r(x, z) = [z1 (.) c + z2, z3], for the standard cell
             i, f, o = sigmoid(.), gg = tanh(.) of W h + U xin,  c' = f (.) c + i (.) gg,  h' = o (.) tanh(c'):
             a = f, b = i (.) gg, c3 = o (.) tanh(f (.) c + i (.) gg).  K = dr/dx = diag([f | 0]): only the
             cell part has a residual path; everything else, the dependence of h' on c included, is J.
             kind = 'transformer' is the pre-norm transformer of the appendix (GPT-2 paragraph), every layer split into
             its two sub-layers, so that L = 2 x layers: block l even is multi-head self-attention on the normed state,
             [q | k | v] = norm(x) Wqkv^T, per sequence and head softmax(q k^T / sqrt(dh)) v (keys after the query
             masked out when causal), heads side by side, times Wo^T; block l odd is the two-matrix MLP.  The residual
             function is r(x, z) = lam (.) x + z as for 'mlp' (the decomposition with gamma applies as for any kind;
             post = 'rms' with norm = 'none' gives the post-norm transformer of the appendix's RoBERTa paragraph);
             a token's block output now depends on the other tokens of its sequence, so J couples the rows of a state.
  exact BP   Section "Backpropagation as a system of equations" and the first
             line of the proof of Theorem 1 (chain rule through J + K).
  Highway-BP Theorem 2 (w^0 and the recursion for w^{k+1}) in its two-step
             "Parallel computation" form: v_i = w_{i+1} J_{i+1} for all i,
             then u_i = v_i + u_{i+1} K_{i+1}, and w^{k+1} = w^0 + u.
  CumSumProd its definition in Section "Parallel computation"
             (sum_{j>=i} a_j M_j ... M_{i+1}); Algorithm 1 (Hillis-Steele) is
             reproduced separately for cross-checking.
  param grad sentence after Theorem 2: dL/dtheta_i = w_i . df_i/dtheta_i.

Indexing (0-based states x_0..x_L, blocks l = 0..L-1, x_{l+1} = lam_l (.) x_l +
block_l(x_l)): the paper's h_i is x_i, its layer i is block i-1, K_i =
diag(lam_{i-1}), J_i = d block_{i-1} / d x at x_{i-1}, dL_i/dh_i is e_i.
Gradients are stored as rows [N, d] (one row per token), matching the paper's
row-vector convention  w J.

Parity status: every function below is pinned by tests/test_oracle_pins.py
(finite differences, closed forms, path enumeration, an independent autograd
library) -- no function is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------
# model description
# --------------------------------------------------------------------------
@dataclass
class Stack:
    """A residual stack.

    kind   'gru'   one standard GRU cell shared by all L (= T) steps, state width H:
                  W1 = [W_z; W_r; W_n] [3H,H], U = [U_z; U_r; U_n] [3H,d_in], no W2, no lam
           'lstm'  one LSTM cell shared by all L (= T) steps, state [c | h] of width 2H:
                  W1 = [W_i; W_f; W_o; W_g] [4H,H] (acts on h), U likewise [4H,d_in], no W2, no lam
           'gated' one recurrent cell shared by all L (= T) steps, state width H:
                  W1 = [W_u; W_c] [2H,H], U = [U_u; U_c] [2H,d_in], no W2, no lam
                  (the coefficient of the residual path is the cell's own 1 - u)
           'mlp'  per-block weights W1[L,d_ff,d], W2[L,d,d_ff]
           'transformer'  L = 2 x layers alternating sub-blocks: l even self-attention with Wqkv[L/2,3d,d] (rows
                  [W_q; W_k; W_v], head h in columns h dh .. (h+1) dh of each third) and Wo[L/2,d,d]; l odd the MLP with
                  W1[L/2,d_ff,d], W2[L/2,d,d_ff].  Tokens are B sequences of T: row n = b T + t.
           'rnn'  weights shared by all L (= T) blocks: W1 = W_h [d_ff,d],
                  W2 = W_o [d,d_ff], U [d_ff,d_in]; block l maps state l to
                  l+1 and consumes xin[l]
    act    'gelu' (exact erf form) | 'tanh' | 'identity'
    norm   'none' | 'rms'  (no gain, eps inside the square root)
    post   'none' | 'relu' | 'rms': what the residual function applies after the sum
           (Section "Notations and assumptions": r need not be linear)
    lam    None (lambda = 1), [L, d] (one coefficient per block and channel,
           shared by all tokens) or [L, N, d] (per token as well: a diagonal
           K_l that depends on the data, given here as data, e.g. gates computed
           from the input of a recurrent cell; Section "Layer decomposition")
    """
    kind: str
    act: str
    norm: str
    W1: np.ndarray
    W2: Optional[np.ndarray]
    lam: Optional[np.ndarray] = None
    U: Optional[np.ndarray] = None
    eps: float = 1e-6
    L: int = 0
    post: str = "none"
    Wqkv: Optional[np.ndarray] = None
    Wo: Optional[np.ndarray] = None
    T: int = 0               # sequence length of the attention sub-blocks
    heads: int = 0
    causal: bool = True

    def __post_init__(self):
        assert self.post in ("none", "relu", "rms")
        assert self.kind in ("mlp", "rnn", "gated", "lstm", "gru", "transformer")
        assert self.act in ("gelu", "tanh", "identity")
        assert self.norm in ("none", "rms")
        self.W1 = np.asarray(self.W1, dtype=F64)
        if self.kind in ("gated", "lstm", "gru"):
            assert self.W2 is None and self.lam is None and self.norm == "none" and self.post == "none"
            assert self.W1.ndim == 2 and self.L > 0
            assert self.W1.shape[0] == {"gated": 2, "gru": 3, "lstm": 4}[self.kind] * self.W1.shape[1]
            self.U = np.asarray(self.U, dtype=F64)
            return
        self.W2 = np.asarray(self.W2, dtype=F64)
        if self.lam is not None:
            self.lam = np.asarray(self.lam, dtype=F64)
        if self.U is not None:
            self.U = np.asarray(self.U, dtype=F64)
        if self.kind == "mlp":
            assert self.W1.ndim == 3 and self.W2.ndim == 3
            self.L = self.W1.shape[0]
        elif self.kind == "transformer":
            assert self.W1.ndim == 3 and self.W2.ndim == 3 and self.post in ("none", "rms")
            self.Wqkv = np.asarray(self.Wqkv, dtype=F64)
            self.Wo = np.asarray(self.Wo, dtype=F64)
            assert self.Wqkv.shape == (self.W1.shape[0], 3 * self.W2.shape[1], self.W2.shape[1])
            assert self.Wo.shape == (self.W1.shape[0], self.W2.shape[1], self.W2.shape[1])
            assert self.T > 0 and self.heads > 0 and self.W2.shape[1] % self.heads == 0
            self.L = 2 * self.W1.shape[0]
        else:
            assert self.W1.ndim == 2 and self.W2.ndim == 2
            assert self.L > 0, "rnn stacks need L (= T) given"

    @property
    def d(self) -> int:
        if self.kind in ("gated", "gru"):
            return self.W1.shape[-1]
        if self.kind == "lstm":
            return 2 * self.W1.shape[-1]
        return self.W2.shape[-2]

    @property
    def d_ff(self) -> int:
        return self.W1.shape[-2]

    def is_attn(self, l: int) -> bool:
        return self.kind == "transformer" and l % 2 == 0

    def w1(self, l: int) -> np.ndarray:
        """The matrix a block applies to its (normed) input: W1, or Wqkv for an attention sub-block."""
        if self.kind == "transformer":
            return self.Wqkv[l // 2] if l % 2 == 0 else self.W1[l // 2]
        return self.W1[l] if self.kind == "mlp" else self.W1

    def w2(self, l: int) -> np.ndarray:
        """The matrix that maps a block's inner result back to the state: W2, or Wo for an attention sub-block."""
        if self.kind == "transformer":
            return self.Wo[l // 2] if l % 2 == 0 else self.W2[l // 2]
        return self.W2[l] if self.kind == "mlp" else self.W2

    def lam_row(self, l: int) -> np.ndarray:
        """Diagonal of K carrying state l+1 to state l, as [1, d] or [N, d]."""
        if self.lam is None:
            return np.ones((1, self.d), dtype=F64)
        return np.atleast_2d(self.lam[l])


# --------------------------------------------------------------------------
# activations
# --------------------------------------------------------------------------
def act_fn(name: str, a: np.ndarray) -> np.ndarray:
    if name == "gelu":          # a * Phi(a), Phi = standard normal CDF
        return 0.5 * a * (1.0 + _erf(a / math.sqrt(2.0)))
    if name == "tanh":
        return np.tanh(a)
    return a


def act_grad(name: str, a: np.ndarray) -> np.ndarray:
    if name == "gelu":          # Phi(a) + a * pdf(a)
        return 0.5 * (1.0 + _erf(a / math.sqrt(2.0))) + a * np.exp(-0.5 * a * a) / math.sqrt(2.0 * math.pi)
    if name == "tanh":
        t = np.tanh(a)
        return 1.0 - t * t
    return np.ones_like(a)


# --------------------------------------------------------------------------
# multi-head self-attention on [q | k | v] rows (the attention sub-block between its two matrices)
# --------------------------------------------------------------------------
def _heads(st: Stack, m: np.ndarray) -> np.ndarray:
    """[B T, heads dh] -> [B, heads, T, dh]"""
    B = m.shape[0] // st.T
    return m.reshape(B, st.T, st.heads, -1).transpose(0, 2, 1, 3)


def _merge(m: np.ndarray) -> np.ndarray:
    """[B, heads, T, dh] -> [B T, heads dh]"""
    B, Hn, T, dh = m.shape
    return m.transpose(0, 2, 1, 3).reshape(B * T, Hn * dh)


def attn_probs(st: Stack, q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """softmax over the keys of q k^T / sqrt(dh), [B, heads, T, T]; causal: a query sees keys up to its own position."""
    dh = q.shape[-1]
    s = q @ k.transpose(0, 1, 3, 2) / math.sqrt(dh)
    if st.causal:
        s = np.where(np.tril(np.ones((st.T, st.T), dtype=bool)), s, -np.inf)
    p = np.exp(s - s.max(axis=-1, keepdims=True))
    return p / p.sum(axis=-1, keepdims=True)


def attention(st: Stack, qkv: np.ndarray) -> np.ndarray:
    """o = softmax(q k^T / sqrt(dh)) v per sequence and head; qkv [N,3d] -> o [N,d]."""
    d = qkv.shape[1] // 3
    q, k, v = (_heads(st, qkv[:, j * d:(j + 1) * d]) for j in range(3))
    return _merge(attn_probs(st, q, k) @ v)


def attention_vjp(st: Stack, qkv: np.ndarray, do: np.ndarray) -> np.ndarray:
    """Gradient w.r.t. [q | k | v] given the gradient do of o:  dv = P^T do,  dP = do v^T,
    dS = P (.) (dP - rowsum(dP (.) P)),  dq = dS k / sqrt(dh),  dk = dS^T q / sqrt(dh)."""
    d = qkv.shape[1] // 3
    q, k, v = (_heads(st, qkv[:, j * d:(j + 1) * d]) for j in range(3))
    doh = _heads(st, do)
    P = attn_probs(st, q, k)
    dv = P.transpose(0, 1, 3, 2) @ doh
    dP = doh @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - np.sum(dP * P, axis=-1, keepdims=True))
    sc = 1.0 / math.sqrt(q.shape[-1])
    dq = dS @ k * sc
    dk = dS.transpose(0, 1, 3, 2) @ q * sc
    return np.concatenate([_merge(dq), _merge(dk), _merge(dv)], axis=1)


# --------------------------------------------------------------------------
# forward: produces the states and what the backward pass needs
# --------------------------------------------------------------------------
def forward(st: Stack, x0: np.ndarray, xin: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """x_{l+1} = lam_l (.) x_l + W2_l . act(W1_l . norm(x_l) [+ U . xin_l]).

    Returns x[L+1,N,d] and the saved tensors y = norm(x_l) [L,N,d],
    rinv = 1/rms [L,N] (ones without a norm), a (pre-activation), z = act(a),
    dphi = act'(a), all [L,N,d_ff]; with post = 'relu' the sum goes through a
    ReLU and mask[l] = 1 where the sum that made x_{l+1} was positive (all ones otherwise).
    kind = 'transformer' also returns qkv [L,N,3d] and o [L,N,d] (attention output before Wo); rows of a, z, dphi
    belonging to attention sub-blocks and rows of qkv, o belonging to MLP sub-blocks are zero.
    """
    x0 = np.asarray(x0, dtype=F64)
    N, d = x0.shape
    if st.kind == "gated":
        return _forward_gated(st, x0, xin)
    if st.kind == "lstm":
        return _forward_lstm(st, x0, xin)
    if st.kind == "gru":
        return _forward_gru(st, x0, xin)
    L, dff = st.L, st.d_ff
    x = np.zeros((L + 1, N, d), F64)
    y = np.zeros((L, N, d), F64)
    rinv = np.ones((L, N), F64)
    a = np.zeros((L, N, dff), F64)
    mask = np.ones((L, N, d), F64)
    rpost = np.ones((L, N), F64)
    tr = st.kind == "transformer"
    qkv = np.zeros((L, N, 3 * d), F64) if tr else None
    o = np.zeros((L, N, d), F64) if tr else None
    x[0] = x0
    for l in range(L):
        if st.norm == "rms":
            r = np.sqrt(np.mean(x[l] * x[l], axis=1) + st.eps)
            rinv[l] = 1.0 / r
            y[l] = x[l] / r[:, None]
        else:
            y[l] = x[l]
        if st.is_attn(l):
            qkv[l] = y[l] @ st.w1(l).T
            o[l] = attention(st, qkv[l])
            x[l + 1] = st.lam_row(l) * x[l] + o[l] @ st.w2(l).T
        else:
            a[l] = y[l] @ st.w1(l).T
            if st.kind == "rnn":
                a[l] += np.asarray(xin[l], dtype=F64) @ st.U.T
            x[l + 1] = st.lam_row(l) * x[l] + act_fn(st.act, a[l]) @ st.w2(l).T
        if st.post == "relu":
            mask[l] = (x[l + 1] > 0.0).astype(F64)
            x[l + 1] = np.maximum(x[l + 1], 0.0)
        if st.post == "rms":
            rpost[l] = 1.0 / np.sqrt(np.mean(x[l + 1] * x[l + 1], axis=1) + st.eps)
            x[l + 1] = x[l + 1] * rpost[l][:, None]
    out = {"x": x, "y": y, "rinv": rinv, "a": a, "mask": mask, "rpost": rpost,
           "z": act_fn(st.act, a), "dphi": act_grad(st.act, a)}
    if tr:
        out["qkv"], out["o"] = qkv, o
        for l in range(0, L, 2):      # no MLP in these blocks
            out["z"][l] = 0.0
            out["dphi"][l] = 0.0
    return out


def _forward_gated(st: Stack, x0: np.ndarray, xin: np.ndarray) -> Dict[str, np.ndarray]:
    """x_{l+1} = (1 - u_l) (.) x_l + u_l (.) c_l,  u = sigmoid(W_u x + U_u xin),  c = tanh(W_c x + U_c xin).
    Saved: x, u, c and a = 1 - u (the coefficient of the residual path, kept as its own tensor as the
    layer decomposition has it: z1 = a(x)), all [L,N,H] (and y = x, rinv = 1, mask = 1 so that the
    shared code reads them)."""
    N, H = x0.shape
    L = st.L
    x = np.zeros((L + 1, N, H), F64)
    u = np.zeros((L, N, H), F64)
    c = np.zeros((L, N, H), F64)
    x[0] = x0
    for l in range(L):
        pre = x[l] @ st.W1.T + np.asarray(xin[l], dtype=F64) @ st.U.T
        u[l] = 1.0 / (1.0 + np.exp(-pre[:, :H]))
        c[l] = np.tanh(pre[:, H:])
        x[l + 1] = (1.0 - u[l]) * x[l] + u[l] * c[l]
    return {"x": x, "y": x[:-1], "rinv": np.ones((L, N), F64), "u": u, "c": c, "a": 1.0 - u,
            "mask": np.ones((L, N, H), F64)}


def _sigmoid(a: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-a))


def _forward_gru(st: Stack, x0: np.ndarray, xin: np.ndarray) -> Dict[str, np.ndarray]:
    """The standard GRU: z = sigmoid(W_z x + U_z xin), r = sigmoid(W_r x + U_r xin),
    n = tanh(W_n (r (.) x) + U_n xin), x' = (1 - z) (.) x + z (.) n.  Saved: x, the gates zrn = [z | r | n]
    [L,N,3H] and a = 1 - z (the coefficient of the residual path)."""
    N, H = x0.shape
    L = st.L
    Wz, Wr, Wn = st.W1[:H], st.W1[H:2 * H], st.W1[2 * H:]
    x = np.zeros((L + 1, N, H), F64)
    zrn = np.zeros((L, N, 3 * H), F64)
    x[0] = x0
    for l in range(L):
        ux = np.asarray(xin[l], dtype=F64) @ st.U.T
        z = _sigmoid(x[l] @ Wz.T + ux[:, :H])
        r = _sigmoid(x[l] @ Wr.T + ux[:, H:2 * H])
        n = np.tanh((r * x[l]) @ Wn.T + ux[:, 2 * H:])
        x[l + 1] = (1.0 - z) * x[l] + z * n
        zrn[l] = np.concatenate([z, r, n], axis=1)
    return {"x": x, "y": x[:-1], "rinv": np.ones((L, N), F64), "zrn": zrn, "a": 1.0 - zrn[:, :, :H],
            "mask": np.ones((L, N, H), F64)}


def _forward_lstm(st: Stack, x0: np.ndarray, xin: np.ndarray) -> Dict[str, np.ndarray]:
    """x = [c | h];  [i, f, o, gg] = [sigmoid, sigmoid, sigmoid, tanh](W h + U xin);  c' = f (.) c + i (.) gg;
    h' = o (.) tanh(c').  Saved: x [L+1,N,2H], gates = [i | f | o | gg] [L,N,4H], a = [f | 0] [L,N,2H] (the
    diagonal of dr/dx: the hidden part has no residual path)."""
    N, d = x0.shape
    H = d // 2
    L = st.L
    x = np.zeros((L + 1, N, d), F64)
    gates = np.zeros((L, N, 4 * H), F64)
    a = np.zeros((L, N, d), F64)
    x[0] = x0
    for l in range(L):
        c, h = x[l][:, :H], x[l][:, H:]
        pre = h @ st.W1.T + np.asarray(xin[l], dtype=F64) @ st.U.T
        i, f, o = _sigmoid(pre[:, :H]), _sigmoid(pre[:, H:2 * H]), _sigmoid(pre[:, 2 * H:3 * H])
        gg = np.tanh(pre[:, 3 * H:])
        cn = f * c + i * gg
        x[l + 1] = np.concatenate([cn, o * np.tanh(cn)], axis=1)
        gates[l] = np.concatenate([i, f, o, gg], axis=1)
        a[l, :, :H] = f
    return {"x": x, "y": x[:-1], "rinv": np.ones((L, N), F64), "gates": gates, "a": a,
            "mask": np.ones((L, N, d), F64)}


def k_diag(st: Stack, l: int, saved: Dict[str, np.ndarray]) -> np.ndarray:
    """Diagonal of dr/dx for the layer that carries state l+1 to state l, before any mask: lam_l, or for the
    gated cell its own coefficient a_l = 1 - u_l (per token)."""
    if st.kind in ("gated", "lstm", "gru"):
        return saved["a"][l]
    return st.lam_row(l)


# --------------------------------------------------------------------------
# step (i): vector-Jacobian product through one block,  v_l = g_{l+1} J_{l+1}
# --------------------------------------------------------------------------
def block_preact_grad(st: Stack, l: int, saved: Dict[str, np.ndarray], g_next: np.ndarray) -> np.ndarray:
    """Gradient w.r.t. the pre-activation of block l: (g W2) (.) act'(a).  Gated cell: with r = z1 (.) x + z2,
    z1 = 1 - u, z2 = u (.) c:  dL/du = g (.) (c - x), dL/dc = g (.) u, taken through sigmoid' = u (1 - u) and
    tanh' = 1 - c^2, side by side as [N, 2H]."""
    if st.kind == "gated":
        u, c, x = saved["u"][l], saved["c"][l], saved["x"][l]
        return np.concatenate([g_next * (c - x) * u * (1.0 - u), g_next * u * (1.0 - c * c)], axis=1)
    if st.kind == "gru":
        # dL/dz = g (.) (n - x), dL/dn = g (.) z, through sigmoid' and tanh'; the reset gate receives what comes back
        # from the candidate's product through r (.) x:  d(r (.) x) = dn_pre W_n,  dL/dr = d(r (.) x) (.) x
        H = st.d
        z, r, n = (saved["zrn"][l][:, j * H:(j + 1) * H] for j in range(3))
        x = saved["x"][l]
        dn = g_next * z * (1.0 - n * n)
        dz = g_next * (n - x) * z * (1.0 - z)
        drx = dn @ st.W1[2 * H:]
        dr = drx * x * r * (1.0 - r)
        return np.concatenate([dz, dr, dn], axis=1)
    if st.kind == "lstm":
        # g = [Gc | Gh] at the next state.  Everything that reaches c' : Gc and, through h' = o tanh(c'), Gh.
        H = st.d // 2
        Gc, Gh = g_next[:, :H], g_next[:, H:]
        i, f, o, gg = (saved["gates"][l][:, j * H:(j + 1) * H] for j in range(4))
        c = saved["x"][l][:, :H]
        tc = np.tanh(saved["x"][l + 1][:, :H])
        dct = Gc + Gh * o * (1.0 - tc * tc)
        return np.concatenate([dct * gg * i * (1.0 - i), dct * c * f * (1.0 - f), Gh * tc * o * (1.0 - o),
                               dct * i * (1.0 - gg * gg)], axis=1)
    if st.is_attn(l):      # the gradient of [q | k | v]: back through Wo, then through the attention
        return attention_vjp(st, saved["qkv"][l], g_next @ st.w2(l))
    return (g_next @ st.w2(l)) * saved["dphi"][l]


def block_vjp(st: Stack, l: int, saved: Dict[str, np.ndarray], g_next: np.ndarray) -> np.ndarray:
    da = block_preact_grad(st, l, saved, g_next)
    if st.kind == "lstm":
        # J only: into h through the gates' weights; into c the part of d c'/d c = f that carries Gh (the part that
        # carries Gc is K)
        H = st.d // 2
        Gh = g_next[:, H:]
        f, o = saved["gates"][l][:, H:2 * H], saved["gates"][l][:, 2 * H:3 * H]
        tc = np.tanh(saved["x"][l + 1][:, :H])
        return np.concatenate([Gh * o * (1.0 - tc * tc) * f, da @ st.W1], axis=1)
    if st.kind == "gru":
        # into the state: through the two gates' weights, and through r (.) x directly (scaled by r)
        H = st.d
        r = saved["zrn"][l][:, H:2 * H]
        return da[:, :2 * H] @ st.W1[:2 * H] + (da[:, 2 * H:] @ st.W1[2 * H:]) * r
    dn = da @ st.w1(l)
    if st.norm == "rms":
        # y = x / r, r = sqrt(mean(x^2) + eps):  dx = (dn - y * mean(dn (.) y)) / r
        y = saved["y"][l]
        m = np.mean(dn * y, axis=1, keepdims=True)
        return (dn - y * m) * saved["rinv"][l][:, None]
    return dn


def through_r(st: Stack, l: int, saved: Dict[str, np.ndarray], g_next: np.ndarray) -> np.ndarray:
    """g_{l+1} . dr/d(sum): the gradient of state l+1 taken back through what the residual function applies after
    the sum (the ReLU's mask, the norm's backward, or nothing): the gradient with respect to the sum, which is what
    the block VJP and the parameter gradients start from."""
    if st.post == "relu":
        return saved["mask"][l] * g_next
    if st.post == "rms":
        xn = saved["x"][l + 1]
        m = np.mean(g_next * xn, axis=1, keepdims=True)
        return (g_next - xn * m) * saved["rpost"][l][:, None]
    return g_next


def k_full(st: Stack, l: int, saved: Dict[str, np.ndarray]) -> np.ndarray:
    """Diagonal of K_l = dr/dx for the layer between states l and l+1, as [1,d] or [N,d]."""
    k = k_diag(st, l, saved)
    if st.post == "relu":
        return saved["mask"][l] * k
    if st.post == "rms":
        return saved["rpost"][l][:, None] * k
    return k


def j_vjp(st: Stack, l: int, saved: Dict[str, np.ndarray], g_next: np.ndarray) -> np.ndarray:
    """g_{l+1} J_l with J_l = (the layer's whole Jacobian) - K_l."""
    gs = through_r(st, l, saved, g_next)
    v = block_vjp(st, l, saved, gs)
    if st.post == "rms":     # what the sum's own lam (.) x contributes beyond K: lam (.) (P(G) - rho G)
        v = v + k_diag(st, l, saved) * (gs - saved["rpost"][l][:, None] * g_next)
    return v


def _e_full(st: Stack, e: np.ndarray, N: int) -> np.ndarray:
    """Per-state loss gradients e_0..e_L.  A [N,d] array means only e_L != 0."""
    e = np.asarray(e, dtype=F64)
    if e.ndim == 2:
        full = np.zeros((st.L + 1, N, st.d), F64)
        full[st.L] = e
        return full
    assert e.shape[0] == st.L + 1
    return e


# --------------------------------------------------------------------------
# exact sequential backpropagation
# --------------------------------------------------------------------------
def exact_backward(st: Stack, saved: Dict[str, np.ndarray], e: np.ndarray) -> np.ndarray:
    """G_L = e_L ; G_l = e_l + G_{l+1} (K_{l+1} + J_{l+1}),  l = L-1 .. 0."""
    N = saved["y"].shape[1]
    ef = _e_full(st, e, N)
    G = np.zeros_like(ef)
    G[st.L] = ef[st.L]
    for l in range(st.L - 1, -1, -1):
        G[l] = ef[l] + k_full(st, l, saved) * G[l + 1] + j_vjp(st, l, saved, G[l + 1])
    return G


# --------------------------------------------------------------------------
# CumSumProd along the residual path (sequential form of the recurrence)
# --------------------------------------------------------------------------
def cumsumprod_reverse(a: np.ndarray, lam_rows) -> np.ndarray:
    """u_i = sum_{j>=i} a_j M_j ... M_{i+1} with diagonal M: the multiplier that
    carries position i+1 to position i is lam_rows(i).

    a has shape [P, N, d] (positions 0..P-1); returns u of the same shape,
    computed by u_{P-1} = a_{P-1}, u_i = a_i + lam_i (.) u_{i+1}.
    """
    P = a.shape[0]
    u = np.zeros_like(a)
    u[P - 1] = a[P - 1]
    for i in range(P - 2, -1, -1):
        u[i] = a[i] + np.atleast_2d(lam_rows(i)) * u[i + 1]
    return u


# --------------------------------------------------------------------------
# Highway-BP, k iterations (Theorem 2, two-step form)
# --------------------------------------------------------------------------
def hbp_backward(st: Stack, saved: Dict[str, np.ndarray], e: np.ndarray, k: int,
                 return_all: bool = False, gamma: float = 0.0):
    """w^0 = CumSumProd(e, K);  repeat k times: v_l = w_{l+1} J_{l+1} for every
    l from the current estimate, u = CumSumProd(v, K), w <- w^0 + u.

    gamma re-splits each layer between its block and its residual connection
    (appendix, the decomposition with gamma used for pre-norm transformers,
    written there for lambda = 1 and taken here for any diagonal coefficient):
    the residual connection keeps (1 - gamma) lambda_l (.) x and the block gains
    gamma lambda_l (.) x, i.e. K' = (1 - gamma) K and J' = J + gamma K.  The
    function and its exact gradient are unchanged; the iterates are not.
    gamma = 0 is the plain method, gamma = 1 the fixed-point iteration."""
    assert k >= 0
    N = saved["y"].shape[1]
    L = st.L
    ef = _e_full(st, e, N)
    k_row = lambda l: (1.0 - gamma) * k_full(st, l, saved)
    w0 = cumsumprod_reverse(ef, k_row)
    w = w0.copy()
    hist = [w0.copy()]
    for _ in range(k):
        v = np.zeros_like(w)                       # v_L = 0: no block above x_L
        for l in range(L):
            v[l] = j_vjp(st, l, saved, w[l + 1])
            if gamma != 0.0:
                v[l] = v[l] + gamma * k_full(st, l, saved) * w[l + 1]
        u = cumsumprod_reverse(v, k_row)
        w = w0 + u
        hist.append(w.copy())
    return hist if return_all else w


# --------------------------------------------------------------------------
# parameter gradients from a given state-gradient estimate
# --------------------------------------------------------------------------
def param_grads(st: Stack, saved: Dict[str, np.ndarray], g: np.ndarray,
                xin: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """dW2_l = sum_n g_{l+1}[n]^T z_l[n] ; dW1_l = sum_n da_l[n]^T y_l[n] ;
    dU = sum da^T xin, with da from the given g.  Shared weights (rnn) sum
    over l as well.  (With post = 'relu' or 'rms', g_{l+1} is first taken through it: through_r.)"""
    L = st.L
    if st.post != "none":
        g = np.concatenate([g[:1]] + [through_r(st, l, saved, g[l + 1])[None] for l in range(L)], axis=0)
    if st.kind == "mlp":
        dW1 = np.zeros_like(st.W1)
        dW2 = np.zeros_like(st.W2)
        for l in range(L):
            da = block_preact_grad(st, l, saved, g[l + 1])
            dW2[l] = g[l + 1].T @ saved["z"][l]
            dW1[l] = da.T @ saved["y"][l]
        return {"dW1": dW1, "dW2": dW2}
    if st.kind == "transformer":
        out = {"dW1": np.zeros_like(st.W1), "dW2": np.zeros_like(st.W2), "dWqkv": np.zeros_like(st.Wqkv),
               "dWo": np.zeros_like(st.Wo)}
        for l in range(L):
            da = block_preact_grad(st, l, saved, g[l + 1])
            if st.is_attn(l):
                out["dWo"][l // 2] = g[l + 1].T @ saved["o"][l]
                out["dWqkv"][l // 2] = da.T @ saved["y"][l]
            else:
                out["dW2"][l // 2] = g[l + 1].T @ saved["z"][l]
                out["dW1"][l // 2] = da.T @ saved["y"][l]
        return out
    if st.kind in ("gated", "lstm"):
        dW1 = np.zeros_like(st.W1)
        dU = np.zeros_like(st.U)
        H = st.W1.shape[1]
        for l in range(L):
            da = block_preact_grad(st, l, saved, g[l + 1])
            dW1 += da.T @ (saved["x"][l] if st.kind == "gated" else saved["x"][l][:, H:])
            dU += da.T @ np.asarray(xin[l], dtype=F64)
        return {"dW1": dW1, "dU": dU}
    if st.kind == "gru":      # the candidate's weights see r (.) x, the gates' weights x
        dW1 = np.zeros_like(st.W1)
        dU = np.zeros_like(st.U)
        H = st.d
        for l in range(L):
            da = block_preact_grad(st, l, saved, g[l + 1])
            x, r = saved["x"][l], saved["zrn"][l][:, H:2 * H]
            dW1[:2 * H] += da[:, :2 * H].T @ x
            dW1[2 * H:] += da[:, 2 * H:].T @ (r * x)
            dU += da.T @ np.asarray(xin[l], dtype=F64)
        return {"dW1": dW1, "dU": dU}
    dW1 = np.zeros_like(st.W1)
    dW2 = np.zeros_like(st.W2)
    dU = np.zeros_like(st.U)
    for l in range(L):
        da = block_preact_grad(st, l, saved, g[l + 1])
        dW2 += g[l + 1].T @ saved["z"][l]
        dW1 += da.T @ saved["y"][l]
        dU += da.T @ np.asarray(xin[l], dtype=F64)
    return {"dW1": dW1, "dW2": dW2, "dU": dU}


# --------------------------------------------------------------------------
# Algorithm 1 (Hillis-Steele CumSumProd) -- only used to cross-check the scan
# --------------------------------------------------------------------------
def cumsumprod_hillis_steele(a: np.ndarray, lam_rows) -> np.ndarray:
    """ceil(log2 P) sweeps over pairs (u_i, P_i); P_i starts as the multiplier
    that carries position i+1 to i (the reading that matches the algorithm's
    stated post-condition), and a sweep with stride s does
    u_i += u_{i+s} P_i ; P_i <- P_{i+s} P_i  for i + s < P."""
    P = a.shape[0]
    u = a.astype(F64).copy()
    d = a.shape[-1]
    Pm = np.ones((P, d), F64)
    for i in range(P - 1):
        Pm[i] = lam_rows(i)
    s = 1
    while s < P:
        un, Pn = u.copy(), Pm.copy()
        for i in range(P - s):
            un[i] = u[i] + Pm[i][None, :] * u[i + s]
            Pn[i] = Pm[i + s] * Pm[i]
        u, Pm = un, Pn
        s *= 2
    return u


# --------------------------------------------------------------------------
# error measures used in reports
# --------------------------------------------------------------------------
def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    """||a - b||_2 / ||b||_2 (b is the reference)."""
    a = np.asarray(a, F64).ravel()
    b = np.asarray(b, F64).ravel()
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a - b))


def cosine(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, F64).ravel()
    b = np.asarray(b, F64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


# --------------------------------------------------------------------------
# a training step around the backward pass (Section "Discussion and conclusion": the number of iterations can be
# raised during training, ending with exact backpropagation; appendix "Training scheme": SGD with momentum and
# weight decay for the ResNets, AdamW with gradient clipping for the transformers and RNNs)
# --------------------------------------------------------------------------
def mse_loss_and_grad(x_states: np.ndarray, target: np.ndarray, every_state: bool):
    """The stand-in training loss: half the squared distance of the states to targets, averaged over tokens.
    every_state: states 1..L each have a target (target [L+1,N,d], row 0 unused); else only x_L (target [N,d]).
    Returns (loss, e) with e = dL/dx in the layout the backward pass takes ([L+1,N,d] with e[0] = 0, or [N,d])."""
    x = np.asarray(x_states, F64)
    t = np.asarray(target, F64)
    N = x.shape[1]
    if every_state:
        diff = x - t
        diff[0] = 0.0
        return 0.5 * float(np.sum(diff * diff)) / N, diff / N
    diff = x[-1] - t
    return 0.5 * float(np.sum(diff * diff)) / N, diff / N


def clip_scale(grads, max_norm: float) -> float:
    """Factor that brings the global L2 norm of all gradients down to max_norm (1 when it is below, or when
    max_norm <= 0: no clipping): min(1, max_norm / (norm + 1e-6))."""
    if max_norm <= 0.0:
        return 1.0
    tot = math.sqrt(sum(float(np.sum(np.asarray(g, F64) ** 2)) for g in grads))
    return min(1.0, max_norm / (tot + 1e-6))


def sgd_momentum_step(w, g, buf, lr: float, momentum: float, weight_decay: float, scale: float = 1.0):
    """SGD with momentum and L2 weight decay, in the form the ResNet recipe uses:
    g' = scale g + weight_decay w;  buf <- momentum buf + g';  w <- w - lr buf.  Returns (w, buf)."""
    w = np.asarray(w, F64)
    gp = scale * np.asarray(g, F64) + weight_decay * w
    buf = momentum * np.asarray(buf, F64) + gp
    return w - lr * buf, buf


def adamw_step(w, g, m, v, step: int, lr: float, beta1: float, beta2: float, eps: float, weight_decay: float,
               scale: float = 1.0):
    """AdamW (weight decay decoupled from the gradient), step counted from 1:
    w <- w (1 - lr wd);  m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
    w <- w - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).  Returns (w, m, v)."""
    w = np.asarray(w, F64) * (1.0 - lr * weight_decay)
    g = scale * np.asarray(g, F64)
    m = beta1 * np.asarray(m, F64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, F64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v


def lr_schedule(step: int, total: int, base_lr: float, warmup: int) -> float:
    """Linear warm-up over `warmup` steps, then a cosine from base_lr down to a tenth of it at step `total`
    (appendix "Training scheme").  step counts from 0."""
    if warmup > 0 and step < warmup:
        return base_lr * (step + 1) / warmup
    p = min(1.0, (step - warmup) / max(1, total - warmup))
    return base_lr * (0.1 + 0.9 * 0.5 * (1.0 + math.cos(math.pi * p)))
