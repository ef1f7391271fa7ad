"""Glue shared by the GPU parity tests: builds the oracle's Stack and the GPU
Problem from the same seeded inputs and compares results.  Holds no arithmetic
of the method itself."""
from __future__ import annotations

import numpy as np

from oracle import hbp_oracle as O
from paper_2501_17086_amd import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}   # relative L2, GPU vs oracle


def oracle_stack(w: synth.Workload, inp) -> O.Stack:
    if w.kind in ("gated", "lstm", "gru"):
        return O.Stack(w.kind, w.act, w.norm, inp["W1"], None, U=inp["U"], L=w.L)
    if w.kind == "transformer":
        return O.Stack(w.kind, w.act, w.norm, inp["W1"], inp["W2"], lam=inp["lam"], eps=w.eps, Wqkv=inp["Wqkv"],
                       Wo=inp["Wo"], T=w.seq_len, heads=w.heads, causal=w.causal, post=w.post)
    return O.Stack(w.kind, w.act, w.norm, inp["W1"], inp["W2"], lam=inp["lam"], U=inp["U"], eps=w.eps, L=w.L,
                   post=w.post)


def attn_row_stats(st: O.Stack, qkv: np.ndarray) -> np.ndarray:
    """What the library keeps of an attention sub-block's probabilities: per (sequence, head, position) the base-2
    logarithm of sum_j exp2(s_j log2 e) over the keys the query sees, s = q k^T / sqrt(dh); qkv [N,3d] -> [N heads]."""
    d = qkv.shape[1] // 3
    q, k = (O._heads(st, qkv[:, j * d:(j + 1) * d]) for j in range(2))
    s = q @ k.transpose(0, 1, 3, 2) / np.sqrt(q.shape[-1])
    if st.causal:
        s = np.where(np.tril(np.ones((st.T, st.T), dtype=bool)), s, -np.inf)
    m = s.max(axis=-1)
    return ((m + np.log(np.exp(s - m[..., None]).sum(axis=-1))) / np.log(2.0)).reshape(-1)


def to_np(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def oracle_saved_rounded(w: synth.Workload, sv):
    """The oracle's forward state rounded to the storage type, as float64
    arrays: the values a backward call reads from memory."""
    r = lambda a: synth.storage_round(w, a.astype(np.float32)).astype(np.float64)
    out = dict(sv)
    if w.kind == "gated":      # x, the two gates and the residual coefficient, each stored on its own
        for k in ("x", "u", "c", "a"):
            out[k] = r(sv[k])
        out["y"] = out["x"][:-1]
        return out
    if w.kind == "lstm":
        for k in ("x", "gates", "a"):
            out[k] = r(sv[k])
        out["y"] = out["x"][:-1]
        return out
    if w.kind == "gru":
        for k in ("x", "zrn", "a"):
            out[k] = r(sv[k])
        out["y"] = out["x"][:-1]
        return out
    for k in ("x", "y", "z", "dphi") + (("qkv", "o") if w.kind == "transformer" else ()):
        out[k] = r(sv[k])
    out["rinv"] = sv["rinv"].astype(np.float32).astype(np.float64)
    if "rpost" in sv:
        out["rpost"] = sv["rpost"].astype(np.float32).astype(np.float64)
    if w.act == "tanh":        # the GPU derives act' from the stored z
        out["dphi"] = 1.0 - out["z"] ** 2
    if w.norm == "none":
        out["y"] = out["x"][:-1]
    return out


def upload_saved(p, w: synth.Workload, sv_r):
    """Writes a (rounded) forward state into the Problem's device tensors."""
    import torch
    dev = p.x.device

    def put(dst, a):
        if dst is not None:
            dst.copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(dst.dtype))
    put(p.x, sv_r["x"])
    if w.kind == "gated":      # z = [u | c] side by side, lambda = a
        put(p.z, np.concatenate([sv_r["u"], sv_r["c"]], axis=-1))
        put(p.lam, sv_r["a"])
        return
    if w.kind == "lstm":       # z = the four gates side by side, lambda = [f | 0]
        put(p.z, sv_r["gates"])
        put(p.lam, sv_r["a"])
        return
    if w.kind == "gru":        # z = [z | r | n], lambda = 1 - z
        put(p.z, sv_r["zrn"])
        put(p.lam, sv_r["a"])
        return
    put(p.y, sv_r["y"])
    put(p.rinv, sv_r["rpost"] if w.post == "rms" else sv_r["rinv"])
    if w.kind == "transformer":   # inner state of the MLP sub-blocks (odd l) and of the attention sub-blocks (even l)
        put(p.z, sv_r["z"][1::2])
        put(p.dphi, sv_r["dphi"][1::2])
        put(p.qkv, sv_r["qkv"][0::2])
        put(p.attn_o, sv_r["o"][0::2])
        st = sv_r["_stack"]
        put(p.lse, np.stack([attn_row_stats(st, sv_r["qkv"][l]) for l in range(0, w.L, 2)]))
        return
    put(p.z, sv_r["z"])
    put(p.dphi, sv_r["dphi"])
    if p.mask is not None:     # one bit per element, channel 8c+j in bit j of byte c
        bits = np.packbits(sv_r["mask"].astype(np.uint8), axis=-1, bitorder="little")
        p.mask.copy_(torch.from_numpy(bits).to(dev))


def mask_bits(p) -> np.ndarray:
    """The Problem's mask unpacked to [L,N,d] of 0/1."""
    return np.unpackbits(p.mask.cpu().numpy(), axis=-1, bitorder="little").astype(np.float64)


def as_kept(st: O.Stack, sv, G: np.ndarray) -> np.ndarray:
    """State gradients in the form the library keeps them: with a ReLU or a norm after the sum, g[l >= 1] is the
    oracle's gradient of state l taken through it (the oracle's own through_r); unchanged otherwise."""
    if st.post == "none":
        return G
    out = G.copy()
    for l in range(st.L):
        out[l + 1] = O.through_r(st, l, sv, G[l + 1])
    return out


def rel(a, b) -> float:
    return O.rel_l2(a, b)


def assert_close(got, want, tol, tag, row_factor=4.0, abs_factor=8.0, row_floor=0.1):
    """got against want ([..., rows, width]) by three measures, so that an error confined to a few rows or
    elements (a tile edge, a ragged tail, the last chunk of a scan) cannot hide inside a whole-tensor norm:
      whole tensor   relative L2 below tol;
      per row        relative L2 of every row (last axis) below row_factor * tol, the row's norm floored at
                     row_floor times the tensor's typical row norm (rows that are nearly zero carry the others'
                     rounding; a weight-gradient row summed over a handful of tokens is one rounded number times
                     a vector, so its floor is set higher by the callers);
      per element    |got - want| below abs_factor * tol * (rms(want) + |want|) everywhere (an element's rounding
                     error grows with its own size; a wrong element is off by about its size or the rms).
    Returns the three figures (whole, worst row, worst element)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{tag}: shape {got.shape} vs {want.shape}"
    assert np.isfinite(got).all(), f"{tag}: non-finite values"
    whole = rel(got, want)
    assert whole < tol, f"{tag}: rel L2 {whole:.3e} (bar {tol:g})"
    rms = float(np.sqrt(np.mean(want * want)))
    diff = got - want
    if rms == 0.0:
        assert float(np.abs(got).max()) == 0.0, f"{tag}: reference is zero, result is not"
        return whole, 0.0, 0.0
    width = want.shape[-1]
    rn = np.linalg.norm(want.reshape(-1, width), axis=1)
    floor = row_floor * rms * np.sqrt(width)
    rows = np.linalg.norm(diff.reshape(-1, width), axis=1) / np.maximum(rn, floor)
    worst_row = float(rows.max())
    assert worst_row < row_factor * tol, \
        f"{tag}: row {int(rows.argmax())} rel L2 {worst_row:.3e} (bar {row_factor * tol:g}; whole tensor {whole:.3e})"
    ratio = np.abs(diff) / (rms + np.abs(want))
    worst_abs = float(ratio.max())
    assert worst_abs < abs_factor * tol, \
        f"{tag}: element {np.unravel_index(int(ratio.argmax()), diff.shape)} off by {worst_abs:.3e} of rms + |value| " \
        f"(bar {abs_factor * tol:g}; whole tensor {whole:.3e})"
    return whole, worst_row, worst_abs


def forward_rounded_stepwise(w: synth.Workload, st: O.Stack, x0):
    """The oracle's forward of a depth stack one block at a time, every state rounded to the storage type before
    the next block reads it: the states a forward pass that STORES each x_l in that type produces (rounding
    accumulates over the depth), computed with the oracle's own forward on one-block stacks.  Returns a saved
    state of the oracle's layout, the other saved tensors rounded once (oracle_saved_rounded)."""
    assert st.kind == "mlp"
    r = lambda a: synth.storage_round(w, np.asarray(a, np.float32)).astype(np.float64)
    x = r(x0)
    per = []
    xs = [x]
    for l in range(st.L):
        one = O.Stack("mlp", st.act, st.norm, st.W1[l:l + 1], st.W2[l:l + 1],
                      lam=None if st.lam is None else st.lam[l:l + 1], eps=st.eps, post=st.post)
        sv1 = O.forward(one, x)
        x = r(sv1["x"][1])
        xs.append(x)
        per.append(sv1)
    out = {k: np.concatenate([s1[k] for s1 in per], axis=0) for k in ("y", "rinv", "a", "mask", "rpost", "z", "dphi")}
    out["x"] = np.stack(xs)
    return oracle_saved_rounded(w, out)
