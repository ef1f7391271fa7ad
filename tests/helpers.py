"""Glue shared by the GPU parity tests: builds the oracle's Stack and the GPU
Problem from the same seeded inputs and compares results.  Holds no arithmetic
of the method itself."""
from __future__ import annotations

import numpy as np

from oracle import hbp_oracle as O
from paper_2501_17086_amd import synth

TOL = {"f32": 1e-5, "bf16": 2e-2}   # relative L2, GPU vs oracle


def oracle_stack(w: synth.Workload, inp) -> O.Stack:
    if w.kind in ("gated", "lstm"):
        return O.Stack(w.kind, w.act, w.norm, inp["W1"], None, U=inp["U"], L=w.L)
    return O.Stack(w.kind, w.act, w.norm, inp["W1"], inp["W2"], lam=inp["lam"], U=inp["U"], eps=w.eps, L=w.L,
                   post=w.post)


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
    for k in ("x", "y", "z", "dphi"):
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
    put(p.y, sv_r["y"])
    put(p.rinv, sv_r["rpost"] if w.post == "rms" else sv_r["rinv"])
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
