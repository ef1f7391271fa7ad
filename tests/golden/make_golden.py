"""Writes tests/golden/oracle_small.txt: the oracle's own results on tiny seeded stacks, one per kind of layer.

The paper prints no numerical worked example, so no file here holds values of the paper's.  This fixture is a
regression pin of the oracle against itself as it stood when its pins (tests/test_oracle_pins.py) last passed:
it catches an accidental change of its arithmetic.  It is written by this script, which calls only oracle/ (and
numpy's generator for the inputs), never by the GPU path.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "..", ".."))
from oracle import hbp_oracle as O  # noqa: E402


def cases():
    """name -> (stack, x0, xin, e): every tensor from numpy's PCG64 with a fixed seed per case."""
    out = {}

    def rnd(seed):
        return np.random.Generator(np.random.PCG64(seed))
    L, N, d, dff, I = 3, 2, 4, 6, 3
    for name, norm, post in (("mlp_rms", "rms", "none"), ("mlp_relu", "rms", "relu"), ("mlp_postnorm", "none", "rms")):
        r = rnd(len(out) + 1)
        st = O.Stack("mlp", "gelu", norm, r.standard_normal((L, dff, d)) / 2, r.standard_normal((L, d, dff)) / 2,
                     lam=r.uniform(0.6, 1.0, (L, d)), post=post)
        out[name] = (st, r.standard_normal((N, d)), None, r.standard_normal((L + 1, N, d)))
    r = rnd(11)
    st = O.Stack("rnn", "tanh", "none", r.standard_normal((d, d)) / 2, r.standard_normal((d, d)) / 2,
                 lam=r.uniform(0.6, 1.0, (L, d)), U=r.standard_normal((d, I)) / 2, L=L)
    out["rnn"] = (st, np.zeros((N, d)), r.standard_normal((L, N, I)), r.standard_normal((L + 1, N, d)))
    r = rnd(12)
    st = O.Stack("gated", "tanh", "none", r.standard_normal((2 * d, d)) / 2, None, U=r.standard_normal((2 * d, I)) / 2, L=L)
    out["gated"] = (st, r.standard_normal((N, d)) / 2, r.standard_normal((L, N, I)), r.standard_normal((L + 1, N, d)))
    r = rnd(13)
    H = d // 2
    st = O.Stack("lstm", "tanh", "none", r.standard_normal((4 * H, H)) / 2, None, U=r.standard_normal((4 * H, I)) / 2, L=L)
    out["lstm"] = (st, r.standard_normal((N, d)) / 2, r.standard_normal((L, N, I)), r.standard_normal((L + 1, N, d)))
    return out


def results(st, x0, xin, e):
    sv = O.forward(st, x0, xin)
    rows = {"x_L": sv["x"][-1]}
    for k in (0, 1, 2):
        rows[f"w{k}_state0"] = O.hbp_backward(st, sv, e, k)[0]
    rows["w1_gamma0.5_state0"] = O.hbp_backward(st, sv, e, 1, gamma=0.5)[0]
    G = O.exact_backward(st, sv, e)
    rows["exact_state0"] = G[0]
    pg = O.param_grads(st, sv, G, xin)
    rows["dW1_first_row"] = pg["dW1"].reshape(-1, pg["dW1"].shape[-1])[0]
    return rows


def main():
    lines = ["# written by tests/golden/make_golden.py from oracle/hbp_oracle.py; see that script's header",
             "# case quantity values..."]
    for name, (st, x0, xin, e) in cases().items():
        for q, v in results(st, x0, xin, e).items():
            lines.append(" ".join([name, q] + [repr(float(t)) for t in np.asarray(v).ravel()]))
    with open(os.path.join(HERE, "oracle_small.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
