"""Pins for the CPU oracle: every check compares the oracle with something the
paper or the mathematics fixes independently of the oracle's own code
(finite differences, closed forms, explicit path enumeration, an independent
autograd library), so a dropped term, wrong index, sign or transposed operand
fails at least one of them.  CPU only.
"""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import hbp_oracle as O

RNG = np.random.default_rng(1234)


def small_mlp(L=4, d=6, dff=10, act="gelu", norm="rms", lam="rand", seed=0):
    r = np.random.default_rng(seed)
    W1 = r.standard_normal((L, dff, d)) / math.sqrt(d)
    W2 = r.standard_normal((L, d, dff)) / math.sqrt(dff)
    lm = None if lam == "one" else r.uniform(0.5, 1.1, (L, d))
    return O.Stack("mlp", act, norm, W1, W2, lam=lm)


def small_rnn(T=5, H=6, I=4, seed=0):
    r = np.random.default_rng(seed)
    Wh = r.standard_normal((H, H)) / math.sqrt(H)
    Wo = r.standard_normal((H, H)) / math.sqrt(H)
    U = r.standard_normal((H, I)) / math.sqrt(I)
    lm = 1.0 / (1.0 + np.exp(-r.normal(3.0, 0.5, (T, H))))
    return O.Stack("rnn", "tanh", "none", Wh, Wo, lam=lm, U=U, L=T)


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("family", ["mlp_rms", "mlp_plain", "rnn"])
def test_finite_termination_and_exact_top_states(family):
    """Theorem 2, last sentence: w_i^k is exact for k >= L - i.  So k = L is exact
    everywhere and after k iterations the top k+1 states already are."""
    r = np.random.default_rng(5)
    if family == "rnn":
        st = small_rnn(T=6)
        N = 3
        xin = r.standard_normal((st.L, N, 4))
        sv = O.forward(st, np.zeros((N, st.d)), xin)
        e = r.standard_normal((st.L + 1, N, st.d))
        e[0] = 0
    else:
        st = small_mlp(L=6, norm="rms" if family == "mlp_rms" else "none",
                       lam="rand" if family == "mlp_rms" else "one")
        N = 3
        sv = O.forward(st, r.standard_normal((N, st.d)))
        e = r.standard_normal((N, st.d))
    G = O.exact_backward(st, sv, e)
    L = st.L
    for k in range(L + 2):
        w = O.hbp_backward(st, sv, e, k)
        lo = max(L - k, 0)
        np.testing.assert_allclose(w[lo:], G[lo:], rtol=1e-11, atol=1e-12)
        if k < L - 1:      # and it is a genuine truncation below that
            assert O.rel_l2(w[0], G[0]) > 1e-6
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L), G, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- P2
def test_k0_is_cumulative_product_of_lambda_depth():
    """Initial estimate of Theorem 2 with a loss on the last state only:
    w_i^0 = e_L K_L ... K_{i+1}."""
    st = small_mlp(L=5)
    N = 4
    sv = O.forward(st, RNG.standard_normal((N, st.d)))
    e = RNG.standard_normal((N, st.d))
    w0 = O.hbp_backward(st, sv, e, 0)
    for l in range(st.L + 1):
        prod = np.ones(st.d)
        for m in range(l, st.L):
            prod = prod * st.lam[m]
        np.testing.assert_allclose(w0[l], e * prod[None, :], rtol=1e-13)


def test_k0_rnn_double_sum():
    """w_i^0 = sum_{j>=i} e_j K_j ... K_{i+1} with a loss at every state."""
    st = small_rnn(T=6)
    N = 2
    xin = RNG.standard_normal((st.L, N, 4))
    sv = O.forward(st, np.zeros((N, st.d)), xin)
    e = RNG.standard_normal((st.L + 1, N, st.d))
    w0 = O.hbp_backward(st, sv, e, 0)
    for i in range(st.L + 1):
        acc = np.zeros((N, st.d))
        for j in range(i, st.L + 1):
            prod = np.ones(st.d)
            for m in range(i, j):
                prod = prod * st.lam[m]
            acc += e[j] * prod[None, :]
        np.testing.assert_allclose(w0[i], acc, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- P3
def test_zero_block_closed_form():
    """Blocks with W2 = 0: the stack is x_l = x_0 prod(lam), every iteration
    returns w^0, dW1 = 0 and dW2_l = sum_n w^0_{l+1}[n]^T act(W1 norm(x_l)[n])."""
    st = small_mlp(L=4)
    st.W2[:] = 0.0
    N = 5
    x0 = RNG.standard_normal((N, st.d))
    sv = O.forward(st, x0)
    e = RNG.standard_normal((N, st.d))
    prod = np.ones(st.d)
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], x0 * prod[None, :], rtol=1e-13)
        if l < st.L:
            prod = prod * st.lam[l]
    w0 = O.hbp_backward(st, sv, e, 0)
    for k in (1, 3):
        np.testing.assert_allclose(O.hbp_backward(st, sv, e, k), w0, rtol=0, atol=0)
    pg = O.param_grads(st, sv, w0)
    assert np.all(pg["dW1"] == 0)
    for l in range(st.L):
        xl = sv["x"][l]
        yl = xl / np.sqrt(np.mean(xl ** 2, axis=1, keepdims=True) + st.eps)
        al = yl @ st.W1[l].T
        zl = np.array([[0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in row] for row in al])
        tail = np.ones(st.d)
        for m in range(l + 1, st.L):
            tail = tail * st.lam[m]
        want = (e * tail[None, :]).T @ zl
        np.testing.assert_allclose(pg["dW2"][l], want, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- P4
def _loss(st, x0, xin, c):
    sv = O.forward(st, x0, xin)
    return float(np.sum(c * sv["x"]))


@pytest.mark.parametrize("family", ["mlp_rms_gelu", "mlp_none_gelu", "mlp_rms_tanh", "rnn"])
def test_exact_gradient_by_finite_differences(family):
    """Central differences of loss = sum_l <c_l, x_l> against exact_backward (state
    gradient at x_0) and param_grads (every weight entry of a tiny stack)."""
    r = np.random.default_rng(11)
    N = 2
    if family == "rnn":
        st = small_rnn(T=4, H=5, I=3)
        xin = r.standard_normal((st.L, N, 3))
        x0 = r.standard_normal((N, st.d)) * 0.3     # non-zero h_0 exercises g[0]
    else:
        _, norm, act = family.split("_")
        st = small_mlp(L=3, d=5, dff=7, act=act, norm=norm)
        xin = None
        x0 = r.standard_normal((N, st.d))
    c = r.standard_normal((st.L + 1, N, st.d))
    sv = O.forward(st, x0, xin)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G, xin)
    h = 1e-6

    def fd(arr):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h
            lp = _loss(st, x0, xin, c)
            arr[i] = old - h
            lm = _loss(st, x0, xin, c)
            arr[i] = old
            out[i] = (lp - lm) / (2 * h)
        return out

    np.testing.assert_allclose(G[0], fd(x0), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(pg["dW1"], fd(st.W1), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(pg["dW2"], fd(st.W2), rtol=2e-6, atol=2e-8)
    if family == "rnn":
        np.testing.assert_allclose(pg["dU"], fd(st.U), rtol=2e-6, atol=2e-8)


# ---------------------------------------------------------------- P5
def test_scalar_linear_binomial_closed_form():
    """J = c I and K = a I: paths with exactly j Jacobians among L - i layers
    number C(L-i, j), so w_i^k = e_L sum_{j<=min(k,L-i)} C(L-i,j) c^j a^(L-i-j)."""
    L, d, N = 7, 3, 2
    c, a = 0.37, 0.9
    W1 = np.tile(np.eye(d)[None], (L, 1, 1))
    W2 = np.tile((c * np.eye(d))[None], (L, 1, 1))
    st = O.Stack("mlp", "identity", "none", W1, W2, lam=np.full((L, d), a))
    sv = O.forward(st, RNG.standard_normal((N, d)))
    e = RNG.standard_normal((N, d))
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k)
        for i in range(L + 1):
            n = L - i
            coef = sum(math.comb(n, j) * c ** j * a ** (n - j) for j in range(min(k, n) + 1))
            np.testing.assert_allclose(w[i], coef * e, rtol=1e-12)


# ---------------------------------------------------------------- P6
def _dense_block_jacobians(st, sv, n):
    """J_l[out, in] = d block_l(x)[out] / d x[in] for token n, by central
    differences of the block's forward map (independent of block_vjp)."""
    L, d = st.L, st.d
    Js = []
    for l in range(L):
        x = sv["x"][l][n].copy()

        def blk(xv):
            if st.norm == "rms":
                yv = xv / math.sqrt(np.mean(xv * xv) + st.eps)
            else:
                yv = xv
            return O.act_fn(st.act, st.w1(l) @ yv) @ st.w2(l).T

        J = np.zeros((d, d))
        for i in range(d):
            h = 1e-6
            xp, xm = x.copy(), x.copy()
            xp[i] += h
            xm[i] -= h
            J[:, i] = (blk(xp) - blk(xm)) / (2 * h)
        Js.append(J)
    return Js


def test_path_enumeration_matches_theorem():
    """Theorems 1 and 2: w_i^k is the sum over end states j >= i and subsets of
    blocks of size <= k of e_j times the product of J (chosen) or K (not)."""
    st = small_mlp(L=5, d=3, dff=4)
    N = 1
    r = np.random.default_rng(3)
    sv = O.forward(st, r.standard_normal((N, st.d)))
    e = r.standard_normal((st.L + 1, N, st.d))
    e[0] = 0
    Js = _dense_block_jacobians(st, sv, 0)
    Ks = [np.diag(st.lam[l]) for l in range(st.L)]
    L = st.L
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k)
        for i in range(L + 1):
            acc = np.zeros(st.d)
            for j in range(i, L + 1):
                layers = list(range(i, j))          # blocks between state i and state j
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):   # row vector times matrices, top block first
                            vec = vec @ (Js[l] if l in chosen else Ks[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=2e-6, atol=2e-8)
    # k = L enumerates all 2^L paths: the full gradient (Theorem 1)
    G = O.exact_backward(st, sv, e)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L), G, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- P7
@pytest.mark.parametrize("P", [1, 2, 5, 8, 13])
def test_cumsumprod_definition_and_hillis_steele(P):
    """CumSumProd(a, M)_i = sum_{j>=i} a_j M_j ... M_{i+1}, and the parallel
    Hillis-Steele form of the appendix gives the same result."""
    r = np.random.default_rng(P)
    d, N = 4, 3
    a = r.standard_normal((P, N, d))
    lam = r.uniform(0.3, 1.2, (P, d))
    rows = lambda i: lam[i]
    u = O.cumsumprod_reverse(a, rows)
    want = np.zeros_like(a)
    for i in range(P):
        for j in range(i, P):
            prod = np.ones(d)
            for m in range(i, j):
                prod = prod * lam[m]
            want[i] += a[j] * prod[None, :]
    np.testing.assert_allclose(u, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(O.cumsumprod_hillis_steele(a, rows), want, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- P8
def test_fixed_point_iteration_special_case():
    """K = 0 (lambda = 0): only the pure-Jacobian path survives, so with a loss
    on the last state w_i^k is the exact gradient for i >= L - k and 0 below."""
    st = small_mlp(L=5)
    st.lam[:] = 0.0
    N = 2
    sv = O.forward(st, RNG.standard_normal((N, st.d)))
    e = RNG.standard_normal((N, st.d))
    G = O.exact_backward(st, sv, e)
    for k in range(st.L + 1):
        w = O.hbp_backward(st, sv, e, k)
        for i in range(st.L + 1):
            if i >= st.L - k:
                np.testing.assert_allclose(w[i], G[i], rtol=1e-12, atol=1e-14)
            else:
                assert np.all(w[i] == 0)


# ---------------------------------------------------------------- P8b, P9b
@pytest.mark.parametrize("gamma", [0.2, 0.8, 1.0])
def test_gamma_iterates_by_path_enumeration(gamma):
    """With gamma the layer is split into J' = J + gamma K and K' = (1 - gamma) K;
    Theorem 2 applied to that pair: w_i^k sums, over end states j >= i and at most
    k blocks taken through J', the products of J' (chosen) and K' (not)."""
    st = small_mlp(L=5, d=3, dff=4)
    N = 1
    r = np.random.default_rng(11)
    sv = O.forward(st, r.standard_normal((N, st.d)))
    e = r.standard_normal((st.L + 1, N, st.d))
    e[0] = 0
    Js = _dense_block_jacobians(st, sv, 0)
    Ks = [np.diag(st.lam[l]) for l in range(st.L)]
    Jg = [Js[l] + gamma * Ks[l] for l in range(st.L)]
    Kg = [(1.0 - gamma) * Ks[l] for l in range(st.L)]
    L = st.L
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(st.d)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):
                            vec = vec @ (Jg[l] if l in chosen else Kg[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=2e-6, atol=2e-8)
    G = O.exact_backward(st, sv, e)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), G, rtol=1e-10, atol=1e-12)


def test_gamma_one_is_the_fixed_point_iteration():
    """gamma = 1 leaves nothing on the residual path: the iterates are those of
    k sweeps w_l <- e_l + w_{l+1} (J_l + K_l) through all layers at once, from
    w = e (the fixed-point-iteration baseline), written here with dense matrices."""
    st = small_mlp(L=6, d=4, dff=5)
    r = np.random.default_rng(5)
    sv = O.forward(st, r.standard_normal((1, st.d)))
    e = r.standard_normal((st.L + 1, 1, st.d))
    e[0] = 0
    Js = _dense_block_jacobians(st, sv, 0)
    T = [Js[l] + np.diag(st.lam[l]) for l in range(st.L)]
    w = e[:, 0, :].copy()
    for k in range(st.L + 2):
        got = O.hbp_backward(st, sv, e, k, gamma=1.0)[:, 0, :]
        np.testing.assert_allclose(got, w, rtol=2e-6, atol=2e-8)
        nxt = e[:, 0, :].copy()
        for l in range(st.L):
            nxt[l] = e[l, 0] + w[l + 1] @ T[l]
        w = nxt


def test_gamma_zero_is_the_plain_method():
    st = small_rnn()
    r = np.random.default_rng(2)
    xin = r.standard_normal((st.L, 2, st.U.shape[1]))
    sv = O.forward(st, np.zeros((2, st.d)), xin)
    e = r.standard_normal((st.L + 1, 2, st.d))
    e[0] = 0
    for k in (0, 1, 3):
        assert np.array_equal(O.hbp_backward(st, sv, e, k), O.hbp_backward(st, sv, e, k, gamma=0.0))


# ---------------------------------------------------------------- P10b: per-token diagonal K
def _per_token(st, N, seed):
    """The same stack with a coefficient per (block, token, channel)."""
    r = np.random.default_rng(seed)
    lam = r.uniform(0.4, 1.1, (st.L, N, st.d))
    return O.Stack(st.kind, st.act, st.norm, st.W1, st.W2, lam=lam, U=st.U, eps=st.eps, L=st.L)


@pytest.mark.parametrize("family", ["mlp", "rnn"])
def test_per_token_coefficients_token_by_token(family):
    """Tokens are independent: a stack with coefficients [L, N, d] gives, for token
    n, what the per-channel stack built from lam[:, n, :] gives for that token alone
    (forward state, exact gradient, every Highway-BP iterate, with and without gamma)."""
    r = np.random.default_rng(21)
    N = 3
    if family == "rnn":
        base = small_rnn(T=5, H=4, I=3)
        xin = r.standard_normal((base.L, N, 3))
        x0 = np.zeros((N, base.d))
    else:
        base = small_mlp(L=4, d=5, dff=6)
        xin = None
        x0 = r.standard_normal((N, base.d))
    st = _per_token(base, N, 5)
    e = r.standard_normal((st.L + 1, N, st.d))
    e[0] = 0
    sv = O.forward(st, x0, xin)
    G = O.exact_backward(st, sv, e)
    for n in range(N):
        one = O.Stack(st.kind, st.act, st.norm, st.W1, st.W2, lam=st.lam[:, n, :], U=st.U, eps=st.eps, L=st.L)
        xin1 = None if xin is None else xin[:, n:n + 1]
        sv1 = O.forward(one, x0[n:n + 1], xin1)
        np.testing.assert_allclose(sv["x"][:, n], sv1["x"][:, 0], rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(G[:, n], O.exact_backward(one, sv1, e[:, n:n + 1])[:, 0], rtol=1e-12, atol=1e-14)
        for k in (0, 1, 2, st.L):
            for gamma in (0.0, 0.3):
                w = O.hbp_backward(st, sv, e, k, gamma=gamma)
                w1 = O.hbp_backward(one, sv1, e[:, n:n + 1], k, gamma=gamma)
                np.testing.assert_allclose(w[:, n], w1[:, 0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, st.L), G, rtol=1e-11, atol=1e-13)


def test_per_token_coefficients_by_finite_differences():
    """Exact gradient with per-token coefficients (held fixed as data) against central
    differences of the loss in x_0 and in every weight; k = 0 is the per-token
    cumulative product of the coefficients."""
    r = np.random.default_rng(8)
    N = 2
    st = _per_token(small_mlp(L=3, d=4, dff=5), N, 9)
    x0 = r.standard_normal((N, st.d))
    c = r.standard_normal((st.L + 1, N, st.d))
    sv = O.forward(st, x0)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G)
    h = 1e-6

    def fd(arr):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h
            lp = _loss(st, x0, None, c)
            arr[i] = old - h
            lm = _loss(st, x0, None, c)
            arr[i] = old
            out[i] = (lp - lm) / (2 * h)
        return out

    np.testing.assert_allclose(G[0], fd(x0), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(pg["dW1"], fd(st.W1), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(pg["dW2"], fd(st.W2), rtol=2e-6, atol=2e-8)
    eL = r.standard_normal((N, st.d))
    w0 = O.hbp_backward(st, sv, eL, 0)
    for i in range(st.L + 1):
        prod = np.ones((N, st.d))
        for m in range(i, st.L):
            prod = prod * st.lam[m]
        np.testing.assert_allclose(w0[i], eL * prod, rtol=1e-13)


# ---------------------------------------------------------------- P9
def test_gamma_reparametrisation_leaves_exact_gradient_unchanged():
    """Moving gamma*x from the residual connection into the block changes J and K
    but not J + K, so the exact gradient is the same (identity activation lets
    the block absorb gamma*x as extra hidden units)."""
    L, d, dff, N, gamma = 4, 4, 6, 3, 0.2
    r = np.random.default_rng(9)
    W1 = r.standard_normal((L, dff, d)) / 2
    W2 = r.standard_normal((L, d, dff)) / 2
    lam = r.uniform(0.6, 1.0, (L, d))
    stA = O.Stack("mlp", "identity", "none", W1, W2, lam=lam)
    W1b = np.concatenate([W1, np.tile(np.eye(d)[None], (L, 1, 1))], axis=1)
    W2b = np.concatenate([W2, np.tile((gamma * np.eye(d))[None], (L, 1, 1))], axis=2)
    stB = O.Stack("mlp", "identity", "none", W1b, W2b, lam=lam - gamma)
    x0 = r.standard_normal((N, d))
    e = r.standard_normal((N, d))
    svA, svB = O.forward(stA, x0), O.forward(stB, x0)
    np.testing.assert_allclose(svA["x"], svB["x"], rtol=1e-11, atol=1e-13)
    GA, GB = O.exact_backward(stA, svA, e), O.exact_backward(stB, svB, e)
    np.testing.assert_allclose(GA, GB, rtol=1e-11, atol=1e-13)
    # the truncated estimates do differ
    assert O.rel_l2(O.hbp_backward(stA, svA, e, 1), O.hbp_backward(stB, svB, e, 1)) > 1e-4


# ---------------------------------------------------------------- P10
@pytest.mark.parametrize("family", ["mlp", "rnn"])
def test_exact_gradient_against_torch_autograd(family):
    """The same stack written with torch fp64 ops and differentiated by torch's
    autograd: forward states, all state gradients and all parameter gradients."""
    r = np.random.default_rng(21)
    N = 4
    if family == "mlp":
        st = small_mlp(L=4, d=8, dff=12)
        xin = None
        x0 = r.standard_normal((N, st.d))
    else:
        st = small_rnn(T=5, H=8, I=6)
        xin = r.standard_normal((st.L, N, 6))
        x0 = np.zeros((N, st.d))
    c = r.standard_normal((st.L + 1, N, st.d))
    c[0] = 0
    sv = O.forward(st, x0, xin)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G, xin)

    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W1, W2, lam = t(st.W1), t(st.W2), torch.tensor(st.lam)
    U = t(st.U) if st.U is not None else None
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        if st.norm == "rms":
            y = x / torch.sqrt((x * x).mean(dim=1, keepdim=True) + st.eps)
        else:
            y = x
        if family == "mlp":
            a = y @ W1[l].T
            z = torch.nn.functional.gelu(a)       # exact erf form
            nxt = lam[l] * x + z @ W2[l].T
        else:
            a = y @ W1.T + torch.tensor(xin[l]) @ U.T
            nxt = lam[l] * x + torch.tanh(a) @ W2.T
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW1"], W1.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW2"], W2.grad.numpy(), rtol=1e-10, atol=1e-12)
    if U is not None:
        np.testing.assert_allclose(pg["dU"], U.grad.numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- P11
def test_param_grads_use_the_given_estimate():
    """Parameter gradients are linear in the state-gradient estimate handed in
    (sentence after Theorem 2): dtheta(w^k) for k < L differs from the exact one
    and equals it at k = L."""
    st = small_mlp(L=4)
    N = 3
    sv = O.forward(st, RNG.standard_normal((N, st.d)))
    e = RNG.standard_normal((N, st.d))
    G = O.exact_backward(st, sv, e)
    full = O.param_grads(st, sv, G)
    at_L = O.param_grads(st, sv, O.hbp_backward(st, sv, e, st.L))
    np.testing.assert_allclose(at_L["dW1"], full["dW1"], rtol=1e-11, atol=1e-13)
    w1 = O.hbp_backward(st, sv, e, 1)
    p1 = O.param_grads(st, sv, w1)
    p1b = O.param_grads(st, sv, 2.0 * w1)
    np.testing.assert_allclose(p1b["dW2"], 2.0 * p1["dW2"], rtol=1e-12)
    # top block sees the exact gradient at any k; lower ones do not at k = 1
    np.testing.assert_allclose(p1["dW2"][-1], full["dW2"][-1], rtol=1e-11, atol=1e-13)
    assert O.rel_l2(p1["dW1"][0], full["dW1"][0]) > 1e-4


# ---------------------------------------------------------------- P12: r(x, z) = ReLU(lam (.) x + z)
def small_relu_mlp(L=4, d=6, dff=10, norm="rms", seed=5):
    st = small_mlp(L=L, d=d, dff=dff, norm=norm, seed=seed)
    st.post = "relu"
    return st


@pytest.mark.parametrize("norm", ["rms", "none"])
def test_relu_after_the_sum_against_torch_autograd(norm):
    """The original-ResNet residual function (table of layer decompositions): forward states, every
    state gradient and every parameter gradient against torch's autograd of the same stack in fp64."""
    r = np.random.default_rng(31)
    N = 5
    st = small_relu_mlp(L=5, d=8, dff=12, norm=norm)
    x0 = r.standard_normal((N, st.d))
    c = r.standard_normal((st.L + 1, N, st.d))
    sv = O.forward(st, x0)
    assert 0.1 < sv["mask"].mean() < 0.9            # both branches of the ReLU occur
    assert np.all(sv["x"][1:] >= 0)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G)

    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W1, W2, lam = t(st.W1), t(st.W2), torch.tensor(st.lam)
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        y = x / torch.sqrt((x * x).mean(dim=1, keepdim=True) + st.eps) if norm == "rms" else x
        nxt = torch.relu(lam[l] * x + torch.nn.functional.gelu(y @ W1[l].T) @ W2[l].T)
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW1"], W1.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW2"], W2.grad.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("gamma", [0.0, 0.3])
def test_relu_after_the_sum_by_path_enumeration(gamma):
    """Theorem 2 with K_l = diag(m_l lam_l) and J_l = diag(m_l) . (block Jacobian), m_l the ReLU's mask: every
    iterate is the sum over paths with at most k block steps.  The block Jacobians come from central
    differences of the block's forward map and the masks from the sign of the states."""
    st = small_relu_mlp(L=5, d=3, dff=4, seed=8)
    r = np.random.default_rng(4)
    sv = O.forward(st, r.standard_normal((1, st.d)) + 0.5)
    e = r.standard_normal((st.L + 1, 1, st.d))
    Jb = _dense_block_jacobians(st, sv, 0)
    L = st.L
    Ms = [np.diag((sv["x"][l + 1][0] > 0).astype(float)) for l in range(L)]
    assert 0 < sum(M.trace() for M in Ms) < L * st.d
    Ks = [(1 - gamma) * Ms[l] @ np.diag(st.lam[l]) for l in range(L)]
    Js = [Ms[l] @ Jb[l] + gamma * Ms[l] @ np.diag(st.lam[l]) for l in range(L)]
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(st.d)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):
                            vec = vec @ (Js[l] if l in chosen else Ks[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), O.exact_backward(st, sv, e),
                               rtol=1e-10, atol=1e-12)


def test_relu_after_the_sum_finite_termination():
    """Theorem 2's guarantee (exact for k >= L - i) holds with the non-linear residual function."""
    st = small_relu_mlp(L=6, d=5, dff=7, seed=2)
    r = np.random.default_rng(6)
    sv = O.forward(st, r.standard_normal((3, st.d)))
    e = r.standard_normal((3, st.d))
    G = O.exact_backward(st, sv, e)
    for k in range(st.L + 1):
        w = O.hbp_backward(st, sv, e, k)
        for i in range(st.L + 1):
            if k >= st.L - i:
                np.testing.assert_allclose(w[i], G[i], rtol=1e-11, atol=1e-13)
    assert O.rel_l2(O.hbp_backward(st, sv, e, 1)[0], G[0]) > 1e-3


# ---------------------------------------------------------------- P13: the gated recurrent cell (GRU row of the table)
def small_gated(T=5, H=6, I=4, seed=0):
    r = np.random.default_rng(seed)
    W = r.standard_normal((2 * H, H)) / math.sqrt(H)
    U = r.standard_normal((2 * H, I)) / math.sqrt(I)
    return O.Stack("gated", "tanh", "none", W, None, U=U, L=T)


def test_gated_cell_against_torch_autograd():
    """x' = (1 - u) x + u c with u = sigmoid(.), c = tanh(.): states, every state gradient and the gradients of
    both weight matrices against torch's autograd of the same recurrence in fp64."""
    r = np.random.default_rng(41)
    N, I = 3, 5
    st = small_gated(T=6, H=7, I=I)
    H_ = st.d
    xin = r.standard_normal((st.L, N, I))
    x0 = r.standard_normal((N, H_)) * 0.5
    c = r.standard_normal((st.L + 1, N, H_))
    sv = O.forward(st, x0, xin)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G, xin)
    assert set(pg) == {"dW1", "dU"}

    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W, U = t(st.W1), t(st.U)
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        pre = x @ W.T + torch.tensor(xin[l]) @ U.T
        u, cc = torch.sigmoid(pre[:, :H_]), torch.tanh(pre[:, H_:])
        nxt = (1 - u) * x + u * cc
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW1"], W.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dU"], U.grad.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("gamma", [0.0, 0.4])
def test_gated_cell_by_path_enumeration(gamma):
    """Theorem 2 for r(x, z) = z1 (.) x + z2: K_l = diag(1 - u_l) (a function of the state) and J_l = the Jacobian
    of h -> (1 - u(h)) (.) x_l + u(h) (.) c(h) with x_l held fixed, by central differences."""
    st = small_gated(T=5, H=3, I=2, seed=3)
    r = np.random.default_rng(9)
    xin = r.standard_normal((st.L, 1, 2))
    sv = O.forward(st, r.standard_normal((1, st.d)) * 0.5, xin)
    e = r.standard_normal((st.L + 1, 1, st.d))
    L, H_ = st.L, st.d

    def jac(l):
        x = sv["x"][l][0]

        def via_g(h):
            pre = st.W1 @ h + st.U @ xin[l][0]
            u, c = 1 / (1 + np.exp(-pre[:H_])), np.tanh(pre[H_:])
            return (1 - u) * x + u * c
        J = np.zeros((H_, H_))
        for i in range(H_):
            hp, hm = x.copy(), x.copy()
            hp[i] += 1e-6
            hm[i] -= 1e-6
            J[:, i] = (via_g(hp) - via_g(hm)) / 2e-6
        return J
    np.testing.assert_array_equal(sv["a"], 1 - sv["u"])
    Kd = [np.diag(1 - sv["u"][l][0]) for l in range(L)]
    Js = [jac(l) + gamma * Kd[l] for l in range(L)]
    Ks = [(1 - gamma) * Kd[l] for l in range(L)]
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(H_)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):
                            vec = vec @ (Js[l] if l in chosen else Ks[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), O.exact_backward(st, sv, e),
                               rtol=1e-10, atol=1e-12)


def test_gated_cell_k0_and_finite_termination():
    """w^0 carries e_T down by the products of the cell's own 1 - u; exact once k >= T - i."""
    st = small_gated(T=6, H=4, I=3, seed=5)
    r = np.random.default_rng(2)
    xin = r.standard_normal((st.L, 2, 3))
    sv = O.forward(st, np.zeros((2, st.d)), xin)
    e = r.standard_normal((2, st.d))
    w0 = O.hbp_backward(st, sv, e, 0)
    prod = np.ones_like(e)
    for l in range(st.L - 1, -1, -1):
        prod = prod * (1 - sv["u"][l])
        np.testing.assert_allclose(w0[l], e * prod, rtol=1e-12)
    G = O.exact_backward(st, sv, e)
    for k in range(st.L + 1):
        w = O.hbp_backward(st, sv, e, k)
        for i in range(st.L + 1):
            if k >= st.L - i:
                np.testing.assert_allclose(w[i], G[i], rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- the standard GRU (reset gate included)
def small_gru(T=5, H=6, I=4, seed=0):
    r = np.random.default_rng(seed)
    W = r.standard_normal((3 * H, H)) / math.sqrt(H)
    U = r.standard_normal((3 * H, I)) / math.sqrt(I)
    return O.Stack("gru", "tanh", "none", W, None, U=U, L=T)


def test_gru_cell_against_torch_autograd_and_torch_grucell_form():
    """The standard GRU: states, every state gradient and both weight gradients against torch's autograd of the
    same recurrence written out in fp64."""
    r = np.random.default_rng(43)
    N, I = 3, 5
    st = small_gru(T=6, H=7, I=I)
    H_ = st.d
    xin = r.standard_normal((st.L, N, I))
    x0 = r.standard_normal((N, H_)) * 0.5
    c = r.standard_normal((st.L + 1, N, H_))
    sv = O.forward(st, x0, xin)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G, xin)
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W, U = t(st.W1), t(st.U)
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        ux = torch.tensor(xin[l]) @ U.T
        z = torch.sigmoid(x @ W[:H_].T + ux[:, :H_])
        rr = torch.sigmoid(x @ W[H_:2 * H_].T + ux[:, H_:2 * H_])
        n = torch.tanh((rr * x) @ W[2 * H_:].T + ux[:, 2 * H_:])
        nxt = (1 - z) * x + z * n
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW1"], W.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dU"], U.grad.numpy(), rtol=1e-10, atol=1e-12)
    # with the reset gate held open (its rows of W and U zero, a large constant input) the cell is the gated cell
    H2 = 4
    g2 = small_gated(T=4, H=H2, I=3, seed=8)
    W3 = np.concatenate([g2.W1[:H2], np.zeros((H2, H2)), g2.W1[H2:]])
    U3 = np.concatenate([g2.U[:H2], np.zeros((H2, 3)), g2.U[H2:]])
    U3 = np.concatenate([U3, np.concatenate([np.zeros(H2), np.full(H2, 40.0), np.zeros(H2)])[:, None]], axis=1)
    gr = O.Stack("gru", "tanh", "none", W3, None, U=U3, L=4)
    xin2 = r.standard_normal((4, 2, 3))
    x02 = r.standard_normal((2, H2)) * 0.5
    sv_a = O.forward(g2, x02, xin2)
    sv_b = O.forward(gr, x02, np.concatenate([xin2, np.ones((4, 2, 1))], axis=-1))
    np.testing.assert_allclose(sv_b["x"], sv_a["x"], rtol=1e-12, atol=1e-13)
    e2 = r.standard_normal((5, 2, H2))
    for k in (0, 1, 2, 4):
        np.testing.assert_allclose(O.hbp_backward(gr, sv_b, e2, k), O.hbp_backward(g2, sv_a, e2, k), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("gamma", [0.0, 0.4])
def test_gru_cell_by_path_enumeration(gamma):
    """Theorem 2 with K_l = diag(1 - z_l) and J_l = the Jacobian of h -> (1 - z(h)) (.) x_l + z(h) (.) n(h) with x_l
    held fixed in the residual term, by central differences."""
    st = small_gru(T=5, H=3, I=2, seed=3)
    r = np.random.default_rng(9)
    xin = r.standard_normal((st.L, 1, 2))
    sv = O.forward(st, r.standard_normal((1, st.d)) * 0.5, xin)
    e = r.standard_normal((st.L + 1, 1, st.d))
    L, H_ = st.L, st.d

    def jac(l):
        x = sv["x"][l][0]

        def via_g(h):
            ux = st.U @ xin[l][0]
            z = 1 / (1 + np.exp(-(st.W1[:H_] @ h + ux[:H_])))
            rr = 1 / (1 + np.exp(-(st.W1[H_:2 * H_] @ h + ux[H_:2 * H_])))
            n = np.tanh(st.W1[2 * H_:] @ (rr * h) + ux[2 * H_:])
            return (1 - z) * x + z * n
        J = np.zeros((H_, H_))
        for i in range(H_):
            hp, hm = x.copy(), x.copy()
            hp[i] += 1e-6
            hm[i] -= 1e-6
            J[:, i] = (via_g(hp) - via_g(hm)) / 2e-6
        return J
    Kd = [np.diag(1 - sv["zrn"][l][0][:H_]) for l in range(L)]
    Js = [jac(l) + gamma * Kd[l] for l in range(L)]
    Ks = [(1 - gamma) * Kd[l] for l in range(L)]
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(H_)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):
                            vec = vec @ (Js[l] if l in chosen else Ks[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), O.exact_backward(st, sv, e),
                               rtol=1e-10, atol=1e-12)


def test_gru_cell_parameter_gradients_by_finite_differences():
    """Every entry of W1 = [W_z; W_r; W_n] and of U by central differences of a scalar loss."""
    st = small_gru(T=4, H=3, I=2, seed=6)
    r = np.random.default_rng(12)
    xin = r.standard_normal((st.L, 2, 2))
    x0 = r.standard_normal((2, st.d)) * 0.5
    c = r.standard_normal((st.L + 1, 2, st.d))

    def loss(W, U):
        s2 = O.Stack("gru", "tanh", "none", W, None, U=U, L=st.L)
        return float(np.sum(c * O.forward(s2, x0, xin)["x"]))
    sv = O.forward(st, x0, xin)
    pg = O.param_grads(st, sv, O.exact_backward(st, sv, c), xin)
    for name, M in (("dW1", st.W1), ("dU", st.U)):
        num = np.zeros_like(M)
        for idx in np.ndindex(M.shape):
            Mp, Mm = M.copy(), M.copy()
            Mp[idx] += 1e-6
            Mm[idx] -= 1e-6
            num[idx] = ((loss(Mp, st.U) - loss(Mm, st.U)) if name == "dW1" else (loss(st.W1, Mp) - loss(st.W1, Mm))) / 2e-6
        np.testing.assert_allclose(pg[name], num, rtol=2e-6, atol=2e-8)


# ---------------------------------------------------------------- attention sub-blocks (appendix, GPT-2 paragraph)
def small_transformer(layers=2, d=8, dff=12, T=4, heads=2, causal=True, norm="rms", lam="rand", seed=0, post="none"):
    r = np.random.default_rng(seed)
    W1 = r.standard_normal((layers, dff, d)) / math.sqrt(d)
    W2 = r.standard_normal((layers, d, dff)) / math.sqrt(dff)
    Wqkv = r.standard_normal((layers, 3 * d, d)) / math.sqrt(d) * 1.5
    Wo = r.standard_normal((layers, d, d)) / math.sqrt(d)
    lm = None if lam == "one" else r.uniform(0.5, 1.1, (2 * layers, d))
    return O.Stack("transformer", "gelu", norm, W1, W2, lam=lm, Wqkv=Wqkv, Wo=Wo, T=T, heads=heads, causal=causal, post=post)


@pytest.mark.parametrize("causal,norm,post", [(True, "rms", "none"), (False, "rms", "none"), (True, "none", "none"),
                                              (False, "none", "rms"), (True, "none", "rms")])
def test_transformer_stack_against_torch_autograd(causal, norm, post):
    """The alternating attention / MLP stack written with torch fp64 ops, the attention itself by torch's own
    scaled_dot_product_attention, differentiated by autograd: states, state gradients, all four weight gradients."""
    r = np.random.default_rng(31)
    B, T, heads = 3, 5, 2
    st = small_transformer(layers=2, d=8, dff=12, T=T, heads=heads, causal=causal, norm=norm, post=post)
    d = st.d
    x0 = r.standard_normal((B * T, d))
    c = r.standard_normal((st.L + 1, B * T, d))
    sv = O.forward(st, x0)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G)
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W1, W2, Wqkv, Wo, lam = t(st.W1), t(st.W2), t(st.Wqkv), t(st.Wo), torch.tensor(st.lam)
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        y = x / torch.sqrt((x * x).mean(dim=1, keepdim=True) + st.eps) if norm == "rms" else x
        if l % 2 == 0:
            qkv = (y @ Wqkv[l // 2].T).reshape(B, T, 3, heads, d // heads).permute(2, 0, 3, 1, 4)
            o = torch.nn.functional.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=causal)
            nxt = lam[l] * x + o.permute(0, 2, 1, 3).reshape(B * T, d) @ Wo[l // 2].T
        else:
            nxt = lam[l] * x + torch.nn.functional.gelu(y @ W1[l // 2].T) @ W2[l // 2].T
        if post == "rms":      # post-norm: the norm after the residual sum
            nxt = nxt / torch.sqrt((nxt * nxt).mean(dim=1, keepdim=True) + st.eps)
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for k in (0, 1, st.L):     # the iteration ends at the exact gradient for this residual function too
        w = O.hbp_backward(st, sv, c, k, gamma=0.8 if post == "rms" else 0.0)
        if k == st.L:
            np.testing.assert_allclose(w, G, rtol=1e-9, atol=1e-11)
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-9, atol=1e-11)
    for name, w in (("dW1", W1), ("dW2", W2), ("dWqkv", Wqkv), ("dWo", Wo)):
        np.testing.assert_allclose(pg[name], w.grad.numpy(), rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("gamma", [0.0, 0.2])
def test_transformer_stack_by_path_enumeration(gamma):
    """Theorem 2 for one sequence taken as a single state vector of T d entries: K_l = diag(lam_l) repeated per token,
    J_l = the Jacobian of the whole sub-block (attention couples the tokens), by central differences."""
    st = small_transformer(layers=2, d=4, dff=5, T=3, heads=2, seed=4)
    r = np.random.default_rng(17)
    T, d, L = st.T, st.d, st.L
    x0 = r.standard_normal((T, d))
    sv = O.forward(st, x0)
    e = r.standard_normal((L + 1, T, d))

    def block(xflat, l):
        x = xflat.reshape(T, d)
        y = x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + st.eps)
        if l % 2 == 0:
            qkv = y @ st.Wqkv[l // 2].T
            out = np.zeros((T, d))
            dh = d // st.heads
            for h in range(st.heads):
                q, k, v = (qkv[:, j * d + h * dh: j * d + (h + 1) * dh] for j in range(3))
                for i in range(T):          # one query at a time, its own softmax over the keys it may see
                    sc = np.array([q[i] @ k[j] / math.sqrt(dh) for j in range(i + 1)])
                    pr = np.exp(sc) / np.exp(sc).sum()
                    out[i, h * dh:(h + 1) * dh] = sum(pr[j] * v[j] for j in range(i + 1))
            return (out @ st.Wo[l // 2].T).ravel()
        a = y @ st.W1[l // 2].T
        return ((0.5 * a * (1 + np.vectorize(math.erf)(a / math.sqrt(2)))) @ st.W2[l // 2].T).ravel()

    def jac(l):
        xf = sv["x"][l].ravel()
        J = np.zeros((T * d, T * d))
        for i in range(T * d):
            hp, hm = xf.copy(), xf.copy()
            hp[i] += 1e-6
            hm[i] -= 1e-6
            J[:, i] = (block(hp, l) - block(hm, l)) / 2e-6
        return J
    # the forward state the oracle produced is the one this independent block function produces
    for l in range(L):
        np.testing.assert_allclose(sv["x"][l + 1].ravel(), np.tile(st.lam[l], T) * sv["x"][l].ravel() + block(sv["x"][l].ravel(), l),
                                   rtol=1e-12, atol=1e-13)
    Kd = [np.diag(np.tile(st.lam[l], T)) for l in range(L)]
    Js = [jac(l) + gamma * Kd[l] for l in range(L)]
    Ks = [(1 - gamma) * Kd[l] for l in range(L)]
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(T * d)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j].ravel().copy()
                        for l in reversed(layers):
                            vec = vec @ (Js[l] if l in chosen else Ks[l])
                        acc += vec
            np.testing.assert_allclose(w[i].ravel(), acc, rtol=5e-6, atol=5e-8)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), O.exact_backward(st, sv, e), rtol=1e-10, atol=1e-12)


def test_transformer_parameter_gradients_by_finite_differences():
    """Every entry of Wqkv, Wo, W1, W2 by central differences of a scalar loss (two sequences, non-causal as well)."""
    for causal in (True, False):
        st = small_transformer(layers=2, d=4, dff=5, T=3, heads=2, causal=causal, seed=9)
        r = np.random.default_rng(5)
        x0 = r.standard_normal((2 * st.T, st.d))
        c = r.standard_normal((st.L + 1, 2 * st.T, st.d))
        sv = O.forward(st, x0)
        pg = O.param_grads(st, sv, O.exact_backward(st, sv, c))

        def loss(**kw):
            a = dict(W1=st.W1, W2=st.W2, Wqkv=st.Wqkv, Wo=st.Wo)
            a.update(kw)
            s2 = O.Stack("transformer", "gelu", "rms", a["W1"], a["W2"], lam=st.lam, Wqkv=a["Wqkv"], Wo=a["Wo"], T=st.T,
                         heads=st.heads, causal=causal)
            return float(np.sum(c * O.forward(s2, x0)["x"]))
        for name in ("W1", "W2", "Wqkv", "Wo"):
            M = getattr(st, name)
            num = np.zeros_like(M)
            for idx in np.ndindex(M.shape):
                Mp, Mm = M.copy(), M.copy()
                Mp[idx] += 1e-6
                Mm[idx] -= 1e-6
                num[idx] = (loss(**{name: Mp}) - loss(**{name: Mm})) / 2e-6
            np.testing.assert_allclose(pg["d" + name], num, rtol=5e-6, atol=5e-8)


def test_attention_special_cases():
    """What the attention must reduce to: with one token per sequence the softmax is 1 and o = v; with zero query
    weights every visible key weighs the same, so o is the running mean of v (causal) or its mean (not causal); and with
    a causal mask the gradient of a loss on token t reaches no later token."""
    r = np.random.default_rng(3)
    d, heads = 8, 2
    st1 = small_transformer(layers=1, d=d, T=1, heads=heads, lam="one", norm="none")
    qkv = r.standard_normal((5, 3 * d))
    np.testing.assert_allclose(O.attention(st1, qkv), qkv[:, 2 * d:], rtol=0, atol=1e-15)
    dqkv = O.attention_vjp(st1, qkv, np.ones((5, d)))
    np.testing.assert_allclose(dqkv, np.concatenate([np.zeros((5, 2 * d)), np.ones((5, d))], axis=1), atol=1e-15)
    T = 6
    for causal in (True, False):
        st = small_transformer(layers=1, d=d, T=T, heads=heads, causal=causal)
        qkv = r.standard_normal((2 * T, 3 * d))
        qkv[:, :d] = 0.0
        v = qkv[:, 2 * d:].reshape(2, T, d)
        want = np.cumsum(v, axis=1) / np.arange(1, T + 1)[None, :, None] if causal else np.repeat(v.mean(axis=1, keepdims=True), T, axis=1)
        np.testing.assert_allclose(O.attention(st, qkv), want.reshape(2 * T, d), rtol=1e-13, atol=1e-14)
    st = small_transformer(layers=2, d=d, T=T, heads=heads, causal=True)
    sv = O.forward(st, r.standard_normal((T, d)))
    e = np.zeros((st.L + 1, T, d))
    e[st.L, 2] = r.standard_normal(d)
    for k in (1, 2, st.L):
        w = O.hbp_backward(st, sv, e, k)
        assert np.all(w[:, 3:] == 0.0) and np.abs(w[0, :3]).min() > 0.0
    # rows of the probabilities sum to one and respect the mask
    q, k_ = (O._heads(st, sv["qkv"][0][:, j * d:(j + 1) * d]) for j in range(2))
    P = O.attn_probs(st, q, k_)
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=1e-14)
    assert np.all(P[..., np.triu_indices(T, 1)[0], np.triu_indices(T, 1)[1]] == 0.0)


# ---------------------------------------------------------------- P14: the LSTM cell (LSTM row of the table)
def small_lstm(T=5, H=4, I=3, seed=0):
    r = np.random.default_rng(seed)
    W = r.standard_normal((4 * H, H)) / math.sqrt(H)
    U = r.standard_normal((4 * H, I)) / math.sqrt(I)
    return O.Stack("lstm", "tanh", "none", W, None, U=U, L=T)


def test_lstm_cell_against_torch_autograd():
    """State [c | h], c' = f c + i g, h' = o tanh(c'): states, every state gradient (both parts) and the gradients
    of both weight matrices against torch's autograd of the same recurrence in fp64."""
    r = np.random.default_rng(51)
    N, I = 3, 4
    st = small_lstm(T=6, H=5, I=I)
    H_ = st.d // 2
    xin = r.standard_normal((st.L, N, I))
    x0 = r.standard_normal((N, st.d)) * 0.5
    c = r.standard_normal((st.L + 1, N, st.d))
    sv = O.forward(st, x0, xin)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G, xin)

    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W, U = t(st.W1), t(st.U)
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        cc, h = x[:, :H_], x[:, H_:]
        pre = h @ W.T + torch.tensor(xin[l]) @ U.T
        i, f, o = (torch.sigmoid(pre[:, j * H_:(j + 1) * H_]) for j in range(3))
        g = torch.tanh(pre[:, 3 * H_:])
        cn = f * cc + i * g
        nxt = torch.cat([cn, o * torch.tanh(cn)], dim=1)
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW1"], W.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dU"], U.grad.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("gamma", [0.0, 0.5])
def test_lstm_cell_by_path_enumeration(gamma):
    """Theorem 2 with K_l = diag([f_l | 0]) and J_l = (Jacobian of the whole step) - K_l, the step's Jacobian by
    central differences of the cell's forward map on [c | h]."""
    st = small_lstm(T=4, H=2, I=2, seed=7)
    r = np.random.default_rng(12)
    xin = r.standard_normal((st.L, 1, 2))
    sv = O.forward(st, r.standard_normal((1, st.d)) * 0.5, xin)
    e = r.standard_normal((st.L + 1, 1, st.d))
    L, d = st.L, st.d
    H_ = d // 2

    def step(x, l):
        cc, h = x[:H_], x[H_:]
        pre = st.W1 @ h + st.U @ xin[l][0]
        sg = lambda a: 1 / (1 + np.exp(-a))
        i, f, o, g = sg(pre[:H_]), sg(pre[H_:2 * H_]), sg(pre[2 * H_:3 * H_]), np.tanh(pre[3 * H_:])
        cn = f * cc + i * g
        return np.concatenate([cn, o * np.tanh(cn)])
    Kd, Js = [], []
    for l in range(L):
        x = sv["x"][l][0]
        F = np.zeros((d, d))
        for i in range(d):
            xp, xm = x.copy(), x.copy()
            xp[i] += 1e-6
            xm[i] -= 1e-6
            F[:, i] = (step(xp, l) - step(xm, l)) / 2e-6
        K = np.diag(np.concatenate([sv["gates"][l][0][H_:2 * H_], np.zeros(H_)]))
        Kd.append(K)
        Js.append(F - K)
    np.testing.assert_array_equal(sv["a"][:, 0], np.stack([np.diag(K) for K in Kd]))
    Jg = [Js[l] + gamma * Kd[l] for l in range(L)]
    Kg = [(1 - gamma) * Kd[l] for l in range(L)]
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(d)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):
                            vec = vec @ (Jg[l] if l in chosen else Kg[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), O.exact_backward(st, sv, e),
                               rtol=1e-10, atol=1e-12)


def test_lstm_cell_k0_follows_the_forget_gates_only():
    """w^0: the cell part of e_T travels down through the products of the forget gates, the hidden part not at all."""
    st = small_lstm(T=5, H=3, I=2, seed=9)
    r = np.random.default_rng(3)
    xin = r.standard_normal((st.L, 2, 2))
    sv = O.forward(st, np.zeros((2, st.d)), xin)
    e = r.standard_normal((2, st.d))
    H_ = st.d // 2
    w0 = O.hbp_backward(st, sv, e, 0)
    prod = np.ones((2, H_))
    for l in range(st.L - 1, -1, -1):
        prod = prod * sv["gates"][l][:, H_:2 * H_]
        np.testing.assert_allclose(w0[l][:, :H_], e[:, :H_] * prod, rtol=1e-12)
        np.testing.assert_array_equal(w0[l][:, H_:], 0.0)


# ---------------------------------------------------------------- P15: post-norm, x' = RMSnorm(lam (.) x + block(x))
def small_postnorm_mlp(L=4, d=6, dff=10, seed=5):
    st = small_mlp(L=L, d=d, dff=dff, norm="none", seed=seed)
    st.post = "rms"
    return st


def test_post_norm_against_torch_autograd():
    """The post-norm row of the table of layer decompositions (RMS norm without gain after the sum): forward
    states, every state gradient and every parameter gradient against torch's autograd in fp64."""
    r = np.random.default_rng(61)
    N = 5
    st = small_postnorm_mlp(L=5, d=8, dff=12)
    x0 = r.standard_normal((N, st.d))
    c = r.standard_normal((st.L + 1, N, st.d))
    sv = O.forward(st, x0)
    np.testing.assert_allclose(np.mean(sv["x"][1:] ** 2, axis=-1), 1.0, rtol=1e-5)
    G = O.exact_backward(st, sv, c)
    pg = O.param_grads(st, sv, G)

    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    W1, W2, lam = t(st.W1), t(st.W2), torch.tensor(st.lam)
    xs = [t(x0)]
    for l in range(st.L):
        x = xs[-1]
        s = lam[l] * x + torch.nn.functional.gelu(x @ W1[l].T) @ W2[l].T
        nxt = s / torch.sqrt((s * s).mean(dim=1, keepdim=True) + st.eps)
        nxt.retain_grad()
        xs.append(nxt)
    loss = sum((torch.tensor(c[l]) * xs[l]).sum() for l in range(st.L + 1))
    loss.backward()
    for l in range(st.L + 1):
        np.testing.assert_allclose(sv["x"][l], xs[l].detach().numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(G[l], xs[l].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW1"], W1.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(pg["dW2"], W2.grad.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("gamma", [0.0, 0.3])
def test_post_norm_by_path_enumeration(gamma):
    """Theorem 2 with K_l = diag(lam_l rho_l) (rho_l the token's 1/rms of the sum, held as data) and J_l = F_l - K_l,
    F_l the whole layer's Jacobian by central differences of x -> RMSnorm(lam (.) x + block(x))."""
    st = small_postnorm_mlp(L=5, d=3, dff=4, seed=8)
    r = np.random.default_rng(4)
    sv = O.forward(st, r.standard_normal((1, st.d)))
    e = r.standard_normal((st.L + 1, 1, st.d))
    L, d = st.L, st.d

    def layer(x, l):
        s = st.lam[l] * x + O.act_fn(st.act, st.W1[l] @ x) @ st.W2[l].T
        return s / math.sqrt(np.mean(s * s) + st.eps)
    Kd, Js = [], []
    for l in range(L):
        x = sv["x"][l][0]
        F = np.zeros((d, d))
        for i in range(d):
            xp, xm = x.copy(), x.copy()
            xp[i] += 1e-6
            xm[i] -= 1e-6
            F[:, i] = (layer(xp, l) - layer(xm, l)) / 2e-6
        s = st.lam[l] * x + O.act_fn(st.act, st.W1[l] @ x) @ st.W2[l].T
        K = np.diag(st.lam[l] / math.sqrt(np.mean(s * s) + st.eps))
        Kd.append(K)
        Js.append(F - K)
    Jg = [Js[l] + gamma * Kd[l] for l in range(L)]
    Kg = [(1 - gamma) * Kd[l] for l in range(L)]
    for k in range(L + 1):
        w = O.hbp_backward(st, sv, e, k, gamma=gamma)
        for i in range(L + 1):
            acc = np.zeros(d)
            for j in range(i, L + 1):
                layers = list(range(i, j))
                for size in range(min(k, len(layers)) + 1):
                    for chosen in itertools.combinations(layers, size):
                        vec = e[j][0].copy()
                        for l in reversed(layers):
                            vec = vec @ (Jg[l] if l in chosen else Kg[l])
                        acc += vec
            np.testing.assert_allclose(w[i][0], acc, rtol=5e-6, atol=5e-8)
    np.testing.assert_allclose(O.hbp_backward(st, sv, e, L, gamma=gamma), O.exact_backward(st, sv, e),
                               rtol=1e-10, atol=1e-12)


def test_post_norm_finite_termination_and_k0():
    st = small_postnorm_mlp(L=6, d=5, dff=7, seed=2)
    r = np.random.default_rng(6)
    sv = O.forward(st, r.standard_normal((3, st.d)))
    e = r.standard_normal((3, st.d))
    G = O.exact_backward(st, sv, e)
    w0 = O.hbp_backward(st, sv, e, 0)
    prod = np.ones_like(e)
    for l in range(st.L - 1, -1, -1):      # w^0: e_L times the products of lam rho
        prod = prod * st.lam[l] * sv["rpost"][l][:, None]
        np.testing.assert_allclose(w0[l], e * prod, rtol=1e-12)
    for k in range(st.L + 1):
        w = O.hbp_backward(st, sv, e, k)
        for i in range(st.L + 1):
            if k >= st.L - i:
                np.testing.assert_allclose(w[i], G[i], rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- stored results of the oracle itself
def test_oracle_reproduces_its_stored_results():
    """tests/golden/oracle_small.txt (written by tests/golden/make_golden.py from the oracle alone): one tiny stack
    per kind of layer; guards the oracle's arithmetic against accidental change."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    stored = {}
    for line in open(os.path.join(here, "oracle_small.txt")):
        if line.startswith("#"):
            continue
        parts = line.split()
        stored[(parts[0], parts[1])] = np.array([float(t) for t in parts[2:]])
    seen = 0
    for name, (st, x0, xin, e) in mg.cases().items():
        for q, v in mg.results(st, x0, xin, e).items():
            np.testing.assert_allclose(np.asarray(v).ravel(), stored[(name, q)], rtol=1e-12, atol=1e-14,
                                       err_msg=f"{name} {q}")
            seen += 1
    assert seen == len(stored) and seen >= 6 * 7


def test_error_measures_on_hand_computed_vectors():
    """rel_l2 and cosine, the two measures every comparison goes through, on vectors small enough to do by hand:
    a = (3, 4), b = (0, 4): a - b = (3, 0), |a - b| = 3, |b| = 4, so rel_l2 = 3/4 (the SECOND argument is the
    reference: swapped, |a| = 5 gives 3/5); cosine((3, 4), (4, 3)) = 24/25; a zero reference leaves the plain
    norm of the difference; shapes are flattened."""
    assert O.rel_l2([3.0, 4.0], [0.0, 4.0]) == pytest.approx(0.75, abs=1e-15)
    assert O.rel_l2([0.0, 4.0], [3.0, 4.0]) == pytest.approx(0.6, abs=1e-15)
    assert O.rel_l2([[1.0, 2.0], [2.0, 0.0]], np.zeros((2, 2))) == pytest.approx(3.0, abs=1e-15)
    assert O.rel_l2([1.0, -2.0, 0.5], [1.0, -2.0, 0.5]) == 0.0
    assert O.rel_l2([2.0, 0.0], [1.0, 0.0]) == pytest.approx(1.0, abs=1e-15)       # not symmetric, not capped
    assert O.cosine([3.0, 4.0], [4.0, 3.0]) == pytest.approx(24.0 / 25.0, abs=1e-15)
    assert O.cosine([1.0, 0.0], [0.0, 5.0]) == 0.0
    assert O.cosine([[1.0, 2.0]], [[-2.0, -4.0]]) == pytest.approx(-1.0, abs=1e-15)


def test_assert_close_catches_a_wrong_row_and_a_wrong_element():
    """The comparison helper of the GPU tests: a perturbation too small for the whole-tensor norm must still be
    caught when it sits in one row or one element (planted here in a copy of the reference, on the CPU)."""
    from tests import helpers as H
    rng = np.random.default_rng(0)
    want = rng.standard_normal((333, 512))
    tol = 2e-2
    noisy = want * (1.0 + 2e-3 * rng.standard_normal(want.shape))      # rounding-sized noise passes
    H.assert_close(noisy, want, tol, "noise")
    bad_row = noisy.copy()
    bad_row[332] = rng.standard_normal(512)                            # one wrong row of 333: whole tensor 7.7e-2
    assert H.rel(bad_row, want) < 0.1
    with pytest.raises(AssertionError):
        H.assert_close(bad_row, want, 0.1, "row")
    bad_el = noisy.copy()
    bad_el[17, 300] += 1.5                                             # one wrong element: whole tensor 3.6e-3, its
    assert H.rel(bad_el, want) < tol                                   # row 6.6e-2 (below the row bar of 8e-2)
    with pytest.raises(AssertionError, match="element"):
        H.assert_close(bad_el, want, tol, "element")
    few = noisy.copy()
    few[100, :48] = 0.0                                                # 48 elements of a row left unwritten
    assert H.rel(few, want) < tol
    with pytest.raises(AssertionError):
        H.assert_close(few, want, tol, "corner")


def test_optimizer_steps_against_torch_optim():
    """The oracle's SGD-with-momentum and AdamW steps against torch.optim (an independent implementation) over
    several steps in fp64, and a one-step closed form done by hand."""
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal((5, 7))
    grads = [rng.standard_normal((5, 7)) for _ in range(4)]
    # SGD: lr 0.1, momentum 0.9, weight decay 1e-2
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=0.1, momentum=0.9, weight_decay=1e-2)
    w, buf = w0.copy(), np.zeros_like(w0)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, buf = O.sgd_momentum_step(w, g, buf, 0.1, 0.9, 1e-2)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-13, atol=1e-13)
    # AdamW: lr 1e-2, betas (0.9, 0.98), eps 1e-8, weight decay 0.1
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=1e-2, betas=(0.9, 0.98), eps=1e-8, weight_decay=0.1)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = O.adamw_step(w, g, m, v, t, 1e-2, 0.9, 0.98, 1e-8, 0.1)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-12)
    # by hand: one AdamW step from zero moments moves every weight by lr sign(g) (up to eps) after the decay
    w1, _, _ = O.adamw_step(np.array([2.0]), np.array([0.5]), np.zeros(1), np.zeros(1), 1, 0.1, 0.9, 0.999, 0.0, 0.5)
    assert w1[0] == pytest.approx(2.0 * (1 - 0.05) - 0.1, abs=1e-12)
    # by hand: SGD, first step, no momentum history: w - lr (g + wd w)
    w1, b1 = O.sgd_momentum_step(np.array([2.0]), np.array([0.5]), np.zeros(1), 0.1, 0.9, 0.25)
    assert w1[0] == pytest.approx(2.0 - 0.1 * (0.5 + 0.5), abs=1e-15) and b1[0] == pytest.approx(1.0)


def test_clip_scale_and_schedule_and_loss():
    """Gradient clipping against torch's clip_grad_norm_, the learning-rate schedule at its fixed points, and the
    stand-in loss against autograd."""
    rng = np.random.default_rng(4)
    gs = [rng.standard_normal((3, 4)), rng.standard_normal(6)]
    ps = [torch.nn.Parameter(torch.zeros(3, 4, dtype=torch.float64)), torch.nn.Parameter(torch.zeros(6, dtype=torch.float64))]
    for p, g in zip(ps, gs):
        p.grad = torch.tensor(g)
    torch.nn.utils.clip_grad_norm_(ps, 1.0)
    s = O.clip_scale(gs, 1.0)
    for p, g in zip(ps, gs):
        assert np.allclose(p.grad.numpy(), s * g, rtol=1e-12)
    assert O.clip_scale(gs, 0.0) == 1.0 and O.clip_scale([np.array([0.3, 0.4])], 1.0) == 1.0
    assert O.clip_scale([np.array([3.0, 4.0])], 1.0) == pytest.approx(1.0 / (5.0 + 1e-6))
    # schedule: warm-up reaches the base rate, the cosine ends at a tenth of it, half-way it is 0.55 of it
    assert O.lr_schedule(0, 100, 1.0, 10) == pytest.approx(0.1)
    assert O.lr_schedule(9, 100, 1.0, 10) == pytest.approx(1.0)
    assert O.lr_schedule(10, 100, 1.0, 10) == pytest.approx(1.0)
    assert O.lr_schedule(55, 100, 1.0, 10) == pytest.approx(0.55)
    assert O.lr_schedule(100, 100, 1.0, 10) == pytest.approx(0.1)
    # loss: e is the gradient of the loss w.r.t. the states
    x = rng.standard_normal((4, 3, 5)); t = rng.standard_normal((4, 3, 5))
    for every in (True, False):
        xt = torch.tensor(x, requires_grad=True)
        if every:
            loss = 0.5 * ((xt[1:] - torch.tensor(t[1:])) ** 2).sum() / 3
        else:
            loss = 0.5 * ((xt[-1] - torch.tensor(t[-1])) ** 2).sum() / 3
        loss.backward()
        val, e = O.mse_loss_and_grad(x, t if every else t[-1], every)
        assert val == pytest.approx(float(loss.detach()), rel=1e-13)
        want = xt.grad.numpy() if every else xt.grad.numpy()[-1]
        assert np.allclose(e, want, rtol=1e-13, atol=1e-15)


def test_training_with_few_iterations_then_exact_reduces_the_loss():
    """The conclusion's recipe on a tiny stack, all in the oracle: SGD on the stand-in loss with gradients from
    Highway-BP at k = 1, then k = 2, then exact backpropagation; the loss goes down in every phase, and a step
    with k >= L equals a step with exact backpropagation."""
    rng = np.random.default_rng(5)
    L, N, d, dff = 4, 16, 6, 12
    W1 = rng.standard_normal((L, dff, d)) / np.sqrt(d)
    W2 = rng.standard_normal((L, d, dff)) / np.sqrt(dff) * 0.5
    x0 = rng.standard_normal((N, d)); target = rng.standard_normal((N, d)) * 0.1
    b1, b2 = np.zeros_like(W1), np.zeros_like(W2)
    losses = []
    for step in range(30):
        st = O.Stack("mlp", "gelu", "rms", W1, W2)
        sv = O.forward(st, x0)
        loss, e = O.mse_loss_and_grad(sv["x"], target, False)
        losses.append(loss)
        k = 1 if step < 10 else 2 if step < 20 else None
        g = O.exact_backward(st, sv, e) if k is None else O.hbp_backward(st, sv, e, k)
        if step == 29:
            assert np.allclose(O.hbp_backward(st, sv, e, L), O.exact_backward(st, sv, e), rtol=1e-12, atol=1e-14)
        pg = O.param_grads(st, sv, g)
        W1, b1 = O.sgd_momentum_step(W1, pg["dW1"], b1, 0.05, 0.9, 0.0)
        W2, b2 = O.sgd_momentum_step(W2, pg["dW2"], b2, 0.05, 0.9, 0.0)
    assert losses[10] < losses[0] and losses[20] < losses[10] and losses[29] < losses[20]
