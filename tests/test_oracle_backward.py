"""Pins of the oracle's backward pass against things other than itself: central differences of the
forward definition (the explicit-loop quadratic form), the two algebraic forms against each other,
and invariants of the normalized mixer."""
import numpy as np
import pytest

from oracle import linattn_oracle as orc


def _inputs(n, d, seed, shift=0.0):
    rng = np.random.default_rng(seed)
    q = rng.normal(size=(n, d)) + shift
    k = rng.normal(size=(n, d)) + shift
    v = rng.normal(size=(n, d))
    g = rng.normal(size=(n, d))
    # keep every element away from the kink of elu+1 / relu at 0 so that central differences are valid
    for t in (q, k):
        t[np.abs(t) < 1e-3] = 0.5
    return q, k, v, g


def _numeric_grad(fn, x, g, h=1e-6):
    """d/dx sum(fn(x) * g) by central differences, element by element."""
    out = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = (fn(x) * g).sum()
        x[i] = old - h
        fm = (fn(x) * g).sum()
        x[i] = old
        out[i] = (fp - fm) / (2 * h)
    return out


@pytest.mark.parametrize("fm", [orc.ELU_PLUS_ONE, orc.RELU, orc.IDENTITY])
@pytest.mark.parametrize("normalize,eps", [(True, 0.0), (True, 0.3), (False, 0.0)])
@pytest.mark.parametrize("backward", ["quadratic", "linear"])
def test_backward_matches_central_differences_of_the_explicit_forward(fm, normalize, eps, backward):
    n, d = 5, 3
    q, k, v, g = _inputs(n, d, seed=11 + fm, shift=1.5 if fm == orc.IDENTITY else 0.0)
    if fm == orc.IDENTITY:
        q, k = np.abs(q) + 0.1, np.abs(k) + 0.1
    if fm == orc.RELU:                                    # one active channel per token keeps den > 0
        q[:, 0], k[:, 0] = np.abs(q[:, 0]) + 0.2, np.abs(k[:, 0]) + 0.2
    fn = orc.attention_backward_quadratic if backward == "quadratic" else orc.attention_backward_linear
    dq, dk, dv = fn(q, k, v, g, fm, eps, normalize)
    fwd = lambda q_, k_, v_: orc.attention_quadratic(q_, k_, v_, fm, eps, normalize)
    nq = _numeric_grad(lambda x: fwd(x, k, v), q.copy(), g)
    nk = _numeric_grad(lambda x: fwd(q, x, v), k.copy(), g)
    nv = _numeric_grad(lambda x: fwd(q, k, x), v.copy(), g)
    for got, want, name in ((dq, nq, "dq"), (dk, nk, "dk"), (dv, nv, "dv")):
        assert np.abs(got - want).max() <= 2e-7 * max(1.0, np.abs(want).max()), name


@pytest.mark.parametrize("fm", [orc.ELU_PLUS_ONE, orc.RELU])
@pytest.mark.parametrize("normalize", [True, False])
def test_linear_and_quadratic_backward_agree(fm, normalize):
    q, k, v, g = _inputs(67, 12, seed=5)
    q[:, 0], k[:, 0] = np.abs(q[:, 0]) + 0.2, np.abs(k[:, 0]) + 0.2
    a = orc.attention_backward_quadratic(q, k, v, g, fm, 1e-6, normalize)
    b = orc.attention_backward_linear(q, k, v, g, fm, 1e-6, normalize)
    for x, y in zip(a, b):
        assert np.abs(x - y).max() <= 1e-11 * max(1.0, np.abs(x).max())


def test_dv_sums_to_the_summed_upstream_gradient():
    """Rows of the weight matrix sum to one (Sec. 2.3), so sum_j dv_j = sum_i g_i at eps = 0."""
    q, k, v, g = _inputs(40, 8, seed=3)
    _, _, dv = orc.attention_backward_linear(q, k, v, g, orc.ELU_PLUS_ONE, 0.0, True)
    assert np.abs(dv.sum(axis=0) - g.sum(axis=0)).max() <= 1e-12 * np.abs(g).sum()


def test_gradient_is_orthogonal_to_the_scaling_directions():
    """At eps = 0 the output does not change when phi(q_i) or all phi(k_j) are scaled, so
    d phi(q_i) . phi(q_i) = 0 for every token and sum_j d phi(k_j) . phi(k_j) = 0."""
    q, k, v, g = _inputs(30, 6, seed=4, shift=1.5)
    q, k = np.abs(q) + 0.1, np.abs(k) + 0.1               # IDENTITY: dq = d phi(q)
    dq, dk, _ = orc.attention_backward_linear(q, k, v, g, orc.IDENTITY, 0.0, True)
    assert np.abs((dq * q).sum(axis=1)).max() <= 1e-12 * np.abs(dq).max() * np.abs(q).max() * q.shape[1]
    assert abs((dk * k).sum()) <= 1e-11 * np.abs(dk).sum() * np.abs(k).max()


def test_constant_v_has_zero_gradient_to_q_and_k():
    """Prop. 1's setting: with every v_j equal the output is that constant whatever q and k are."""
    q, k, v, g = _inputs(25, 5, seed=6)
    v[:] = v[0]
    dq, dk, _ = orc.attention_backward_linear(q, k, v, g, orc.ELU_PLUS_ONE, 0.0, True)
    assert np.abs(dq).max() <= 1e-12 and np.abs(dk).max() <= 1e-12


def test_backward_is_linear_in_the_upstream_gradient():
    q, k, v, g = _inputs(20, 4, seed=7)
    g2 = np.random.default_rng(8).normal(size=g.shape)
    a = orc.attention_backward_linear(q, k, v, g, 0, 1e-6, True)
    b = orc.attention_backward_linear(q, k, v, g2, 0, 1e-6, True)
    c = orc.attention_backward_linear(q, k, v, 2.0 * g - 3.0 * g2, 0, 1e-6, True)
    for x, y, w in zip(a, b, c):
        assert np.abs(2.0 * x - 3.0 * y - w).max() <= 1e-11 * max(1.0, np.abs(w).max())


def test_planted_mistakes_in_the_backward_are_caught():
    """Mutants of the linear form: each must disagree with the central differences."""
    n, d = 5, 3
    q, k, v, g = _inputs(n, d, seed=21)
    fwd = lambda q_, k_, v_: orc.attention_quadratic(q_, k_, v_, 0, 0.0, True)
    nq = _numeric_grad(lambda x: fwd(x, k, v), q.copy(), g)
    nk = _numeric_grad(lambda x: fwd(q, x, v), k.copy(), g)
    r, p = orc.phi(q), orc.phi(k)
    S, z = p.T @ v, p.sum(axis=0)
    den = r @ z
    out = (r @ S) / den[:, None]
    gn = g / den[:, None]
    mutants = {
        "sign of the normalizer term": +(g * out).sum(axis=1) / den,
        "normalizer term dropped": np.zeros(n),
        "normalizer term not divided by den": -(g * out).sum(axis=1),
    }
    for name, e in mutants.items():
        dr = gn @ S.T + e[:, None] * z[None, :]
        assert np.abs(dr * orc.phi_prime(q) - nq).max() > 1e-3, name
    e = -(g * out).sum(axis=1) / den
    dS, dz = r.T @ gn, r.T @ e
    assert np.abs((v @ dS + dz[None, :]) * orc.phi_prime(k) - nk).max() > 1e-3, "dS not transposed"
    assert np.abs((v @ dS.T) * orc.phi_prime(k) - nk).max() > 1e-3, "dz dropped"
