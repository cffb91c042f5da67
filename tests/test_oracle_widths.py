"""Pins for the oracle with a feature width of q, k other than the value width (Prop. 3: the state is
d_qk x d_v; the computational form is unchanged).  CPU only."""
import numpy as np
import pytest

from oracle import linattn_oracle as orc


@pytest.mark.parametrize("dk,dv", [(1, 2), (3, 5), (6, 2), (8, 3)])
@pytest.mark.parametrize("fm", [orc.ELU_PLUS_ONE, orc.RELU, orc.IDENTITY])
def test_linear_form_equals_the_explicit_quadratic_form(dk, dv, fm):
    r = np.random.default_rng(10 * dk + dv)
    n = 9
    q, k, v = r.normal(size=(n, dk)), r.normal(size=(n, dk)), r.normal(size=(n, dv))
    if fm != orc.ELU_PLUS_ONE:
        q, k = np.abs(q) + 0.1, np.abs(k) + 0.1
    for normalize in (True, False):
        lin = orc.attention_linear(q, k, v, fm, 1e-3, normalize)
        quad = orc.attention_quadratic(q, k, v, fm, 1e-3, normalize)
        assert lin.shape == (n, dv)
        np.testing.assert_allclose(lin, quad, rtol=1e-12, atol=1e-12)


def test_state_shapes_and_hand_worked_values():
    # two tokens, features of width 2, values of width 3, identity feature map
    k = np.array([[1.0, 2.0], [3.0, 0.5]])
    v = np.array([[1.0, 0.0, -1.0], [2.0, 4.0, 6.0]])
    S, z = orc.state(k, v, orc.IDENTITY)
    np.testing.assert_array_equal(S, np.array([[7.0, 12.0, 17.0], [3.0, 2.0, 1.0]]))   # k^T v: 2 x 3
    np.testing.assert_array_equal(z, np.array([4.0, 2.5]))
    q = np.array([[2.0, 2.0]])
    out = orc.apply_state(q, S, z, orc.IDENTITY, eps=0.0)
    np.testing.assert_allclose(out, np.array([[20.0, 28.0, 36.0]]) / 13.0, rtol=0, atol=1e-15)


def test_scalar_feature_gives_a_key_weighted_mean_of_the_values():
    """Feature width 1: phi(q_i) cancels between numerator and denominator, every token receives the same
    mean of V weighted by phi(k_j)."""
    r = np.random.default_rng(3)
    n, dv = 12, 4
    q, k, v = r.normal(size=(n, 1)), r.normal(size=(n, 1)), r.normal(size=(n, dv))
    w = orc.phi(k)[:, 0]
    want = (w[:, None] * v).sum(axis=0) / w.sum()
    got = orc.attention_linear(q, k, v)
    np.testing.assert_allclose(got, np.tile(want, (n, 1)), rtol=1e-12, atol=1e-12)


def test_extra_feature_channels_that_are_constant_in_k_only_rescale_the_weights():
    """Appending a feature channel whose phi(k) is the same for every token adds c * phi(q_extra) * sum_j v_j to
    the numerator and c * phi(q_extra) * n to the denominator: checked against that closed form."""
    r = np.random.default_rng(4)
    n, dk, dv = 7, 3, 2
    q, k, v = r.normal(size=(n, dk)), r.normal(size=(n, dk)), r.normal(size=(n, dv))
    qe = np.concatenate([q, r.normal(size=(n, 1))], axis=1)
    ke = np.concatenate([k, np.full((n, 1), 0.7)], axis=1)
    S, z = orc.state(k, v)
    rq = orc.phi(qe)
    c = orc.phi(np.array(0.7))
    num = orc.phi(q) @ S + c * rq[:, 3:4] * v.sum(axis=0)[None, :]
    den = orc.phi(q) @ z + c * rq[:, 3] * n
    np.testing.assert_allclose(orc.attention_linear(qe, ke, v), num / den[:, None], rtol=1e-12, atol=1e-12)


def test_planted_mistakes_are_caught():
    r = np.random.default_rng(5)
    n, dk, dv = 10, 4, 6
    q, k, v = r.normal(size=(n, dk)), r.normal(size=(n, dk)), r.normal(size=(n, dv))
    good = orc.attention_linear(q, k, v)
    p, rq = orc.phi(k), orc.phi(q)
    S, z = p.T @ v, p.sum(axis=0)
    mutants = {
        "normalizer from the values' side": (rq @ S) / (rq @ S).sum(axis=1, keepdims=True),
        "phi on v as well": (rq @ (p.T @ orc.phi(v))) / (rq @ z)[:, None],
        "z over features instead of tokens": (rq @ S) / (rq.sum(axis=1) * p.sum())[:, None],
    }
    for name, bad in mutants.items():
        assert np.abs(bad - good).max() > 1e-3, name
