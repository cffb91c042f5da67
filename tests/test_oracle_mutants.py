"""Planted-mistake check: each plausible slip in the oracle must fail at least one pin.

The mistakes are planted in the oracle module on the CPU (monkeypatched copies of its
functions); the battery below re-runs a compact subset of the pins of test_oracle_pins.py.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import linattn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


def _num(tok):
    if isinstance(tok, str):
        if tok.endswith("ln2"):
            return math.copysign(math.log(2.0), -1.0 if tok.startswith("-") else 1.0)
        return float(Fraction(tok))
    return float(tok)


def _arr(x):
    return np.array([[_num(t) for t in row] for row in x], dtype=np.float64)


def _battery() -> bool:
    """True when every pin in the compact battery holds for the oracle as currently patched."""
    try:
        with open(GOLDEN) as f:
            cases = json.load(f)["cases"]
        for c in cases:
            q, k, v = _arr(c["q"]), _arr(c["k"]), _arr(c["v"])
            got = orc.attention_linear(q, k, v, c["feature_map"], c["eps"], c["normalize"])
            np.testing.assert_allclose(got, _arr(c["out"]), rtol=1e-14, atol=1e-14)
            got = orc.attention_quadratic(q, k, v, c["feature_map"], c["eps"], c["normalize"])
            np.testing.assert_allclose(got, _arr(c["out"]), rtol=1e-14, atol=1e-14)
        rng = np.random.default_rng(99)
        q, k, v = rng.normal(size=(3, 12, 5))
        np.testing.assert_allclose(orc.attention_linear(q, k, v, 0, 1e-3),
                                   orc.attention_quadratic(q, k, v, 0, 1e-3), rtol=1e-12)
        qp, kp = rng.uniform(0.1, 1.0, size=(2, 12, 5))
        want = (qp @ (kp.T @ v)) / (qp @ kp.sum(axis=0))[:, None]
        np.testing.assert_allclose(orc.attention_linear(qp, kp, v, orc.IDENTITY, 0.0), want, rtol=1e-12)
        c = rng.normal(size=5)
        np.testing.assert_allclose(orc.attention_linear(q, k, np.tile(c, (12, 1)), 0, 0.0),
                                   np.tile(c, (12, 1)), rtol=1e-12)
        return True
    except AssertionError:
        return False


def test_battery_passes_unmutated():
    assert _battery()


def _m_state_transposed(mp):
    def state(k, v, fm=0):
        p = orc.phi(k, fm)
        return np.asarray(v, dtype=np.float64).T @ p, p.sum(axis=0)
    mp.setattr(orc, "state", state)


def _m_apply_transposed(mp):
    def apply_state(q, S, z, fm=0, eps=0.0, normalize=True):
        r = orc.phi(q, fm)
        num = r @ S.T
        return num / (r @ z + eps)[:, None] if normalize else num
    mp.setattr(orc, "apply_state", apply_state)


def _m_z_without_phi(mp):
    def state(k, v, fm=0):
        p = orc.phi(k, fm)
        return p.T @ np.asarray(v, dtype=np.float64), np.asarray(k, dtype=np.float64).sum(axis=0)
    mp.setattr(orc, "state", state)


def _m_eps_inside_sum(mp):
    def apply_state(q, S, z, fm=0, eps=0.0, normalize=True):
        r = orc.phi(q, fm)
        num = r @ S
        return num / (r @ (z + eps))[:, None] if normalize else num
    mp.setattr(orc, "apply_state", apply_state)


def _m_eps_dropped(mp):
    def apply_state(q, S, z, fm=0, eps=0.0, normalize=True):
        r = orc.phi(q, fm)
        num = r @ S
        return num / (r @ z)[:, None] if normalize else num
    mp.setattr(orc, "apply_state", apply_state)


def _m_phi_on_v(mp):
    def state(k, v, fm=0):
        p = orc.phi(k, fm)
        return p.T @ orc.phi(v, fm), p.sum(axis=0)
    mp.setattr(orc, "state", state)


def _m_elu_without_plus_one(mp):
    real = orc.phi

    def phi(x, fm=0):
        return real(x, fm) - 1.0 if fm == 0 else real(x, fm)
    mp.setattr(orc, "phi", phi)


def _m_phi_not_on_q(mp):
    def apply_state(q, S, z, fm=0, eps=0.0, normalize=True):
        r = np.asarray(q, dtype=np.float64)
        num = r @ S
        return num / (r @ z + eps)[:, None] if normalize else num
    mp.setattr(orc, "apply_state", apply_state)


def _m_softmax_scale(mp):
    def apply_state(q, S, z, fm=0, eps=0.0, normalize=True):
        r = orc.phi(q, fm) / math.sqrt(S.shape[0])
        num = r @ S
        return num / (r @ z + eps)[:, None] if normalize else num
    mp.setattr(orc, "apply_state", apply_state)


def _m_den_is_plain_sum_of_z(mp):
    def apply_state(q, S, z, fm=0, eps=0.0, normalize=True):
        r = orc.phi(q, fm)
        num = r @ S
        return num / (z.sum() + eps) if normalize else num
    mp.setattr(orc, "apply_state", apply_state)


def _m_branch_flipped(mp):
    real = orc.phi

    def phi(x, fm=0):
        x = np.asarray(x, dtype=np.float64)
        if fm == 0:
            return np.where(x < 0.0, x + 1.0, np.exp(np.minimum(x, 0.0)))
        return real(x, fm)
    mp.setattr(orc, "phi", phi)


MUTANTS = [_m_state_transposed, _m_apply_transposed, _m_z_without_phi, _m_eps_inside_sum,
           _m_eps_dropped, _m_phi_on_v, _m_elu_without_plus_one, _m_phi_not_on_q,
           _m_softmax_scale, _m_den_is_plain_sum_of_z, _m_branch_flipped]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda f: f.__name__[3:])
def test_planted_mistake_is_caught(mutant, monkeypatch):
    mutant(monkeypatch)
    assert not _battery(), "a planted mistake slipped through every pin"
