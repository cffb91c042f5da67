"""Pins for the fp64 oracle: everything here is CPU-only and independent of the HIP path.

Each test fixes the oracle to something other than itself: hand-worked exact values
(tests/golden/worked_examples.json), the explicit-loop quadratic definition, the sequential
state-space recurrence of Eq. 3 / Eq. 5 with every gate equal to one, closed forms, and
invariants the paper states (Sec. 2.3 row-stochastic M, Prop. 1, Sec. 2.4 non-causality,
the Kronecker identity in the proof of Prop. 2).
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
        if tok == "ln2":
            return math.log(2.0)
        if tok == "-ln2":
            return -math.log(2.0)
        return float(Fraction(tok))
    return float(tok)


def _arr(x):
    return np.array([[_num(t) for t in row] for row in x], dtype=np.float64)


def _cases():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_worked_examples(case):
    q, k, v = _arr(case["q"]), _arr(case["k"]), _arr(case["v"])
    fm, eps, norm = case["feature_map"], case["eps"], case["normalize"]
    S, z = orc.state(k, v, fm)
    np.testing.assert_allclose(S, _arr(case["S"]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(z, np.array([_num(t) for t in case["z"]]), rtol=0, atol=1e-15)
    want = _arr(case["out"])
    got_l = orc.attention_linear(q, k, v, fm, eps, norm)
    got_q = orc.attention_quadratic(q, k, v, fm, eps, norm)
    np.testing.assert_allclose(got_l, want, rtol=1e-15, atol=1e-15)
    np.testing.assert_allclose(got_q, want, rtol=1e-15, atol=1e-15)


def test_phi_values():
    # elu(x)+1 with alpha=1: x+1 above zero, exp(x) at and below zero; strictly positive.
    x = np.array([-math.log(2.0), -40.0, 0.0, 3.0, 1e-300, -1e-300, 700.0, -800.0])
    got = orc.phi(x, orc.ELU_PLUS_ONE)
    assert got[0] == pytest.approx(0.5, rel=1e-15)
    assert got[1] == pytest.approx(math.exp(-40.0), rel=1e-15) and got[1] > 0
    assert got[2] == 1.0
    assert got[3] == 4.0
    assert got[4] == 1.0 and got[5] == 1.0
    assert got[6] == 701.0            # no overflow from evaluating exp on the positive side
    assert got[7] == 0.0              # exp underflows to zero in fp64, not nan
    assert np.all(np.isfinite(got))
    # derivative-level check of the two branches meeting continuously at zero
    h = 1e-6
    assert orc.phi(np.array([h]))[0] - orc.phi(np.array([-h]))[0] == pytest.approx(2 * h, rel=1e-4)
    np.testing.assert_array_equal(orc.phi(np.array([-2.0, 0.0, 2.5]), orc.RELU), [0.0, 0.0, 2.5])
    np.testing.assert_array_equal(orc.phi(np.array([-2.0, 0.0, 2.5]), orc.IDENTITY), [-2.0, 0.0, 2.5])


def test_decoders_known_bit_patterns():
    # binary16: 1.0, max normal, smallest subnormal, -2.0, smallest normal, +inf
    bits = np.array([0x3C00, 0x7BFF, 0x0001, 0xC000, 0x0400, 0x7C00, 0x3555], dtype=np.uint16)
    got = orc.decode_f16_bits(bits)
    assert got[0] == 1.0 and got[1] == 65504.0 and got[2] == 2.0 ** -24
    assert got[3] == -2.0 and got[4] == 2.0 ** -14 and np.isinf(got[5])
    assert got[6] == (1.0 + 0x155 / 1024.0) * 0.25
    assert np.isnan(orc.decode_f16_bits(np.array([0x7E00], dtype=np.uint16))[0])
    # bfloat16: 1.0, 3.140625, -0.5, largest normal, smallest subnormal
    bits = np.array([0x3F80, 0x4049, 0xBF00, 0x7F7F, 0x0001], dtype=np.uint16)
    got = orc.decode_bf16_bits(bits)
    assert got[0] == 1.0 and got[1] == 3.140625 and got[2] == -0.5
    assert got[3] == (2.0 - 2.0 ** -7) * 2.0 ** 127 and got[4] == 2.0 ** -133


def test_decoders_exhaustive_against_library_views():
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    lib16 = allbits.view(np.float16).astype(np.float64)
    got16 = orc.decode_f16_bits(allbits)
    np.testing.assert_array_equal(np.isnan(lib16), np.isnan(got16))
    ok = ~np.isnan(lib16)
    np.testing.assert_array_equal(lib16[ok], got16[ok])
    libbf = (allbits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    gotbf = orc.decode_bf16_bits(allbits)
    np.testing.assert_array_equal(np.isnan(libbf), np.isnan(gotbf))
    ok = ~np.isnan(libbf)
    np.testing.assert_array_equal(libbf[ok], gotbf[ok])


def test_half_ulp():
    assert orc.half_ulp(np.array([1.0]), "f16")[0] == 2.0 ** -11
    assert orc.half_ulp(np.array([1.5]), "bf16")[0] == 2.0 ** -8
    assert orc.half_ulp(np.array([-3.0]), "f16")[0] == 2.0 ** -10
    assert orc.half_ulp(np.array([2.0 ** -20]), "f16")[0] == 2.0 ** -25   # subnormal spacing 2^-24
    assert orc.half_ulp(np.array([1.0]), "f32")[0] == 2.0 ** -24
    assert orc.half_ulp(np.array([0.0]), "f16")[0] == 2.0 ** -25


@pytest.mark.parametrize("d", [1, 2, 5, 8])
@pytest.mark.parametrize("n", [1, 2, 7, 33])
@pytest.mark.parametrize("fm", [orc.ELU_PLUS_ONE, orc.RELU])
def test_linear_equals_quadratic(n, d, fm):
    # Prop. 2: the linear form reaches exactly the quadratic form's result.
    rng = np.random.default_rng(1000 * n + 10 * d + fm)
    q, k, v = rng.normal(size=(3, n, d))
    eps = 1e-6
    a = orc.attention_linear(q, k, v, fm, eps)
    b = orc.attention_quadratic(q, k, v, fm, eps)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    a = orc.attention_linear(q, k, v, fm, eps, normalize=False)
    b = orc.attention_quadratic(q, k, v, fm, eps, normalize=False)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)


def test_rectangular_query_count():
    # the number of query rows need not equal the number of key/value rows
    rng = np.random.default_rng(5)
    q = rng.normal(size=(3, 4))
    k, v = rng.normal(size=(2, 9, 4))
    np.testing.assert_allclose(orc.attention_linear(q, k, v, 0, 1e-6),
                               orc.attention_quadratic(q, k, v, 0, 1e-6), rtol=1e-12)


def test_weights_nonnegative_rows_sum_to_one():
    # Sec. 2.3: sum_k M_ik = 1 (up to the eps deficit eps / (den + eps)).
    rng = np.random.default_rng(7)
    q, k, v = rng.normal(size=(3, 19, 6))
    eps = 1e-3
    _, w = orc.attention_quadratic(q, k, v, 0, eps, return_weights=True)
    assert np.all(w >= 0.0)
    r, p = orc.phi(q), orc.phi(k)
    den = (r @ p.T).sum(axis=1)
    np.testing.assert_allclose(w.sum(axis=1), 1.0 - eps / (den + eps), rtol=1e-13)
    _, w0 = orc.attention_quadratic(q, k, v, 0, 0.0, return_weights=True)
    np.testing.assert_allclose(w0.sum(axis=1), 1.0, rtol=1e-14)


def test_ssm_recurrence_with_unit_gates():
    # Eq. 3 with A_i = 1 run to the last token gives the hidden state every token sees once
    # the causal mask is removed (Sec. 2.4); Eq. 5 gives the normalizer the same way.
    rng = np.random.default_rng(11)
    n, dp, d = 13, 5, 5
    C = orc.phi(rng.normal(size=(n, dp)))
    Bm = orc.phi(rng.normal(size=(n, dp)))
    X = rng.normal(size=(n, d))
    H = np.zeros((dp, d))
    Z = np.zeros(dp)
    for i in range(n):
        H = 1.0 * H + np.outer(Bm[i], X[i])
        Z = 1.0 * Z + Bm[i]
    Y = np.stack([(C[i] / np.dot(C[i], Z)) @ H for i in range(n)])
    got = orc.attention_linear(C, Bm, X, orc.IDENTITY, 0.0)
    np.testing.assert_allclose(got, Y, rtol=1e-13)


def test_constant_v_gives_constant_output():
    # Prop. 1 with sum_k M_ik = 1: a constant channel stays constant.
    rng = np.random.default_rng(3)
    n, d = 50, 8
    q, k = rng.normal(size=(2, n, d))
    c = rng.normal(size=d)
    v = np.tile(c, (n, 1))
    out = orc.attention_linear(q, k, v, 0, 0.0)
    np.testing.assert_allclose(out, np.tile(c, (n, 1)), rtol=1e-13)
    eps = 0.25
    den = orc.phi(q) @ orc.phi(k).sum(axis=0)
    out = orc.attention_linear(q, k, v, 0, eps)
    np.testing.assert_allclose(out, np.outer(den / (den + eps), c), rtol=1e-13)


def test_channel_mean_proposition_1():
    # Prop. 1: mean over tokens j of channel c of Y equals mu_c-weighted row sums when rows of
    # X are replaced by their channel means; checked through linearity in V.
    rng = np.random.default_rng(4)
    n, d = 21, 3
    q, k, v = rng.normal(size=(3, n, d))
    _, w = orc.attention_quadratic(q, k, v, 0, 0.0, return_weights=True)
    mu = v.mean(axis=0)
    vbar = np.tile(mu, (n, 1))
    np.testing.assert_allclose(w @ vbar, np.outer(w.sum(axis=1), mu), rtol=1e-13)
    np.testing.assert_allclose(orc.attention_linear(q, k, vbar, 0, 0.0), vbar, rtol=1e-13)


def test_non_causal_permutation_invariance():
    rng = np.random.default_rng(5)
    n, d = 40, 6
    q, k, v = rng.normal(size=(3, n, d))
    base = orc.attention_linear(q, k, v, 0, 1e-6)
    perm = rng.permutation(n)
    np.testing.assert_allclose(orc.attention_linear(q, k[perm], v[perm], 0, 1e-6), base, rtol=1e-12)
    np.testing.assert_allclose(orc.attention_linear(q[perm], k, v, 0, 1e-6), base[perm], rtol=1e-15)
    # permuting K without V must change the result (guards against a vacuous test)
    assert np.abs(orc.attention_linear(q, k[perm], v, 0, 1e-6) - base).max() > 1e-3


def test_token_tiling_invariance():
    # the normalizer keeps the total impact the same at any number of tokens (Sec. 1, Introduction; Sec. 2.3)
    rng = np.random.default_rng(6)
    q, k, v = rng.normal(size=(3, 17, 4))
    base = orc.attention_linear(q, k, v, 0, 0.0)
    np.testing.assert_allclose(orc.attention_linear(q, np.tile(k, (3, 1)), np.tile(v, (3, 1)), 0, 0.0),
                               base, rtol=1e-13)
    # without normalization the output grows with the token count instead
    un = orc.attention_linear(q, k, v, 0, 0.0, normalize=False)
    un3 = orc.attention_linear(q, np.tile(k, (3, 1)), np.tile(v, (3, 1)), 0, 0.0, normalize=False)
    np.testing.assert_allclose(un3, 3.0 * un, rtol=1e-13)


def test_kronecker_identity_from_proof_of_prop_2():
    # ((C B^T) o (F G^T)) X with f' = c (x) f, g' = b (x) g.
    rng = np.random.default_rng(8)
    n, dp, r, d = 11, 3, 2, 6
    C, Bm = rng.uniform(0.1, 2.0, size=(2, n, dp))
    F, G = rng.uniform(0.1, 2.0, size=(2, n, r))
    X = rng.normal(size=(n, d))
    M = (C @ Bm.T) * (F @ G.T)
    fq = np.stack([np.kron(C[i], F[i]) for i in range(n)])
    gk = np.stack([np.kron(Bm[i], G[i]) for i in range(n)])
    # value width (6) equals feature width (3*2) so the square-state oracle applies
    np.testing.assert_allclose(orc.attention_linear(fq, gk, X, orc.IDENTITY, 0.0, normalize=False),
                               M @ X, rtol=1e-12)
    np.testing.assert_allclose(orc.attention_linear(fq, gk, X, orc.IDENTITY, 0.0),
                               (M / M.sum(axis=1, keepdims=True)) @ X, rtol=1e-12)


def test_affine_equivariance_in_v():
    rng = np.random.default_rng(9)
    q, k, v = rng.normal(size=(3, 23, 5))
    alpha, c = -1.75, rng.normal(size=5)
    base = orc.attention_linear(q, k, v, 0, 0.0)
    np.testing.assert_allclose(orc.attention_linear(q, k, alpha * v + c, 0, 0.0), alpha * base + c, rtol=1e-12)


def test_single_channel_is_weighted_mean():
    rng = np.random.default_rng(10)
    q, k, v = rng.normal(size=(3, 31, 1))
    p = orc.phi(k)[:, 0]
    want = np.sum(p * v[:, 0]) / np.sum(p)
    np.testing.assert_allclose(orc.attention_linear(q, k, v, 0, 0.0), np.full((31, 1), want), rtol=1e-13)


def test_all_equal_keys_give_plain_mean():
    rng = np.random.default_rng(12)
    n, d = 29, 4
    q, v = rng.normal(size=(2, n, d))
    k = np.tile(rng.normal(size=d), (n, 1))
    np.testing.assert_allclose(orc.attention_linear(q, k, v, 0, 0.0), np.tile(v.mean(axis=0), (n, 1)), rtol=1e-13)


def test_identity_phi_is_two_library_gemms():
    rng = np.random.default_rng(13)
    n, d = 64, 8
    q, k = rng.uniform(0.1, 1.0, size=(2, n, d))
    v = rng.normal(size=(n, d))
    want = (q @ (k.T @ v)) / (q @ k.sum(axis=0))[:, None]
    np.testing.assert_allclose(orc.attention_linear(q, k, v, orc.IDENTITY, 0.0), want, rtol=1e-12)


def test_eps_enters_once_in_the_denominator():
    rng = np.random.default_rng(14)
    q, k, v = rng.normal(size=(3, 9, 3))
    eps = 0.75
    un = orc.attention_linear(q, k, v, 0, 0.0, normalize=False)
    den = orc.phi(q) @ orc.phi(k).sum(axis=0)
    np.testing.assert_allclose(orc.attention_linear(q, k, v, 0, eps), un / (den + eps)[:, None], rtol=1e-13)


def test_batched_heads_are_independent():
    rng = np.random.default_rng(15)
    q, k, v = rng.normal(size=(3, 2, 3, 10, 4))
    full = orc.attention_linear(q, k, v, 0, 1e-6)
    for b in range(2):
        for h in range(3):
            np.testing.assert_array_equal(full[b, h], orc.attention_linear(q[b, h], k[b, h], v[b, h], 0, 1e-6))
    # changing one head's keys leaves all other heads untouched
    k2 = k.copy()
    k2[1, 2] += 1.0
    full2 = orc.attention_linear(q, k2, v, 0, 1e-6)
    assert np.abs(full2[1, 2] - full[1, 2]).max() > 1e-3
    full2[1, 2] = full[1, 2]
    np.testing.assert_array_equal(full2, full)


def test_large_n_accumulation_order():
    # plain BLAS sum vs chunked pairwise-style sum at 2^18 tokens agree far below tolerance
    rng = np.random.default_rng(16)
    n, d = 1 << 18, 8
    k, v = rng.normal(size=(2, n, d))
    S, z = orc.state(k, v)
    S2 = np.zeros_like(S)
    z2 = np.zeros_like(z)
    for c in range(0, n, 4096):
        s_c, z_c = orc.state(k[c:c + 4096], v[c:c + 4096])
        S2 += s_c
        z2 += z_c
    np.testing.assert_allclose(z, z2, rtol=1e-12)
    np.testing.assert_allclose(S, S2, rtol=0, atol=1e-10 * np.abs(S).max())


def test_stored_entry_matches_widened_inputs():
    rng = np.random.default_rng(17)
    x = rng.normal(size=(3, 12, 4)).astype(np.float32)
    h = x.astype(np.float16)
    got = orc.attention_linear_stored(h[0].view(np.uint16), h[1].view(np.uint16), h[2].view(np.uint16), "f16", 0, 1e-6)
    want = orc.attention_linear(h[0].astype(np.float64), h[1].astype(np.float64), h[2].astype(np.float64), 0, 1e-6)
    np.testing.assert_array_equal(got, want)
    b = (x.view(np.uint32) >> 16).astype(np.uint16)
    xb = (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = orc.attention_linear_stored(b[0], b[1], b[2], "bf16", 0, 1e-6)
    np.testing.assert_array_equal(got, orc.attention_linear(xb[0], xb[1], xb[2], 0, 1e-6))
