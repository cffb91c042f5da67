"""Pins for the oracle's upstream part: the two-branch MLPs f', g' of Sec. 3.1 (Implementation Details) (a linear branch plus one
Linear-LayerNorm-LeakyReLU block, results added) in front of the mixer.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import linattn_oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


@pytest.mark.parametrize("C", [8, 40, 320])
def test_against_the_library_layer_norm_and_leaky_relu(C):
    r = _rng(C)
    a, t = r.normal(size=(5, 7, C)), r.normal(1.5, 3.0, size=(5, 7, C))
    gamma, beta = r.normal(size=C), r.normal(size=C)
    ours = orc.mlp_branch_sum(a, t, gamma, beta, ln_eps=1e-5, slope=0.01)
    tt = torch.from_numpy(t)
    lib = torch.nn.functional.leaky_relu(
        torch.nn.functional.layer_norm(tt, (C,), torch.from_numpy(gamma), torch.from_numpy(beta), 1e-5), 0.01)
    np.testing.assert_allclose(ours, a + lib.numpy(), rtol=0, atol=1e-12)


def test_hand_worked_row():
    # t = (1, 2, 3, 6): mean 3, deviations (-2, -1, 0, 3), variance 14/4 = 3.5
    t = np.array([[1.0, 2.0, 3.0, 6.0]])
    gamma = np.array([1.0, 2.0, 1.0, 0.5])
    beta = np.array([0.0, 0.0, -1.0, 0.25])
    s = np.sqrt(3.5)
    ln = np.array([-2 / s, -2 / s, -1.0, 1.5 / s + 0.25])
    want = np.array([[10.0, 20.0, 30.0, 40.0]]) + np.where(ln >= 0, ln, 0.1 * ln)
    got = orc.mlp_branch_sum([[10.0, 20.0, 30.0, 40.0]], t, gamma, beta, ln_eps=0.0, slope=0.1)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


def test_rows_are_standardised_over_all_channels():
    r = _rng(3)
    t = r.normal(-2.0, 5.0, size=(4, 9, 64))
    ln = orc.layer_norm_rows(t, np.ones(64), np.zeros(64), ln_eps=0.0)
    np.testing.assert_allclose(ln.mean(axis=-1), 0.0, atol=1e-13)
    np.testing.assert_allclose((ln * ln).mean(axis=-1), 1.0, atol=1e-12)
    # per row, not per tensor or per head: another row's values do not matter
    t2 = t.copy()
    t2[0, 0] *= 100.0
    ln2 = orc.layer_norm_rows(t2, np.ones(64), np.zeros(64), ln_eps=0.0)
    np.testing.assert_allclose(ln2[1:], ln[1:], atol=0)
    np.testing.assert_allclose(ln2[0, 1:], ln[0, 1:], atol=0)


def test_shift_and_scale_of_the_layer_norm_input_cancel():
    r = _rng(4)
    t = r.normal(size=(3, 16))
    gamma, beta = r.normal(size=16), r.normal(size=16)
    base = orc.layer_norm_rows(t, gamma, beta, ln_eps=0.0)
    np.testing.assert_allclose(orc.layer_norm_rows(3.0 * t + 7.0, gamma, beta, ln_eps=0.0), base, atol=1e-12)
    # ln_eps sits inside the square root next to the variance: scaling t by s equals dividing ln_eps by s^2
    np.testing.assert_allclose(orc.layer_norm_rows(4.0 * t, gamma, beta, ln_eps=1.6),
                               orc.layer_norm_rows(t, gamma, beta, ln_eps=0.1), atol=1e-12)


def test_leaky_relu_slope():
    x = np.array([-2.0, -0.0, 0.0, 3.0])
    np.testing.assert_array_equal(orc.leaky_relu(x, 0.01), np.array([-0.02, 0.0, 0.0, 3.0]))


def test_zero_start_reduces_the_module_to_the_plain_mixer():
    """Sec. 3.1 (Implementation Details): the second branch starts at zero, so at initialisation q = X W_Q and k = X W_K exactly."""
    r = _rng(5)
    B, N, H, d = 2, 33, 4, 8
    C = H * d
    a_q, t_q, a_k, t_k, v = (r.normal(size=(B, N, C)) for _ in range(5))
    zero = np.zeros(C)
    got = orc.module_mixer(a_q, t_q, a_k, t_k, v, zero, zero, zero, zero, H, eps=1e-6)
    heads = lambda x: x.reshape(B, N, H, d).transpose(0, 2, 1, 3)
    want = orc.attention_linear(heads(a_q), heads(a_k), heads(v), eps=1e-6).transpose(0, 2, 1, 3).reshape(B, N, C)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_module_equals_mixer_on_explicitly_formed_q_and_k():
    r = _rng(6)
    B, N, H, d = 1, 20, 2, 8
    C = H * d
    a_q, t_q, a_k, t_k, v = (r.normal(size=(B, N, C)) for _ in range(5))
    gq, bq, gk, bk = (r.normal(size=C) for _ in range(4))
    got = orc.module_mixer(a_q, t_q, a_k, t_k, v, gq, bq, gk, bk, H, eps=1e-6, normalize=False)
    q = a_q + torch.nn.functional.leaky_relu(
        torch.nn.functional.layer_norm(torch.from_numpy(t_q), (C,), torch.from_numpy(gq), torch.from_numpy(bq)), 0.01).numpy()
    k = a_k + torch.nn.functional.leaky_relu(
        torch.nn.functional.layer_norm(torch.from_numpy(t_k), (C,), torch.from_numpy(gk), torch.from_numpy(bk)), 0.01).numpy()
    for h in range(H):
        c = slice(h * d, (h + 1) * d)
        want = orc.attention_quadratic(q[0, :, c], k[0, :, c], v[0, :, c], eps=1e-6, normalize=False)
        np.testing.assert_allclose(got[0, :, c], want, rtol=1e-11, atol=1e-11)


def test_planted_mistakes_are_caught():
    r = _rng(7)
    C = 24
    a, t = r.normal(size=(6, C)), r.normal(2.0, 2.0, size=(6, C))
    gamma, beta = r.normal(size=C), r.normal(size=C)
    good = orc.mlp_branch_sum(a, t, gamma, beta)
    mean = t.mean(-1, keepdims=True)
    var = ((t - mean) ** 2).mean(-1, keepdims=True)
    lk = lambda x: np.where(x >= 0, x, 0.01 * x)
    mutants = {
        "unbiased variance": a + lk((t - mean) / np.sqrt(var * C / (C - 1) + 1e-5) * gamma + beta),
        "statistics per head of 8 channels": a + lk(orc.layer_norm_rows(t.reshape(6, 3, 8), 1.0, 0.0).reshape(6, C) * gamma + beta),
        "activation before the affine": a + lk((t - mean) / np.sqrt(var + 1e-5)) * gamma + beta,
        "mean not removed": a + lk(t / np.sqrt(var + 1e-5) * gamma + beta),
        "relu instead of leaky": a + np.maximum((t - mean) / np.sqrt(var + 1e-5) * gamma + beta, 0.0),
        "linear branch through the activation too": lk(a + (t - mean) / np.sqrt(var + 1e-5) * gamma + beta),
        "gamma and beta swapped": a + lk((t - mean) / np.sqrt(var + 1e-5) * beta + gamma),
    }
    for name, bad in mutants.items():
        assert np.abs(bad - good).max() > 1e-3, name
