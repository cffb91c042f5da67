"""fp64 CPU oracle for the normalized, non-causal linear-attention token mixer of LinFusion.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: only tests,
the smoke check and the benchmark's `cpu_baseline` leg call it.  It shares no code, table or
helper with the HIP library and never imports it.

What it computes, per (batch, head), for Q, K, V in R^{N x d}, a non-negative elementwise
feature map phi and eps >= 0:

    p_j = phi(k_j)            r_i = phi(q_i)
    quadratic form (the definition):
        a_ij  = r_i . p_j                               attention score before normalization
        den_i = sum_j a_ij + eps
        out_i = sum_j (a_ij / den_i) v_j                rows of M sum to one (Sec. 2.3, Eq. 5)
    linear form (what the method evaluates, Prop. 2 / Prop. 3):
        S = sum_j p_j^T v_j   (d x d state, g'(X)^T X)
        z = sum_j p_j         (normalizer state, the non-causal Z of Eq. 5)
        out_i = (r_i S) / (r_i . z + eps)

The two forms are equal in real arithmetic; `attention_quadratic` is the definition written
out with explicit loops, `attention_linear` is the reordered sum with one matmul per step.

Readings of points on which the paper is silent (fixed by this build's task statement):
  * phi is elu(x)+1 (alpha = 1): x + 1 for x > 0, exp(x) otherwise.  RELU and IDENTITY are
    test aids.  phi acts on Q and K only; V enters raw.
  * eps is added once, to the denominator, after the dot product.
  * no 1/sqrt(d) scale (that belongs to softmax attention, Eq. 2, not to Prop. 2's form).
  * heads are independent; Q/K feature width equals the value width d.
  * `normalize=False` gives the un-normalized variant of the paper's Tab. 2 ablation:
    out_i = r_i S.

Pins (tests/test_oracle_pins.py): hand-derived exact worked examples (tests/golden/), the
explicit-loop quadratic form, the sequential SSM recurrence of Eq. 3 + Eq. 5 with all gates
equal to one, row-stochastic weights, Prop. 1 (constant V), joint K/V permutation invariance,
token-tiling invariance, the Kronecker identity from the proof of Prop. 2, affine
equivariance, the d = 1 weighted mean, all-equal K = plain mean, IDENTITY phi = two library
GEMMs, and a mutant check showing that planted mistakes are caught.
Backward pass (needed by the distillation of Sec. 2.5 (Training Objectives), Eq. 8; the paper gives no formula, so the
definition is the derivative of the forward definition): `attention_backward_quadratic` differentiates
the quadratic form with the n x n weights written out, `attention_backward_linear` is the same gradient
reordered through the d x d states (S, z, dS, dz) and is what large-N parity tests call.  Pins
(tests/test_oracle_backward.py): central differences of `attention_quadratic`, agreement of the two
forms, dV column sums, orthogonality of d phi(q) to phi(q) at eps = 0, linearity in the upstream gradient.
Upstream of the mixer (Sec. 3.1 (Implementation Details), implementation details): f' and g' are two-branch MLPs, a plain
linear branch plus one Linear-LayerNorm-LeakyReLU block, the two results added; the linear branch starts
from the softmax layer's W_Q / W_K and the other branch starts at zero.  `mlp_branch_sum` is that sum given
the two Linear outputs, `module_mixer` feeds it to the mixer over all heads of a token-major tensor.
Readings where the text names no value: LayerNorm over the whole channel axis C = H d of a token (the MLP
acts before the split into heads), biased variance, ln_eps = 1e-5 inside the square root, affine gamma and
beta per channel (gamma = beta = 0 is the zero start), LeakyReLU slope 0.01.  Pins
(tests/test_oracle_mlp.py): a library layer norm + leaky ReLU, zero mean / unit variance rows, invariance
to shifting and scaling the LayerNorm input, the zero start reducing the module to the plain mixer,
a hand-worked row, mutants.
Unpinned: that elu(x)+1 is the activation the authors trained with (their figure naming it
is not in the text available to this build) -- "parity unpinned" for that choice only.
"""
from __future__ import annotations

import numpy as np

ELU_PLUS_ONE = 0
RELU = 1
IDENTITY = 2


# ----------------------------------------------------------------------------------------
# Exact widening of stored 16-bit patterns to fp64 (own decoders: no library float16 path).
# ----------------------------------------------------------------------------------------
def decode_f16_bits(bits) -> np.ndarray:
    """IEEE binary16 bit patterns (uint16) -> fp64, exactly (normals, subnormals, inf, nan)."""
    b = np.asarray(bits).astype(np.uint16).astype(np.int64)
    sign = np.where((b >> 15) & 1, -1.0, 1.0)
    e = (b >> 10) & 0x1F
    m = (b & 0x3FF).astype(np.float64)
    normal = np.ldexp(1.0 + m / 1024.0, (e - 15).astype(np.int64))
    sub = np.ldexp(m / 1024.0, -14)
    val = np.where(e == 0, sub, normal)
    special = np.where(m == 0, np.inf, np.nan)
    val = np.where(e == 31, special, val)
    return sign * val


def decode_bf16_bits(bits) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> fp64, exactly (8 exponent bits, 7 fraction bits)."""
    b = np.asarray(bits).astype(np.uint16).astype(np.int64)
    sign = np.where((b >> 15) & 1, -1.0, 1.0)
    e = (b >> 7) & 0xFF
    m = (b & 0x7F).astype(np.float64)
    normal = np.ldexp(1.0 + m / 128.0, (e - 127).astype(np.int64))
    sub = np.ldexp(m / 128.0, -126)
    val = np.where(e == 0, sub, normal)
    special = np.where(m == 0, np.inf, np.nan)
    val = np.where(e == 255, special, val)
    return sign * val


def widen(x, dtype: str) -> np.ndarray:
    """Stored tensor -> fp64.  dtype: 'f32' (float array), 'f16' / 'bf16' (uint16 bit patterns)."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "f16":
        return decode_f16_bits(x)
    if dtype == "bf16":
        return decode_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype!r}")


# ----------------------------------------------------------------------------------------
# Feature map (Sec. 2.3: a non-negative activation on the B / C branches, here K / Q).
# ----------------------------------------------------------------------------------------
def phi(x, feature_map: int = ELU_PLUS_ONE) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if feature_map == ELU_PLUS_ONE:
        # exp is evaluated on min(x, 0) only so that large positive x cannot overflow it.
        return np.where(x > 0.0, x + 1.0, np.exp(np.minimum(x, 0.0)))
    if feature_map == RELU:
        return np.maximum(x, 0.0)
    if feature_map == IDENTITY:
        return x.copy()
    raise ValueError(f"unknown feature_map {feature_map!r}")


# ----------------------------------------------------------------------------------------
# The definition: quadratic form with the n x n matrix M written out (Eq. 4 with the mask
# removed and A~ = F G^T, rows normalised as in Sec. 2.3).  Tiny N only.
# ----------------------------------------------------------------------------------------
def attention_quadratic(q, k, v, feature_map: int = ELU_PLUS_ONE, eps: float = 0.0,
                        normalize: bool = True, return_weights: bool = False):
    """q, k, v: [N, d] (one head).  Explicit loops over (i, j); O(N^2 d)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n_q, d = q.shape
    n_k = k.shape[0]
    r = phi(q, feature_map)
    p = phi(k, feature_map)
    w = np.zeros((n_q, n_k), dtype=np.float64)
    out = np.zeros((n_q, v.shape[1]), dtype=np.float64)
    for i in range(n_q):
        a = np.zeros(n_k, dtype=np.float64)
        for j in range(n_k):
            s = 0.0
            for c in range(d):
                s += r[i, c] * p[j, c]
            a[j] = s
        den = 1.0
        if normalize:
            den = eps
            for j in range(n_k):
                den += a[j]
        for j in range(n_k):
            w[i, j] = a[j] / den
            out[i, :] += w[i, j] * v[j, :]
    if return_weights:
        return out, w
    return out


# ----------------------------------------------------------------------------------------
# The linear form (Prop. 2): state, normalizer, apply.
# ----------------------------------------------------------------------------------------
def state(k, v, feature_map: int = ELU_PLUS_ONE):
    """S = phi(K)^T V  (d x d)  and  z = sum_j phi(k_j)  (d), for one head."""
    p = phi(k, feature_map)
    v = np.asarray(v, dtype=np.float64)
    S = p.T @ v
    z = p.sum(axis=0)
    return S, z


def apply_state(q, S, z, feature_map: int = ELU_PLUS_ONE, eps: float = 0.0,
                normalize: bool = True) -> np.ndarray:
    """out_i = phi(q_i) S / (phi(q_i) . z + eps)  for the given rows of Q."""
    r = phi(q, feature_map)
    num = r @ S
    if not normalize:
        return num
    den = r @ z + eps
    return num / den[:, None]


def attention_linear(q, k, v, feature_map: int = ELU_PLUS_ONE, eps: float = 0.0,
                     normalize: bool = True) -> np.ndarray:
    """q, k, v: [..., N, d]; leading axes are independent (batch, head) slices."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if q.ndim == 2:
        S, z = state(k, v, feature_map)
        return apply_state(q, S, z, feature_map, eps, normalize)
    lead = q.shape[:-2]
    out = np.empty(lead + (q.shape[-2], v.shape[-1]), dtype=np.float64)
    for idx in np.ndindex(*lead):
        S, z = state(k[idx], v[idx], feature_map)
        out[idx] = apply_state(q[idx], S, z, feature_map, eps, normalize)
    return out


def attention_linear_stored(q, k, v, dtype: str, feature_map: int = ELU_PLUS_ONE,
                            eps: float = 0.0, normalize: bool = True) -> np.ndarray:
    """Same, on stored tensors: the oracle sees exactly the quantised inputs the GPU sees."""
    return attention_linear(widen(q, dtype), widen(k, dtype), widen(v, dtype),
                            feature_map, eps, normalize)


# ----------------------------------------------------------------------------------------
# The two-branch MLPs f', g' in front of the mixer (Sec. 3.1 (Implementation Details)): what they add after their Linears.
# ----------------------------------------------------------------------------------------
def layer_norm_rows(t, gamma, beta, ln_eps: float = 1e-5) -> np.ndarray:
    """LayerNorm over the last axis (all C channels of a token): (t - mean) / sqrt(var + ln_eps),
    var the mean squared deviation, then the per-channel affine gamma, beta."""
    t = np.asarray(t, dtype=np.float64)
    mean = t.mean(axis=-1, keepdims=True)
    dev = t - mean
    var = (dev * dev).mean(axis=-1, keepdims=True)
    return dev / np.sqrt(var + ln_eps) * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)


def leaky_relu(x, slope: float = 0.01) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    return np.where(x >= 0.0, x, slope * x)


def mlp_branch_sum(a, t, gamma, beta, ln_eps: float = 1e-5, slope: float = 0.01) -> np.ndarray:
    """Output of f' (or g') for tokens whose linear-branch result is `a` [..., C] and whose second
    branch's Linear result is `t` [..., C]:  a + LeakyReLU(LayerNorm(t))."""
    return np.asarray(a, dtype=np.float64) + leaky_relu(layer_norm_rows(t, gamma, beta, ln_eps), slope)


def module_mixer(a_q, t_q, a_k, t_k, v, gamma_q, beta_q, gamma_k, beta_k, H: int,
                 feature_map: int = ELU_PLUS_ONE, eps: float = 0.0, normalize: bool = True,
                 ln_eps: float = 1e-5, slope: float = 0.01) -> np.ndarray:
    """Token-major tensors [B, N, C], C = H d, head h owning channels h d .. (h + 1) d - 1:
    q = f'(X), k = g'(X) from their branch results, then the mixer per (batch, head).  Returns [B, N, C]."""
    q = mlp_branch_sum(a_q, t_q, gamma_q, beta_q, ln_eps, slope)
    k = mlp_branch_sum(a_k, t_k, gamma_k, beta_k, ln_eps, slope)
    v = np.asarray(v, dtype=np.float64)
    B, N, C = q.shape
    d = C // H
    out = np.empty_like(v)
    for b in range(B):
        for h in range(H):
            c = slice(h * d, (h + 1) * d)
            S, z = state(k[b, :, c], v[b, :, c], feature_map)
            out[b, :, c] = apply_state(q[b, :, c], S, z, feature_map, eps, normalize)
    return out


# ----------------------------------------------------------------------------------------
# Backward pass: gradients of a scalar loss L with respect to q, k, v, given g = dL/d out.
# ----------------------------------------------------------------------------------------
def phi_prime(x, feature_map: int = ELU_PLUS_ONE) -> np.ndarray:
    """d phi / dx, elementwise (one-sided value 1 at x = 0 for elu+1, 0 for relu)."""
    x = np.asarray(x, dtype=np.float64)
    if feature_map == ELU_PLUS_ONE:
        return np.where(x > 0.0, 1.0, np.exp(np.minimum(x, 0.0)))
    if feature_map == RELU:
        return np.where(x > 0.0, 1.0, 0.0)
    if feature_map == IDENTITY:
        return np.ones_like(x)
    raise ValueError(f"unknown feature_map {feature_map!r}")


def attention_backward_quadratic(q, k, v, g, feature_map: int = ELU_PLUS_ONE, eps: float = 0.0,
                                 normalize: bool = True):
    """Derivative of the quadratic form, one head, with the n x n matrices written out.
    out_i = sum_j w_ij v_j,  w_ij = a_ij / den_i,  a_ij = r_i . p_j,  den_i = sum_j a_ij + eps:
        dv_j  = sum_i w_ij g_i
        da_ij = (g_i . v_j - g_i . out_i) / den_i          (normalized; g_i . v_j otherwise)
        dr_i  = sum_j da_ij p_j ,  dp_j = sum_i da_ij r_i ,  dq = dr * phi'(q) ,  dk = dp * phi'(k)
    Returns (dq, dk, dv).  O(N^2 d): small N only."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    r = phi(q, feature_map)
    p = phi(k, feature_map)
    a = r @ p.T                                   # [n_q, n_k]
    gv = g @ v.T                                  # g_i . v_j
    if normalize:
        den = a.sum(axis=1) + eps
        w = a / den[:, None]
        out = w @ v
        da = (gv - (g * out).sum(axis=1)[:, None]) / den[:, None]
    else:
        w = a
        da = gv
    dv = w.T @ g
    dr = da @ p
    dp = da.T @ r
    return dr * phi_prime(q, feature_map), dp * phi_prime(k, feature_map), dv


def attention_backward_linear(q, k, v, g, feature_map: int = ELU_PLUS_ONE, eps: float = 0.0,
                              normalize: bool = True):
    """The same gradient with every sum over tokens taken through a d x d (or d) state:
        S = P^T V, z = P^T 1;  den = R z + eps;  out = R S / den
        gn_i = g_i / den_i ;  e_i = -(g_i . out_i) / den_i        (gn = g, e = 0 if not normalized)
        dS = R^T gn ,  dz = R^T e
        dr = gn S^T + e z^T ;  dp = V dS^T + 1 dz^T ;  dv = P dS
    One head; O(N d^2)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    r = phi(q, feature_map)
    p = phi(k, feature_map)
    S = p.T @ v
    z = p.sum(axis=0)
    if normalize:
        den = r @ z + eps
        out = (r @ S) / den[:, None]
        gn = g / den[:, None]
        e = -(g * out).sum(axis=1) / den
    else:
        gn = g
        e = np.zeros(q.shape[0], dtype=np.float64)
    dS = r.T @ gn
    dz = r.T @ e
    dr = gn @ S.T + e[:, None] * z[None, :]
    dp = v @ dS.T + dz[None, :]
    dv = p @ dS
    return dr * phi_prime(q, feature_map), dp * phi_prime(k, feature_map), dv


# ----------------------------------------------------------------------------------------
# Output-format helper for tolerance checks: half a unit in the last place of `ref` in the
# storage format the library writes (the stated tolerance governs the arithmetic before the
# final round-to-nearest cast; the cast itself may move a value by up to this much).
# ----------------------------------------------------------------------------------------
_FMT = {"f32": (24, -126), "f16": (11, -14), "bf16": (8, -126)}


def half_ulp(ref, dtype: str) -> np.ndarray:
    prec, emin = _FMT[dtype]
    a = np.abs(np.asarray(ref, dtype=np.float64))
    _, e = np.frexp(a)                               # a = m * 2^e, m in [0.5, 1); frexp(0) = (0, 0)
    e = np.where(a == 0.0, emin, np.maximum(e - 1, emin))   # leading-bit exponent, clamped to subnormal spacing
    return np.ldexp(0.5, (e - (prec - 1)).astype(np.int64))
