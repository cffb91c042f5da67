"""Tolerance rule for comparing the library with the fp64 oracle (shared by the GPU tests).

The task states "max relative error 2e-3 for fp16/bf16 inputs with fp32 accumulation, 1e-5 for
fp32 inputs".  Outputs are convex combinations of zero-mean values and cross zero, so an
element-by-element ratio is ill-posed; the error is measured per (batch, head) slice against
the slice's largest reference magnitude, and in relative L2 norm.  The tolerance governs the
arithmetic before the final round-to-nearest cast to the storage type; that cast may move a
value by half a unit in the last place of the reference, which is added element-wise
(uniform rounding noise of that size has relative L2 norm 2^-(p-1) / sqrt(12), p = precision).

    |gpu - ref| <= tol * max|ref_slice| + half_ulp_out(ref)          for every element
    (check_slice also returns max(|gpu - ref| - half_ulp_out(ref), 0) / max|ref_slice|: the error the final cast
     does not explain, to be read against `tol` alone)
    ||gpu - ref||_2 <= (tol + 2^-(p-1) / sqrt(12)) ||ref||_2 + ||h||_2   for every slice

where h holds half_ulp_out(ref) for the reference values below the smallest normal number of the storage
type and 0 elsewhere: there the spacing of representable values is absolute, not relative (a reference
of 1e-16 is correctly stored as 0 in fp16), so the relative-noise term does not cover the final cast.
"""
import math

import numpy as np

from oracle import linattn_oracle as orc

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}
PREC = {"f32": 24, "f16": 11, "bf16": 8}
MIN_NORMAL = {"f32": 2.0 ** -126, "f16": 2.0 ** -14, "bf16": 2.0 ** -126}


def to_f64(t):
    """Library output tensor -> fp64 numpy (exact widening)."""
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


def check_slice(gpu, ref, dtype, what=""):
    """gpu, ref: [n, d] fp64 arrays of one (b, h) slice (or a sample of its rows)."""
    tol = TOL[dtype]
    assert np.all(np.isfinite(ref)), f"{what}: oracle produced non-finite values"
    assert np.all(np.isfinite(gpu)), f"{what}: library produced non-finite values"
    scale = np.abs(ref).max()
    err = np.abs(gpu - ref)
    bound = tol * scale + orc.half_ulp(ref, dtype)
    worst = (err - bound).max()
    # the part of the error that the final cast's half ulp does not explain, against the arithmetic budget `tol`
    arith = float(np.maximum(err - orc.half_ulp(ref, dtype), 0.0).max() / max(scale, 1e-300))
    assert worst <= 0, (f"{what}: max-norm error {err.max():.3e} vs scale {scale:.3e} "
                        f"(ratio {err.max() / max(scale, 1e-300):.3e}; {arith:.3e} beyond the output's half ulp; "
                        f"tol {tol:g})")
    nref = math.sqrt(float((ref * ref).sum()))
    if nref > 0:
        rel = math.sqrt(float((err * err).sum())) / nref
        lim = tol + 2.0 ** -(PREC[dtype] - 1) / math.sqrt(12.0)
        tiny = np.abs(ref) < MIN_NORMAL[dtype]
        if tiny.any():
            h = orc.half_ulp(ref, dtype)[tiny]
            lim += math.sqrt(float((h * h).sum())) / nref
        assert rel <= lim, f"{what}: relative L2 error {rel:.3e} > {lim:.3e}"
        return err.max() / max(scale, 1e-300), rel, arith
    return err.max() / max(scale, 1e-300), 0.0, arith


def check_all(out_t, q_t, k_t, v_t, dtype, feature_map=0, eps=1e-6, normalize=True, what=""):
    """Full element-by-element comparison over every (b, h) slice.  Returns worst ratios."""
    from paper_2409_02097_amd.workloads import stored_numpy
    qs, ks, vs = stored_numpy(q_t), stored_numpy(k_t), stored_numpy(v_t)
    gpu = to_f64(out_t)
    B, H = qs.shape[:2]
    worst = (0.0, 0.0, 0.0)      # max-norm ratio, relative L2, max-norm ratio beyond the output's half ulp
    for b in range(B):
        for h in range(H):
            ref = orc.attention_linear_stored(qs[b, h], ks[b, h], vs[b, h], dtype, feature_map, eps, normalize)
            r = check_slice(gpu[b, h], ref, dtype, f"{what} b={b} h={h}")
            worst = tuple(max(a, c) for a, c in zip(worst, r))
    return worst


def gradient_term_scales(q, k, v, g, fm, eps, normalize):
    """Largest magnitude, per gradient, of the sums of absolute terms that the gradient is made of:
        dq: (|g / den| |S|^T + |e| |z|) phi'(q),  dk: (|v| |dS|^T + |dz|) phi'(k),  dv: |p| |dS|.
    Gradients cancel (with one token dq is exactly zero: the output does not depend on q), so an error
    bound has to be relative to what is summed, not to what is left; these are the classical |A| |B| bounds."""
    r, p = orc.phi(q, fm), orc.phi(k, fm)
    S, z = orc.state(k, v, fm)
    if normalize:
        den = r @ z + eps
        gn = g / den[:, None]
        e = -(g * ((r @ S) / den[:, None])).sum(axis=1) / den
    else:
        gn, e = g, np.zeros(q.shape[0])
    dS, dz = r.T @ gn, r.T @ e
    sq = (np.abs(gn) @ np.abs(S).T + np.abs(e)[:, None] * np.abs(z)[None, :]) * np.abs(orc.phi_prime(q, fm))
    sk = (np.abs(v) @ np.abs(dS).T + np.abs(dz)[None, :]) * np.abs(orc.phi_prime(k, fm))
    sv = np.abs(p) @ np.abs(dS)
    return sq.max(), sk.max(), sv.max()


# Result-relative bound on a whole gradient tensor (beyond the half ulp of its storage type): ||gpu - ref|| / ||ref||.
# Gradients cancel, so single elements cannot be held to a relative bound, but the tensor as a whole can.
GRAD_REL_L2 = {"f16": 2e-3, "bf16": 2e-3, "f32": 1e-5}   # the forward budgets; measured 7e-4, 5e-7, 4e-7
REL_L2_SEEN = {}


def check_gradients(got, q, k, v, g, dtype, fm=0, eps=1e-6, normalize=True, what=""):
    """got = (dq, dk, dv) of one (b, h) slice as fp64 arrays; q, k, v, g the slice's widened inputs.
    |gpu - ref| <= tol * (largest sum of absolute terms in the slice) + half an ulp of the output type."""
    tol = TOL[dtype]
    ref = orc.attention_backward_linear(q, k, v, g, fm, eps, normalize)
    scales = gradient_term_scales(q, k, v, g, fm, eps, normalize)
    worst = 0.0
    for gpu, want, scale, name in zip(got, ref, scales, ("dq", "dk", "dv")):
        assert np.all(np.isfinite(gpu)), f"{what} {name}: non-finite values"
        err = np.abs(gpu - want)
        bound = tol * scale + orc.half_ulp(want, dtype)
        assert (err - bound).max() <= 0, (f"{what} {name}: error {err.max():.3e} vs term scale "
                                          f"{scale:.3e} (ratio {err.max() / scale:.3e}, tol {tol:g})")
        worst = max(worst, float((err / scale).max()))
        # result-relative as well: the error of the whole gradient tensor against its own size (half an ulp of every
        # output allowed for, as above)
        beyond = np.maximum(err - orc.half_ulp(want, dtype), 0.0)
        rel = float(np.sqrt((beyond ** 2).sum()) / max(np.sqrt((want ** 2).sum()), 1e-300))
        # (only where the tensor is not itself a cancellation: with a single token dq is exactly zero, and the measure
        #  would divide rounding noise by rounding noise)
        if np.sqrt((want ** 2).mean()) >= 1e-2 * scale:
            REL_L2_SEEN[(dtype, name)] = max(REL_L2_SEEN.get((dtype, name), 0.0), rel)
            assert rel <= GRAD_REL_L2[dtype], f"{what} {name}: relative L2 error {rel:.3e} (bound {GRAD_REL_L2[dtype]:g})"
    return worst
