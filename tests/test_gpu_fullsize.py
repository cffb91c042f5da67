"""Full-size parity at the benchmark workload (16384x8192 image, 2,097,152 tokens per head), in the
launch configuration bench.py times.

Forward: EVERY element of EVERY head is compared with the oracle.  Per head the oracle accumulates the
exact fp64 state (S, z) over all tokens, streamed in slices to bound host memory, then evaluates all
2,097,152 output rows slice by slice; each slice goes through tests/parity.py: check_slice (whose error
scale is then the slice's own largest reference magnitude, never larger than the head's).  One test per
head, so that a long run keeps reporting.  The same reference rows serve the contiguous [B, H, N, d] call
and the token-major [B, N, H*d] call (row-piece kernels on groups of eight heads); a bf16 run of the same
shape has its own references.  The state entry point is checked on every head as well.

Backward and the MLP-fed call: sampled rows (the oracle evaluates them one by one from full-size states)."""
import numpy as np
import pytest
import torch

import paper_2409_02097_amd as lf
from oracle import linattn_oracle as orc
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu

NAME = "sd15_16k_f16"
STEP = 1 << 19          # oracle slice, in token rows


def _stream_head(t, h, step=STEP, dtype="f16"):
    """One head of a [1, H, N, d] device tensor, widened to fp64, in slices that bound host memory."""
    N = t.shape[2]
    for s0 in range(0, N, step):
        yield s0, orc.widen(wl.stored_numpy(t[0, h, s0:s0 + step]), dtype)


class _FullRun:
    """The library's outputs for the whole workload in one storage type: contiguous call, token-major call
    (f16 only) and the state entry point; q, k, v stay on the device for the oracle to stream."""

    def __init__(self, dtype, token_major):
        c = wl.CONFIGS[NAME]
        self.B, self.H, self.N, self.d = c["B"], c["H"], c["N"], c["d"]
        self.dtype = dtype
        B, H, N, d = self.B, self.H, self.N, self.d
        code = wl.DTYPE_CODE[dtype]
        if dtype == c["dtype"]:
            self.q, self.k, self.v = wl.make_config(NAME, device="cuda")
        else:      # the same shape and seeds, values rounded to the other storage type
            self.q, self.k, self.v = wl.make_qkv(B, H, N, d, dtype, idx=c["idx"], device="cuda")
        ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
        self.plan = lf.linfusion_attn_plan(B, H, N, d, code)
        self.out = torch.full_like(self.q, float("nan"))
        lf.linfusion_attn_fwd_ex(self.q, self.k, self.v, self.out, lf.PHI_ELU_PLUS_ONE, wl.EPS, lf.FLAG_NONE, ws)
        st = torch.empty(B * H * (d * d + d), dtype=torch.float32, device="cuda")
        lf.linfusion_attn_state(self.k, self.v, st, lf.PHI_ELU_PLUS_ONE, ws)
        torch.cuda.synchronize()
        self.state = st.cpu().numpy().astype(np.float64).reshape(B * H, d * d + d)
        self.out_tm = None
        if token_major:
            tm = lambda t: t.permute(0, 2, 1, 3).contiguous()
            qt, kt, vt = tm(self.q), tm(self.k), tm(self.v)
            ot = torch.full_like(qt, float("nan"))
            view = lambda t: t.permute(0, 2, 1, 3)
            lf.linfusion_attn_fwd_strided(view(qt), view(kt), view(vt), view(ot), lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, ws)
            torch.cuda.synchronize()
            self.out_tm = ot      # [1, N, H, d]
            del qt, kt, vt

    def check_head(self, h):
        d, dtype, N = self.d, self.dtype, self.N
        S, z = np.zeros((d, d)), np.zeros(d)
        for (s0, ks), (_, vs) in zip(_stream_head(self.k, h, dtype=dtype), _stream_head(self.v, h, dtype=dtype)):
            S_c, z_c = orc.state(ks, vs)
            S += S_c
            z += z_c
        gS, gz = self.state[h, :d * d].reshape(d, d), self.state[h, d * d:]
        assert np.abs(gS - S).max() <= parity.TOL[dtype] * np.abs(S).max()
        assert np.abs(gz - z).max() <= parity.TOL[dtype] * np.abs(z).max()
        worst = {"contiguous": (0.0, 0.0, 0.0), "token-major": (0.0, 0.0, 0.0)}
        rows = 0
        for s0, qs in _stream_head(self.q, h, dtype=dtype):
            ref = orc.apply_state(qs, S, z, orc.ELU_PLUS_ONE, wl.EPS)
            n = ref.shape[0]
            outs = [("contiguous", self.out[0, h, s0:s0 + n])]
            if self.out_tm is not None:
                outs.append(("token-major", self.out_tm[0, s0:s0 + n, h]))
            for label, got_t in outs:
                r = parity.check_slice(parity.to_f64(got_t), ref, dtype, f"{NAME} {dtype} {label} head {h} rows {s0}..{s0 + n}")
                worst[label] = tuple(max(a, c) for a, c in zip(worst[label], r))
            rows += n
        assert rows == N
        for label, w in worst.items():
            if label == "contiguous" or self.out_tm is not None:
                print(f"{NAME} {dtype} {label} head {h}: all {N} rows, worst max-norm ratio {w[0]:.2e} "
                      f"({w[2]:.2e} beyond the output's half ulp), worst rel L2 {w[1]:.2e}", flush=True)


@pytest.fixture(scope="module")
def full_f16():
    run = _FullRun("f16", token_major=True)
    assert run.plan["path"] == 0 and run.plan["apply_wgs_per_head"] >= 64   # the launch shape bench.py times
    yield run
    del run
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def full_bf16():
    run = _FullRun("bf16", token_major=False)
    yield run
    del run
    torch.cuda.empty_cache()


@pytest.mark.parametrize("h", range(8))
def test_16k_image_workload_every_row_f16(full_f16, h):
    """All 2,097,152 rows of head h: contiguous call and token-major call against the oracle."""
    full_f16.check_head(h)


@pytest.mark.parametrize("h", range(8))
def test_16k_image_workload_every_row_bf16(full_bf16, h):
    """The same shape in bf16 (hi + lo operands): all rows of head h of the contiguous call."""
    full_bf16.check_head(h)


def test_16k_image_workload_outputs_inside_the_range_of_v(full_f16):
    """A property that holds at any size: the weights are a convex combination (up to eps), so every output
    lies inside the range of its head's values."""
    run = full_f16
    vmin = run.v.amin(dim=2, keepdim=True).float()
    vmax = run.v.amax(dim=2, keepdim=True).float()
    o32 = run.out.float()
    assert bool(torch.isfinite(o32).all())
    assert bool((o32 >= vmin - 1e-3).all()) and bool((o32 <= vmax + 1e-3).all())


def test_16k_image_workload_backward_sampled_rows():
    """Gradients at the benchmark size: the oracle streams one head through its state form (S, z, then dS, dz
    over all 2,097,152 tokens) and evaluates sampled rows of dq, dk and dv."""
    name = "sd15_16k_f16"
    c = wl.CONFIGS[name]
    B, H, N, d, dtype = c["B"], c["H"], c["N"], c["d"], c["dtype"]
    q, k, v = wl.make_config(name, device="cuda")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 99777, dtype, "cuda")
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_bwd(q, k, v, g, dq, dk, dv, lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, ws)
    torch.cuda.synchronize()
    for t in (dq, dk, dv):
        assert bool(torch.isfinite(t).all())
    rng = np.random.default_rng(20240904)
    edges = [0, 31, 32, N // 2, N - 32, N - 1]
    h = 5
    print(f"backward head {h}: oracle states over {N} tokens", flush=True)
    S, z = np.zeros((d, d)), np.zeros(d)
    for (s0, ks), (_, vs) in zip(_stream_head(k, h), _stream_head(v, h)):
        S_c, z_c = orc.state(ks, vs)
        S += S_c
        z += z_c
    dS, dz = np.zeros((d, d)), np.zeros(d)
    a_gn, a_e = 0.0, 0.0
    for (s0, qs), (_, gs) in zip(_stream_head(q, h), _stream_head(g, h)):
        r = orc.phi(qs)
        den = r @ z + wl.EPS
        gn = gs / den[:, None]
        e = -(gs * ((r @ S) / den[:, None])).sum(axis=1) / den
        dS += r.T @ gn
        dz += r.T @ e
    rows = np.unique(np.concatenate([np.array(edges), rng.integers(0, N, size=2048)]))
    idx = torch.from_numpy(rows).cuda()
    sel = lambda t: orc.widen(wl.stored_numpy(t[0, h].index_select(0, idx)), dtype)
    qs, ks, vs, gs = sel(q), sel(k), sel(v), sel(g)
    r, p = orc.phi(qs), orc.phi(ks)
    den = r @ z + wl.EPS
    gn = gs / den[:, None]
    e = -(gs * ((r @ S) / den[:, None])).sum(axis=1) / den
    ref = {"dq": (gn @ S.T + e[:, None] * z[None, :]) * orc.phi_prime(qs),
           "dk": (vs @ dS.T + dz[None, :]) * orc.phi_prime(ks),
           "dv": p @ dS}
    scale = {"dq": ((np.abs(gn) @ np.abs(S).T + np.abs(e)[:, None] * np.abs(z)[None, :]) * orc.phi_prime(qs)).max(),
             "dk": ((np.abs(vs) @ np.abs(dS).T + np.abs(dz)[None, :]) * orc.phi_prime(ks)).max(),
             "dv": (np.abs(p) @ np.abs(dS)).max()}
    for name_, t in (("dq", dq), ("dk", dk), ("dv", dv)):
        got = parity.to_f64(t[0, h].index_select(0, idx))
        err = np.abs(got - ref[name_])
        bound = parity.TOL[dtype] * scale[name_] + orc.half_ulp(ref[name_], dtype)
        assert (err - bound).max() <= 0, f"{name_}: error {err.max():.3e} vs term scale {scale[name_]:.3e}"
        print(f"  {name_}: error / term scale {err.max() / scale[name_]:.2e}", flush=True)


def test_16k_image_workload_mlp_fed_sampled_rows():
    """linfusion_attn_fwd_mlp at the benchmark shape: the oracle forms k = g'(X) for all 2,097,152 tokens in
    slices (LayerNorm over the 320 channels of a token), accumulates the exact fp64 state of a subset of heads,
    and evaluates sampled output rows; finiteness and the range of V are checked over every element."""
    name = "sd15_16k_f16"
    c = wl.CONFIGS[name]
    _mlp_fed_sampled_rows(name, c["B"], c["H"], c["N"], c["d"], c["dtype"], c["idx"], (0, 5, 7))


def test_large_mlp_fed_case_on_per_head_kernels_sampled_rows():
    """The same check where token rows do not fit one workgroup (ten heads of 64 channels, as in the SD-XL
    levels): statistics pass + per-head kernels at 2^20 tokens."""
    _mlp_fed_sampled_rows("10 heads of 64, bf16", 1, 10, 1 << 20, 64, "bf16", 77, (0, 4, 9))


def _mlp_fed_sampled_rows(name, B, H, N, d, dtype, idx_, heads):
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=idx_, device="cuda")
    a_q, t_q, a_k, t_k, v = ins[:5]
    gq, bq, gk, bk = (t.cpu().numpy().astype(np.float64) for t in ins[5:])
    out = torch.empty_like(a_q)
    ws = torch.empty(lf.linfusion_attn_mlp_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype]), dtype=torch.uint8,
                     device="cuda")
    lf.linfusion_attn_fwd_mlp(a_q, t_q, a_k, t_k, v, out, *ins[5:], H, lf.PHI_ELU_PLUS_ONE, wl.EPS, 1e-5, 0.01, 0, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    vmin = v.amin(dim=1, keepdim=True).float()
    vmax = v.amax(dim=1, keepdim=True).float()
    assert bool((out.float() >= vmin - 1e-3).all()) and bool((out.float() <= vmax + 1e-3).all())

    S = {h: np.zeros((d, d)) for h in heads}
    z = {h: np.zeros(d) for h in heads}
    step = 1 << 18
    for s0 in range(0, N, step):
        if s0 % (1 << 20) == 0:
            print(f"oracle keys: tokens {s0} ..", flush=True)
        sl = slice(s0, s0 + step)
        k = orc.mlp_branch_sum(orc.widen(wl.stored_numpy(a_k[0, sl]), dtype), orc.widen(wl.stored_numpy(t_k[0, sl]), dtype),
                               gk, bk, 1e-5, 0.01)
        vs = orc.widen(wl.stored_numpy(v[0, sl]), dtype)
        for h in heads:
            S_c, z_c = orc.state(k[:, h * d:(h + 1) * d], vs[:, h * d:(h + 1) * d])
            S[h] += S_c
            z[h] += z_c
    rng = np.random.default_rng(20240903)
    edges = [0, 31, 32, 255, 256, N // 2 - 1, N // 2, N - 33, N - 32, N - 1]
    rows = np.unique(np.concatenate([np.array(edges), rng.integers(0, N, size=4096)]))
    idx = torch.from_numpy(rows).cuda()
    q = orc.mlp_branch_sum(orc.widen(wl.stored_numpy(a_q[0].index_select(0, idx)), dtype),
                           orc.widen(wl.stored_numpy(t_q[0].index_select(0, idx)), dtype), gq, bq, 1e-5, 0.01)
    got = parity.to_f64(out[0].index_select(0, idx))
    for h in heads:
        ref = orc.apply_state(q[:, h * d:(h + 1) * d], S[h], z[h], orc.ELU_PLUS_ONE, wl.EPS)
        r = parity.check_slice(got[:, h * d:(h + 1) * d], ref, dtype, f"{name} mlp-fed head {h} sampled rows")
        print(f"  head {h} sampled rows: max-norm ratio {r[0]:.2e}, rel L2 {r[1]:.2e}", flush=True)
