"""Seeded random shapes, layouts and launch paths against the fp64 oracle: a net for combinations that the
hand-picked cases of the other GPU tests do not name."""
import numpy as np
import pytest
import torch

import paper_2409_02097_amd as lf
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu

NARROW = [8, 16, 24, 32, 40, 48, 56, 64]
WIDE = [80, 96, 128, 160]


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = ["f16", "bf16", "f32"][int(rng.integers(0, 3))]
    d = int(rng.choice(NARROW + (WIDE if dtype != "f32" else [])))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 10))
    N = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 100, 255, 257, 513, 1000, 2049, 3000]))
    layout = ["contiguous", "token_major", "padded", "fused_projection"][int(rng.integers(0, 4))]
    path = [0, lf.FLAG_FORCE_SPLIT, lf.FLAG_FORCE_FUSED][int(rng.integers(0, 3))]
    if d > 80 and path == lf.FLAG_FORCE_FUSED:
        path = 0
    groups = int(rng.integers(0, 2))          # row-piece kernels wherever the layout allows them, or by size
    fm = int(rng.choice([0, 0, 0, 1]))
    return dtype, d, B, H, N, layout, path, groups, fm


@pytest.mark.parametrize("seed", range(48))
def test_random_case_matches_oracle(seed, monkeypatch, tuning):
    dtype, d, B, H, N, layout, path, groups, fm = _case(seed)
    print(f"seed {seed}: {dtype} d={d} B={B} H={H} N={N} {layout} flags={path} groups={groups} fm={fm}", flush=True)
    if groups:
        monkeypatch.setenv("LINFUSION_HEAD_GROUPS", "3")
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=300 + seed, device="cpu")
    tdt = q.dtype
    if layout == "contiguous":
        qv, kv, vv = q.cuda(), k.cuda(), v.cuda()
        ov = torch.full_like(qv, float("nan"))
    elif layout == "token_major":
        tm = lambda t: t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)
        qv, kv, vv = tm(q), tm(k), tm(v)
        ov = torch.full((B, N, H, d), float("nan"), dtype=tdt, device="cuda").permute(0, 2, 1, 3)
    elif layout == "padded":
        pad = 16

        def padded(t):
            big = torch.full((B, H, N, d + pad), float("nan"), dtype=tdt)
            big[..., :d] = t
            return big.cuda()[..., :d]
        qv, kv, vv = padded(q), padded(k), padded(v)
        ov = torch.full((B, H, N, d + pad), float("nan"), dtype=tdt, device="cuda")[..., :d]
    else:
        buf = torch.stack([t.permute(0, 2, 1, 3) for t in (q, k, v)], dim=2).contiguous().cuda()   # [B, N, 3, H, d]
        qv, kv, vv = (buf[:, :, i].permute(0, 2, 1, 3) for i in range(3))
        ov = torch.full((B, N, H, d), float("nan"), dtype=tdt, device="cuda").permute(0, 2, 1, 3)
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)
    lf.linfusion_attn_fwd_strided(qv, kv, vv, ov, fm, 1e-6, path, ws)
    torch.cuda.synchronize()
    parity.check_all(ov.contiguous(), q, k, v, dtype, fm, 1e-6, True, f"seed {seed}")


NS_RAGGED = [1, 2, 31, 32, 33, 63, 64, 65, 100, 255, 257, 513, 1000, 2049, 3000]


@pytest.mark.parametrize("seed", range(24))
def test_random_mlp_fed_case_matches_oracle(seed):
    """linfusion_attn_fwd_mlp on random shapes of the whole-row kernels (eight heads up to d = 48, four up to 80)."""
    rng = np.random.default_rng(5000 + seed)
    dtype = ["f16", "bf16"][int(rng.integers(0, 2))]
    H = int(rng.choice([4, 8]))
    d = int(rng.choice([8, 16, 24, 32, 40, 48] if H == 8 else [8, 16, 24, 32, 40, 48, 56, 64, 80]))
    _random_mlp_case(seed, rng, dtype, H, d)


@pytest.mark.parametrize("seed", range(24))
def test_random_mlp_fed_case_on_per_head_kernels_matches_oracle(seed):
    """The same on head counts and widths that go through the statistics pass and the per-head kernels."""
    rng = np.random.default_rng(5500 + seed)
    dtype = ["f16", "bf16"][int(rng.integers(0, 2))]
    H = int(rng.choice([1, 2, 3, 5, 6, 8, 10, 12, 16, 20]))
    d = int(rng.choice([56, 64, 80, 96, 128, 160] if H == 8 else [8, 16, 24, 32, 40, 48, 56, 64, 80, 96, 128, 160]))
    _random_mlp_case(500 + seed, rng, dtype, H, d)


def _random_mlp_case(seed, rng, dtype, H, d):
    from oracle import linattn_oracle as orc
    B, N = int(rng.integers(1, 4)), int(rng.choice(NS_RAGGED))
    fm, unnorm = int(rng.choice([0, 0, 1])), bool(rng.integers(0, 2))
    slope, ln_eps = float(rng.choice([0.0, 0.01, 0.2, 1.0])), float(rng.choice([1e-6, 1e-5, 1e-3]))
    print(f"seed {seed}: mlp {dtype} H={H} d={d} B={B} N={N} fm={fm} unnorm={unnorm} slope={slope} ln_eps={ln_eps}", flush=True)
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=400 + seed))
    if fm != 0:
        ins[0] = (ins[0].float().abs() + 1.5).to(ins[0].dtype)      # relu: keep q, k positive after the branch sum
        ins[2] = (ins[2].float().abs() + 1.5).to(ins[2].dtype)
        ins[6] = ins[6].abs()
        ins[8] = ins[8].abs()
    if unnorm:   # the unnormalized sums of a few thousand tokens of wide heads reach fp16's range: smaller values
        ins[4] = (ins[4].float() * 0.0625).to(ins[4].dtype)
    dev = [t.cuda() for t in ins]
    out = torch.full_like(dev[0], float("nan"))
    ws = torch.empty(lf.linfusion_attn_mlp_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_fwd_mlp(*dev[:5], out, *dev[5:], H, fm, 1e-6, ln_eps, slope, lf.FLAG_UNNORMALIZED if unnorm else 0, ws)
    torch.cuda.synchronize()
    wide = [orc.widen(wl.stored_numpy(t), dtype) for t in ins[:5]]
    vecs = [t.numpy().astype(np.float64) for t in ins[5:]]
    ref = orc.module_mixer(*wide, *vecs, H, fm, 1e-6, not unnorm, ln_eps, slope)
    got = parity.to_f64(out)
    for b in range(B):
        for h in range(H):
            c = slice(h * d, (h + 1) * d)
            parity.check_slice(got[b, :, c], ref[b, :, c], dtype, f"seed {seed} b={b} h={h}")


@pytest.mark.parametrize("seed", range(24))
def test_random_unequal_width_case_matches_oracle(seed):
    """linfusion_attn_fwd_qv on random supported width pairs."""
    from oracle import linattn_oracle as orc
    rng = np.random.default_rng(6000 + seed)
    dtype = ["f16", "bf16"][int(rng.integers(0, 2))]
    dv = int(rng.choice([40, 64]))
    dk = int(rng.choice([x for x in (16, 32, 40, 64, 80) if x != dv]))
    B, H, N = int(rng.integers(1, 3)), int(rng.integers(1, 10)), int(rng.choice(NS_RAGGED))
    fm, unnorm = int(rng.choice([0, 0, 1])), bool(rng.integers(0, 2))
    print(f"seed {seed}: qv {dtype} d_qk={dk} d_v={dv} B={B} H={H} N={N} fm={fm} unnorm={unnorm}", flush=True)
    q, k, v = wl.make_qkv_widths(B, H, N, dk, dv, dtype, idx=500 + seed)
    if fm != 0:
        q, k = (q.float().abs() + 0.5).to(q.dtype), (k.float().abs() + 0.5).to(k.dtype)
    out = torch.full(v.shape, float("nan"), dtype=v.dtype, device="cuda")
    ws = torch.empty(lf.linfusion_attn_qv_workspace_bytes(B, H, N, dk, dv, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_fwd_qv(q.cuda(), k.cuda(), v.cuda(), out, fm, 1e-6, lf.FLAG_UNNORMALIZED if unnorm else 0, ws)
    torch.cuda.synchronize()
    got = parity.to_f64(out)
    qs, ks, vs = (wl.stored_numpy(t) for t in (q, k, v))
    for b in range(B):
        for h in range(H):
            ref = orc.attention_linear_stored(qs[b, h], ks[b, h], vs[b, h], dtype, fm, 1e-6, not unnorm)
            parity.check_slice(got[b, h], ref, dtype, f"seed {seed} b={b} h={h}")
