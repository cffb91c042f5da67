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
def test_random_case_matches_oracle(seed, monkeypatch):
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
