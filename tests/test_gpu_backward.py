"""GPU parity of the backward pass (linfusion_attn_bwd) against the fp64 oracle's gradients."""
import numpy as np
import pytest
import torch

import paper_2409_02097_amd as lf
from oracle import linattn_oracle as orc
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def _run(q, k, v, g, fm=0, eps=1e-6, flags=0):
    B, H, N, d = q.shape
    code = wl.DTYPE_CODE[{torch.float16: "f16", torch.bfloat16: "bf16"}[q.dtype]]
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    outs = [torch.full_like(q, float("nan")).cuda() for _ in range(3)]
    lf.linfusion_attn_bwd(q.cuda(), k.cuda(), v.cuda(), g.cuda(), *outs, fm, eps, flags, ws)
    torch.cuda.synchronize()
    return outs


def _check(outs, q, k, v, g, dtype, fm, eps, normalize, what):
    """Every (batch, head) slice against the oracle's gradients, rule of tests/parity.py: check_gradients."""
    qs, ks, vs, gs = (wl.stored_numpy(t) for t in (q, k, v, g))
    B, H = qs.shape[:2]
    worst = 0.0
    for b in range(B):
        for h in range(H):
            w = [orc.widen(x[b, h], dtype) for x in (qs, ks, vs, gs)]
            got = [parity.to_f64(t[b, h]) for t in outs]
            worst = max(worst, parity.check_gradients(got, *w, dtype, fm, eps, normalize, f"{what} b={b} h={h}"))
    return worst


SHAPES = [
    (1, 2, 1, 40, "f16"), (1, 1, 31, 64, "f16"), (2, 3, 33, 40, "f16"), (1, 2, 1000, 40, "f16"),
    (2, 2, 4099, 64, "f16"), (1, 3, 777, 8, "f16"), (1, 1, 130, 16, "f16"), (1, 2, 515, 24, "f16"),
    (1, 2, 300, 32, "f16"), (1, 2, 300, 48, "f16"), (1, 1, 300, 56, "f16"), (1, 2, 700, 80, "f16"),
    (1, 2, 1, 64, "bf16"), (2, 2, 33, 40, "bf16"), (1, 2, 1000, 64, "bf16"), (1, 3, 4099, 40, "bf16"),
    (1, 2, 300, 24, "bf16"), (1, 1, 200, 48, "bf16"), (1, 2, 600, 80, "bf16"), (2, 8, 4096, 40, "f16"),
    (1, 2, 515, 8, "bf16"), (1, 2, 130, 16, "bf16"), (1, 2, 300, 32, "bf16"), (2, 8, 4096, 40, "bf16"),
    (1, 1, 2100, 48, "bf16"), (1, 2, 300, 56, "bf16"),
]


@pytest.mark.parametrize("B,H,N,d,dtype", SHAPES)
def test_backward_matches_oracle(B, H, N, d, dtype):
    print(f"bwd B={B} H={H} N={N} d={d} {dtype}", flush=True)
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=80, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 80777, dtype, "cpu")
    outs = _run(q, k, v, g)
    worst = _check(outs, q, k, v, g, dtype, 0, 1e-6, True, f"bwd N={N} d={d} {dtype}")
    print(f"  worst max-norm ratio {worst:.2e}", flush=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,H,N,d", [(1, 2, 1000, 40), (2, 2, 333, 16), (1, 1, 4099, 48), (1, 2, 700, 64), (1, 1, 300, 80)])
def test_backward_separate_kernels(B, H, N, d, dtype, monkeypatch, tuning):
    """Contiguous heads normally take the merged dQ + state-gradient kernel; the separate kernels (kept for the
    token-major layouts without a row-piece form of the merged one) must give the same gradients to tolerance."""
    monkeypatch.setenv("LINFUSION_BWD_MERGED", "2")
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=84, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 84777, dtype, "cpu")
    outs = _run(q, k, v, g)
    _check(outs, q, k, v, g, dtype, 0, 1e-6, True, f"bwd separate kernels N={N} d={d} {dtype}")


@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 2, 1000, 40, "f16"), (2, 3, 4099, 40, "f16"), (1, 2, 33, 64, "f16"),
                                            (1, 1, 2100, 80, "f16"), (1, 2, 777, 8, "f16"), (1, 2, 1000, 40, "bf16"),
                                            (1, 2, 515, 64, "bf16"), (1, 1, 1, 48, "f16"), (1, 2, 5000, 56, "bf16")])
def test_backward_kv_from_packed_operands(B, H, N, d, dtype, monkeypatch, tuning):
    """Large fp16 problems compute dK, dV with many short-lived workgroups from operands packed once per head; forced
    here at small sizes: the oracle's gradients, and bit for bit what the long-lived workgroups give."""
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=85, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 85777, dtype, "cpu")
    monkeypatch.setenv("LINFUSION_BWD_KV_PACKED", "2")
    plain = _run(q, k, v, g)
    monkeypatch.setenv("LINFUSION_BWD_KV_PACKED", "3")
    monkeypatch.setenv("LINFUSION_BWD_KVP_BLK", "8")
    outs = _run(q, k, v, g)
    _check(outs, q, k, v, g, dtype, 0, 1e-6, True, f"bwd packed kv N={N} d={d} {dtype}")
    for got, want in zip(outs, plain):
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("fm,normalize", [(1, True), (2, True), (0, False), (1, False)])
def test_backward_other_feature_maps_and_unnormalized(dtype, fm, normalize):
    B, H, N, d = 1, 2, 500, 40
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=81, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 81777, dtype, "cpu")
    if fm == 2:
        q, k = q.abs(), k.abs()
    if not normalize:
        v, g = v * 0.05, g * 0.05      # keeps the un-normalized sums inside fp16's range
    outs = _run(q, k, v, g, fm, 1e-6, 0 if normalize else lf.FLAG_UNNORMALIZED)
    _check(outs, q, k, v, g, dtype, fm, 1e-6, normalize, f"bwd fm={fm} norm={normalize} {dtype}")


def test_backward_is_run_to_run_identical_and_leaves_inputs_alone():
    B, H, N, d, dtype = 1, 3, 2100, 40, "f16"
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=82, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 82777, dtype, "cpu")
    qd, kd, vd, gd = q.cuda(), k.cuda(), v.cuda(), g.cuda()
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    a = [torch.empty_like(qd) for _ in range(3)]
    b = [torch.empty_like(qd) for _ in range(3)]
    lf.linfusion_attn_bwd(qd, kd, vd, gd, *a, 0, 1e-6, 0, ws)
    lf.linfusion_attn_bwd(qd, kd, vd, gd, *b, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))
    for dev, host in ((qd, q), (kd, k), (vd, v), (gd, g)):
        assert torch.equal(dev.cpu().view(torch.uint8), host.view(torch.uint8))


@pytest.mark.parametrize("path", [lf.FLAG_FORCE_SPLIT, lf.FLAG_FORCE_FUSED])
def test_backward_with_the_state_a_forward_call_left_in_its_workspace(path):
    B, H, N, d, dtype = 2, 3, 1500, 40, "f16"
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=83, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 83777, dtype, "cpu")
    qd, kd, vd, gd = q.cuda(), k.cuda(), v.cuda(), g.cuda()
    fws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(qd)
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, 1e-6, path, fws)
    off = lf.linfusion_attn_workspace_state_offset(B, H, N, d, 1)
    state = fws[off:off + B * H * (d * d + d) * 4].view(torch.float32)
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    a = [torch.full_like(qd, float("nan")) for _ in range(3)]
    b = [torch.full_like(qd, float("nan")) for _ in range(3)]
    lf.linfusion_attn_bwd(qd, kd, vd, gd, *a, 0, 1e-6, 0, ws, state=state)
    lf.linfusion_attn_bwd(qd, kd, vd, gd, *b, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    _check(a, q, k, v, g, dtype, 0, 1e-6, True, "bwd with saved state")
    if path == lf.FLAG_FORCE_SPLIT:       # same kernels produced the state: the gradients are identical
        for x, y in zip(a, b):
            assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))


def test_backward_argument_checks():
    x = torch.zeros(1, 1, 64, 40, dtype=torch.float16, device="cuda")
    outs = [torch.empty_like(x) for _ in range(3)]
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(1, 1, 64, 40, 1), dtype=torch.uint8, device="cuda")
    assert lf.linfusion_attn_bwd(x, x, x, x, x, outs[1], outs[2], 0, 1e-6, 0, ws, check=False) == -7   # dq aliases q
    assert lf.linfusion_attn_bwd(x, x, x, x, outs[0], outs[0], outs[2], 0, 1e-6, 0, ws, check=False) == -7
    assert lf.linfusion_attn_bwd(x, x, x, x, *outs, 0, 1e-6, lf.FLAG_FORCE_FUSED, ws, check=False) == -1
    assert lf.linfusion_attn_bwd(x, x, x, x, *outs, 0, 1e-6, 0, ws[:64], check=False) == -4
    f = torch.zeros(1, 1, 64, 80, dtype=torch.float32, device="cuda")      # fp32 stops at d = 64, as its forward does
    fo = [torch.empty_like(f) for _ in range(3)]
    assert lf.linfusion_attn_bwd(f, f, f, f, *fo, 0, 1e-6, 0, ws, check=False) == -2
    assert lf.linfusion_attn_bwd_workspace_bytes(1, 1, 64, 80, 0) == 0
    b = torch.zeros(1, 1, 64, 160, dtype=torch.bfloat16, device="cuda")    # bf16 stops at d = 80
    bo = [torch.empty_like(b) for _ in range(3)]
    assert lf.linfusion_attn_bwd(b, b, b, b, *bo, 0, 1e-6, 0, ws, check=False) == -2


@pytest.mark.parametrize("B,H,N,d,dtype", [(2, 3, 33, 40, "f16"), (1, 8, 1000, 40, "f16"), (2, 5, 700, 64, "bf16"),
                                            (1, 4, 515, 80, "f16"), (1, 2, 300, 24, "bf16"), (1, 10, 2049, 64, "f16"),
                                            # groups of eight / four heads on the row-piece dK, dV kernel
                                            (2, 8, 2051, 40, "bf16"), (3, 4, 100, 40, "f16"), (1, 16, 257, 24, "f16"),
                                            (1, 12, 130, 56, "bf16"), (1, 8, 1, 40, "f16"), (2, 8, 33, 80, "bf16"),
                                            (1, 8, 300, 8, "f16"), (1, 4, 700, 16, "bf16"), (1, 8, 515, 48, "f16"),
                                            (1, 8, 96, 32, "bf16")])
def test_backward_on_token_major_views(B, H, N, d, dtype, monkeypatch, tuning):
    """All seven tensors in the UNet's [B, N, H*d] layout, handed over as strided [B, H, N, d] views: the oracle's
    gradients, and what the contiguous entry point gives on the same values.  The row-piece gradient kernels, which
    the library picks from a few tens of MB up, are switched on for every size here."""
    print(f"bwd token-major B={B} H={H} N={N} d={d} {dtype}", flush=True)
    monkeypatch.setenv("LINFUSION_BWD_ROWS", "3")
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=70, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 70707, dtype, "cpu")
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)   # [B, N, H, d] in memory
    views = [tm(t) for t in (q, k, v, g)]
    outs = [torch.full((B, N, H, d), float("nan"), dtype=q.dtype, device="cuda").permute(0, 2, 1, 3) for _ in range(3)]
    code = wl.DTYPE_CODE[dtype]
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_bwd_strided(*views, *outs, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    dense = _run(q, k, v, g)
    # the row-piece kernels sum the state and the state gradient over the tiles in another order than the per-head
    # kernels: the gradients agree with the contiguous call's up to that fp32 rounding
    # (two units in the last place of the 16-bit results at most; the oracle check below is the measure of accuracy)
    ulp2 = 2.0 ** -7 if dtype == "bf16" else 2.0 ** -10
    for got, want in zip(outs, dense):
        diff = (got.contiguous().float() - want.float()).abs().max().item()
        assert diff <= ulp2 * want.float().abs().max().item(), f"token-major vs contiguous: {diff}"
    _check([o.contiguous() for o in outs], q, k, v, g, dtype, 0, 1e-6, True, "token-major")
    # and with the per-head kernels only: every gradient bit for bit as the contiguous call
    monkeypatch.setenv("LINFUSION_BWD_ROWS", "2")
    outs2 = [torch.full((B, N, H, d), float("nan"), dtype=q.dtype, device="cuda").permute(0, 2, 1, 3) for _ in range(3)]
    lf.linfusion_attn_bwd_strided(*views, *outs2, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    for got, want in zip(outs2, dense):
        assert torch.equal(got.contiguous().view(torch.int16), want.view(torch.int16))


def test_backward_on_padded_and_mixed_layouts():
    """q and dout padded to a longer row, k and v token-major, gradients written into padded rows whose padding
    must stay untouched."""
    B, H, N, d, dtype, pad = 1, 3, 450, 40, "f16", 24
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=71, device="cpu")
    g = wl.draw((B, H, N, d), wl.BASE_SEED + 71717, dtype, "cpu")

    def padded(t, fill=float("nan")):
        big = torch.full((B, H, N, d + pad), fill, dtype=t.dtype)
        big[..., :d] = t
        return big.cuda()
    qb, gb = padded(q), padded(g)
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)
    bigs = [torch.full((B, H, N, d + pad), 7.0, dtype=q.dtype, device="cuda") for _ in range(3)]
    outs = [b[..., :d] for b in bigs]
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_bwd_strided(qb[..., :d], tm(k), tm(v), gb[..., :d], *outs, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    for b in bigs:
        assert bool((b[..., d:] == 7.0).all()), "padding of a gradient row was written"
    dense = _run(q, k, v, g)
    for got, want in zip(outs, dense):
        assert torch.equal(got.contiguous().view(torch.int16), want.view(torch.int16))


def test_backward_strided_argument_checks():
    B, H, N, d = 1, 2, 64, 40
    q, k, v = (t.cuda() for t in wl.make_qkv(B, H, N, d, "f16", idx=72, device="cpu"))
    g = torch.randn_like(q)
    outs = [torch.empty_like(q) for _ in range(3)]
    ws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    call = lambda *a: lf.linfusion_attn_bwd_strided(*a, 0, 1e-6, 0, ws, check=False)
    fused = torch.empty(B, N, 3, H, d, dtype=q.dtype, device="cuda")           # three gradients interleaved
    inter = [fused[:, :, i].permute(0, 2, 1, 3) for i in range(3)]
    assert call(q, k, v, g, *inter) == -7                                      # spans overlap: not accepted
    bcast = torch.empty(B, 1, N, d, dtype=q.dtype, device="cuda").expand(B, H, N, d)
    assert call(q, k, v, g, bcast, outs[1], outs[2]) == -7                     # a written view with stride 0
    odd = torch.empty(B, H, N, d + 4, dtype=q.dtype, device="cuda")[..., :d]   # rows not 16-byte aligned
    assert call(odd, k, v, g, *outs) == -3
