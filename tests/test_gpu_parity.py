"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2409_02097_amd as lf
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def _run(q, k, v, feature_map=0, eps=1e-6, flags=0):
    B, H, N, d = q.shape
    out = torch.full_like(q, float("nan"))
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[_dt(q)]), dtype=torch.uint8, device=q.device)
    lf.linfusion_attn_fwd_ex(q, k, v, out, feature_map, eps, flags, ws)
    torch.cuda.synchronize()
    return out


def _dt(t):
    return {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}[t.dtype]


SMALL = [
    # (B, H, N, d, dtype): several tiles, ragged tails, single token, every head width family
    (1, 2, 1, 40, "f16"), (1, 1, 31, 64, "f16"), (2, 3, 33, 40, "f16"), (1, 2, 257, 64, "f16"),
    (1, 2, 1000, 40, "f16"), (2, 2, 4099, 64, "f16"), (1, 3, 777, 8, "f16"), (1, 1, 130, 16, "f16"),
    (1, 2, 515, 24, "f16"), (1, 2, 300, 32, "f16"), (1, 2, 300, 48, "f16"), (1, 1, 300, 56, "f16"),
    (1, 2, 1, 64, "bf16"), (2, 2, 33, 40, "bf16"), (1, 2, 1000, 64, "bf16"), (1, 3, 4099, 40, "bf16"),
    (1, 2, 300, 24, "bf16"), (1, 1, 200, 48, "bf16"), (1, 2, 1029, 80, "bf16"), (1, 2, 1, 80, "bf16"),
    (2, 3, 1500, 80, "f16"), (1, 1, 33, 80, "f16"),
    (1, 2, 1, 40, "f32"), (1, 2, 17, 64, "f32"), (2, 2, 1000, 40, "f32"), (1, 3, 2051, 64, "f32"),
    (1, 2, 100, 8, "f32"), (1, 2, 100, 24, "f32"), (1, 1, 100, 56, "f32"), (1, 1, 333, 32, "f32"),
]


PATHS = {"split": lf.FLAG_FORCE_SPLIT, "fused": lf.FLAG_FORCE_FUSED, "solo": lf.FLAG_FORCE_SOLO}
PATH_CODE = {"split": 0, "fused": 1, "solo": 2}


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("B,H,N,d,dtype", SMALL)
def test_small_shapes_match_oracle(B, H, N, d, dtype, path):
    print(f"case B={B} H={H} N={N} d={d} {dtype} {path}", flush=True)
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=50, device="cpu")
    if path == "solo" and d > 64:
        with pytest.raises(lf.LinFusionError):       # the replicated-state launch covers head widths up to 64
            lf.linfusion_attn_plan(B, H, N, d, wl.DTYPE_CODE[dtype], PATHS[path])
        return
    assert lf.linfusion_attn_plan(B, H, N, d, wl.DTYPE_CODE[dtype], PATHS[path])["path"] == PATH_CODE[path]
    out = _run(q.cuda(), k.cuda(), v.cuda(), flags=PATHS[path])
    worst = parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"N={N} d={d} {dtype}")
    print(f"  worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)


@pytest.mark.parametrize("waves", [4, 2, 1])
@pytest.mark.parametrize("B,H,N,d,dtype", [c for c in SMALL if c[4] != "f32"])
def test_packed_operand_apply_on_small_shapes(B, H, N, d, dtype, waves, monkeypatch, tuning):
    """The apply kernel of the large workloads (operands packed once per head, many short-lived workgroups),
    forced onto small shapes: the oracle's values, and the bits of the kernel that packs per workgroup."""
    print(f"packed apply B={B} H={H} N={N} d={d} {dtype} waves={waves}", flush=True)
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=51, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    monkeypatch.setenv("LINFUSION_APPLY_PACKED", "2")
    ref = _run(qd, kd, vd, flags=lf.FLAG_FORCE_SPLIT)
    monkeypatch.setenv("LINFUSION_APPLY_PACKED", "3")
    monkeypatch.setenv("LINFUSION_APPLY_WAVES", str(waves))
    monkeypatch.setenv("LINFUSION_APPLY_WGS", str(7 * B * H))      # several workgroups per head, tiles dealt cyclically
    out = _run(qd, kd, vd, flags=lf.FLAG_FORCE_SPLIT)
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"packed apply N={N} d={d} {dtype}")
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    if N >= 1000:      # feature maps and the un-normalized arm on the same kernel
        for fm, flags in ((1, 0), (2, 0), (0, lf.FLAG_UNNORMALIZED)):
            qq, kk = (qd.abs(), kd.abs()) if fm == 2 else (qd, kd)
            out = _run(qq, kk, vd, fm, 1e-6, flags | lf.FLAG_FORCE_SPLIT)
            parity.check_all(out, qq.cpu(), kk.cpu(), v, dtype, fm, 1e-6, not flags, f"packed apply fm={fm} flags={flags}")


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("name", ["sd15_256_f32", "sd15_512_f16", "sd21_768_f16", "sd21_768_f16_peaky",
                                  "sdxl_2048_A_bf16", "sdxl_2048_B_bf16"])
def test_paper_shaped_configs_match_oracle(name, path):
    print(f"config {name} {path}", flush=True)
    c = wl.CONFIGS[name]
    q, k, v = wl.make_config(name, device="cpu")
    out = _run(q.cuda(), k.cuda(), v.cuda(), 0, wl.EPS, PATHS[path])
    worst = parity.check_all(out, q, k, v, c["dtype"], 0, wl.EPS, True, name)
    print(f"  worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("fm", [1, 2])
def test_other_feature_maps(dtype, fm):
    q, k, v = wl.make_qkv(1, 2, 555, 40, dtype, idx=60, device="cpu")
    if fm == 2:   # identity phi needs non-negative q, k for a positive normalizer
        q, k = q.abs(), k.abs()
    out = _run(q.cuda(), k.cuda(), v.cuda(), fm, 1e-6)
    parity.check_all(out, q, k, v, dtype, fm, 1e-6, True, f"fm={fm} {dtype}")


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_unnormalized_variant(dtype):
    q, k, v = wl.make_qkv(1, 2, 700, 64, dtype, idx=61, device="cpu")
    out = _run(q.cuda(), k.cuda(), v.cuda(), 0, 1e-6, lf.FLAG_UNNORMALIZED)
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, False, f"unnormalized {dtype}")


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_constant_v_and_large_mean(dtype):
    # Prop. 1: a constant channel stays constant; a large mean stresses the 16-bit state scaling
    q, k, _ = wl.make_qkv(1, 2, 3000, 40, dtype, idx=62, device="cpu")
    v = torch.full((1, 2, 3000, 40), 3.0).to(q.dtype)
    v[..., 1] = -100.0
    v[..., 2] = 0.001
    out = _run(q.cuda(), k.cuda(), v.cuda(), 0, 1e-6)
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"constant V {dtype}")


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_run_to_run_bit_identical(dtype, path):
    q, k, v = wl.make_qkv(2, 3, 5000, 64, dtype, idx=63, device="cuda")
    a = _run(q, k, v, flags=PATHS[path])
    for _ in range(3):
        b = _run(q, k, v, flags=PATHS[path])
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_fused_calls_back_to_back_share_a_workspace():
    # the barrier words are never reset: consecutive calls on one workspace must not see stale arrivals
    q, k, v = wl.make_qkv(2, 4, 3000, 40, "f16", idx=67, device="cuda")
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(2, 4, 3000, 40, 1), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)            # whatever the caller left there
    ref = _run(q, k, v, flags=lf.FLAG_FORCE_SPLIT)
    outs = [torch.empty_like(q) for _ in range(20)]
    for o in outs:
        lf.linfusion_attn_fwd_ex(q, k, v, o, 0, 1e-6, lf.FLAG_FORCE_FUSED, ws)
    torch.cuda.synchronize()
    for o in outs:
        assert torch.equal(o.view(torch.uint8), outs[0].view(torch.uint8))
    parity.check_all(outs[0], q.cpu(), k.cpu(), v.cpu(), "f16", 0, 1e-6, True, "fused back-to-back")
    assert (outs[0].float() - ref.float()).abs().max().item() < 1e-2


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_in_place_on_q(dtype):
    q, k, v = wl.make_qkv(1, 2, 1234, 40, dtype, idx=64, device="cuda")
    ref = _run(q, k, v)
    q2 = q.clone()
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(1, 2, 1234, 40, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_fwd_ex(q2, k, v, q2, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    assert torch.equal(ref.view(torch.uint8), q2.view(torch.uint8))


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_state_entry_matches_oracle(dtype):
    from oracle import linattn_oracle as orc
    B, H, N, d = 1, 3, 2500, 40
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=65, device="cpu")
    st = torch.empty(B * H * (d * d + d), dtype=torch.float32, device="cuda")
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_state(k.cuda(), v.cuda(), st, 0, ws)
    torch.cuda.synchronize()
    got = st.cpu().numpy().astype(np.float64).reshape(B * H, d * d + d)
    ks, vs = wl.stored_numpy(k), wl.stored_numpy(v)
    tol = parity.TOL[dtype]
    for h in range(H):
        S, z = orc.state(orc.widen(ks[0, h], dtype), orc.widen(vs[0, h], dtype))
        gS, gz = got[h, :d * d].reshape(d, d), got[h, d * d:]
        assert np.abs(gS - S).max() <= tol * np.abs(S).max()
        assert np.abs(gz - z).max() <= tol * np.abs(z).max()


def test_owned_workspace_entry_points():
    for dtype, fn in (("f16", lf.linfusion_attn_fwd), ("f16", lf.linfusion_attn_fwd_f16),
                      ("bf16", lf.linfusion_attn_fwd_bf16), ("f32", lf.linfusion_attn_fwd_f32)):
        q, k, v = wl.make_qkv(1, 2, 900, 40, dtype, idx=66, device="cuda")
        out = torch.empty_like(q)
        fn(q, k, v, out, 0, 1e-6)
        torch.cuda.synchronize()
        # (these entry points always take the three-kernel path)
        assert torch.equal(out.view(torch.uint8), _run(q, k, v, flags=lf.FLAG_FORCE_SPLIT).view(torch.uint8))
    lf.linfusion_release()


def test_single_launch_timeout_is_reported_and_harmless(monkeypatch, tuning):
    # a spin limit of zero makes every workgroup that does not see all arrivals at its first poll give
    # up: the kernel must still end (no hang), the error must be reported, and the next call must work
    B, H, N, d = 2, 4, 20000, 40
    q, k, v = wl.make_qkv(B, H, N, d, "f16", idx=68, device="cuda")
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, 1), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)
    assert lf.linfusion_attn_plan(B, H, N, d, 1, lf.FLAG_FORCE_FUSED)["reduce_wgs_per_head"] > 8
    monkeypatch.setenv("LINFUSION_FUSED_SPIN_LIMIT", "0")
    lf.linfusion_attn_fwd_ex(q, k, v, out, 0, 1e-6, lf.FLAG_FORCE_FUSED, ws)
    rc = lf.linfusion_attn_last_error(ws, B, H, N, d, 1)
    assert rc in (0, -8)          # -8 unless every workgroup happened to arrive before the first poll
    print("forced give-up ->", rc, flush=True)
    monkeypatch.delenv("LINFUSION_FUSED_SPIN_LIMIT")
    # the report belongs to the workspace: single-launch calls on another workspace (and another shape) in
    # between do not hide it
    ws2 = torch.empty_like(ws)
    out2 = torch.empty_like(q)
    lf.linfusion_attn_fwd_ex(q, k, v, out2, 0, 1e-6, lf.FLAG_FORCE_FUSED, ws2)
    assert lf.linfusion_attn_last_error(ws2, B, H, N, d, 1) == 0
    assert lf.linfusion_attn_last_error(ws, B, H, N, d, 1) == rc
    lf.linfusion_attn_fwd_ex(q, k, v, out, 0, 1e-6, lf.FLAG_FORCE_FUSED, ws)
    assert lf.linfusion_attn_last_error(ws, B, H, N, d, 1) == 0
    parity.check_all(out, q.cpu(), k.cpu(), v.cpu(), "f16", 0, 1e-6, True, "after a forced give-up")
    assert torch.equal(out.view(torch.uint8), out2.view(torch.uint8))
    # the split path never reports a timeout
    lf.linfusion_attn_fwd_ex(q, k, v, out, 0, 1e-6, lf.FLAG_FORCE_SPLIT, ws)
    assert lf.linfusion_attn_last_error(ws, B, H, N, d, 1) == 0


@pytest.mark.parametrize("dtype,d", [("f16", 40), ("bf16", 64), ("f32", 40)])
def test_single_launch_on_a_workspace_with_arbitrary_content(dtype, d):
    # The workspace's content is undefined: whatever it holds (zeros, ones, small integers, bytes an earlier
    # tensor left behind), the barrier flags must read as "not arrived" and no timeout may be reported.
    B, H, N = 2, 4, 6000
    code = wl.DTYPE_CODE[dtype]
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=69, device="cuda")
    nbytes = lf.linfusion_attn_workspace_bytes(B, H, N, d, code)
    assert lf.linfusion_attn_plan(B, H, N, d, code, lf.FLAG_FORCE_FUSED)["path"] == 1
    ref = None
    gen = torch.Generator(device="cuda").manual_seed(7)
    fills = [lambda w: w.zero_(), lambda w: w.fill_(1), lambda w: w.fill_(255),
             lambda w: w.view(torch.int32).copy_(torch.arange(w.numel() // 4, device="cuda", dtype=torch.int32) % 7),
             lambda w: w.view(torch.int32).fill_(1),
             lambda w: w.copy_(torch.randint(0, 256, (w.numel(),), device="cuda", dtype=torch.uint8, generator=gen))]
    for i, fill in enumerate(fills):
        ws = torch.empty((nbytes + 3) // 4 * 4, dtype=torch.uint8, device="cuda")
        fill(ws)
        assert lf.linfusion_attn_last_error(ws, B, H, N, d, code) == 0, f"fill {i}: a report before any call"
        out = torch.full_like(q, float("nan"))
        lf.linfusion_attn_fwd_ex(q, k, v, out, 0, 1e-6, lf.FLAG_FORCE_FUSED, ws)
        assert lf.linfusion_attn_last_error(ws, B, H, N, d, code) == 0, f"fill {i}"
        if ref is None:
            ref = out
            parity.check_all(out, q.cpu(), k.cpu(), v.cpu(), dtype, 0, 1e-6, True, "single launch, zeroed workspace")
        else:
            assert torch.equal(out.view(torch.uint8), ref.view(torch.uint8)), f"fill {i}"


def test_single_launch_falls_back_when_heads_exceed_residency():
    # more (batch, head) slices than resident workgroups: the single-launch path is not available
    B, H, N, d = 8, 160, 64, 64
    assert lf.linfusion_attn_plan(B, H, N, d, 1, lf.FLAG_FORCE_FUSED)["path"] == 0
    q, k, v = wl.make_qkv(B, H, N, d, "f16", idx=69, device="cpu")
    out = _run(q.cuda(), k.cuda(), v.cuda(), flags=lf.FLAG_FORCE_FUSED)
    parity.check_all(out, q, k, v, "f16", 0, 1e-6, True, "fallback")


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("case", ["zeros", "large_positive", "large_negative", "tiny"])
def test_extreme_values_match_oracle(dtype, case, path):
    """Inputs at the edges of the feature map: phi(0) = 1 everywhere; q, k = 30 (state entries ~ N * 31 * |v|,
    beyond fp16 without the power-of-two rescaling); q, k = -20 (phi ~ 2e-9 is below fp16's range, and eps
    takes over the denominator); q, k, v ~ 1e-3."""
    B, H, N, d = 1, 2, 777, 40
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=66, device="cpu")
    if case == "zeros":
        q, k, v = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    elif case == "large_positive":
        q, k = q * 0.5 + 30.0, k * 0.5 + 30.0
    elif case == "large_negative":
        q, k = q * 0.5 - 20.0, k * 0.5 - 20.0
    else:
        q, k, v = q * 1e-3, k * 1e-3, v * 1e-3
    out = _run(q.cuda(), k.cuda(), v.cuda(), flags=PATHS[path])
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"{case} {dtype}")


@pytest.mark.parametrize("path", ["split", "fused", "packed", "solo"])
@pytest.mark.parametrize("d", [40, 64])
@pytest.mark.parametrize("case", ["q-20", "q-12", "k-12", "k-20", "q-20_k-20", "some_rows_q-25", "some_tokens_k-25",
                                  "q-60000"])
def test_fp16_inputs_far_below_zero(case, d, path, monkeypatch, tuning):
    """exp(x) of fp16 inputs far below zero leaves the normal range of an fp16 operand (subnormal below -10, zero
    below -17), but the definition gives a proper weighted mean as long as the denominator stays above eps: query
    rows are evaluated relative to their largest channel, key streams relative to their largest key.  Shifts are
    applied to q or k alone (shifting both only makes eps dominate on both sides, which hides the case)."""
    B, H, N = 1, 2, 777
    q, k, v = wl.make_qkv(B, H, N, d, "f32", idx=70, device="cpu")
    if case == "q-20" or case == "q-20_k-20":
        q = q - 20.0
    if case == "q-12":
        q = q - 12.0
    if case == "q-60000":
        q = q * 100.0 - 60000.0
    if case == "k-12":
        k = k - 12.0
    if case == "k-20" or case == "q-20_k-20":
        k = k - 20.0
    if case == "some_rows_q-25":
        q[:, :, ::3] -= 25.0
    if case == "some_tokens_k-25":
        k[:, :, ::2] -= 25.0
    q, k, v = q.half(), k.half(), v.half()
    flags = {"split": lf.FLAG_FORCE_SPLIT, "fused": lf.FLAG_FORCE_FUSED, "packed": lf.FLAG_FORCE_SPLIT,
             "solo": lf.FLAG_FORCE_SOLO}[path]
    monkeypatch.setenv("LINFUSION_APPLY_PACKED", "3" if path == "packed" else "2")
    # (exp(-60000) is zero in every arithmetic: the definition gives 0 / eps = 0 there, and nothing without eps)
    for eps in ((1e-6,) if case == "q-60000" else (1e-6, 0.0)):
        out = _run(q.cuda(), k.cuda(), v.cuda(), 0, eps, flags)
        worst = parity.check_all(out, q, k, v, "f16", 0, eps, True, f"{case} d={d} {path} eps={eps}")
        print(f"{case} d={d} {path} eps={eps}: worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)
    if case in ("q-12", "some_rows_q-25"):      # the un-normalized arm takes the row's factor out again
        out = _run(q.cuda(), k.cuda(), v.cuda(), 0, 1e-6, flags | lf.FLAG_UNNORMALIZED)
        parity.check_all(out, q, k, v, "f16", 0, 1e-6, False, f"{case} d={d} {path} unnormalized")


@pytest.mark.parametrize("B,H,N,d,dtype", [(2, 150, 70, 40, "f16"), (1, 3, 20000, 40, "f16"), (1, 2, 9000, 64, "bf16"),
                                           (1, 2, 5000, 56, "f32"), (3, 100, 33, 16, "f32"), (1, 1, 3000, 48, "bf16")])
def test_replicated_state_launch_on_other_shapes(B, H, N, d, dtype):
    """More heads than compute units (one workgroup per head, several rounds), many tiles per workgroup, the other
    feature maps and the un-normalized arm; the single launch needs no workspace content and repeats itself."""
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=72, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    assert lf.linfusion_attn_plan(B, H, N, d, wl.DTYPE_CODE[dtype], lf.FLAG_FORCE_SOLO)["path"] == 2
    out = _run(qd, kd, vd, flags=lf.FLAG_FORCE_SOLO)
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"solo B={B} H={H} N={N} d={d} {dtype}")
    again = _run(qd, kd, vd, flags=lf.FLAG_FORCE_SOLO)
    assert torch.equal(out.view(torch.uint8), again.view(torch.uint8))
    if H <= 3:
        for fm, flags in ((1, 0), (2, 0), (0, lf.FLAG_UNNORMALIZED)):
            qq, kk = (qd.abs(), kd.abs()) if fm == 2 else (qd, kd)
            out = _run(qq, kk, vd, fm, 1e-6, flags | lf.FLAG_FORCE_SOLO)
            parity.check_all(out, qq.cpu(), kk.cpu(), v, dtype, fm, 1e-6, not flags, f"solo fm={fm} flags={flags} {dtype}")


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_a_nan_stays_inside_its_head(dtype):
    B, H, N, d = 1, 3, 500, 40
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=67, device="cpu")
    k[0, 1, 123, 7] = float("nan")
    out = _run(q.cuda(), k.cuda(), v.cuda())
    assert bool(torch.isnan(out[0, 1]).all()), "the poisoned head must not produce numbers"
    clean = torch.isfinite(out[0, 0]).all() and torch.isfinite(out[0, 2]).all()
    assert bool(clean), "other heads must be unaffected"
    k[0, 1, 123, 7] = 0.0
    for h in (0, 2):
        ref = __import__("oracle.linattn_oracle", fromlist=["x"]).attention_linear_stored(
            wl.stored_numpy(q)[0, h], wl.stored_numpy(k)[0, h], wl.stored_numpy(v)[0, h], dtype, 0, 1e-6, True)
        parity.check_slice(parity.to_f64(out[0, h]), ref, dtype, f"head {h} next to a NaN head")


def test_forward_recorded_into_a_graph_replays_correctly():
    """A mid-sized problem (the single launch would be chosen eagerly) captured once and replayed with new
    inputs in the same buffers, with eager calls and synchronisations in between: every replay must give
    what an eager call on the same inputs gives."""
    B, H, N, d, dtype = 2, 10, 16384, 64, "bf16"          # 168 MB of tensor traffic, d = 64: inside the single-launch window
    code = wl.DTYPE_CODE[dtype]
    assert lf.linfusion_attn_plan(B, H, N, d, code)["path"] == 1
    q, k, v = (t.cuda() for t in wl.make_qkv(B, H, N, d, dtype, idx=68, device="cpu"))
    out = torch.zeros_like(q)
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                          # warm-up outside the capture
        lf.linfusion_attn_fwd_ex(q, k, v, out, 0, 1e-6, 0, ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lf.linfusion_attn_fwd_ex(q, k, v, out, 0, 1e-6, 0, ws, stream=torch.cuda.current_stream())
    for rep in range(3):
        nq, nk, nv = (t.cuda() for t in wl.make_qkv(B, H, N, d, dtype, idx=68, device="cpu", seed_offset=rep + 1))
        q.copy_(nq); k.copy_(nk); v.copy_(nv)
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = torch.empty_like(nq)
        ews = torch.empty_like(ws)
        lf.linfusion_attn_fwd_ex(nq, nk, nv, eager, 0, 1e-6, lf.FLAG_FORCE_SPLIT, ews)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.uint8), eager.view(torch.uint8)), f"replay {rep} differs from the eager call"
    worst = parity.check_all(out[:, :2], q[:, :2].cpu(), k[:, :2].cpu(), v[:, :2].cpu(), dtype, 0, 1e-6, True, "graph replay")


@pytest.mark.parametrize("mode", [3, 2])
@pytest.mark.parametrize("B,H,N,d", [(1, 2, 1, 40), (1, 2, 17, 64), (2, 2, 1000, 40), (1, 3, 2051, 64), (1, 2, 100, 8),
                                     (1, 2, 515, 24), (1, 1, 300, 56), (1, 1, 333, 32), (1, 2, 300, 16), (1, 1, 200, 48),
                                     (1, 2, 9001, 40)])
def test_fp32_state_reduction_on_either_matrix_instruction(B, H, N, d, mode, monkeypatch, tuning):
    """fp32 runs its state reduction through three bf16 terms per value on the 16-bit matrix cores (narrow heads at
    large N) or on the fp32 instruction (the rest); both kernels on every width and on ragged sizes, each against the
    oracle at the fp32 tolerance, split path forced so that the choice is the reduction's alone."""
    print(f"fp32 reduction mode {mode} B={B} H={H} N={N} d={d}", flush=True)
    monkeypatch.setenv("LINFUSION_F32_SPLIT", str(mode))
    q, k, v = wl.make_qkv(B, H, N, d, "f32", idx=45, device="cpu")
    out = _run(q.cuda(), k.cuda(), v.cuda(), flags=lf.FLAG_FORCE_SPLIT)
    worst = parity.check_all(out, q, k, v, "f32", 0, 1e-6, True, f"fp32 reduction mode {mode} N={N} d={d}")
    print(f"  worst max-norm ratio {worst[0]:.2e}", flush=True)


def test_fp32_split_reduction_is_the_default_for_narrow_heads_at_large_n():
    """Default choice (no environment): N = 20,011 tokens of width 40 take the 16-bit route; token-major views too."""
    B, H, N, d = 1, 4, 20011, 40
    q, k, v = wl.make_qkv(B, H, N, d, "f32", idx=46, device="cpu")
    out = _run(q.cuda(), k.cuda(), v.cuda())
    parity.check_all(out, q, k, v, "f32", 0, 1e-6, True, "fp32 default at large N")
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)
    o = tm(torch.full_like(q, float("nan")))
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, lf.DTYPE_F32), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_fwd_strided(tm(q), tm(k), tm(v), o, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    assert torch.equal(o.contiguous().view(torch.int32), out.view(torch.int32)), "token-major differs from contiguous"


@pytest.mark.parametrize("B,H,N,d,dtype,per_cu", [(1, 4, 3200003, 8, "f16", 8), (1, 2, 3300001, 8, "f32", 4)])
def test_narrow_heads_at_large_n_with_more_reduction_workgroups(B, H, N, d, dtype, per_cu):
    """From 768 MB of tensor traffic on the narrowest heads (and bf16 up to 40 channels, which the full-size bf16 test
    covers) are reduced by eight workgroups per CU instead of two (four in fp32): every row of every head of such
    shapes, with a ragged last tile, against the oracle."""
    print(f"narrow heads at large N: B={B} H={H} N={N} d={d} {dtype}", flush=True)
    plan = lf.linfusion_attn_plan(B, H, N, d, wl.DTYPE_CODE[dtype])
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert (per_cu - 1) * cus < plan["reduce_wgs_per_head"] * B * H <= per_cu * cus, plan
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=94, device="cpu")
    out = _run(q.cuda(), k.cuda(), v.cuda())
    worst = parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"narrow heads at large N d={d} {dtype}")
    print(f"  worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)
