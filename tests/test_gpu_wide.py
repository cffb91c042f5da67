"""GPU parity for head widths above 64 (the d = 80 and d = 160 levels of the SD-v1.5 UNet): the wide
kernels against the fp64 oracle, element by element."""
import pytest
import torch

import paper_2409_02097_amd as lf
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def _ws(B, H, N, d, dtype, dev="cuda"):
    return torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device=dev)


SHAPES = [
    # (B, H, N, d, dtype): SD-v1.5 at 512 px has (2, 8, 1024, 80) and (2, 8, 256 / 64, 160)
    (2, 8, 1024, 80, "f16"), (2, 8, 256, 160, "f16"), (2, 8, 64, 160, "f16"),
    (1, 2, 1, 80, "f16"), (1, 3, 33, 160, "f16"), (1, 2, 31, 80, "f16"), (1, 1, 4099, 160, "f16"),
    (1, 2, 2051, 80, "f16"), (1, 2, 1, 160, "bf16"), (1, 2, 1000, 80, "bf16"), (2, 2, 515, 160, "bf16"),
    (1, 8, 1024, 80, "bf16"), (1, 1, 97, 160, "bf16"),
    (1, 2, 700, 96, "f16"), (1, 2, 1, 96, "bf16"), (2, 2, 333, 128, "f16"), (1, 3, 1030, 128, "bf16"),
    (1, 2, 65, 96, "bf16"),
]


@pytest.mark.parametrize("B,H,N,d,dtype", SHAPES)
def test_wide_heads_match_oracle(B, H, N, d, dtype):
    print(f"wide B={B} H={H} N={N} d={d} {dtype}", flush=True)
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=70, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    worst = parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"wide N={N} d={d} {dtype}")
    print(f"  worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)
    out2 = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out2, 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.uint8), out2.view(torch.uint8)), "not run-to-run identical"


@pytest.mark.parametrize("waves", [4, 8])
@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 3, 33, 160, "f16"), (1, 1, 4099, 160, "f16"), (2, 2, 333, 128, "f16"),
                                           (1, 3, 1030, 128, "bf16"), (1, 2, 700, 96, "f16"), (1, 2, 65, 96, "bf16"),
                                           (2, 2, 515, 160, "bf16")])
def test_workgroup_shared_apply_where_the_wave_apply_is_the_default(B, H, N, d, dtype, waves, monkeypatch, tuning):
    """These shapes run apply16_wave (a wave per tile) by default; the workgroup-shared apply16_wide, which the
    MLP-fed call at these widths is built on, is checked on them as well."""
    print(f"shared-tile apply B={B} H={H} N={N} d={d} {dtype} waves={waves}", flush=True)
    code = wl.DTYPE_CODE[dtype]
    assert lf.linfusion_attn_apply_kernel(B, H, N, d, code) == "apply16_wave"
    monkeypatch.setenv("LINFUSION_WIDE_WAVE_APPLY", "2")
    monkeypatch.setenv("LINFUSION_WIDE_APPLY_WAVES", str(waves))
    assert lf.linfusion_attn_apply_kernel(B, H, N, d, code) == "apply16_wide"
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=74, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"shared-tile apply N={N} d={d} {dtype} waves={waves}")


@pytest.mark.parametrize("N,d,dtype,limit", [(1000, 160, "f16", 32), (1000, 160, "f16", 1), (33, 96, "bf16", 2),
                                             (33, 96, "bf16", 1), (420, 128, "bf16", 16)])
def test_heads_of_few_tiles_with_and_without_partials(N, d, dtype, limit, monkeypatch, tuning):
    """Heads of one or two tiles are summed by one workgroup that writes the state itself (no partials, no combine
    launch).  Both routes on the same shapes: the limit raised so that one workgroup walks dozens of tiles to a
    ragged last one, and lowered so that the partials and the combine kernel run."""
    B, H = 2, 3
    print(f"one-workgroup heads N={N} d={d} {dtype} limit={limit}", flush=True)
    monkeypatch.setenv("LINFUSION_WIDE_ONE_SPLIT_TILES", str(limit))
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=91, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"one-workgroup heads N={N} d={d} {dtype} limit={limit}")


@pytest.mark.parametrize("wgs,blk", [(4, 4), (6, 8), (2, 64)])
@pytest.mark.parametrize("N,d,dtype", [(20011, 160, "f16"), (9000, 128, "bf16"), (6000, 96, "bf16"), (20011, 160, "bf16")])
def test_wave_apply_with_many_tiles_per_wave(N, d, dtype, wgs, blk, monkeypatch, tuning):
    """Few long-lived workgroups: every wave walks dozens of tiles through its ring (steady state of the copy /
    store pipeline, block changes, a ragged last tile), which the small shapes never reach."""
    B, H = 1, 2
    print(f"wave apply N={N} d={d} {dtype} wgs={wgs} blk={blk}", flush=True)
    monkeypatch.setenv("LINFUSION_WIDE_APPLY_WGS", str(wgs))
    monkeypatch.setenv("LINFUSION_WIDE_APPLY_BLK", str(blk))
    assert lf.linfusion_attn_apply_kernel(B, H, N, d, wl.DTYPE_CODE[dtype]) == "apply16_wave"
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=75, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"wave apply N={N} d={d} {dtype} wgs={wgs} blk={blk}")


@pytest.mark.parametrize("N,d,dtype,per_cu", [(200003, 128, "f16", 3), (270001, 96, "bf16", 4)])
def test_large_wide_heads_every_row(N, d, dtype, per_cu):
    """From 768 MB of tensor traffic on the widths below 160 run three or four reduction workgroups per CU instead
    of two (more partials for the combine kernel, longer streams): every row of every head against the oracle at
    such sizes, with a ragged last tile."""
    B, H = 1, 4
    print(f"large wide heads N={N} d={d} {dtype}", flush=True)
    plan = lf.linfusion_attn_plan(B, H, N, d, wl.DTYPE_CODE[dtype])
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert plan["reduce_wgs_per_head"] * B * H <= per_cu * cus
    assert plan["reduce_wgs_per_head"] * B * H > (per_cu - 1) * cus, plan
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=93, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    worst = parity.check_all(out, q, k, v, dtype, 0, 1e-6, True, f"large wide heads N={N} d={d} {dtype}")
    print(f"  worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)


def test_wave_apply_is_chosen_at_every_wide_width():
    """fp16 operands for both storage types: (d + 2) x d of them fit one wave's registers up to d = 160."""
    names = {(d, t): lf.linfusion_attn_apply_kernel(1, 8, 4096, d, wl.DTYPE_CODE[t])
             for d in (96, 128, 160) for t in ("f16", "bf16")}
    assert all(v == "apply16_wave" for v in names.values()), names


@pytest.mark.parametrize("d,dtype", [(96, "bf16"), (160, "bf16"), (160, "f16"), (128, "f16")])
@pytest.mark.parametrize("case", ["q-20", "q-60", "some_rows_q-300", "q+3000", "q_near_the_top", "some_rows_q*1e30",
                                  "q*1e-20", "one_channel_up"])
def test_wide_query_rows_of_any_magnitude(case, d, dtype):
    """At the wide widths both storage types are multiplied as fp16 operands; every query row is scaled into fp16's
    range by its own largest channel as it is read (the factor cancels in the ratio once eps carries it), so rows far
    below zero (exp(q) subnormal or zero in fp16), rows of huge values (q + 1 beyond 65504) and rows of tiny ones
    must come out as the definition gives them."""
    if dtype == "f16" and case in ("some_rows_q*1e30", "q*1e-20"):
        pytest.skip("outside what fp16 storage holds")
    B, H, N = 1, 2, 777
    q, k, v = wl.make_qkv(B, H, N, d, "f32", idx=76, device="cpu")
    if case == "q-20":
        q = q - 20.0
    elif case == "q-60":
        q = q * 3.0 - 60.0
    elif case == "some_rows_q-300":
        q[:, :, ::3] -= 300.0
    elif case == "q+3000":
        q = q * 500.0 + 3000.0
    elif case == "q_near_the_top":
        q = q * 2500.0 + 50000.0
    elif case == "some_rows_q*1e30":
        q[:, :, 1::2] *= 1e30
    elif case == "q*1e-20":
        q = q * 1e-20
    else:
        q = q - 30.0
        q[:, :, :, 7] += 25.0 + 10.0 * torch.rand(B, H, N)
    tt = torch.bfloat16 if dtype == "bf16" else torch.float16
    q, k, v = q.to(tt), k.to(tt), v.to(tt)
    assert lf.linfusion_attn_apply_kernel(B, H, N, d, wl.DTYPE_CODE[dtype]) == "apply16_wave"
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    for eps in (1e-6, 0.0):
        out = torch.full_like(qd, float("nan"))
        lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, eps, 0, _ws(B, H, N, d, dtype))
        torch.cuda.synchronize()
        worst = parity.check_all(out, q, k, v, dtype, 0, eps, True, f"{case} d={d} {dtype} eps={eps}")
        print(f"{case} d={d} {dtype} eps={eps}: worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)
    if case in ("q-20", "some_rows_q-300", "q+3000"):      # the un-normalized arm takes the row's factor out again
        vs = (v.float() * (1e-4 if case == "q+3000" else 0.01)).to(tt)
        out = torch.full_like(qd, float("nan"))
        lf.linfusion_attn_fwd_ex(qd, kd, vs.cuda(), out, 0, 1e-6, lf.FLAG_UNNORMALIZED, _ws(B, H, N, d, dtype))
        torch.cuda.synchronize()
        parity.check_all(out, q, k, vs, dtype, 0, 1e-6, False, f"{case} d={d} {dtype} unnormalized")


@pytest.mark.parametrize("d", [96, 160])
@pytest.mark.parametrize("case", ["k-12", "k-20", "k-20_q-20", "some_tokens_k-25", "k-70"])
def test_wide_fp16_keys_far_below_zero(case, d):
    """exp(k) of fp16 keys far below zero is subnormal or zero as an fp16 operand, but the definition still gives a
    proper weighted mean: a stream whose normalizer sums show it is summed again relative to its largest key."""
    B, H, N = 1, 2, 777
    q, k, v = wl.make_qkv(B, H, N, d, "f32", idx=78, device="cpu")
    if case == "k-12":
        k = k - 12.0
    elif case in ("k-20", "k-20_q-20"):
        k = k - 20.0
    elif case == "some_tokens_k-25":
        k[:, :, ::2] -= 25.0
    else:
        k = k * 3.0 - 70.0
    if case == "k-20_q-20":
        q = q - 20.0
    q, k, v = q.half(), k.half(), v.half()
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    for eps in (1e-6, 0.0):
        out = torch.full_like(qd, float("nan"))
        lf.linfusion_attn_fwd_ex(qd, kd, vd, out, 0, eps, 0, _ws(B, H, N, d, "f16"))
        torch.cuda.synchronize()
        worst = parity.check_all(out, q, k, v, "f16", 0, eps, True, f"{case} d={d} eps={eps}")
        print(f"{case} d={d} eps={eps}: worst max-norm ratio {worst[0]:.2e}, rel L2 {worst[1]:.2e}", flush=True)


@pytest.mark.parametrize("d,dtype", [(160, "f16"), (160, "bf16"), (96, "bf16")])
def test_wide_nan_stays_where_it_belongs(d, dtype):
    """A NaN in one query row reaches that token's outputs only (the row's maximum, which scales the row, skips it and
    the other rows are bit-identical to a clean run); a NaN in a key poisons its own head and no other."""
    B, H, N = 1, 3, 333
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=77, device="cpu")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    ws = _ws(B, H, N, d, dtype)
    clean = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, clean, 0, 1e-6, 0, ws)
    qn = qd.clone()
    qn[0, 1, 200, 17] = float("nan")
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qn, kd, vd, out, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    assert bool(torch.isnan(out[0, 1, 200]).all()), "the poisoned token must not produce numbers"
    keep = torch.ones(B, H, N, dtype=torch.bool, device="cuda")
    keep[0, 1, 200] = False
    assert torch.equal(out[keep].view(torch.uint8), clean[keep].view(torch.uint8)), "other tokens changed"
    kn = kd.clone()
    kn[0, 2, 100, 5] = float("nan")
    lf.linfusion_attn_fwd_ex(qd, kn, vd, out, 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    assert bool(torch.isnan(out[0, 2]).all()), "the poisoned head must not produce numbers"
    assert torch.equal(out[0, :2].view(torch.uint8), clean[0, :2].view(torch.uint8)), "other heads changed"


@pytest.mark.parametrize("d,dtype", [(80, "f16"), (160, "f16"), (80, "bf16"), (160, "bf16"), (96, "f16"), (128, "bf16")])
def test_wide_heads_token_major_and_in_place(d, dtype):
    B, H, N = 2, 4, 700
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=71, device="cpu")
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous().cuda()
    qt, kt, vt = tm(q), tm(k), tm(v)
    view = lambda t: t.permute(0, 2, 1, 3)
    ot = torch.full_like(qt, float("nan"))
    lf.linfusion_attn_fwd_strided(view(qt), view(kt), view(vt), view(ot), 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    parity.check_all(view(ot).contiguous(), q, k, v, dtype, 0, 1e-6, True, f"wide token-major d={d} {dtype}")
    lf.linfusion_attn_fwd_strided(view(qt), view(kt), view(vt), view(qt), 0, 1e-6, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    assert torch.equal(qt.view(torch.uint8), ot.view(torch.uint8)), "in place differs from out of place"


@pytest.mark.parametrize("d,dtype", [(80, "f16"), (160, "f16"), (160, "bf16"), (96, "bf16")])
@pytest.mark.parametrize("fm,normalize", [(1, True), (2, True), (0, False)])
def test_wide_heads_other_feature_maps_and_unnormalized(d, dtype, fm, normalize):
    B, H, N = 1, 2, 300
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=72, device="cpu")
    if fm == 2:
        q, k = q.abs(), k.abs()
    if not normalize:
        v = v * 0.01          # keeps the un-normalized sums inside fp16's range
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.full_like(qd, float("nan"))
    lf.linfusion_attn_fwd_ex(qd, kd, vd, out, fm, 1e-6, 0 if normalize else lf.FLAG_UNNORMALIZED, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    parity.check_all(out, q, k, v, dtype, fm, 1e-6, normalize, f"wide d={d} fm={fm} norm={normalize}")


def test_wide_state_entry_matches_oracle():
    import numpy as np
    from oracle import linattn_oracle as orc
    B, H, N, d, dtype = 1, 2, 777, 160, "f16"
    q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=73, device="cpu")
    st = torch.full((B, H, d * d + d), float("nan"), dtype=torch.float32, device="cuda")
    lf.linfusion_attn_state(k.cuda(), v.cuda(), st, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    ks, vs = wl.stored_numpy(k), wl.stored_numpy(v)
    for h in range(H):
        S, z = orc.state(orc.widen(ks[0, h], dtype), orc.widen(vs[0, h], dtype))
        got = st[0, h].double().cpu().numpy()
        scale = np.abs(S).max()
        assert np.abs(got[:d * d].reshape(d, d) - S).max() <= 2e-3 * scale
        assert np.abs(got[d * d:] - z).max() <= 2e-3 * np.abs(z).max()


def test_wide_heads_reject_fp32_and_forced_single_launch():
    x = torch.zeros(1, 1, 64, 160, dtype=torch.float32, device="cuda")
    assert lf.linfusion_attn_workspace_bytes(1, 1, 64, 160, lf.DTYPE_F32) == 0
    assert lf.linfusion_attn_workspace_bytes(1, 1, 64, 80, lf.DTYPE_F32) == 0
    h = torch.zeros(1, 1, 64, 160, dtype=torch.float16, device="cuda")
    ws = _ws(1, 1, 64, 160, "f16")
    assert lf.linfusion_attn_fwd_ex(h, h, h, torch.empty_like(h), 0, 1e-6, lf.FLAG_FORCE_FUSED, ws, check=False) == -2
    assert lf.linfusion_attn_fwd_ex(x, x, x, torch.empty_like(x), 0, 1e-6, 0, ws, check=False) == -2
