"""GPU parity of linfusion_attn_fwd_mlp (the mixer fed by the two-branch MLPs f', g' of Sec. 3.1 (Implementation Details)) against the
fp64 oracle's module_mixer on the same stored inputs, element by element."""
import numpy as np
import pytest
import torch

import paper_2409_02097_amd as lf
from oracle import linattn_oracle as orc
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu

LN_EPS, SLOPE = 1e-5, 0.01


def _ws(B, H, N, d, dtype):
    n = lf.linfusion_attn_mlp_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype])
    assert n > 0
    return torch.empty(n, dtype=torch.uint8, device="cuda")


def _run(ins, H, fm=0, eps=1e-6, flags=0, ln_eps=LN_EPS, slope=SLOPE):
    dev = [t.cuda() for t in ins]
    B, N, C = dev[0].shape
    dtype = {torch.float16: "f16", torch.bfloat16: "bf16"}[dev[0].dtype]
    out = torch.full_like(dev[0], float("nan"))
    lf.linfusion_attn_fwd_mlp(*dev[:5], out, *dev[5:], H, fm, eps, ln_eps, slope, flags, _ws(B, H, N, C // H, dtype))
    torch.cuda.synchronize()
    return out


def _oracle(ins, H, dtype, fm=0, eps=1e-6, normalize=True, ln_eps=LN_EPS, slope=SLOPE):
    a_q, t_q, a_k, t_k, v = (orc.widen(wl.stored_numpy(t), dtype) for t in ins[:5])
    gq, bq, gk, bk = (t.numpy().astype(np.float64) for t in ins[5:])
    return orc.module_mixer(a_q, t_q, a_k, t_k, v, gq, bq, gk, bk, H, fm, eps, normalize, ln_eps, slope)


def _check(out, ref, H, dtype, what):
    gpu = parity.to_f64(out)
    B, N, C = ref.shape
    d = C // H
    worst = (0.0, 0.0)
    for b in range(B):
        for h in range(H):
            c = slice(h * d, (h + 1) * d)
            r = parity.check_slice(gpu[b, :, c], ref[b, :, c], dtype, f"{what} b={b} h={h}")
            worst = (max(worst[0], r[0]), max(worst[1], r[1]))
    return worst


SHAPES = [
    # eight heads (whole rows of the SD-v1.5 first level: 8 x 40 = 320 channels)
    (1, 8, 1, 40, "f16"), (2, 8, 33, 40, "f16"), (1, 8, 1000, 40, "f16"), (2, 8, 4099, 40, "f16"),
    (3, 8, 31, 8, "f16"), (1, 8, 515, 16, "f16"), (1, 8, 300, 24, "f16"), (2, 8, 260, 32, "f16"),
    (1, 8, 777, 48, "f16"),
    (1, 8, 33, 40, "bf16"), (2, 8, 1000, 40, "bf16"), (1, 8, 2100, 48, "bf16"), (1, 8, 130, 8, "bf16"),
    (1, 8, 95, 32, "bf16"),
    # four heads
    (1, 4, 1, 64, "f16"), (2, 4, 1000, 64, "f16"), (1, 4, 333, 80, "f16"), (2, 4, 77, 40, "f16"),
    (1, 4, 600, 56, "f16"), (1, 4, 100, 8, "f16"), (1, 4, 2051, 16, "f16"),
    (1, 4, 500, 80, "bf16"), (2, 4, 300, 64, "bf16"), (1, 4, 1030, 24, "bf16"),
]


@pytest.mark.parametrize("B,H,N,d,dtype", SHAPES)
def test_matches_oracle(B, H, N, d, dtype):
    print(f"mlp B={B} H={H} N={N} d={d} {dtype}", flush=True)
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=80)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, f"mlp {B}x{H}x{N}x{d} {dtype}")


@pytest.mark.parametrize("fm", [0, 1, 2])
@pytest.mark.parametrize("unnorm", [False, True])
@pytest.mark.parametrize("H,d,dtype", [(8, 40, "f16"), (4, 64, "bf16")])
def test_feature_maps_and_unnormalized(H, d, dtype, fm, unnorm):
    print(f"mlp fm={fm} unnorm={unnorm} H={H} d={d} {dtype}", flush=True)
    B, N = 2, 700
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=81))
    if fm != 0:   # identity / relu: keep the denominators away from zero
        ins[0] = (ins[0].float().abs() + 0.5).to(ins[0].dtype)
        ins[2] = (ins[2].float().abs() + 0.5).to(ins[2].dtype)
    out = _run(ins, H, fm=fm, flags=lf.FLAG_UNNORMALIZED if unnorm else 0)
    _check(out, _oracle(ins, H, dtype, fm=fm, normalize=not unnorm), H, dtype, f"fm={fm} unnorm={unnorm}")


@pytest.mark.parametrize("H,d,dtype", [(8, 40, "f16"), (8, 48, "bf16"), (4, 80, "f16")])
def test_zero_start_is_the_plain_mixer(H, d, dtype):
    """Sec. 3.1 (Implementation Details): with the second branch at its initial value zero, q and k are the linear-branch results."""
    B, N = 2, 1500
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=82, zero_start=True)
    out = _run(ins, H)
    heads = lambda t: t.cuda().view(B, N, H, d).permute(0, 2, 1, 3)          # strided [B, H, N, d] views
    plain = torch.empty(B, N, H, d, dtype=out.dtype, device="cuda")
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype]), dtype=torch.uint8, device="cuda")
    lf.linfusion_attn_fwd_strided(heads(ins[0]), heads(ins[2]), heads(ins[4]), plain.permute(0, 2, 1, 3), 0, 1e-6, 0, ws)
    torch.cuda.synchronize()
    ref = parity.to_f64(plain.view(B, N, H * d))
    _check(out, _oracle(ins, H, dtype), H, dtype, "zero start vs oracle")
    # two correct roundings of the same values: they differ by at most one unit in the last place
    diff = np.abs(parity.to_f64(out) - ref)
    assert (diff <= 2.0 * orc.half_ulp(ref, dtype) + 2e-3 * np.abs(ref).max()).all()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_layer_norm_input_far_from_zero_mean(dtype):
    """Rows whose mean is many standard deviations away from zero: the variance must come from centred sums."""
    B, H, N, d = 1, 8, 500, 40
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=83))
    for i in (1, 3):
        ins[i] = (ins[i].float() * 0.5 + 40.0).to(ins[i].dtype)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, "offset LayerNorm input")


def test_layer_norm_epsilon_and_slope_are_honoured():
    B, H, N, d, dtype = 1, 8, 200, 40, "f16"
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=84))
    for i in (1, 3):
        ins[i] = (ins[i].float() * 0.01).to(ins[i].dtype)        # variance ~ 2e-4: ln_eps = 1e-3 matters
    out = _run(ins, H, ln_eps=1e-3, slope=0.2)
    _check(out, _oracle(ins, H, dtype, ln_eps=1e-3, slope=0.2), H, dtype, "ln_eps, slope")
    other = _oracle(ins, H, dtype)                                # the defaults give something else
    assert np.abs(other - parity.to_f64(out)).max() > 1e-2


def test_run_to_run_identical():
    ins = wl.make_mlp_inputs(2, 8, 3000, 40, "f16", idx=85)
    a, b = _run(ins, 8), _run(ins, 8)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_rejected_arguments():
    code = wl.DTYPE_CODE
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 8, 100, 72, code["f16"]) == 0      # no kernel of that width
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 5, 100, 112, code["f16"]) == 0
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 8, 100, 64, code["f16"]) > 0       # per-head kernels
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 8, 100, 40, code["f32"]) == 0
    ins = [t.cuda() for t in wl.make_mlp_inputs(1, 8, 64, 40, "f16", idx=86)]
    out = torch.empty_like(ins[0])
    ws = _ws(1, 8, 64, 40, "f16")
    call = lambda *a, **k: lf.linfusion_attn_fwd_mlp(*a, check=False, **k)
    assert call(*ins[:5], out, *ins[5:], 8, 0, 1e-6, 0.0, 0.01, 0, ws) == -1           # ln_eps must be positive
    assert call(*ins[:5], out, *ins[5:], 8, 0, 1e-6, 1e-5, float("nan"), 0, ws) == -1
    assert call(*ins[:5], out, *ins[5:], 8, 0, 1e-6, 1e-5, 1.5, 0, ws) == -1           # slope must lie in [0, 1]
    assert call(*ins[:5], out, *ins[5:], 8, 0, 1e-6, 1e-5, 0.01, lf.FLAG_FORCE_FUSED, ws) == -1
    assert call(*ins[:5], out, *ins[5:], 8, 0, 1e-6, 1e-5, 0.01, 0, ws[:1024]) == -4   # workspace too small
    assert call(*ins[:5], ins[0], *ins[5:], 8, 0, 1e-6, 1e-5, 0.01, 0, ws) == -7       # out aliases an input
    assert call(*ins[:5], out, *ins[5:], 8, 7, 1e-6, 1e-5, 0.01, 0, ws) == -2          # unknown feature map


@pytest.mark.parametrize("B,H,N,d,dtype", [(2, 8, 1000, 40, "f16"), (1, 8, 4099, 40, "bf16"), (2, 4, 333, 80, "f16"),
                                           (3, 4, 77, 64, "bf16"), (1, 8, 1, 16, "f16")])
def test_strided_rows_of_one_wide_projection(B, H, N, d, dtype):
    """The five branch results as column blocks of one [B, N, 5 C] tensor, out as a block of a [B, N, 2 C] one:
    same bits as the dense call, and the oracle's values; the rest of the output buffer stays untouched."""
    print(f"mlp strided B={B} H={H} N={N} d={d} {dtype}", flush=True)
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=86)
    C = H * d
    dense = _run(ins, H)
    wide = torch.cat([t.cuda() for t in ins[:5]], dim=2).contiguous()               # [B, N, 5 C]
    views = [wide[:, :, i * C:(i + 1) * C] for i in range(5)]
    vecs = [t.cuda() for t in ins[5:]]
    obuf = torch.full((B, N, 2 * C), 7.0, dtype=wide.dtype, device="cuda")
    out = obuf[:, :, C:]
    lf.linfusion_attn_fwd_mlp_strided(*views, out, *vecs, H, 0, 1e-6, LN_EPS, SLOPE, 0, _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    assert torch.equal(out.contiguous().view(torch.int16), dense.view(torch.int16))
    assert bool((obuf[:, :, :C] == 7.0).all())
    _check(out.contiguous(), _oracle(ins, H, dtype), H, dtype, f"mlp strided {B}x{H}x{N}x{d} {dtype}")


def test_strided_entry_with_padded_batches_and_dense_arrays_absent():
    """Batch stride larger than N rows (padding between batches) on both sides; NULL stride arrays = dense."""
    B, H, N, d, dtype = 2, 8, 515, 40, "f16"
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=87)
    C = H * d
    dense = _run(ins, H)
    dev = [t.cuda() for t in ins]
    pad = [torch.zeros(B, N + 5, C, dtype=dev[0].dtype, device="cuda") for _ in range(5)]
    for p, t in zip(pad, dev[:5]):
        p[:, :N].copy_(t)
    # the five views must share strides, not a buffer
    obuf = torch.full((B, N + 3, C), 7.0, dtype=dev[0].dtype, device="cuda")
    lf.linfusion_attn_fwd_mlp_strided(*[p[:, :N] for p in pad], obuf[:, :N], *dev[5:], H, 0, 1e-6, LN_EPS, SLOPE, 0,
                                      _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    assert torch.equal(obuf[:, :N].contiguous().view(torch.int16), dense.view(torch.int16))
    assert bool((obuf[:, N:] == 7.0).all())
    out2 = torch.empty_like(dense)
    ws = _ws(B, H, N, d, dtype)
    rc = lf.library().linfusion_attn_fwd_mlp_strided(
        *[t.data_ptr() for t in dev[:5]], out2.data_ptr(), *[t.data_ptr() for t in dev[5:]], B, H, N, d, 1, 0, 1e-6,
        LN_EPS, SLOPE, 0, None, None, ws.data_ptr(), ws.numel(), None, None)
    torch.cuda.synchronize()
    assert rc == 0 and torch.equal(out2.view(torch.int16), dense.view(torch.int16))


# ---- shapes whose token rows do not fit one workgroup: per-head kernels with a statistics pass ------------------
HEAD_SHAPES = [
    (1, 10, 1000, 64, "f16"), (2, 20, 333, 64, "bf16"), (1, 8, 777, 80, "f16"), (1, 5, 515, 64, "f16"),
    (1, 8, 300, 64, "f16"), (1, 2, 100, 40, "f16"), (1, 3, 2051, 24, "bf16"), (1, 1, 33, 8, "f16"),
    (2, 16, 64, 56, "f16"), (1, 8, 1, 80, "bf16"), (1, 10, 4099, 64, "bf16"), (3, 6, 31, 16, "f16"),
    (1, 12, 130, 32, "bf16"), (1, 16, 257, 48, "f16"),
]


@pytest.mark.parametrize("B,H,N,d,dtype", HEAD_SHAPES)
def test_per_head_route_matches_oracle(B, H, N, d, dtype):
    print(f"mlp heads B={B} H={H} N={N} d={d} {dtype}", flush=True)
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=88)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, f"mlp heads {B}x{H}x{N}x{d} {dtype}")


@pytest.mark.parametrize("B,H,N,d,dtype", [(2, 8, 1000, 40, "f16"), (1, 8, 4099, 40, "bf16"), (1, 4, 333, 80, "f16"),
                                           (2, 4, 77, 64, "bf16"), (1, 8, 33, 8, "f16")])
def test_per_head_route_on_whole_row_shapes(B, H, N, d, dtype, monkeypatch, tuning):
    """Both routes on one shape: each within tolerance of the oracle (their bits may differ: the statistics are
    summed in another order)."""
    print(f"mlp heads forced B={B} H={H} N={N} d={d} {dtype}", flush=True)
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=89)
    ref = _oracle(ins, H, dtype)
    rows = _run(ins, H)
    monkeypatch.setenv("LINFUSION_MLP_ROUTE", "1")
    heads = _run(ins, H)
    monkeypatch.setenv("LINFUSION_MLP_ROUTE", "2")     # statistics pass + row-piece kernels on groups of four heads
    groups = _run(ins, H)
    monkeypatch.delenv("LINFUSION_MLP_ROUTE")
    _check(rows, ref, H, dtype, "whole rows")
    _check(heads, ref, H, dtype, "per head")
    _check(groups, ref, H, dtype, "groups of four heads")


@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 8, 777, 80, "f16"), (2, 8, 2051, 80, "bf16"), (1, 16, 257, 48, "f16"),
                                           (1, 12, 130, 32, "bf16"), (1, 8, 1000, 56, "f16")])
def test_group_shapes_on_the_per_head_kernels(B, H, N, d, dtype, monkeypatch, tuning):
    """Rows of whole groups of four heads whose head rows are no whole cache lines go through the group kernels by
    default (covered by the per-head shape list above); the per-head kernels must serve them too."""
    print(f"mlp group shape forced per head B={B} H={H} N={N} d={d} {dtype}", flush=True)
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=97)
    ref = _oracle(ins, H, dtype)
    groups = _run(ins, H)
    monkeypatch.setenv("LINFUSION_MLP_ROUTE", "1")
    heads = _run(ins, H)
    monkeypatch.delenv("LINFUSION_MLP_ROUTE")
    _check(groups, ref, H, dtype, "groups of four heads")
    _check(heads, ref, H, dtype, "per head")


@pytest.mark.parametrize("fm", [0, 1, 2])
@pytest.mark.parametrize("unnorm", [False, True])
def test_per_head_route_feature_maps_and_unnormalized(fm, unnorm):
    B, H, N, d, dtype = 2, 10, 700, 64, "f16"
    print(f"mlp heads fm={fm} unnorm={unnorm}", flush=True)
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=90))
    if fm != 0:   # identity / relu: keep the denominators away from zero
        ins[0] = (ins[0].float().abs() + 0.5).to(ins[0].dtype)
        ins[2] = (ins[2].float().abs() + 0.5).to(ins[2].dtype)
    out = _run(ins, H, fm=fm, flags=lf.FLAG_UNNORMALIZED if unnorm else 0)
    _check(out, _oracle(ins, H, dtype, fm=fm, normalize=not unnorm), H, dtype, f"mlp heads fm={fm} unnorm={unnorm}")


@pytest.mark.parametrize("H,d,dtype", [(10, 64, "f16"), (8, 80, "bf16"), (3, 8, "f16")])
def test_per_head_route_layer_norm_input_far_from_zero_mean(H, d, dtype):
    B, N = 1, 500
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=92))
    for i in (1, 3):
        ins[i] = (ins[i].float() * 0.5 + 40.0).to(ins[i].dtype)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, "offset LayerNorm input, per head")


@pytest.mark.parametrize("B,H,N,d,dtype", [(2, 10, 515, 64, "bf16"), (2, 8, 515, 80, "f16"), (1, 16, 1000, 40, "bf16")])
def test_per_head_route_strided_and_repeatable(B, H, N, d, dtype):
    """Column blocks of one wide buffer on the routes that start with the statistics pass (per-head kernels; groups of
    four heads): same bits as the dense call, twice."""
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=91)
    C = H * d
    dense = _run(ins, H)
    assert torch.equal(_run(ins, H).view(torch.int16), dense.view(torch.int16))
    wide = torch.cat([t.cuda() for t in ins[:5]], dim=2).contiguous()
    views = [wide[:, :, i * C:(i + 1) * C] for i in range(5)]
    obuf = torch.full((B, N, 2 * C), 7.0, dtype=wide.dtype, device="cuda")
    lf.linfusion_attn_fwd_mlp_strided(*views, obuf[:, :, C:], *[t.cuda() for t in ins[5:]], H, 0, 1e-6, LN_EPS, SLOPE, 0,
                                      _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    assert torch.equal(obuf[:, :, C:].contiguous().view(torch.int16), dense.view(torch.int16))
    assert bool((obuf[:, :, :C] == 7.0).all())
    _check(dense, _oracle(ins, H, dtype), H, dtype, "mlp heads strided")


# ---- head widths above 64 (SD-v1.5's third level: 8 heads of 160): statistics pass + the wide kernels ------------
WIDE_SHAPES = [
    (1, 8, 1000, 160, "f16"), (2, 8, 333, 160, "bf16"), (1, 4, 515, 128, "f16"), (1, 5, 2051, 96, "bf16"),
    (1, 2, 1, 160, "f16"), (2, 3, 33, 96, "f16"), (1, 8, 4099, 160, "bf16"), (1, 1, 64, 128, "bf16"),
]


@pytest.mark.parametrize("B,H,N,d,dtype", WIDE_SHAPES)
def test_wide_heads_match_oracle(B, H, N, d, dtype):
    print(f"mlp wide B={B} H={H} N={N} d={d} {dtype}", flush=True)
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=93)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, f"mlp wide {B}x{H}x{N}x{d} {dtype}")


@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 8, 1000, 160, "f16"), (2, 8, 333, 160, "bf16"), (1, 5, 2051, 96, "bf16"),
                                           (1, 4, 515, 128, "f16")])
def test_wide_heads_on_the_workgroup_shared_apply(B, H, N, d, dtype, monkeypatch, tuning):
    """By default apply runs a wave per 16-token tile (apply16_wave_mlp); the workgroup-shared kernel that it replaced
    stays in the library as a tuning aid and is checked against the oracle too."""
    monkeypatch.setenv("LINFUSION_MLPW_WAVE_APPLY", "2")
    ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=93)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, f"mlp wide, shared tiles {B}x{H}x{N}x{d} {dtype}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("case", ["a-20", "a+3000", "some_rows_a-300"])
def test_wide_heads_query_rows_far_from_one(case, dtype):
    """The formed query a + LeakyReLU(LayerNorm(t)) far below zero or large: bf16 rows are scaled into fp16's range
    as they are formed; fp16 rows keep fp16's own range (so -20 stays inside what exp leaves representable)."""
    if dtype == "f16" and case == "some_rows_a-300":
        pytest.skip("exp(-300) is zero in an fp16 operand: covered for bf16, whose rows are scaled")
    B, H, N, d = 1, 8, 333, 160
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=96))
    a = ins[0].float()
    if case == "a-20":
        a = a - (8.0 if dtype == "f16" else 20.0)
    elif case == "a+3000":
        a = a * 500.0 + 3000.0
    else:
        a[:, ::3] -= 300.0
    ins[0] = a.to(ins[0].dtype)
    out = _run(ins, H)
    _check(out, _oracle(ins, H, dtype), H, dtype, f"mlp wide {case} {dtype}")


@pytest.mark.parametrize("fm", [0, 1, 2])
@pytest.mark.parametrize("unnorm", [False, True])
def test_wide_heads_feature_maps_and_unnormalized(fm, unnorm):
    B, H, N, d, dtype = 2, 8, 300, 160, "f16"
    print(f"mlp wide fm={fm} unnorm={unnorm}", flush=True)
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=94))
    if fm != 0:   # identity / relu: keep the denominators away from zero
        ins[0] = (ins[0].float().abs() + 0.5).to(ins[0].dtype)
        ins[2] = (ins[2].float().abs() + 0.5).to(ins[2].dtype)
    if unnorm:
        ins[4] = (ins[4].float() * 0.0625).to(ins[4].dtype)
    out = _run(ins, H, fm=fm, flags=lf.FLAG_UNNORMALIZED if unnorm else 0)
    _check(out, _oracle(ins, H, dtype, fm=fm, normalize=not unnorm), H, dtype, f"mlp wide fm={fm} unnorm={unnorm}")


def test_wide_heads_strided_repeatable_and_far_from_zero_mean():
    B, H, N, d, dtype = 2, 8, 515, 160, "bf16"
    ins = list(wl.make_mlp_inputs(B, H, N, d, dtype, idx=95))
    for i in (1, 3):
        ins[i] = (ins[i].float() * 0.5 + 40.0).to(ins[i].dtype)
    C = H * d
    dense = _run(ins, H)
    assert torch.equal(_run(ins, H).view(torch.int16), dense.view(torch.int16))
    _check(dense, _oracle(ins, H, dtype), H, dtype, "mlp wide, offset LayerNorm input")
    wide = torch.cat([t.cuda() for t in ins[:5]], dim=2).contiguous()
    views = [wide[:, :, i * C:(i + 1) * C] for i in range(5)]
    obuf = torch.full((B, N, 2 * C), 7.0, dtype=wide.dtype, device="cuda")
    lf.linfusion_attn_fwd_mlp_strided(*views, obuf[:, :, C:], *[t.cuda() for t in ins[5:]], H, 0, 1e-6, LN_EPS, SLOPE, 0,
                                      _ws(B, H, N, d, dtype))
    torch.cuda.synchronize()
    assert torch.equal(obuf[:, :, C:].contiguous().view(torch.int16), dense.view(torch.int16))
    assert bool((obuf[:, :, :C] == 7.0).all())
