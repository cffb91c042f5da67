"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is enqueued."""
import ctypes
import os
import re

import pytest

import paper_2409_02097_amd as lf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "linfusion.h")


def _device_present():
    import torch
    return torch.cuda.is_available()


# The validation tests hand the library made-up device addresses.  Nothing dereferences them as long as every
# call ends in an error code, which without a device even a valid call does (no device); on a machine that has
# one a valid call would launch kernels on those addresses, so there these tests do not run at all.
fake_addresses = pytest.mark.skipif(_device_present(), reason="passes made-up device addresses: only where no "
                                                              "GPU could be handed them")


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(linfusion_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    syms = _declared_symbols()
    for name in ("linfusion_attn_fwd", "linfusion_attn_fwd_ex", "linfusion_attn_fwd_strided",
                 "linfusion_attn_workspace_bytes",
                 "linfusion_attn_state", "linfusion_status_string", "linfusion_version"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(lf.library_path()) if os.path.exists(lf.library_path()) else lf.library()
    for name in _declared_symbols():
        assert hasattr(lib, name), f"{name} declared in linfusion.h but not exported"


def test_version_and_status_strings():
    assert lf.linfusion_version() >= 100
    seen = set()
    for code in range(0, -9, -1):
        s = lf.linfusion_status_string(code)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert lf.linfusion_status_string(-99) == "unknown status"


def test_workspace_bytes_is_a_pure_function_of_the_shape():
    a = lf.linfusion_attn_workspace_bytes(1, 8, 2097152, 40, lf.DTYPE_F16)
    assert a == lf.linfusion_attn_workspace_bytes(1, 8, 2097152, 40, lf.DTYPE_F16) and a > 0
    plan = lf.linfusion_attn_plan(1, 8, 2097152, 40, lf.DTYPE_F16)
    need = 8 * (plan["reduce_wgs_per_head"] + 1) * (40 * 40 + 40) * 4
    # room for the launch shapes with more partials per head (single launch, grouped heads of strided layouts)
    assert need <= a <= 8 * need
    # rejected arguments need no workspace
    assert lf.linfusion_attn_workspace_bytes(1, 8, 1024, 12, lf.DTYPE_F16) == 0
    assert lf.linfusion_attn_workspace_bytes(0, 8, 1024, 40, lf.DTYPE_F16) == 0
    assert lf.linfusion_attn_workspace_bytes(1, 8, 1024, 40, 7) == 0


def test_environment_is_ignored_unless_tuning_is_switched_on(monkeypatch):
    shape = (1, 8, 2097152, 40, lf.DTYPE_F16)
    base_ws = lf.linfusion_attn_workspace_bytes(*shape)
    base_plan = lf.linfusion_attn_plan(*shape)
    monkeypatch.setenv("LINFUSION_REDUCE_WGS", "4096")
    monkeypatch.setenv("LINFUSION_APPLY_WGS", "512")
    assert lf.linfusion_attn_workspace_bytes(*shape) == base_ws         # no environment on the default path
    assert lf.linfusion_attn_plan(*shape) == base_plan
    lf.linfusion_set_tuning(True)
    try:
        tuned = lf.linfusion_attn_plan(*shape)
        assert tuned["reduce_wgs_per_head"] == 512 and tuned["apply_wgs_per_head"] == 64
        assert lf.linfusion_attn_workspace_bytes(*shape) > base_ws
    finally:
        lf.linfusion_set_tuning(False)
    assert lf.linfusion_attn_plan(*shape) == base_plan


def test_probe_entry_points_validate_on_the_host():
    assert lf.library().linfusion_hbm_probe(0, 0, None, None, None, None, 1024, 64, None, None) == -1
    assert lf.library().linfusion_hbm_probe(1, 0, None, None, None, None, 1024, 64, None, None) == -1   # no source
    assert lf.library().linfusion_hbm_probe(4, 0, 4096, None, None, None, 1024, 64, 4096, None) == -1
    assert lf.library().linfusion_hbm_probe(1, 1, 4096, None, None, 8192, 1000, 64, None, None) == -1    # not whole chunks
    assert lf.library().linfusion_hbm_probe(1, 1, 4100, None, None, 8192, 1024, 64, None, None) == -3
    assert lf.library().linfusion_launch_probe(0, 64, None, None) == -1
    assert lf.library().linfusion_launch_probe(3, 0, None, None) == -1


@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 8, 1024, 40, 0), (2, 8, 4096, 40, 1), (2, 5, 9216, 64, 1),
                                          (2, 10, 16384, 64, 2), (2, 20, 4096, 64, 2), (1, 8, 2097152, 40, 1),
                                          (1, 1, 1, 8, 1), (1, 1, 31, 64, 0)])
def test_plan_covers_every_token_tile(B, H, N, d, dtype):
    plan = lf.linfusion_attn_plan(B, H, N, d, dtype)
    tile = plan["tile_tokens"]
    n_tiles = -(-N // tile)
    assert 1 <= plan["reduce_wgs_per_head"] <= n_tiles
    assert 1 <= plan["apply_wgs_per_head"] <= n_tiles
    assert plan["path"] in (0, 1, 2)


def _call(q=4096, k=1 << 20, v=2 << 20, out=3 << 20, B=1, H=2, N=64, d=40, dtype=1, fm=0, eps=1e-6, flags=0,
          ws=8 << 20, ws_bytes=1 << 20):
    """Raw C call with fake (never dereferenced) device addresses: every check below fails on the host."""
    return lf.library().linfusion_attn_fwd_ex(q, k, v, out, B, H, N, d, dtype, fm, eps, flags, ws, ws_bytes, None)


@fake_addresses
def test_argument_validation_happens_on_the_host():
    assert _call(q=None) == -1 and _call(k=None) == -1 and _call(v=None) == -1 and _call(out=None) == -1
    assert _call(B=0) == -1 and _call(H=-1) == -1 and _call(N=0) == -1 and _call(d=0) == -1
    assert _call(eps=-1.0) == -1 and _call(eps=float("nan")) == -1 and _call(eps=float("inf")) == -1
    assert _call(flags=1 << 9) == -1 and _call(flags=2 | 4) == -1
    assert _call(d=12) == -2 and _call(d=72) == -2 and _call(dtype=3) == -2 and _call(fm=5) == -2
    assert _call(d=80, dtype=0) == -2 and _call(d=160, dtype=0) == -2 and _call(d=168) == -2 and _call(d=112) == -2   # wide heads: 16-bit only
    assert _call(d=160, flags=4, ws_bytes=64 << 20) == -2                                         # no single launch there
    assert _call(q=4096 + 8) == -3 and _call(out=(3 << 20) + 2) == -3 and _call(ws=(8 << 20) + 4) == -3
    assert _call(ws=None) == -4 and _call(ws_bytes=16) == -4
    assert _call(out=1 << 20) == -7                      # out aliases k
    assert _call(out=(2 << 20) + 64) == -7               # out overlaps v partially
    assert _call(q=4096, out=4096 + 160) == -7           # partial overlap with q
    assert _call(ws=3 << 20) == -7                       # workspace overlaps out


def _strided(sq=None, skv=None, so=None, q=4096, k=1 << 20, v=2 << 20, out=3 << 20, B=2, H=4, N=64, d=40, dtype=1,
             ws=64 << 20, ws_bytes=1 << 20):
    arr = lambda s: None if s is None else ctypes.byref((ctypes.c_longlong * 3)(*s))
    return lf.library().linfusion_attn_fwd_strided(q, k, v, out, B, H, N, d, dtype, 0, 1e-6, 0, arr(sq), arr(skv),
                                                   arr(so), ws, ws_bytes, None)


@fake_addresses
def test_stride_validation_happens_on_the_host():
    import torch
    ok = -6 if not torch.cuda.is_available() else None      # valid arguments reach the device check
    dense = (4 * 64 * 40, 64 * 40, 40)
    token_major = (64 * 4 * 40, 40, 4 * 40)
    if ok is not None:
        assert _strided() == ok and _strided(dense, dense, dense) == ok
        assert _strided(token_major, token_major, token_major) == ok
        assert _strided(dense, (64 * 40, 0, 40), dense) == ok            # k, v shared by all heads
        assert _strided(token_major, token_major, token_major, q=4096, out=4096, k=8 << 20, v=16 << 20) == ok
    assert _strided(so=(4 * 64 * 40, 64 * 40, -40)) == -1                # negative stride
    assert _strided(sq=(4 * 64 * 40, 64 * 40, 44)) == -3                 # rows not 16-byte aligned
    assert _strided(so=(4 * 64 * 40 + 4, 64 * 40, 40)) == -3
    assert _strided(sq=dense, skv=dense, so=(4 * 64 * 40, 64 * 40, 40), dtype=0, d=40) in (-6, 0, ok)
    assert _strided(sq=(0, 0, 4), dtype=1) == -3                         # 4 fp16 elements = 8 bytes
    assert _strided(sq=(0, 0, 4), dtype=0, ws_bytes=4 << 20) in (-6, ok) # 4 fp32 elements = 16 bytes
    assert _strided(so=(4 * 64 * 40, 64 * 40, 32)) == -7                 # output rows overlap each other
    assert _strided(so=(4 * 64 * 40, 40, 40)) == -7                      # heads on top of tokens
    assert _strided(so=(0, 64 * 40, 40)) == -7                           # batches on top of each other
    assert _strided(so=(4 * 64 * 40, 64 * 40, 40), sq=token_major, q=4096, out=4096) == -7   # alias, other view
    assert _strided(sq=(1 << 46, 64 * 40, 40)) == -1                     # span beyond the addressable range
    assert _strided(sq=(4 * 64 * 40, 64 * 40, 8 << 24)) == -1            # token stride too large
    # the span of a strided k reaches into out although the dense extents would not
    assert _strided(skv=(64 * 4 * 80, 80, 4 * 80), k=(3 << 20) - 4 * 64 * 80 * 2 * 2 + 4096) == -7


@fake_addresses
def test_backward_argument_validation_happens_on_the_host():
    lib = lf.library()

    def call(state=None, q=4096, k=1 << 20, v=2 << 20, g=3 << 20, dq=4 << 20, dk=5 << 20, dv=6 << 20, d=40, dtype=1, fm=0, eps=1e-6,
             flags=0, ws=64 << 20, ws_bytes=8 << 20):
        return lib.linfusion_attn_bwd(q, k, v, g, state, dq, dk, dv, 1, 2, 64, d, dtype, fm, eps, flags, ws, ws_bytes, None)
    assert call(g=None) == -1 and call(dk=None) == -1 and call(eps=-1.0) == -1 and call(flags=2) == -1
    assert call(d=160, dtype=2) == -2 and call(d=12) == -2 and call(fm=3) == -2 and call(d=80, dtype=0) == -2
    # fp16 at the wide widths and fp32 are supported (the composed pass): validation goes on to the workspace size
    # (-4) and, past it, to the device check (-6: there is none here)
    assert call(d=160, dtype=1) == -6 and call(dtype=0) == -6 and call(dtype=0, ws_bytes=1 << 10) == -4
    assert call(dq=(4 << 20) + 8) == -3 and call(ws=(64 << 20) + 4) == -3
    assert call(ws=None) == -4 and call(ws_bytes=64) == -4
    assert call(dq=4096) == -7 and call(dk=4 << 20) == -7 and call(dv=(2 << 20) + 256) == -7 and call(ws=6 << 20) == -7
    assert call(state=(7 << 20) + 4) == -3 and call(state=4 << 20) == -7 and call(state=64 << 20) == -7
    assert lf.linfusion_attn_bwd_workspace_bytes(1, 2, 64, 40, 1) > 0
    assert 0 < lf.linfusion_attn_workspace_state_offset(1, 2, 64, 40, 1) < lf.linfusion_attn_workspace_bytes(1, 2, 64, 40, 1)
    assert lf.linfusion_attn_bwd_workspace_bytes(1, 2, 64, 40, 0) > 0 and lf.linfusion_attn_bwd_workspace_bytes(1, 2, 64, 80, 0) == 0


@fake_addresses
def test_valid_call_without_a_gfx950_device_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; the no-device error path is a CPU-box check")
    assert _call() == -6
    assert _call(q=4096, out=4096) == -6                 # exact in-place alias passes validation
    rc = lf.library().linfusion_attn_fwd(4096, 1 << 20, 2 << 20, 3 << 20, 1, 2, 64, 40, 0, 1e-6, None)
    assert rc == -6
    st = lf.library().linfusion_attn_state(1 << 20, 2 << 20, 3 << 20, 1, 2, 64, 40, 1, 0, 8 << 20, 1 << 20, None)
    assert st == -6


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 8, dtype=torch.float16)
    with pytest.raises(ValueError):
        lf.linfusion_attn_fwd_ex(x, x, x, x.clone(), 0, 1e-6, 0, None)


def _mlp(B=1, H=8, N=64, d=40, dtype=1, fm=0, eps=1e-6, ln_eps=1e-5, slope=0.01, flags=0, out=5 << 20, ws=64 << 20,
         ws_bytes=4 << 20, a_q=1 << 20, gamma_q=48 << 20):
    """Raw C call of linfusion_attn_fwd_mlp with fake device addresses (never dereferenced)."""
    return lf.library().linfusion_attn_fwd_mlp(a_q, 2 << 20, 3 << 20, 4 << 20, 6 << 20, out, gamma_q, 49 << 20, 50 << 20,
                                               51 << 20, B, H, N, d, dtype, fm, eps, ln_eps, slope, flags, ws, ws_bytes,
                                               None, None)


@fake_addresses
def test_mlp_fed_entry_validates_on_the_host():
    import torch
    ok = -6 if not torch.cuda.is_available() else None
    if ok is not None:
        assert _mlp() == ok and _mlp(H=4, d=80) == ok and _mlp(dtype=2, d=48) == ok
    assert _mlp(a_q=None) == -1 and _mlp(gamma_q=None) == -1 and _mlp(out=None) == -1
    assert _mlp(ln_eps=0.0) == -1 and _mlp(ln_eps=float("inf")) == -1 and _mlp(slope=-0.1) == -1 and _mlp(slope=2.0) == -1
    assert _mlp(eps=-1.0) == -1 and _mlp(flags=2) == -1 and _mlp(B=0) == -1
    if ok is not None:   # head counts and widths beyond the whole-row kernels go the per-head way
        assert _mlp(H=8, d=64) == ok and _mlp(H=5) == ok and _mlp(H=20, d=64, ws_bytes=16 << 20) == ok
        assert _mlp(H=8, d=160, ws_bytes=16 << 20) == ok and _mlp(H=2, d=96, ws_bytes=16 << 20) == ok
    assert _mlp(B=40000, H=1, d=64) == -1 and _mlp(B=9000, H=8, d=64) == -1       # launch grid limits
    assert _mlp(d=72) == -2 and _mlp(d=112) == -2 and _mlp(d=12) == -2 and _mlp(dtype=0) == -2 and _mlp(fm=9) == -2
    assert _mlp(a_q=(1 << 20) + 8) == -3 and _mlp(gamma_q=(48 << 20) + 2) == -3
    assert _mlp(ws=None) == -4 and _mlp(ws_bytes=1024) == -4
    assert _mlp(out=1 << 20) == -7 and _mlp(ws=5 << 20) == -7
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 8, 2097152, 40, 1) > 0
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 8, 64, 56, 1) > 0       # per-head kernels + statistics
    assert lf.linfusion_attn_mlp_workspace_bytes(1, 8, 64, 72, 1) == 0


def _mlps(sin=None, sout=None, B=2, N=64, out=40 << 20, **kw):
    """Raw C call of linfusion_attn_fwd_mlp_strided; the five inputs interleave in one [B, N, 5 C] buffer."""
    C = 320
    arr = lambda s: None if s is None else ctypes.byref((ctypes.c_longlong * 2)(*s))
    base = 1 << 20
    a = dict(H=8, d=40, dtype=1, fm=0, eps=1e-6, ln_eps=1e-5, slope=0.01, flags=0)
    a.update(kw)
    return lf.library().linfusion_attn_fwd_mlp_strided(
        base, base + 2 * C, base + 4 * C, base + 6 * C, base + 8 * C, out, 48 << 20, 49 << 20, 50 << 20, 51 << 20, B,
        a["H"], N, a["d"], a["dtype"], a["fm"], a["eps"], a["ln_eps"], a["slope"], a["flags"], arr(sin), arr(sout),
        64 << 20, 4 << 20, None, None)


@fake_addresses
def test_strided_mlp_entry_validates_on_the_host():
    import torch
    ok = -6 if not torch.cuda.is_available() else None
    C, N = 320, 64
    inter = (N * 5 * C, 5 * C)
    if ok is not None:
        assert _mlps(inter, None) == ok and _mlps(inter, (N * 2 * C, 2 * C)) == ok
        assert _mlps(inter, None, B=1, N=1) == ok
    assert _mlps((N * 5 * C, 5 * C + 4), None) == -3 and _mlps(inter, (N * C + 4, C)) == -3     # 16-byte rows
    assert _mlps((N * 5 * C, -8), None) == -1 and _mlps((N * 5 * C, C - 8), None) == -1         # rows too short
    assert _mlps(inter, (N * C, C - 8)) == -7 and _mlps(inter, (N * C - 8, C)) == -7            # out rows intersect
    assert _mlps(inter, (0, C)) == -7
    assert _mlps((N * 5 * C, 8 << 27), None) == -1 and _mlps((1 << 46, 5 * C), None) == -1      # index ranges
    # the inputs' extent is that of the wide buffer: an out inside it is caught, one behind it is not
    assert _mlps(inter, None, out=(1 << 20) + 2 * (2 * N * 5 * C) - 64) == -7
    if ok is not None:
        assert _mlps(inter, None, out=(1 << 20) + 2 * (2 * N * 5 * C) + 8 * C * 2) == ok
    assert _mlps(inter, None, flags=2) == -1 and _mlps(inter, None, H=8, d=72) == -2


def _qv(B=1, H=2, N=64, dk=80, dv=40, dtype=1, fm=0, eps=1e-6, flags=0, q=1 << 20, out=4 << 20, ws=64 << 20,
        ws_bytes=4 << 20):
    return lf.library().linfusion_attn_fwd_qv(q, 2 << 20, 3 << 20, out, B, H, N, dk, dv, dtype, fm, eps, flags, ws,
                                              ws_bytes, None, None)


@fake_addresses
def test_unequal_width_entry_validates_on_the_host():
    import torch
    ok = -6 if not torch.cuda.is_available() else None
    if ok is not None:
        assert _qv() == ok and _qv(dk=16, dv=64, dtype=2) == ok
    assert _qv(q=None) == -1 and _qv(out=None) == -1 and _qv(N=0) == -1 and _qv(eps=float("nan")) == -1
    assert _qv(flags=4) == -1
    assert _qv(dk=40, dv=40) == -2 and _qv(dk=24) == -2 and _qv(dv=48) == -2 and _qv(dtype=0) == -2 and _qv(fm=3) == -2
    assert _qv(q=(1 << 20) + 4) == -3
    assert _qv(ws=None) == -4 and _qv(ws_bytes=64) == -4
    assert _qv(out=3 << 20) == -7 and _qv(ws=4 << 20) == -7
    # q and k are d_qk wide: an out placed right behind v's span but inside q's is caught with the right widths
    assert _qv(q=1 << 20, out=(1 << 20) + 64 * 2 * 80 * 2 - 16) == -7
    assert lf.linfusion_attn_qv_workspace_bytes(2, 8, 4096, 80, 40, 1) > 0


def _bwds(strides=(None,) * 5, B=1, H=2, N=64, d=40, dq=5 << 20, dk=6 << 20, dv=7 << 20, ws=64 << 20, ws_bytes=4 << 20):
    arr = lambda s: None if s is None else ctypes.byref((ctypes.c_longlong * 3)(*s))
    return lf.library().linfusion_attn_bwd_strided(1 << 20, 2 << 20, 3 << 20, 4 << 20, None, dq, dk, dv, B, H, N, d, 1, 0,
                                                   1e-6, 0, *[arr(s) for s in strides], ws, ws_bytes, None)


@fake_addresses
def test_strided_backward_validates_on_the_host():
    import torch
    ok = -6 if not torch.cuda.is_available() else None
    dense, tm = (2 * 64 * 40, 64 * 40, 40), (64 * 2 * 40, 40, 2 * 40)
    if ok is not None:
        assert _bwds() == ok and _bwds((tm,) * 5) == ok and _bwds((dense, tm, dense, tm, dense)) == ok
    assert _bwds((dense, dense, dense, (2 * 64 * 40, 64 * 40, 44), dense)) == -3        # dq rows not 16-byte aligned
    assert _bwds((dense, dense, dense, (2 * 64 * 40, 0, 40), dense)) == -7              # dq heads on top of each other
    assert _bwds((dense, (2 * 64 * 40, 0, 40), dense, dense, dense)) in (-6, ok)        # inputs may repeat
    assert _bwds(dk=5 << 20) == -7 and _bwds(dq=1 << 20) == -7 and _bwds(ws=7 << 20) == -7
    assert _bwds(ws_bytes=128) == -4
