"""The entry point that allocates nothing (linfusion_attn_fwd_static: scratch in a fixed array of the
library's device image) against the general entry point with a caller-owned workspace, through the C ABI.
Same kernels, same launch plan, so the outputs must agree bit for bit; two calls in a row, the second on a
smaller input (the array keeps the first call's contents), then a third with another dtype and width."""
import pytest
import torch

import paper_2409_02097_amd as lf
from paper_2409_02097_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def _reference(q, k, v, flags):
    B, H, N, d = q.shape
    code = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}[q.dtype]
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
    out = torch.full_like(q, float("nan"))
    lf.linfusion_attn_fwd_ex(q, k, v, out, lf.PHI_ELU_PLUS_ONE, wl.EPS, flags | lf.FLAG_FORCE_SPLIT, ws)
    torch.cuda.synchronize()
    return out


def test_static_scratch_entry_matches_the_general_entry_on_two_calls_in_a_row():
    assert lf.linfusion_attn_static_scratch_bytes() == 16 << 20
    lf.linfusion_init()
    cases = [(2, 8, 40000, 40, "f16", 0),            # several tiles per workgroup, ragged tail
             (1, 3, 1237, 40, "f16", 0),             # smaller input right after: stale partials beyond it
             (2, 5, 9216, 64, "bf16", lf.FLAG_UNNORMALIZED),
             (1, 8, 1024, 40, "f32", 0),
             (1, 2, 1, 8, "f16", 0)]
    for i, (B, H, N, d, dtype, flags) in enumerate(cases):
        q, k, v = wl.make_qkv(B, H, N, d, dtype, idx=40 + i, device="cuda")
        want = _reference(q, k, v, flags)
        out = torch.full_like(q, float("nan"))
        before = torch.cuda.memory_allocated()
        lf.linfusion_attn_fwd_static(q, k, v, out, lf.PHI_ELU_PLUS_ONE, wl.EPS, flags)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out.view(torch.uint8), want.view(torch.uint8)), f"case {i}: {B, H, N, d, dtype}"
        if i < 2:
            parity.check_all(out, q.cpu(), k.cpu(), v.cpu(), dtype, 0, wl.EPS, True, f"static scratch case {i}")


def test_static_scratch_entry_rejects_what_does_not_fit_and_bad_flags():
    q, k, v = wl.make_qkv(1, 2, 64, 40, "f16", idx=46, device="cuda")
    out = torch.empty_like(q)
    assert lf.linfusion_attn_fwd_static(q, k, v, out, 0, wl.EPS, lf.FLAG_FORCE_FUSED, check=False) == -1
    # 160-channel heads: the partial states of the wide kernels exceed the array
    q, k, v = wl.make_qkv(1, 8, 131072, 160, "f16", idx=47, device="cuda")
    out = torch.full_like(q, 7.0)
    assert lf.linfusion_attn_fwd_static(q, k, v, out, 0, wl.EPS, 0, check=False) == -4
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())        # nothing was enqueued
