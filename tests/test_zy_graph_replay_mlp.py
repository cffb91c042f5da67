"""HIP-graph capture of the MLP-fed call (kept in a file of its own, collected late: every replay is compared with
an eager call bit for bit, on new inputs, with the program's own eager work in between)."""
import pytest
import torch

import paper_2409_02097_amd as lf
from paper_2409_02097_amd import workloads as wl

pytestmark = pytest.mark.gpu

LN_EPS, SLOPE = 1e-5, 0.01


def _ws(B, H, N, d, dtype):
    n = lf.linfusion_attn_mlp_workspace_bytes(B, H, N, d, wl.DTYPE_CODE[dtype])
    assert n > 0
    return torch.empty(n, dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 8, 2000, 40, "f16"), (2, 10, 1500, 64, "bf16"), (1, 8, 700, 80, "f16"),
                                           (1, 8, 300, 160, "bf16")])
def test_recorded_into_a_graph_replays_correctly(B, H, N, d, dtype):
    """The MLP-fed call enqueues kernels only (on either route), so it can be captured; every replay (new inputs in
    the same buffers, eager work in between) must equal the eager result bit for bit."""
    dev = [t.cuda() for t in wl.make_mlp_inputs(B, H, N, d, dtype, idx=87)]
    out = torch.zeros_like(dev[0])
    ws = _ws(B, H, N, d, dtype)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lf.linfusion_attn_fwd_mlp(*dev[:5], out, *dev[5:], H, 0, 1e-6, LN_EPS, SLOPE, 0, ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lf.linfusion_attn_fwd_mlp(*dev[:5], out, *dev[5:], H, 0, 1e-6, LN_EPS, SLOPE, 0, ws,
                                  stream=torch.cuda.current_stream())
    for rep in range(3):
        fresh = [t.cuda() for t in wl.make_mlp_inputs(B, H, N, d, dtype, idx=88 + rep)]
        for dst, src in zip(dev, fresh):
            dst.copy_(src)
        out.fill_(float("nan"))
        torch.cuda.synchronize()      # the program's own eager work is complete before the replay starts
        graph.replay()
        torch.cuda.synchronize()
        eager = torch.empty_like(out)
        lf.linfusion_attn_fwd_mlp(*dev[:5], eager, *dev[5:], H, 0, 1e-6, LN_EPS, SLOPE, 0, _ws(B, H, N, d, dtype))
        torch.cuda.synchronize()
        if not torch.equal(out.view(torch.int16), eager.view(torch.int16)):
            # say what differs before failing: which rows, whether the eager call repeats itself, whether the replay does
            ne = (out.view(torch.int16) != eager.view(torch.int16)).nonzero()
            rows = sorted(set((ne[:, 0] * N + ne[:, 1]).tolist()))
            eager2 = torch.empty_like(out)
            lf.linfusion_attn_fwd_mlp(*dev[:5], eager2, *dev[5:], H, 0, 1e-6, LN_EPS, SLOPE, 0, _ws(B, H, N, d, dtype))
            first = out.clone()
            graph.replay()
            torch.cuda.synchronize()
            raise AssertionError(
                f"replay {rep}: {ne.shape[0]} elements in {len(rows)} rows differ from the eager call (rows {rows[:8]} .. "
                f"{rows[-3:]}); eager repeats itself: {torch.equal(eager.view(torch.int16), eager2.view(torch.int16))}; "
                f"replay repeats itself: {torch.equal(first.view(torch.int16), out.view(torch.int16))}; "
                f"second replay equals eager: {torch.equal(out.view(torch.int16), eager.view(torch.int16))}")
