"""The block calls enqueue kernels only (no allocation, no memset, no host synchronisation), so they can be recorded
into a HIP graph: a recorded forward + backward must reproduce the eager result bit for bit on every replay."""
import numpy as np
import pytest

from paper_2506_19645_amd import binding as B
from paper_2506_19645_amd import inputs as I
from tests.util import make_inputs

pytestmark = pytest.mark.gpu


def test_block_fwd_bwd_graph_replay_matches_eager():
    import torch
    cfg = I.C1
    d = make_inputs(cfg, seed=3)
    desc = B.make_desc(cfg)
    w = [B.to_device(d["A"]), B.to_device(d["B"]), B.to_device(d["gamma"]), B.to_device(d["beta"])]
    x, r = B.to_device(d["X"]), B.to_device(d["R"])
    dxo, dro = B.to_device(d["dXo"]), B.to_device(d["dRo"])
    outs = [torch.zeros_like(x) for _ in range(4)]          # r_out, x_out, dx, dr
    dw = [torch.zeros_like(w[0]), torch.zeros_like(w[1])]
    dg, db = torch.zeros(cfg.h, device="cuda"), torch.zeros(cfg.h, device="cuda")
    ws = torch.zeros(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")

    def step():
        B.block_fwd(desc, w, x, r, outs[0], outs[1], ws)
        B.block_bwd(desc, w, x, outs[0], ws, dxo, dro, outs[2], outs[3], dw, dg, db)

    def snapshot():
        torch.cuda.synchronize()
        return [B.to_host_bits(t).copy() for t in outs + dw] + [dg.cpu().numpy().copy(), db.cpu().numpy().copy()]

    step()                                                   # eager reference (also warms the library up)
    ref = snapshot()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                               # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for t in outs + dw + [dg, db]:
            t.zero_()                                        # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, ref):
            assert np.array_equal(a, b), "replay %d differs from the eager result" % rep
