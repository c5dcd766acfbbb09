"""The library allocates nothing, never synchronises and clears its scratch with
kernels, so a whole decode cycle (draft + scores + table, then verification) can be
captured into a HIP graph.  Every replay is checked against the eager result, with
eager work and synchronisations of the same head between replays."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi

from gpu_util import make_head

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("family", ["cp", "hmm", "btree"])
def test_decode_cycle_replays_from_a_graph(family):
    B, n, r, v = 8, 8, 16, 320
    inp = mi.make_inputs(family, B=B, d=512, n=n, r=r, v=v, dtype="bf16", seed=41, h_scale=1.0)
    head = make_head(inp)
    dev = "cuda"
    pver = torch.from_numpy(mi.verifier_noise(B, n, v, seed=2, peak=1.0).astype(np.float32)).to(dev)
    table = torch.empty(B, n, r, v, dtype=torch.float32, device=dev)

    def cycle(out, tab):
        d, l, s = head.sample(1, seed=5, offset=2, want_prefix=True, out=out, logphi=tab)
        return head.verify(d[:, 0], pver, prefix_logq=s[:, 0], logphi=tab, seed=5, offset=3)

    def buffers():
        nl = {"cp": 1, "hmm": n, "btree": n - 1}[family]
        return (torch.empty(B, 1, n, dtype=torch.int32, device=dev), torch.empty(B, 1, nl, dtype=torch.int32, device=dev),
                torch.empty(B, 1, n, dtype=torch.float32, device=dev))

    out_e = buffers()
    acc_e, tok_e = cycle(out_e, table)                     # eager reference (also sizes the workspace)
    torch.cuda.synchronize()
    out_g, table_g = buffers(), torch.empty_like(table)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cycle(out_g, table_g)                              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        acc_g, tok_g = cycle(out_g, table_g)
    tg = torch.from_numpy(inp.targets).cuda()
    for k in range(4):
        for t in out_g:
            t.zero_()
        acc_g.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g[0], out_e[0]) and torch.equal(out_g[2], out_e[2]), k
        assert torch.equal(acc_g, acc_e) and torch.equal(tok_g, tok_e), k
        assert torch.equal(table_g, table), k
        head.loglik(tg)                                    # eager work on the same head and workspace
        torch.cuda.synchronize()
