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


@pytest.mark.parametrize("family", ["cp", "hmm"])
def test_training_sized_step_replays_from_a_graph(family):
    """Drafts through the buckets (their counters are cleared by a kernel, atomics decide only
    the order inside a bucket) and the fused scoring of targets and drafts."""
    B, n, r, v = 300, 4, 8, 268
    inp = mi.make_inputs(family, B=B, d=256, n=n, r=r, v=v, dtype="bf16", seed=43, h_scale=1.0)
    head = make_head(inp)
    dev = "cuda"
    tg = torch.from_numpy(inp.targets).cuda().view(B, 1, n)
    nl = {"cp": 1, "hmm": n}[family]

    def buffers():
        return ((torch.empty(B, 2, n, dtype=torch.int32, device=dev), torch.empty(B, 2, nl, dtype=torch.int32, device=dev), None),
                torch.empty(B, 3, n, dtype=torch.float32, device=dev))

    def step(out, P):
        d, _, _ = head.sample(2, seed=8, offset=1, out=out)
        head.window_scores(tg, d, prefix=True, out=P)

    out_e, P_e = buffers()
    step(out_e, P_e)
    torch.cuda.synchronize()
    out_g, P_g = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(out_g, P_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(out_g, P_g)
    for k in range(4):
        out_g[0].zero_()
        P_g.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g[0], out_e[0]) and torch.equal(out_g[1], out_e[1]), k
        assert torch.equal(P_g, P_e), k
        head.loglik(tg[:, 0].contiguous())                 # eager work on the same head and workspace
        torch.cuda.synchronize()


@pytest.mark.parametrize("family", ["cp", "btree"])
def test_greedy_cycle_of_a_few_positions_replays_from_a_graph(family):
    """Greedy draft without scores (only the slabs the draft selects are read) + greedy verification."""
    B, n, r, v = 2, 8, 16, 300
    inp = mi.make_inputs(family, B=B, d=256, n=n, r=r, v=v, dtype="bf16", seed=47, h_scale=1.0)
    head = make_head(inp)
    dev = "cuda"
    pver = torch.from_numpy(mi.verifier_noise(B, n, v, seed=3, peak=1.0).astype(np.float32)).to(dev)

    def cycle():
        g, _, _ = head.greedy_draft(want_latents=False)
        acc, tok = head.verify(g, pver, mode="greedy")
        return g, acc, tok

    g_e, acc_e, tok_e = cycle()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cycle()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g_g, acc_g, tok_g = cycle()
    tg = torch.from_numpy(inp.targets).cuda()
    for k in range(4):
        g_g.zero_()
        acc_g.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_g, g_e) and torch.equal(acc_g, acc_e) and torch.equal(tok_g, tok_e), k
        head.loglik(tg)                                    # eager work on the same head and workspace
        torch.cuda.synchronize()
