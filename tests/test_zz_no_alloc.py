"""The entry point that allocates nothing (mtpc_sample_static: scratch in a static device array)
against the existing sampling entry points, through the C ABI: same arguments, results bit for
bit - two calls in a row, the second on a smaller input, then the rejection of a call whose
scratch does not fit."""
import numpy as np
import pytest
import torch

import mtpc_inputs as mi

from gpu_util import make_head

pytestmark = pytest.mark.gpu


def both_ways(inp, S, seed, offset, want_prefix, want_table):
    from paper_2511_11346_amd.binding import n_latents
    head = make_head(inp)
    B, n, r, v = inp.B, inp.n, inp.r, inp.v
    nl = n_latents(inp.family, n)
    dev = head.h.device

    def buffers():
        # filled with a pattern so that an output the call did not write would show
        return (torch.full((B, S, n), -7, dtype=torch.int32, device=dev),
                torch.full((B, S, nl), -7, dtype=torch.int32, device=dev),
                torch.full((B, S, n), 7.0, dtype=torch.float32, device=dev) if want_prefix else None,
                torch.full((B, n, r, v), 7.0, dtype=torch.float32, device=dev) if want_table else None)

    d0, l0, p0, t0 = buffers()
    head.sample(S, seed=seed, offset=offset, out=(d0, l0, p0), logphi=t0)
    d1, l1, p1, t1 = buffers()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    head.sample_static(S, seed, offset, d1, latents=l1, prefix_logq=p1, logphi=t1)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(d0, d1) and int(d1.min()) >= 0 and int(d1.max()) < v
    if nl:
        assert torch.equal(l0, l1) and int(l1.min()) >= 0
    if want_prefix:
        assert torch.equal(p0, p1) and bool(torch.all(p1 <= 0))
    if want_table:
        assert torch.equal(t0, t1)
    return head


def test_static_scratch_entry_point_matches_the_sampling_entry_points():
    # a decode-shaped call: draft + prefix scores + table of input units
    big = mi.make_inputs("hmm", B=48, d=256, n=16, r=32, v=320, dtype="bf16", seed=41, h_scale=1.0)
    both_ways(big, S=1, seed=5, offset=2, want_prefix=True, want_table=True)
    # right after it a smaller one of another family: the array still holds the first call's contents
    small = mi.make_inputs("btree", B=5, d=64, n=8, r=6, v=100, dtype="f32", seed=42, h_scale=1.0)
    both_ways(small, S=3, seed=6, offset=0, want_prefix=True, want_table=True)
    tiny = mi.make_inputs("cp", B=3, d=64, n=4, r=8, v=33, dtype="f32", seed=43, h_scale=1.0)
    both_ways(tiny, S=2, seed=7, offset=1, want_prefix=False, want_table=False)
    # more positions than a decode batch: the draws go through buckets kept in the scratch
    wide = mi.make_inputs("cp", B=300, d=64, n=4, r=8, v=200, dtype="bf16", seed=44, h_scale=1.0)
    both_ways(wide, S=2, seed=8, offset=3, want_prefix=True, want_table=False)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    from paper_2511_11346_amd.binding import MtpcError
    inp = mi.make_inputs("cp", B=64, d=64, n=16, r=32, v=320, dtype="bf16", seed=45, h_scale=1.0)
    head = make_head(inp)
    drafts = torch.full((64, 1, 16), -7, dtype=torch.int32, device="cuda")
    scores = torch.full((64, 1, 16), 7.0, dtype=torch.float32, device="cuda")
    # scores of a decode-sized batch without the caller's table: 42 MB of input units would have to
    # live in the 4 MiB array
    with pytest.raises(MtpcError, match="workspace"):
        head.sample_static(1, 0, 0, drafts, prefix_logq=scores)
    torch.cuda.synchronize()
    assert int(drafts.min()) == -7 and float(scores.min()) == 7.0      # nothing was launched
    # the same call with the table handed in fits
    table = torch.empty(64, 16, 32, 320, dtype=torch.float32, device="cuda")
    head.sample_static(1, 0, 0, drafts, prefix_logq=scores, logphi=table)
    ref = head.sample(1, seed=0, offset=0, want_prefix=True, logphi=torch.empty_like(table))
    assert torch.equal(ref[0], drafts) and torch.equal(ref[2], scores)
