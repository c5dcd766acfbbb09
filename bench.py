#!/usr/bin/env python3
"""Throughput of the MtPC head hot path on one MI355X.

Workload: the CP head of the second named configuration at full size - r=16, bf16 inputs with
fp32 accumulation, B=8192 positions, d=4096, n=8, v=320 - on seeded synthetic inputs
already resident in HBM.  One step = one pass of the whole hot path over the
batch: sum-unit parameters, one ancestral draft per position (latents, then each token
from the one input unit it is drawn from), then ONE fused pass (unembedding + log-softmax
+ gather) that scores the targets and the drafts, and the circuit layers with prefix
marginals of both (the last one is the log-likelihood).

Prints ONE JSON line (see the keys below).  `roofline` is for the dominant
kernel (the fused unembedding kernel of that scoring pass), timed with HIP
events recorded by the library right around its launch; `cpu_baseline` is the
float64 NumPy oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E
WORKLOAD = dict(family="cp", B=8192, d=4096, n=8, r=16, v=320)


class HipEvents:
    """hipEvent pairs through the HIP runtime (the events are recorded by libmtpc
    on the stream of the call, see mtpc_profile_unembed)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self):
        ev = C.c_void_p()
        assert self.hip.hipEventCreate(C.byref(ev)) == 0
        return ev

    def elapsed_ms(self, a, b):
        assert self.hip.hipEventSynchronize(b) == 0
        ms = C.c_float()
        assert self.hip.hipEventElapsedTime(C.byref(ms), a, b) == 0
        return float(ms.value)


def cpu_baseline(inp, rows: int, S: int, seed: int):
    """The oracle, as it stands, on the first `rows` positions of the workload."""
    import numpy as np
    from oracle import mtpc_oracle as oc
    from oracle import philox
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    h = inp.h[:rows]
    tg = inp.targets[:rows]
    t0 = time.perf_counter()
    logphi, logw, _ = oc._params(inp.family, h, inp.W, inp.Wsum, None)
    P = oc.prefix_marginals_from(inp.family, logphi, logw, None, tg)
    u = philox.uniforms(rows, S, inp.n + oc.n_latents(inp.family, inp.n), seed)
    drafts, lat = oc.sample_from(inp.family, logphi, logw, None, u)
    for s in range(S):
        oc.prefix_marginals_from(inp.family, logphi, logw, None, drafts[:, s])
    dt = time.perf_counter() - t0
    return {"value": rows / dt, "unit": "windows/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {rows} of {inp.B} positions, same W; loglik+prefix marginals+1 draft+draft scores; {dt:.1f} s"}, P


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--cpu-rows", type=int, default=8192)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-shaped (HBM-bound) side measurement")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run a plain 1 GiB device copy (known HBM traffic) to calibrate rocprofv3 counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import mtpc_inputs as mi
    from paper_2511_11346_amd import Head, binding, profile_unembed

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    t_gen = time.perf_counter()
    inp = mi.config2(r=WORKLOAD["r"], B=WORKLOAD["B"])
    as_bf16 = lambda bits: torch.from_numpy(bits).view(torch.bfloat16).to(dev)
    head = Head("cp", as_bf16(inp.h_bits), as_bf16(inp.W_bits), as_bf16(inp.Wsum_bits))
    tg = torch.from_numpy(inp.targets).to(dev)
    B, n, S = inp.B, inp.n, 1
    P = torch.empty(B, n, dtype=torch.float32, device=dev)
    drafts = torch.empty(B, S, n, dtype=torch.int32, device=dev)
    lat = torch.empty(B, S, 1, dtype=torch.int32, device=dev)
    pl = torch.empty(B, S, n, dtype=torch.float32, device=dev)
    tg3 = tg.view(B, 1, n)
    P2 = torch.empty(B, 1 + S, n, dtype=torch.float32, device=dev)
    # workspace sized once for the largest of the ops
    head._head(max(head.workspace_bytes(binding.OP_MARGINALS), head.workspace_bytes(binding.OP_SAMPLE, S=S),
                   head.workspace_bytes(binding.OP_WINDOWS, S=1 + S)))
    t_gen = time.perf_counter() - t_gen

    if args.copy_calib:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ev = HipEvents()

    def step(k, pairs=None):
        # drafts: latents, then each token from the one input unit it is drawn from (1/r of a pass
        # over W); then ONE fused pass scores the targets and the drafts of every position
        # (prefix marginals, the last of which is the log-likelihood)
        head.sample(S, seed=0, offset=k, out=(drafts, lat, None))
        if pairs is not None:
            profile_unembed(pairs[k][0], pairs[k][1])
        head.window_scores(tg3, drafts, prefix=True, out=P2)
        if pairs is not None:
            profile_unembed(None, None)

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    pairs = [(ev.create(), ev.create()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k, pairs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt * 1e3 / args.steps
    k1_ms = sum(ev.elapsed_ms(a, b) for a, b in pairs) / len(pairs)

    # per-op timings (outside the timed region, for the record)
    def time_op(fn, reps=10):
        fn(); torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps
    ms_marg = time_op(lambda: head.prefix_marginals(tg, out=P))
    ms_samp = time_op(lambda: head.sample(S, seed=0, out=(drafts, lat, pl)))
    ms_win = time_op(lambda: head.window_scores(tg3, drafts, prefix=True, out=P2))
    # the other route to the same results: one pass that leaves the table of normalised input
    # units log phi[B][n][r][v] (1.34 GB), from which tokens are drawn and windows scored
    table = torch.empty(B, n, inp.r, inp.v, dtype=torch.float32, device=dev)
    ms_samp_tab = time_op(lambda: head.sample(S, seed=0, out=(drafts, lat, pl), logphi=table))
    ms_tab = time_op(lambda: head.table_scores(table, tg, prefix=True, out=P))
    del table
    ms_samp_only = time_op(lambda: head.sample(S, seed=0, out=(drafts, lat, None)))
    uni = torch.empty(B, n, inp.v, dtype=torch.float32, device=dev)
    ms_uni = time_op(lambda: head.univariate_marginals(out=uni), 5)
    del uni

    flops = 2.0 * B * inp.n * inp.r * inp.v * inp.d
    # training step of the same workload (Sec. 4.1 loss + gradients w.r.t. h, W, Wsum): the forward
    # product (its probabilities are kept) and the two contractions = 3 passes of `flops`
    coef = (torch.full((B, n), 1.0 / B, device=dev) * 0.8 ** torch.arange(n, device=dev)).contiguous()
    grads = head.loss_backward(tg, coef)
    ms_train = time_op(lambda: head.loss_backward(tg, coef, out=grads), 5)
    del grads
    torch.cuda.empty_cache()
    achieved = flops / (k1_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "k_unembed (evidence of targets and drafts, the step's one pass over all of W)",
                "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS,
                # L2 <-> fabric bytes per launch of this kernel on this workload, from two rocprofv3
                # --pmc runs of this script (FETCH_SIZE 1,709,262 x 2 KiB, WRITE_SIZE 16,384 x 1 KiB,
                # factors calibrated on a 1 GiB device copy); reads served by the Infinity Cache count
                "traffic": 1709262 * 2048 + 16384 * 1024, "traffic_unit": "bytes/launch",
                "algorithmic_bytes": (B * inp.d + inp.n * inp.r * inp.v * inp.d) * 2 + (1 + S) * B * inp.n * inp.r * 4,
                "avg_launch_ms": k1_ms, "flop_per_launch": flops}

    out = {
        "metric": "MtPC head windows/sec (loglik + draft sample)",
        "value": B / (ms_step * 1e-3), "unit": "windows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: CP r=16, B=8192, d=4096, n=8, v=320, bf16 in / fp32 acc; "
                               "step = 1 draft per position (tokens drawn through buckets of their input unit) + prefix "
                               "marginals (last = loglik) of the targets and of the draft in one fused unembedding pass",
                   **WORKLOAD, "S": S},
        "roofline": roofline,
        "ops_ms": {"sample_only": ms_samp_only, "window_scores_targets_and_drafts": ms_win,
                   "prefix_marginals_call": ms_marg, "sample_with_scores": ms_samp,
                   "sample_with_scores_and_table": ms_samp_tab, "table_scores_of_targets": ms_tab,
                   "univariate_marginals_call": ms_uni},
        "loglik_windows_per_s": B / (ms_marg * 1e-3),
        "train_step": {"loss_backward_ms": ms_train, "windows_per_s": B / (ms_train * 1e-3),
                       "matrix_passes": 3, "TFLOPs": 3 * flops / (ms_train * 1e-3) / 1e12},
        "input_generation_s": t_gen,
    }
    # context for the roofline fraction: what the matrix pipes sustain on this machine with
    # register operands only (random data makes the chip hit its power limit)
    probe = os.path.join(ROOT, "paper_2511_11346_amd", "probes", "mfma_ceiling")
    if os.path.exists(probe):
        try:
            res = subprocess.run([probe], capture_output=True, text=True, timeout=120)
            roofline["register_only_mfma_ceiling"] = json.loads(res.stdout.strip().splitlines()[-1])
        except Exception as exc:                                   # the probe is optional context
            roofline["register_only_mfma_ceiling"] = {"error": str(exc)}

    if not args.no_decode:
        # side measurement (not part of `value`): the decode-shaped workload of configs[4]
        # - CP r=32, n=16, d=4096, v=320 - where the unembedding kernel streams the 1.34 GB
        # of W once and is bound by HBM; one call = 1 draft per position + its prefix scores
        del head
        torch.cuda.empty_cache()
        dec = []
        inp5 = mi.config5(B=64)
        W5 = as_bf16(inp5.W_bits)
        Ws5 = as_bf16(inp5.Wsum_bits)
        h5 = as_bf16(inp5.h_bits)
        for Bd in (1, 8, 64):
            hd = Head("cp", h5[:Bd].contiguous(), W5, Ws5)
            o = (torch.empty(Bd, 1, inp5.n, dtype=torch.int32, device=dev),
                 torch.empty(Bd, 1, 1, dtype=torch.int32, device=dev),
                 torch.empty(Bd, 1, inp5.n, dtype=torch.float32, device=dev))
            for k in range(3):
                hd.sample(1, seed=0, offset=k, out=o)
            torch.cuda.synchronize()
            reps = 20
            prs = [(ev.create(), ev.create()) for _ in range(reps)]
            t = time.perf_counter()
            for k in range(reps):
                profile_unembed(prs[k][0], prs[k][1])
                hd.sample(1, seed=0, offset=k, out=o)
                profile_unembed(None, None)
            torch.cuda.synchronize()
            call_ms = (time.perf_counter() - t) * 1e3 / reps
            kms = sum(ev.elapsed_ms(a, b) for a, b in prs) / reps
            # W streamed once, h, and the table of input units the sampling pass writes
            byts = inp5.n * inp5.r * inp5.v * inp5.d * 2 + Bd * inp5.d * 2 + Bd * inp5.n * inp5.r * inp5.v * 4
            # the verification step of the same cycle (Alg. 2): the sampler also keeps its
            # table of input units, then accept / reject against a synthetic verifier that is
            # 90 % the component each draft was drawn from and 10 % random tables
            table = torch.empty(Bd, inp5.n, inp5.r, inp5.v, dtype=torch.float32, device=dev)
            hd.sample(1, seed=0, offset=0, out=o, logphi=table)
            comp = o[1][:, 0, 0].long()
            q_comp = torch.exp(table[torch.arange(Bd, device=dev), :, comp, :])
            noise = torch.from_numpy(mi.verifier_noise(Bd, inp5.n, inp5.v, seed=9)).float().to(dev)
            pver = torch.cat([0.9 * q_comp + 0.1 * noise[:, :inp5.n], noise[:, inp5.n:]], dim=1)
            pver = (pver / pver.sum(-1, keepdim=True)).contiguous()
            dr, sc = o[0][:, 0].contiguous(), o[2][:, 0].contiguous()
            ms_table = time_op(lambda: hd.sample(1, seed=0, offset=0, out=o, logphi=table), reps)
            ms_verify = time_op(lambda: hd.verify(dr, pver, prefix_logq=sc, logphi=table, seed=1, offset=1), reps)
            acc, _ = hd.verify(dr, pver, prefix_logq=sc, logphi=table, seed=1, offset=1)
            # the workload's other reading of "16 verified prefixes per draft": 16 prefixes of random
            # length of each draft (later variables summed out), scored from the table
            gen = torch.Generator().manual_seed(16)
            lens = torch.randint(1, inp5.n + 1, (Bd, 16), generator=gen).to(dev)
            x16 = dr[:, None, :].repeat(1, 16, 1)
            x16[torch.arange(inp5.n, device=dev)[None, None, :] >= lens[:, :, None]] = -1
            x16 = x16.contiguous()
            ms_16 = time_op(lambda: hd.table_scores(table, x16), reps)
            # the same cycle (draft + scores + table, verification) replayed from a HIP graph
            def cycle():
                hd.sample(1, seed=0, offset=0, out=o, logphi=table)
                return hd.verify(o[0][:, 0], pver, prefix_logq=o[2][:, 0], logphi=table, seed=1, offset=1)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                cycle()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                cycle()
            ms_graph = time_op(graph.replay, reps)
            del graph
            # greedy speculative decoding (Sec. 3.4): the draft is the argmax traversal, a token
            # survives iff it is the verifier's argmax - no scores and no table are needed, so for
            # a handful of positions only the n slabs the draft selects are read
            # (synthetic verifier: the drafted component, with half of the mass moved onto the drafted
            # token at 9 of 10 places and onto a random token at the others)
            gdr, glat, _ = hd.greedy_draft()
            qg = torch.exp(table[torch.arange(Bd, device=dev), :, glat[:, 0].long(), :])
            gen = torch.Generator().manual_seed(17)
            agree = (torch.rand(Bd, inp5.n, generator=gen) < 0.9).to(dev)
            other = torch.randint(0, inp5.v, (Bd, inp5.n), generator=gen).to(dev)
            peak = torch.where(agree, gdr.long(), other)
            pverg = torch.cat([0.5 * qg + 0.5 * torch.nn.functional.one_hot(peak, inp5.v).float(), noise[:, inp5.n:]], dim=1)
            pverg = (pverg / pverg.sum(-1, keepdim=True)).contiguous()
            def greedy_cycle():
                g, _, _ = hd.greedy_draft(want_latents=False)
                return hd.verify(g, pverg, mode="greedy")
            ms_gdraft = time_op(lambda: hd.greedy_draft(want_latents=False), reps)
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                greedy_cycle()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            ggraph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(ggraph):
                gacc, _ = greedy_cycle()
            ms_ggraph = time_op(ggraph.replay, reps)
            mean_gacc = float(gacc.float().mean())
            del ggraph
            dec.append({"B": Bd, "call_ms": call_ms, "drafts_per_s": Bd / (call_ms * 1e-3),
                        "k_unembed_ms": kms, "achieved_GBps": byts / (kms * 1e-3) / 1e9,
                        "frac_of_hbm_peak": byts / (kms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                        "call_ms_keeping_table": ms_table, "verify_call_ms": ms_verify,
                        "cycle_ms_from_graph": ms_graph, "score_16_prefixes_per_draft_ms": ms_16,
                        "mean_accepted": float(acc.float().mean()),
                        "greedy_draft_call_ms": ms_gdraft, "greedy_cycle_ms_from_graph": ms_ggraph,
                        "greedy_mean_accepted": mean_gacc})
        out["decode_cp_r32_n16"] = dec

    if not args.no_cpu:
        base, P_cpu = cpu_baseline(inp, min(args.cpu_rows, B), S, seed=0)
        out["cpu_baseline"] = base
        err = float(np.max(np.abs(P[:P_cpu.shape[0]].cpu().numpy() - P_cpu)))
        out["max_abs_err_vs_oracle_on_sample"] = err
    print(json.dumps(out))


if __name__ == "__main__":
    main()
