#!/usr/bin/env python3
"""Benchmark of the ASL per-layer token-importance pass on one MI355X.

One "step" = the whole hot path for one layer of the headline workload (8B shape, 128K context,
window 32, pool 7, budget 2048) with inputs resident in HBM: asl_score_layer (two passes over K:
row statistics + column sums, then pooling), asl_rank_stat (RankDesc into the ring + the rank-
variance statistic over a full 8-row ring), asl_select_topk on the Hk per-head rows and the all-head row, and asl_gather_kv of K and V.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|5] [--lse] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
# HBM traffic of one launch of the pass-2 kernel at workload C3, from two rocprofv3 --pmc runs
# (profiles/hot_path_c3_128k_counters.md): FETCH_SIZE 131260.0 and WRITE_SIZE 4095.0 KiB-units per
# dispatch, scaled by what the same counters read for a 256 MiB copy (x2.0 and x1.0).
PMC_TRAFFIC_BYTES = {3: int((131260.0 * 2.0 + 4095.0 * 1.0) * 1024)}
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16


def attention_lse(q, k, sh):
    """Input preparation for the one-pass mode: the natural-log sum-exp of every window row's
    scaled, causally masked logits, [Hq, W] fp32.  In a prefill this comes out of the layer's
    attention kernel; here plain torch ops stand in for that kernel (not part of the timed path)."""
    import torch
    G, W, N, T = sh.G, sh.W, sh.N, sh.T
    out = torch.empty((sh.Hq, W), dtype=torch.float32, device=q.device)
    causal = torch.ones((W, W), dtype=torch.bool, device=q.device).triu(1)     # key index > row index
    for h in range(sh.Hq):
        logits = (q[h].float() @ k[h // G].float().T) * sh.scale              # [W, N]
        logits[:, T:].masked_fill_(causal, float("-inf"))
        out[h] = torch.logsumexp(logits, dim=1)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 5])
    ap.add_argument("--lse", action="store_true", help="hand the rows' log-sum-exp to the scorer (one K pass)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-lse-leg", action="store_true", help="skip the extra timed region with lse supplied")
    ap.add_argument("--eager", action="store_true", help="time eager launches instead of HIP-graph replay")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run a plain 256 MiB device copy (a reference of known traffic for counter runs)")
    ap.add_argument("--one-stream", action="store_true", help="no fork: rank/statistic and top-k/gather back to back")
    ap.add_argument("--defer-join", action="store_true",
                    help="leave a step's top-k + compaction on the second stream while the next step scores "
                         "(ASL_FLAG_DEFER_JOIN); by default every step joins before it returns")
    ap.add_argument("--no-batched-gather", action="store_true", help="skip the 32-layer batched KV-compaction leg")
    ap.add_argument("--breakdown", action="store_true", help="also time every kernel with events (untimed extra loop)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2601_07667_amd import asl, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    L = synth.config_layer(args.config)
    sh = L.shape
    ctx = asl.Asl(sh.N, sh.Hk + 1, sh.Hq * sh.W)
    p = asl.make_params(sh.Hq, sh.Hk, sh.d, sh.N, sh.W, sh.S, sh.budget)
    # steps that leave their top-k + compaction running on the second stream while the next step scores
    p_defer = asl.make_params(sh.Hq, sh.Hk, sh.d, sh.N, sh.W, sh.S, sh.budget, flags=asl.ASL_FLAG_DEFER_JOIN)
    up = lambda x: torch.from_numpy(x).to(dev).to(torch.bfloat16).contiguous()
    q, k, v = up(L.q_obs), up(L.k), up(L.v)
    # Every layer of a real prefill has its own K/V, so consecutive steps must not find the previous
    # step's K in the last-level cache: the steps cycle through N_SETS separately allocated K/V
    # copies (each rolled along the token axis), about 0.5 GB per set at 128K.
    N_SETS = 4
    ks = [k] + [torch.roll(k, shifts=1000 * j, dims=1).contiguous() for j in range(1, N_SETS)]
    vs = [v] + [torch.roll(v, shifts=1000 * j, dims=1).contiguous() for j in range(1, N_SETS)]
    T, n_idx = sh.T, sh.k + sh.W
    # P [Hk,T] and s [T] share one allocation so that one top-k call covers the Hk per-head rows
    # (Alg. 1) and the all-head row (Alg. 2) together
    PS = torch.empty((sh.Hk + 1, T), dtype=torch.float32, device=dev)
    P, s = PS[:sh.Hk], PS[sh.Hk]
    ring = torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev)
    state, stat = asl.new_state(dev), asl.new_stat(dev)
    I = torch.empty((sh.Hk + 1, n_idx), dtype=torch.int32, device=dev)   # rows 0..Hk-1 per head, row Hk all-head
    Kc = torch.empty((sh.Hk, n_idx, sh.d), dtype=torch.bfloat16, device=dev)
    Vc = torch.empty_like(Kc)
    lses = [None] * N_SETS
    if args.lse:
        for j in range(N_SETS):
            lses[j] = attention_lse(q, ks[j], sh)
    lse = lses[0]

    # Fill the rank ring with L_obs-1 earlier "layers" (perturbed scores) so that every timed step
    # evaluates the statistic over a full ring; tau = 0 never selects, so the ring stays full.
    ctx.asl_score_layer(p, q, k, P, s, lse=lse)
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    layer = 0
    for _ in range(sh.L_obs - 1):
        noisy = s * (1.0 + 0.05 * torch.randn(T, device=dev, generator=g))
        ctx.asl_rank_stat(p, noisy, layer, 0, sh.L_obs, 0.0, ring, state, stat)
        layer += 1
    torch.cuda.synchronize()

    # One step = asl_layer_step: scoring, then ranking + statistic on the launch stream while top-k
    # + KV compaction run on the context's second stream (both depend only on the scores and use
    # disjoint parts of the workspace), joined before the call returns.  --one-stream issues the
    # same work as four single calls back to back.
    def step(layer_idx: int) -> None:
        kk, vv = ks[layer_idx % N_SETS], vs[layer_idx % N_SETS]
        if args.one_stream:
            ctx.asl_score_layer(p, q, kk, P, s, lse=lses[layer_idx % N_SETS])
            ctx.asl_rank_stat(p, s, layer_idx, 0, sh.L_obs, 0.0, ring, state, stat)
            ctx.asl_select_topk(p, PS, sh.Hk + 1, I)
            ctx.asl_gather_kv(p, kk, vv, I, sh.Hk, n_idx, Kc, Vc)
        else:
            ctx.asl_layer_step(p_defer if args.defer_join else p, q, kk, vv, layer_idx, 0, sh.L_obs, 0.0, PS,
                               ring, state, stat, I, Kc, Vc, lse=lses[layer_idx % N_SETS])

    for _ in range(args.warmup):
        step(layer)
        layer += 1
    ctx.asl_join()
    torch.cuda.synchronize()
    if args.copy_ref:
        # 64 Mi fp32 elements = 256 MiB read + 256 MiB written by one elementwise copy kernel
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Timed region: exactly `steps` steps.  By default the steps are replayed from a HIP graph that
    # holds L_obs consecutive layers (one trip round the rank ring), which takes the host's launch
    # cost out of the measurement; --eager launches every kernel from Python instead.
    use_graph = not args.eager
    if use_graph and (args.steps % sh.L_obs != 0 or args.steps < sh.L_obs):
        print(f"bench.py: --steps {args.steps} is not a multiple of L_obs={sh.L_obs} (one graph holds L_obs "
              f"layers): timing eager launches instead", file=sys.stderr)
        use_graph = False
    if use_graph:
        layer = ((layer + sh.L_obs - 1) // sh.L_obs) * sh.L_obs      # graph starts on ring row 0
        cap_stream = torch.cuda.Stream()
        cap_stream.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(cap_stream):
            # bring the ring in phase with the graph's first layer, then capture one trip
            while asl.read_struct(state, asl.AslState).last_layer % sh.L_obs != sh.L_obs - 1:
                nxt = asl.read_struct(state, asl.AslState).last_layer + 1
                step(nxt)
                ctx.asl_join()
                torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=cap_stream):
                for j in range(sh.L_obs):
                    step(layer + j)
                ctx.asl_join()                         # a capture must end with every forked stream joined
            for _ in range(2):
                graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // sh.L_obs):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(layer)
            layer += 1
        ctx.asl_join()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    st = asl.read_struct(stat, asl.AslStat)
    assert st.evaluated == 1 and st.n_rows == sh.L_obs, "statistic was not evaluated over a full ring"

    # Duration of the dominant kernel (pass-2 column sums): HIP events recorded by the library on
    # the launch stream around that kernel alone, in an eager loop of the same `steps` steps run
    # right after the timed region (events cannot bracket a single node of a replayed graph).
    DOM = asl.KERNEL_NAMES.index("score_colsum")
    ctx.asl_profile_enable(1 << DOM, args.steps)
    layer = asl.read_struct(state, asl.AslState).last_layer + 1
    torch.cuda.synchronize()
    e0 = time.perf_counter()
    for _ in range(args.steps):
        step(layer)
        layer += 1
    ctx.asl_join()
    torch.cuda.synchronize()
    e1 = time.perf_counter()
    dom_ms, dom_n = ctx.asl_profile_collect(DOM)
    ctx.asl_profile_enable(0, 0)
    eager_ms_per_step = (e1 - e0) * 1e3 / args.steps

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = sh.N / (ms_per_step * 1e-3)

    # Extra leg: the same steps with the rows' log-sum-exp handed over (what the layer's attention
    # kernel already has), so K is streamed once per layer instead of twice.  Eager launches.
    lse_leg = None
    if not args.lse and not args.no_lse_leg:
        for j in range(N_SETS):
            lses[j] = attention_lse(q, ks[j], sh)
        for _ in range(8):
            step(layer)
            layer += 1
        ctx.asl_join()
        torch.cuda.synchronize()
        l0 = time.perf_counter()
        for _ in range(args.steps):
            step(layer)
            layer += 1
        ctx.asl_join()
        torch.cuda.synchronize()
        l1 = time.perf_counter()
        lse_ms = (l1 - l0) * 1e3 / args.steps
        lse_leg = {"ms_per_step": round(lse_ms, 5), "value": round(sh.N / (lse_ms * 1e-3), 1),
                   "note": "lse [Hq,W] supplied by the caller: one pass over K"}
        lses = [None] * N_SETS

    # Extra leg: a layer before the selection layer only scores, ranks and evaluates the statistic
    # (no top-k, no compaction).  Eager launches of the two single calls.
    ordinary_leg = None
    if not args.no_lse_leg:
        def ordinary(layer_idx: int) -> None:
            ctx.asl_score_layer(p, q, ks[layer_idx % N_SETS], P, s)
            ctx.asl_rank_stat(p, s, layer_idx, 0, sh.L_obs, 0.0, ring, state, stat)
        for _ in range(8):
            ordinary(layer)
            layer += 1
        torch.cuda.synchronize()
        o0 = time.perf_counter()
        for _ in range(args.steps):
            ordinary(layer)
            layer += 1
        torch.cuda.synchronize()
        o_ms = (time.perf_counter() - o0) * 1e3 / args.steps
        ordinary_leg = {"ms_per_step": round(o_ms, 5), "value": round(sh.N / (o_ms * 1e-3), 1),
                        "note": "score + pool + rank + statistic only (a layer that does not select), eager"}

    # Extra leg: the same step on ONE K/V copy every time ("warm": whatever part of K the last-level
    # cache keeps between layers is found there; at 128K K alone is larger than that cache).
    warm_leg = None
    if not args.no_lse_leg:
        def warm_step(layer_idx: int) -> None:
            ctx.asl_layer_step(p, q, ks[0], vs[0], layer_idx, 0, sh.L_obs, 0.0, PS, ring, state, stat, I, Kc, Vc)
        for _ in range(8):
            warm_step(layer)
            layer += 1
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        for _ in range(args.steps):
            warm_step(layer)
            layer += 1
        torch.cuda.synchronize()
        w_ms = (time.perf_counter() - w0) * 1e3 / args.steps
        warm_leg = {"ms_per_step": round(w_ms, 5), "value": round(sh.N / (w_ms * 1e-3), 1),
                    "note": "same K/V copy every step (not cold), eager"}

    # Algorithmic HBM bytes of one pass-2 launch: every past key once (bf16), the window queries,
    # and the group-summed column sums written once.
    eb = 2
    dom_bytes = sh.Hk * T * sh.d * eb + sh.Hq * sh.W * sh.d * eb + sh.Hk * T * 4
    dom_avg_ms = dom_ms / max(dom_n, 1)
    dom_gbs = dom_bytes / (dom_avg_ms * 1e-3) / 1e9
    useful_flops = 2.0 * sh.Hq * sh.W * sh.N * sh.d          # one QK^T over the window rows
    roofline = {"bound": "hbm", "kernel": "score_colsum_kernel (pass 2)", "achieved": round(dom_gbs, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                "traffic": PMC_TRAFFIC_BYTES.get(args.config), "avg_launch_ms": round(dom_avg_ms, 5), "launches": dom_n,
                "timing": "HIP events around this kernel, eager loop of the same steps after the timed region",
                "algorithmic_bytes": dom_bytes,
                "mfma_tflops": round(useful_flops / (dom_avg_ms * 1e-3) / 1e12, 1),
                "mfma_frac_of_bf16_peak": round(useful_flops / (dom_avg_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}

    kernels = None
    if args.breakdown:
        n_b = max(10, min(50, args.steps))
        ctx.asl_profile_enable((1 << len(asl.KERNEL_NAMES)) - 1, 64 * n_b)
        for _ in range(n_b):
            step(layer)
            layer += 1
        ctx.asl_join()
        torch.cuda.synchronize()
        kernels = {}
        for i, name in enumerate(asl.KERNEL_NAMES):
            try:
                ms, n = ctx.asl_profile_collect(i)
            except asl.AslError:                              # an older library that lacks this kernel id
                continue
            if n:
                kernels[name] = {"us_per_step": round(ms * 1e3 / n_b, 2), "launches_per_step": n / n_b}
        ctx.asl_profile_enable(0, 0)

    # Bandwidth of the KV compaction where bandwidth, not launch latency, is the limit: one
    # asl_gather_kv call over 32 layers x Hk heads stacked as rows (what SnapKV-style compression of
    # every layer before the selection layer moves in total), indices from this layer's top-k.
    gather_leg = None
    if not args.no_batched_gather:
        n_layers = 32
        rows = n_layers * sh.Hk
        try:
            bctx = asl.Asl(sh.N, rows, n_layers * sh.Hq * sh.W)
            bp = asl.make_params(n_layers * sh.Hq, rows, sh.d, sh.N, sh.W, sh.S, sh.budget)
            k_all = torch.empty((rows, sh.N, sh.d), dtype=torch.bfloat16, device=dev).normal_()
            v_all = torch.empty((rows, sh.N, sh.d), dtype=torch.bfloat16, device=dev).normal_()
            idx_all = I[:sh.Hk].repeat(n_layers, 1).contiguous()
            ko = torch.empty((rows, n_idx, sh.d), dtype=torch.bfloat16, device=dev)
            vo = torch.empty_like(ko)
            GK = asl.KERNEL_NAMES.index("gather")
            for _ in range(3):
                bctx.asl_gather_kv(bp, k_all, v_all, idx_all, rows, n_idx, ko, vo)
            bctx.asl_profile_enable(1 << GK, 32)
            for _ in range(20):
                bctx.asl_gather_kv(bp, k_all, v_all, idx_all, rows, n_idx, ko, vo)
            torch.cuda.synchronize()
            g_ms, g_n = bctx.asl_profile_collect(GK)
            bctx.asl_profile_enable(0, 0)
            g_bytes = 2 * 2 * rows * n_idx * sh.d * 2 + rows * n_idx * 4      # K,V read + written, indices
            g_gbs = g_bytes / (g_ms / g_n * 1e-3) / 1e9
            gather_leg = {"layers": n_layers, "bytes": g_bytes, "avg_launch_ms": round(g_ms / g_n, 5),
                          "achieved_GBps": round(g_gbs, 1), "frac_of_hbm_peak": round(g_gbs / HBM_PEAK_GBS, 4)}
            del k_all, v_all, ko, vo
            bctx.close()
        except Exception as e:                                # noqa: BLE001 - report, do not hide the headline
            gather_leg = {"error": str(e)}

    cpu = None
    if not args.no_cpu:
        from oracle import asl_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        reps, t_cpu = 0, 0.0
        ost = orc.SelectState.new(sh.L_obs)
        rng = np.random.default_rng(0)
        while t_cpu < 12.0 and reps < 40:                     # bounded sample: whole layers, ~10-30 s
            c0 = time.perf_counter()
            out = orc.get_ranks(L.q_obs, L.k, L.v, sh.W, sh.S, sh.budget)
            ost.push(reps, out["rank"])
            orc.select_tokens(ost, reps, sh.budget, sh.W, 0, 0.0)
            orc.select_indices(out["s"], out["k"], sh.W)
            t_cpu += time.perf_counter() - c0
            reps += 1
        cpu = {"value": round(sh.N * reps / t_cpu, 1), "unit": "KV tokens/s per layer", "cores": cores,
               "kind": "oracle", "sample": f"{reps} whole layer(s) of the same workload, float64 numpy "
               f"(score+pool+rank+statistic+per-head top-k+gather), {t_cpu:.1f} s"}

    workload = {2: "C2: Llama-3-8B shape, N=32768, W=32, S=7, budget 2048, bf16 N(0,1)",
                3: "C3: Llama-3-8B shape (Hq32/Hk8/d128), N=131072, W=32, S=7, budget 2048, bf16 N(0,1) + 64 needles",
                5: "C5: Llama-3-8B shape, N=262144, W=64, S=7, budget 4096, heavy-tailed keys + 256 needles"}
    line = {
        "metric": "KV tokens scored+selected/sec per layer @128K (8B shape)" if args.config == 3
                  else f"KV tokens scored+selected/sec per layer @N={sh.N} (8B shape)",
        "value": round(tokens_per_s, 1), "unit": "KV tokens/s per layer", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (seeded numpy PCG64, bf16-rounded), resident in HBM; steps cycle through 4 K/V copies",
        "config": {"workload": workload[args.config], "seq_len": sh.N, "window": sh.W, "pool_kernel": sh.S,
                   "budget": sh.budget, "L_obs": sh.L_obs,
                   "score_mode": "lse supplied (one K pass)" if args.lse else "self-contained (two K passes)",
                   "launch": ("HIP graph replay (8 layers per graph)" if use_graph else "eager launches from Python")
                             + ("" if args.one_stream else "; rank+statistic and top-k+gather on two streams")
                             + ("" if (args.one_stream or not args.defer_join) else
                                "; a step's top-k+gather may still run while the next step scores (joined before its "
                                "scores are overwritten and at the end of the timed region)"),
                   "eager_ms_per_step": round(eager_ms_per_step, 5),
                   "step": "asl_layer_step = score_layer + rank_stat(full ring) + select_topk(Hk per-head rows + the all-head row) + gather_kv(K,V per head)"},
        "roofline": roofline, "cpu_baseline": cpu, "lse_supplied": lse_leg,
        "ordinary_layer": ordinary_leg, "warm_k": warm_leg, "gather_batched": gather_leg,
    }
    if kernels is not None:
        line["kernels"] = kernels
    print(json.dumps(line))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
