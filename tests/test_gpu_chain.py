"""Chained GPU parity: the whole hot path (score -> pool -> rank -> statistic -> top-k -> gather)
from the same seeded Q/K/V as the oracle, through the C ABI, in the launch configuration the
benchmark times.  Floating-point scores are compared within tolerance; integer results are
compared exactly where the oracle's scores separate them by more than that tolerance."""
import numpy as np
import pytest

import gpu_util as gu
from oracle import asl_oracle as orc
from paper_2601_07667_amd import asl, synth

pytestmark = pytest.mark.gpu


def _rank_order_consistent(rank_gpu: np.ndarray, s_ref: np.ndarray, what: str):
    """Tokens taken in GPU rank order must have non-increasing oracle scores up to the score tolerance:
    a token may precede, in the GPU's order, only tokens whose oracle score exceeds its own by at most
    1e-5 + 2e-3 |score|."""
    T = s_ref.shape[0]
    assert np.array_equal(np.sort(rank_gpu), np.arange(T)), f"{what}: ranks are not a permutation"
    if T < 2:
        return
    order = np.empty(T, dtype=np.int64)
    order[rank_gpu] = np.arange(T)
    so = s_ref[order]
    prefmin = np.minimum.accumulate(so)
    tol = gu.ATOL + gu.RTOL * np.abs(so)
    excess = (so[1:] - prefmin[:-1]) / tol[1:]
    gu.note_margin(f"{what} rank-order inversion", max(float(excess.max()), 0.0))
    assert excess.max() <= 1.0, f"{what}: rank order contradicts oracle scores by {excess.max()} x tolerance"


def _pipeline(dev, L, layer_idx=0, ctx=None, state=None, ring=None, l_min=None, l_obs=None, tau=None):
    import torch
    sh = L.shape
    own = ctx is None
    ctx = ctx or gu.ctx_for(sh)
    p = gu.params_of(sh)
    l_obs = l_obs or sh.L_obs
    l_min = sh.L_min if l_min is None else l_min
    tau = sh.tau if tau is None else tau
    qd, kd, vd = (gu.to_dev(x, sh.dtype, dev) for x in (L.q_obs, L.k, L.v))
    P = torch.empty((sh.Hk, sh.T), dtype=torch.float32, device=dev)
    s = torch.empty((sh.T,), dtype=torch.float32, device=dev)
    ring = ring if ring is not None else torch.zeros((l_obs, sh.T), dtype=torch.int32, device=dev)
    state = state if state is not None else asl.new_state(dev)
    stat = asl.new_stat(dev)
    n_idx = sh.k + sh.W
    I_head = torch.empty((sh.Hk, n_idx), dtype=torch.int32, device=dev)
    I_all = torch.empty((1, n_idx), dtype=torch.int32, device=dev)
    Kc = torch.empty((sh.Hk, n_idx, sh.d), dtype=kd.dtype, device=dev)
    Vc = torch.empty_like(Kc)
    Ks = torch.empty_like(Kc)
    Vs = torch.empty_like(Kc)
    ctx.asl_score_layer(p, qd, kd, P, s)
    ctx.asl_rank_stat(p, s, layer_idx, l_min, l_obs, tau, ring, state, stat)
    ctx.asl_select_topk(p, P, sh.Hk, I_head)
    ctx.asl_gather_kv(p, kd, vd, I_head, sh.Hk, n_idx, Kc, Vc)
    ctx.asl_select_topk(p, s, 1, I_all)
    ctx.asl_gather_kv(p, kd, vd, I_all, 1, n_idx, Ks, Vs)
    out = dict(P=P.cpu().numpy(), s=s.cpu().numpy(), rank=ring[layer_idx % l_obs].cpu().numpy().astype(np.int64),
               stat=asl.read_struct(stat, asl.AslStat), I_head=I_head.cpu().numpy().astype(np.int64),
               I_all=I_all.cpu().numpy().astype(np.int64)[0], Kc=Kc.float().cpu().numpy(),
               Vc=Vc.float().cpu().numpy(), Ks=Ks.float().cpu().numpy(), Vs=Vs.float().cpu().numpy(),
               ring=ring, state=state)
    assert ctx.asl_device_fault() == 0, "a workgroup gave up waiting for its peers"
    if own:
        ctx.close()
    return out


def _check_layer(L, out):
    sh = L.shape
    ref = orc.get_ranks(L.q_obs, L.k, L.v, sh.W, sh.S, sh.budget)
    gu.assert_scores_close(out["P"], ref["P"], f"{L.name} P")
    gu.assert_scores_close(out["s"], ref["s"], f"{L.name} s")
    # ranks: exactly the oracle's RankDesc of the GPU's own fp32 scores, and consistent with the
    # oracle's scores wherever those separate two tokens by more than the tolerance
    np.testing.assert_array_equal(out["rank"], orc.rank_desc(out["s"].astype(np.float64)))
    _rank_order_consistent(out["rank"], ref["s"], L.name)
    k, W, T = sh.k, sh.W, sh.T
    n_diff = gu.check_topk_within_tolerance(out["I_all"], ref["s"], k, f"{L.name} all-head top-k")
    np.testing.assert_array_equal(out["I_all"][k:], np.arange(T, T + W))
    np.testing.assert_array_equal(out["I_all"][:k], np.nonzero(out["rank"] < k)[0])      # top-k == {rank < k}
    for g in range(sh.Hk):
        gu.check_topk_within_tolerance(out["I_head"][g], ref["P"][g], k, f"{L.name} head {g} top-k")
        np.testing.assert_array_equal(out["I_head"][g][k:], np.arange(T, T + W))
        # gathered KV is bit-exact given the GPU's own indices
        assert np.array_equal(out["Kc"][g], L.k[g][out["I_head"][g]])
        assert np.array_equal(out["Vc"][g], L.v[g][out["I_head"][g]])
        assert np.array_equal(out["Ks"][g], L.k[g][out["I_all"]])
        assert np.array_equal(out["Vs"][g], L.v[g][out["I_all"]])
    if len(L.needles):
        assert np.isin(L.needles, orc.topk_indices(ref["s"], k)).all(), "oracle does not recover the needles"
        assert np.isin(L.needles, out["I_all"]).all(), "GPU top-k misses planted needles"
    assert out["stat"].evaluated == 0                          # a single layer: nothing to evaluate yet
    return ref, n_diff


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_config_chain(gpu_device, cfg):
    L = synth.config_layer(cfg)
    print(f"chain {L.name}", flush=True)
    out = _pipeline(gpu_device, L)
    _check_layer(L, out)
    gu.report_margins(L.name)


def test_one_million_tokens(gpu_device):
    """A context four times the longest one of the paper's workloads (N = 2^20, two KV heads):
    every kernel runs with several thousand tiles per row and 64-bit offsets are exercised."""
    sh = synth.Shape(Hq=4, Hk=2, d=128, N=1 << 20, W=32, S=7, budget=8192)
    L = synth.iid_layer(sh, 77, name="1M")
    print("chain 1M", flush=True)
    _check_layer(L, _pipeline(gpu_device, L))


@pytest.mark.parametrize("N,W,budget", [(17, 16, 64), (40, 8, 4096), (65, 64, 65)])
def test_degenerate_sizes_chain(gpu_device, N, W, budget):
    """One past token (T = 1), a budget above the sequence length (everything is kept) and
    k = 1: the whole chain on shapes where every stage degenerates."""
    sh = synth.Shape(Hq=4, Hk=2, d=64, N=N, W=W, S=7, budget=budget)
    L = synth.iid_layer(sh, N, name=f"tiny-{N}-{W}-{budget}")
    out = _pipeline(gpu_device, L)
    _check_layer(L, out)
    if budget >= N:
        np.testing.assert_array_equal(out["I_all"], np.arange(N))


def test_config1_bf16_chain(gpu_device):
    sh = synth.shape_of(1)
    sh.dtype = "bf16"
    L = synth.iid_layer(sh, synth.BASE_SEED + 1, name="C1-bf16")
    _check_layer(L, _pipeline(gpu_device, L))


def test_config3_literal_needles_are_not_recoverable(gpu_device):
    """At the stated gain 4 a needle scores below an average token: the oracle does not rank them
    in the top-k and neither may the GPU (reported, not a defect of either side)."""
    L = synth.config_layer(3, strong_needles=False)
    sh = L.shape
    import torch
    ctx = gu.ctx_for(sh)
    p = gu.params_of(sh)
    P = torch.empty((sh.Hk, sh.T), dtype=torch.float32, device=gpu_device)
    s = torch.empty((sh.T,), dtype=torch.float32, device=gpu_device)
    ctx.asl_score_layer(p, gu.to_dev(L.q_obs, "bf16", gpu_device), gu.to_dev(L.k, "bf16", gpu_device), P, s)
    I = torch.empty((1, sh.k + sh.W), dtype=torch.int32, device=gpu_device)
    ctx.asl_select_topk(p, s, 1, I)
    _, s_ref = orc.score_layer(L.q_obs, L.k, sh.W, sh.S)
    gu.assert_scores_close(s.cpu().numpy(), s_ref, "literal needles s")
    in_ref = np.isin(L.needles, orc.topk_indices(s_ref, sh.k)).sum()
    in_gpu = np.isin(L.needles, I.cpu().numpy()[0]).sum()
    assert in_ref == in_gpu == 0
    ctx.close()


def _sweep_through_pipeline(dev, tau, rho_end, what):
    """The 32-layer sweep through the whole pipeline.  Returns the oracle's selection layer after
    asserting that the GPU agrees with it at every layer.
    The chained statistic is not a score: it depends on the ranks of tens of thousands of tokens
    whose scores are closer together than the score tolerance, so GPU and oracle ranks (hence
    var_top) legitimately differ a little.  The decision must be identical wherever the oracle's
    relative variance is at least 1e-3 away from tau (asserted first); the statistic itself is
    compared at 2 % relative as a sanity bound and the worst observed deviation is printed.  Its
    exactness is established by the stage-isolated tests, which feed identical ranks to both sides."""
    import torch
    sh = synth.shape_of(4)
    z = synth.sweep_latents(sh.T, sh.n_layers, rho_end=rho_end)
    ctx = gu.ctx_for(sh)
    ring = torch.zeros((sh.L_obs, sh.T), dtype=torch.int32, device=dev)
    state = asl.new_state(dev)
    ost = orc.SelectState.new(sh.L_obs)
    sel_gpu = sel_ref = None
    rel_ref, rel_gpu = {}, {}
    worst_rel = 0.0
    for l in range(sh.n_layers):
        L = synth.sweep_layer(sh, z[l], l)
        out = _pipeline(dev, L, layer_idx=l, ctx=ctx, state=state, ring=ring, tau=tau)
        _, s_ref = orc.score_layer(L.q_obs, L.k, sh.W, sh.S)
        gu.assert_scores_close(out["s"], s_ref, f"{what} s")
        ost.push(l, orc.rank_desc(s_ref))
        d = orc.select_tokens(ost, l, sh.budget, sh.W, sh.L_min, tau)
        st = out["stat"]
        print(f"{what} layer {l}: oracle rel={d.rel_var:.4f} gpu rel={st.rel_var:.4f} union {d.union_size}/{st.union_size}",
              flush=True)
        assert bool(st.evaluated) == d.evaluated
        if d.evaluated:
            rel_ref[l], rel_gpu[l] = d.rel_var, st.rel_var
            assert abs(d.rel_var - tau) > 1e-3, "oracle decision too close to tau: reseed"
            dev_rel = abs(st.rel_var - d.rel_var) / max(d.rel_var, 1e-3)
            worst_rel = max(worst_rel, dev_rel)
            assert dev_rel < 2e-2
            assert bool(st.selected) == d.selected
        if d.selected:
            sel_ref, sel_gpu = l, (l if st.selected else None)
            gu.check_topk_within_tolerance(out["I_all"], s_ref, sh.k, f"{what} selection top-k")
            break
    print(f"{what}: worst relative deviation of the chained relative variance {worst_rel:.3g}", flush=True)
    gu.report_margins(what)
    assert sel_ref is not None and sh.L_min < sel_ref <= 31 and sel_gpu == sel_ref
    assert asl.read_struct(state, asl.AslState).n_valid_rows == 0      # rank cache released
    assert rel_ref[sh.L_min] == 1.0 and rel_gpu[sh.L_min] == 1.0       # relative variance is 1 at L_min
    ctx.close()
    return sel_ref, rel_ref, rel_gpu


def test_config4_sweep_selection_layer(gpu_device):
    """32-layer sweep through the whole pipeline with the stated correlation schedule (0.2 -> 0.95):
    the GPU must pick the same selection layer as the oracle.  With this recipe the relative variance
    falls to about 0.34 at the last layer, so the run uses tau = 0.5 from the paper's ablation grid
    (selection near layer 29); the first-crossing layer is also compared for the other grid values
    whose oracle margin is large enough to make the agreement meaningful."""
    _, rel_ref, rel_gpu = _sweep_through_pipeline(gpu_device, 0.5, synth.SWEEP_RHO_END, "sweep tau=0.5")
    first = lambda rel, t: next((l for l in sorted(rel) if rel[l] < t), None)
    for t in (0.6, 0.7, 0.8, 0.9):
        if min(abs(r - t) for r in rel_ref.values()) > 1e-3:
            assert first(rel_ref, t) == first(rel_gpu, t)


def test_config4_variant_selects_at_default_tau(gpu_device):
    """LABELLED VARIANT of the sweep: the correlation schedule ends at SWEEP_RHO_END_CONVERGED instead
    of 0.95, everything else as stated, so that the relative variance of the full pipeline does fall
    below the paper's default tau = 0.3 (Sec. 5.1) before the last layer is over, and the selection
    happens after L_min and at or before layer 31."""
    sel, _, _ = _sweep_through_pipeline(gpu_device, 0.3, synth.SWEEP_RHO_END_CONVERGED, "sweep-variant tau=0.3")
    assert sel > synth.shape_of(4).L_min


def test_sweep_score_level_bit_exact(gpu_device):
    """Score-level sweep: identical fp32 score vectors go to asl_rank_stat and to the oracle, so the
    ranks, the statistic's integers, var_top, rel_var and the decision must match exactly."""
    import torch
    sh = synth.shape_of(4)
    z = synth.sweep_latents(sh.T, sh.n_layers)
    ctx = gu.ctx_for(sh)
    p = gu.params_of(sh)
    for tau in (0.3, 0.5):
        ring = torch.zeros((sh.L_obs, sh.T), dtype=torch.int32, device=gpu_device)
        state = asl.new_state(gpu_device)
        stat = asl.new_stat(gpu_device)
        ost = orc.SelectState.new(sh.L_obs)
        selected_at = None
        for l in range(sh.n_layers):
            s = synth.sweep_scores(z[l])
            ctx.asl_rank_stat(p, torch.from_numpy(s).to(gpu_device), l, sh.L_min, sh.L_obs, tau, ring, state, stat)
            ost.push(l, orc.rank_desc(s.astype(np.float64)))
            np.testing.assert_array_equal(ring[l % sh.L_obs].cpu().numpy(), ost.rows[-1][1])
            d = orc.select_tokens(ost, l, sh.budget, sh.W, sh.L_min, tau)
            st = asl.read_struct(stat, asl.AslStat)
            assert bool(st.evaluated) == d.evaluated and bool(st.selected) == d.selected
            if d.evaluated:
                assert st.union_size == d.union_size and st.n_rows == d.n_rows
                assert st.var_top == d.var_top and st.rel_var == d.rel_var
            if d.selected:
                selected_at = l
                break
        assert selected_at is not None and selected_at > sh.L_min
    ctx.close()


def test_bench_launch_configuration(gpu_device):
    """The configuration bench.py times on workload C3: P and s in one [Hk+1, T] allocation, one
    top-k call over the Hk per-head rows plus the all-head row, ranking/statistic and top-k/gather
    forked on two streams that share one context."""
    import torch
    L = synth.config_layer(3)
    sh = L.shape
    dev = gpu_device
    ctx = asl.Asl(sh.N, sh.Hk + 1, sh.Hq * sh.W)
    p = gu.params_of(sh)
    qd, kd, vd = (gu.to_dev(x, sh.dtype, dev) for x in (L.q_obs, L.k, L.v))
    T, n_idx = sh.T, sh.k + sh.W
    PS = torch.empty((sh.Hk + 1, T), dtype=torch.float32, device=dev)
    P, s = PS[:sh.Hk], PS[sh.Hk]
    ring = torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev)
    state, stat = asl.new_state(dev), asl.new_stat(dev)
    I = torch.empty((sh.Hk + 1, n_idx), dtype=torch.int32, device=dev)
    Kc = torch.empty((sh.Hk, n_idx, sh.d), dtype=torch.bfloat16, device=dev)
    Vc = torch.empty_like(Kc)
    side = torch.cuda.Stream()
    ev_a, ev_b = torch.cuda.Event(), torch.cuda.Event()
    main = torch.cuda.current_stream()
    for layer_idx in range(2):                       # second pass re-uses every workspace region
        ctx.asl_score_layer(p, qd, kd, P, s)
        ev_a.record(main)
        with torch.cuda.stream(side):
            side.wait_event(ev_a)
            ctx.asl_select_topk(p, PS, sh.Hk + 1, I)
            ctx.asl_gather_kv(p, kd, vd, I, sh.Hk, n_idx, Kc, Vc)
            ev_b.record(side)
        ctx.asl_rank_stat(p, s, layer_idx, 0, sh.L_obs, 0.3, ring, state, stat)
        main.wait_event(ev_b)
    torch.cuda.synchronize()
    P_ref, s_ref = orc.score_layer(L.q_obs, L.k, sh.W, sh.S)
    gu.assert_scores_close(P.cpu().numpy(), P_ref, "bench config P")
    gu.assert_scores_close(s.cpu().numpy(), s_ref, "bench config s")
    Ig = I.cpu().numpy().astype(np.int64)
    sg = s.cpu().numpy().astype(np.float64)
    Pg = P.cpu().numpy().astype(np.float64)
    # integer stages are exact given the GPU's own fp32 scores
    np.testing.assert_array_equal(Ig[sh.Hk], orc.select_indices(sg, sh.k, sh.W))
    np.testing.assert_array_equal(Ig[:sh.Hk], orc.select_indices(Pg, sh.k, sh.W))
    for r in range(2):
        np.testing.assert_array_equal(ring[r].cpu().numpy(), orc.rank_desc(sg))
    for g in range(sh.Hk):
        gu.check_topk_within_tolerance(Ig[g], P_ref[g], sh.k, f"bench config head {g}")
        assert np.array_equal(Kc[g].float().cpu().numpy(), L.k[g][Ig[g]])
        assert np.array_equal(Vc[g].float().cpu().numpy(), L.v[g][Ig[g]])
    assert np.isin(L.needles, Ig[sh.Hk]).all()
    st = asl.read_struct(stat, asl.AslStat)
    assert st.evaluated == 1 and st.n_rows == 2 and st.var_top == 0.0      # two identical rank rows
    ctx.close()


def _layer_step_case(dev, L, layer_idx=0):
    import torch
    sh = L.shape
    ctx = asl.Asl(sh.N, sh.Hk + 1, sh.Hq * sh.W)
    p = gu.params_of(sh)
    qd, kd, vd = (gu.to_dev(x, sh.dtype, dev) for x in (L.q_obs, L.k, L.v))
    T, n_idx = sh.T, sh.k + sh.W
    scores = torch.empty((sh.Hk + 1, T), dtype=torch.float32, device=dev)
    ring = torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev)
    state, stat = asl.new_state(dev), asl.new_stat(dev)
    I = torch.empty((sh.Hk + 1, n_idx), dtype=torch.int32, device=dev)
    Kc = torch.empty((sh.Hk, n_idx, sh.d), dtype=kd.dtype, device=dev)
    Vc = torch.empty_like(Kc)
    ctx.asl_layer_step(p, qd, kd, vd, layer_idx, sh.L_min, sh.L_obs, sh.tau, scores, ring, state, stat, I, Kc, Vc)
    torch.cuda.synchronize()
    # the same layer through the single calls
    P2 = torch.empty((sh.Hk, T), dtype=torch.float32, device=dev)
    s2 = torch.empty((T,), dtype=torch.float32, device=dev)
    ring2 = torch.zeros_like(ring)
    state2, stat2 = asl.new_state(dev), asl.new_stat(dev)
    Ih = torch.empty((sh.Hk, n_idx), dtype=torch.int32, device=dev)
    Ia = torch.empty((1, n_idx), dtype=torch.int32, device=dev)
    K2 = torch.empty_like(Kc)
    V2 = torch.empty_like(Kc)
    ctx.asl_score_layer(p, qd, kd, P2, s2)
    ctx.asl_rank_stat(p, s2, layer_idx, sh.L_min, sh.L_obs, sh.tau, ring2, state2, stat2)
    ctx.asl_select_topk(p, P2, sh.Hk, Ih)
    ctx.asl_select_topk(p, s2, 1, Ia)
    ctx.asl_gather_kv(p, kd, vd, Ih, sh.Hk, n_idx, K2, V2)
    torch.cuda.synchronize()
    for what, a, b in (("P", scores[:sh.Hk], P2), ("s", scores[sh.Hk], s2), ("rank ring", ring, ring2),
                       ("per-head indices", I[:sh.Hk], Ih), ("all-head indices", I[sh.Hk:], Ia), ("K[I]", Kc, K2),
                       ("V[I]", Vc, V2), ("state", state, state2)):
        if not torch.equal(a, b):
            d = torch.nonzero(a.reshape(-1) != b.reshape(-1)).reshape(-1)
            raise AssertionError(f"{L.name}: {what} of asl_layer_step differs from the single calls at {d.numel()} of "
                                 f"{a.numel()} places, first at flat index {int(d[0])}: {a.reshape(-1)[d[0]].item()} vs "
                                 f"{b.reshape(-1)[d[0]].item()}; fault word {ctx.asl_device_fault()}")
    out = dict(P=scores[:sh.Hk].cpu().numpy(), s=scores[sh.Hk].cpu().numpy(),
               rank=ring[layer_idx % sh.L_obs].cpu().numpy().astype(np.int64),
               stat=asl.read_struct(stat, asl.AslStat), I_head=I[:sh.Hk].cpu().numpy().astype(np.int64),
               I_all=I[sh.Hk].cpu().numpy().astype(np.int64), Kc=Kc.float().cpu().numpy(),
               Vc=Vc.float().cpu().numpy())
    out["Ks"] = np.stack([L.k[g][out["I_all"]] for g in range(sh.Hk)])      # shared-row gather not part of the step
    out["Vs"] = np.stack([L.v[g][out["I_all"]] for g in range(sh.Hk)])
    ctx.close()
    return out


def test_layer_step_matches_single_calls_and_oracle(gpu_device):
    """asl_layer_step (fork/join on the context's own side stream) gives bit-identical results to the
    single calls, and both match the oracle."""
    for cfg in (1, 2):
        L = synth.config_layer(cfg)
        if cfg == 1:
            sh = synth.shape_of(1)
            sh.dtype = "bf16"
            L = synth.iid_layer(sh, synth.BASE_SEED + 1, name="C1-bf16")
        _check_layer(L, _layer_step_case(gpu_device, L))


@pytest.mark.parametrize("Hq,Hk,d,N,W,S,budget", [(6, 2, 64, 10007, 13, 5, 777), (3, 3, 128, 4099, 7, 3, 64),
                                                   (8, 1, 128, 33333, 32, 7, 5000), (2, 2, 64, 70, 3, 1, 9)])
def test_layer_step_ragged_shapes(gpu_device, Hq, Hk, d, N, W, S, budget):
    """Sizes that are multiples of no tile: odd N and W (score rows that do not start on 16-byte boundaries,
    ragged last tiles in every kernel), one to three KV heads, a budget above and below one tile."""
    sh = synth.Shape(Hq=Hq, Hk=Hk, d=d, N=N, W=W, S=S, budget=budget, L_min=0)
    L = synth.iid_layer(sh, 1000 + N, name=f"ragged-{N}-{W}")
    _check_layer(L, _layer_step_case(gpu_device, L))


def test_layer_step_at_bench_size_and_beyond(gpu_device):
    """asl_layer_step at the size the benchmark times (C3: 64 sort tiles beside the top-k stages) and at
    2^20 tokens (the ranking sort switches to its large tiles): bit-identical to the single calls, and
    both match the oracle."""
    L = synth.config_layer(3)
    _check_layer(L, _layer_step_case(gpu_device, L))
    sh = synth.Shape(Hq=4, Hk=2, d=128, N=1 << 20, W=32, S=7, budget=8192)
    L = synth.iid_layer(sh, 78, name="1M-step")
    _check_layer(L, _layer_step_case(gpu_device, L))
    # the other shapes the benchmark times: 256K / W = 64 (128 sort tiles) and the second model shape with
    # budget 8192 (5 score rows); here against the single calls only (their oracle parity is tested above)
    _layer_step_case(gpu_device, synth.config_layer(5), layer_idx=12)
    sh = synth.Shape(Hq=28, Hk=4, d=128, N=131072, W=32, S=7, budget=8192, L_min=9)
    _layer_step_case(gpu_device, synth.needle_layer(sh, 123, 64, synth.needle_gain_strong(sh), name="second-shape-128K"),
                     layer_idx=3)


def test_layer_step_is_reproducible(gpu_device):
    """200 repetitions of asl_layer_step on the C3 layer, and of the single ranking and top-k calls on its
    scores: every output has the same bits every time (the workgroups of the ranking and statistic
    launches hand counts to each other inside the launch; nothing may depend on who came first)."""
    import torch
    dev = gpu_device
    L = synth.config_layer(3)
    sh = L.shape
    ctx = asl.Asl(sh.N, sh.Hk + 1, sh.Hq * sh.W)
    p = gu.params_of(sh)
    qd, kd, vd = (gu.to_dev(x, sh.dtype, dev) for x in (L.q_obs, L.k, L.v))
    T, n_idx = sh.T, sh.k + sh.W

    def step():
        scores = torch.empty((sh.Hk + 1, T), dtype=torch.float32, device=dev)
        ring = torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev)
        state, stat = asl.new_state(dev), asl.new_stat(dev)
        I = torch.full((sh.Hk + 1, n_idx), -1, dtype=torch.int32, device=dev)
        Kc = torch.zeros((sh.Hk, n_idx, sh.d), dtype=kd.dtype, device=dev)
        Vc = torch.zeros_like(Kc)
        ctx.asl_layer_step(p, qd, kd, vd, 0, sh.L_min, sh.L_obs, sh.tau, scores, ring, state, stat, I, Kc, Vc)
        return scores, ring, I, Kc, Vc, stat, state

    def single(scores):
        ring = torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev)
        state, stat = asl.new_state(dev), asl.new_stat(dev)
        I = torch.full((sh.Hk + 1, n_idx), -1, dtype=torch.int32, device=dev)
        ctx.asl_rank_stat(p, scores[sh.Hk], 0, sh.L_min, sh.L_obs, sh.tau, ring, state, stat)
        ctx.asl_select_topk(p, scores, sh.Hk + 1, I)
        return ring, I, stat, state

    ref = step()
    ref1 = single(ref[0])
    for i in range(200):
        for what, outs, refs in (("asl_layer_step", step(), ref), ("single calls", single(ref[0]), ref1)):
            for j, (a, b) in enumerate(zip(outs, refs)):
                assert torch.equal(a, b), f"run {i}: output {j} of {what} differs from the first run"
    assert ctx.asl_device_fault() == 0
    ctx.close()


def test_second_model_shape_and_large_budget(gpu_device):
    """The 28-layer model's head geometry (4 KV heads, 7 query heads per group: 224 query rows per
    KV head, seven 32-row blocks) and the paper's larger KV budget of 8192."""
    sh = synth.Shape(Hq=28, Hk=4, d=128, N=20000, W=32, S=7, budget=8192, L_min=9)
    L = synth.needle_layer(sh, 77, 32, synth.needle_gain_strong(sh), name="qwen-like-20k-b8192")
    _check_layer(L, _pipeline(gpu_device, L))


def test_hidden_state_propagation(gpu_device):
    """asl_gather_rows on [N, 4096] bf16 hidden states with the selection of a scored layer."""
    import torch
    rng = np.random.default_rng(5)
    N, D = 5000, 4096
    hidden = synth.round_bf16(rng.standard_normal((N, D)).astype(np.float32))
    idx = np.sort(rng.choice(N, 777, replace=False)).astype(np.int32)
    ctx = asl.Asl(N, 1, 32)
    hd = gu.to_dev(hidden, "bf16", gpu_device)
    out = torch.zeros((len(idx), D), dtype=torch.bfloat16, device=gpu_device)
    ctx.asl_gather_rows(hd, D * 2, D * 2, torch.from_numpy(idx).to(gpu_device), len(idx), out)
    assert np.array_equal(out.float().cpu().numpy(), orc.propagate_tokens(hidden, idx))
    ctx.asl_gather_rows(hd, D * 2, D * 2, torch.from_numpy(idx).to(gpu_device), 0, out)      # empty selection
    with pytest.raises(asl.AslError):
        ctx.asl_gather_rows(hd, D * 2, 24, torch.from_numpy(idx).to(gpu_device), 4, out)    # rows not 16-byte multiples
    ctx.close()


def test_two_pass_handoff_from_a_selecting_step(gpu_device):
    """Sec. 4.2, two-pass variant: the first pass runs layer steps until one selects; its select_idx
    (row Hk of idx_out, valid because out->selected is set) then picks the rows of the embedding
    matrix from which the second pass restarts at layer 0.  Score-correlated layers make the
    statistic collapse, so the step at the last layer really selects."""
    import torch
    dev = gpu_device
    sh = synth.Shape(Hq=8, Hk=2, d=128, N=6000, W=32, S=7, budget=512, L_obs=4, L_min=3, tau=0.3)
    rng = np.random.default_rng(9)
    base = synth.iid_layer(sh, 500, name="two-pass")
    ctx = asl.Asl(sh.N, sh.Hk + 1, sh.Hq * sh.W)
    p = gu.params_of(sh)
    T, n_idx = sh.T, sh.k + sh.W
    qd = gu.to_dev(base.q_obs, "bf16", dev)
    scores = torch.empty((sh.Hk + 1, T), dtype=torch.float32, device=dev)
    ring = torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev)
    state, stat = asl.new_state(dev), asl.new_stat(dev)
    I = torch.empty((sh.Hk + 1, n_idx), dtype=torch.int32, device=dev)
    ost = orc.SelectState.new(sh.L_obs)
    selected_at = None
    for l in range(12):
        # layers 0-3 have unrelated keys, from layer 4 on every layer sees the same keys: the ranks stop moving
        kl = synth.iid_layer(sh, 600 + l).k if l < 4 else base.k
        kd, vd = gu.to_dev(kl, "bf16", dev), gu.to_dev(base.v, "bf16", dev)
        ctx.asl_layer_step(p, qd, kd, vd, l, sh.L_min, sh.L_obs, sh.tau, scores, ring, state, stat, I)
        torch.cuda.synchronize()
        sg = scores[sh.Hk].cpu().numpy().astype(np.float64)
        ost.push(l, orc.rank_desc(sg))                     # the oracle's Alg. 2 on the GPU's own scores: exact
        d = orc.select_tokens(ost, l, sh.budget, sh.W, sh.L_min, sh.tau)
        st = asl.read_struct(stat, asl.AslStat)
        assert bool(st.evaluated) == d.evaluated and bool(st.selected) == d.selected
        if d.evaluated:
            assert st.var_top == d.var_top and st.rel_var == d.rel_var and st.union_size == d.union_size
        if d.selected:
            selected_at = l
            break
    assert selected_at is not None and selected_at > sh.L_min
    select_idx = I[sh.Hk]
    np.testing.assert_array_equal(select_idx.cpu().numpy().astype(np.int64), d.select_idx)
    # second pass input: the embeddings of the selected tokens only
    D = 1024
    emb = synth.round_bf16(rng.standard_normal((sh.N, D)).astype(np.float32))
    embd = gu.to_dev(emb, "bf16", dev)
    out = torch.zeros((n_idx, D), dtype=torch.bfloat16, device=dev)
    ctx.asl_gather_rows(embd, D * 2, D * 2, select_idx, n_idx, out)
    assert np.array_equal(out.float().cpu().numpy(), orc.propagate_tokens(emb, d.select_idx))
    ctx.close()


@pytest.mark.parametrize("shared_idx", [False, True])
def test_gather_many_layers_from_separate_allocations(gpu_device, shared_idx):
    """asl_gather_kv_layers: every layer's K/V cache is its own allocation, named by a device array of
    pointers; the result must equal the per-layer oracle gather bit for bit, and the single-layer call."""
    import torch
    dev = gpu_device
    n_layers, Hk, N, d, n_idx = 5, 3, 1777, 128, 301
    rng = np.random.default_rng(17)
    sh = synth.Shape(Hq=Hk, Hk=Hk, d=d, N=N, W=8, S=7, budget=n_idx)
    ctx = gu.ctx_for(sh)
    p = gu.params_of(sh)
    ks, vs, kd, vd, ko, vo = [], [], [], [], [], []
    pad = []                                                    # odd-sized allocations between the caches
    for l in range(n_layers):
        ks.append(synth.round_bf16(rng.standard_normal((Hk, N, d)).astype(np.float32)))
        vs.append(synth.round_bf16(rng.standard_normal((Hk, N, d)).astype(np.float32)))
        kd.append(gu.to_dev(ks[-1], "bf16", dev))
        pad.append(torch.empty(4096 * (l + 1) + 48, dtype=torch.uint8, device=dev))
        vd.append(gu.to_dev(vs[-1], "bf16", dev))
        ko.append(torch.zeros((Hk, n_idx, d), dtype=torch.bfloat16, device=dev))
        vo.append(torch.zeros((Hk, n_idx, d), dtype=torch.bfloat16, device=dev))
    rows = 1 if shared_idx else Hk
    idx = np.stack([np.stack([np.sort(rng.choice(N, n_idx, replace=False)) for _ in range(rows)])
                    for _ in range(n_layers)]).astype(np.int32)
    idxd = torch.from_numpy(idx).to(dev)
    ptrs = lambda ts: torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=dev)
    ctx.asl_gather_kv_layers(p, ptrs(kd), ptrs(vd), idxd, rows, n_idx, n_layers, ptrs(ko), ptrs(vo))
    torch.cuda.synchronize()
    k1 = torch.zeros_like(ko[0])
    v1 = torch.zeros_like(vo[0])
    for l in range(n_layers):
        ref_k, ref_v = orc.gather_kv(ks[l], vs[l], idx[l, 0] if shared_idx else idx[l])
        assert np.array_equal(ko[l].float().cpu().numpy(), ref_k), f"layer {l} K"
        assert np.array_equal(vo[l].float().cpu().numpy(), ref_v), f"layer {l} V"
        ctx.asl_gather_kv(p, kd[l], vd[l], idxd[l], rows, n_idx, k1, v1)
        assert torch.equal(k1, ko[l]) and torch.equal(v1, vo[l])
    # K only, and an empty call
    ko2 = [torch.zeros_like(t) for t in ko]
    ctx.asl_gather_kv_layers(p, ptrs(kd), None, idxd, rows, n_idx, n_layers, ptrs(ko2), None)
    ctx.asl_gather_kv_layers(p, ptrs(kd), None, idxd, rows, n_idx, 0, ptrs(ko2), None)
    torch.cuda.synchronize()
    for l in range(n_layers):
        assert torch.equal(ko2[l], ko[l])
    with pytest.raises(asl.AslError):
        ctx.asl_gather_kv_layers(p, ptrs(kd), ptrs(vd), idxd, rows, n_idx, n_layers, ptrs(ko), None)
    ctx.close()


def test_ring_restart_and_cyclic_continuity(gpu_device):
    """Only the next layer index, or the same index one trip round the ring earlier (a replayed graph
    of L_obs layers), continues the rank cache; any other index restarts it, also one whose ring row
    happens to be the next one."""
    import torch
    sh = synth.shape_of(1)
    ctx = gu.ctx_for(sh)
    p = gu.params_of(sh)
    T, L_obs = sh.T, 4
    rng = np.random.default_rng(0)
    ring = torch.zeros((L_obs, T), dtype=torch.int32, device=gpu_device)
    state, stat = asl.new_state(gpu_device), asl.new_stat(gpu_device)
    rows = {}
    def push(layer):
        s = rng.random(T, dtype=np.float32)
        rows[layer % L_obs] = orc.rank_desc(s.astype(np.float64))
        ctx.asl_rank_stat(p, torch.from_numpy(s).to(gpu_device), layer, 0, L_obs, 0.0, ring, state, stat)
        return asl.read_struct(state, asl.AslState), asl.read_struct(stat, asl.AslStat)
    assert push(0)[0].n_valid_rows == 1
    assert push(1)[0].n_valid_rows == 2
    st, out = push(2)
    assert st.n_valid_rows == 3 and out.evaluated == 1 and out.n_rows == 3
    assert push(3)[0].n_valid_rows == 4
    st, out = push(0)                              # 0 == 3 + 1 - L_obs: a replayed trip, still consecutive rows
    assert st.n_valid_rows == 4 and out.n_rows == 4
    ref = orc.rank_variance(np.stack([rows[r] for r in (1, 2, 3, 0)]), sh.k)
    assert out.numerator == ref.numerator and out.union_size == ref.union_size
    assert push(1)[0].n_valid_rows == 4
    st, out = push(6)                              # 6 % 4 == 2 is the next ring row, but 6 != 1 + 1: restart
    assert st.n_valid_rows == 1 and st.last_layer == 6 and out.evaluated == 0
    st, out = push(7)
    assert st.n_valid_rows == 2 and out.evaluated == 1 and out.n_rows == 2
    ref = orc.rank_variance(np.stack([rows[2], rows[3]]), sh.k)
    assert out.numerator == ref.numerator and out.union_size == ref.union_size
    st, out = push(16)                             # a jump by a multiple of L_obs plus one: restart as well
    assert st.n_valid_rows == 1 and out.evaluated == 0
    ctx.close()


@pytest.mark.parametrize("defer", [False, True])
def test_layer_step_graph_replay_matches_eager(gpu_device, defer):
    """Capture L_obs consecutive asl_layer_step calls in a HIP graph, replay it several times with
    eager work and synchronisations in between, and compare every replay with the eager result.
    defer: the steps leave their top-k + compaction on the second stream (ASL_FLAG_DEFER_JOIN) and all
    layers share ONE score buffer, so a step's top-k must have read it before the next step's pooling
    overwrites it; the reference is the same sequence with every step joined."""
    import torch
    sh = synth.Shape(Hq=8, Hk=2, d=128, N=6000, W=32, S=7, budget=256, L_obs=4, L_min=0)
    layers = [synth.iid_layer(sh, 100 + j) for j in range(sh.L_obs)]
    dev = gpu_device
    ctx = asl.Asl(sh.N, sh.Hk + 1, sh.Hq * sh.W)
    p = gu.params_of(sh)
    p_defer = gu.params_of(sh, flags=asl.ASL_FLAG_DEFER_JOIN)
    T, n_idx = sh.T, sh.k + sh.W
    qs = [gu.to_dev(L.q_obs, "bf16", dev) for L in layers]
    kss = [gu.to_dev(L.k, "bf16", dev) for L in layers]
    vss = [gu.to_dev(L.v, "bf16", dev) for L in layers]
    n_score_bufs = 1 if defer else sh.L_obs

    def buffers():
        return dict(scores=torch.zeros((n_score_bufs, sh.Hk + 1, T), dtype=torch.float32, device=dev),
                    ring=torch.zeros((sh.L_obs, T), dtype=torch.int32, device=dev),
                    state=asl.new_state(dev), stats=torch.zeros((sh.L_obs, 40), dtype=torch.uint8, device=dev),
                    I=torch.zeros((sh.L_obs, sh.Hk + 1, n_idx), dtype=torch.int32, device=dev),
                    K=torch.zeros((sh.L_obs, sh.Hk, n_idx, sh.d), dtype=torch.bfloat16, device=dev),
                    V=torch.zeros((sh.L_obs, sh.Hk, n_idx, sh.d), dtype=torch.bfloat16, device=dev))

    def trip(b, first_layer, params):
        for j in range(sh.L_obs):
            ctx.asl_layer_step(params, qs[j], kss[j], vss[j], first_layer + j, 0, sh.L_obs, 0.0,
                               b["scores"][j % n_score_bufs], b["ring"], b["state"], b["stats"][j], b["I"][j],
                               b["K"][j], b["V"][j])
        ctx.asl_join()                               # no-op unless the steps were deferred

    ref = buffers()
    trip(ref, 0, p)
    trip(ref, sh.L_obs, p)                           # second trip: the ring is full, statistic over 4 rows
    torch.cuda.synchronize()
    pg = p_defer if defer else p
    if defer:                                        # eager deferred steps first
        e = buffers()
        trip(e, 0, pg)
        trip(e, sh.L_obs, pg)
        torch.cuda.synchronize()
        for name in ("scores", "ring", "I", "K", "V", "stats"):
            assert torch.equal(e[name], ref[name]), f"eager deferred steps: {name} differs"
    g = buffers()
    trip(g, 0, pg)                                   # warm the ring eagerly, then capture the second trip
    torch.cuda.synchronize()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            trip(g, sh.L_obs, pg)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (g["scores"], g["I"], g["K"], g["V"], g["stats"]):
            t.zero_()                                # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ("scores", "ring", "I", "K", "V", "stats"):
            assert torch.equal(g[name], ref[name]), f"replay {rep}: {name} differs from the eager result"
    st = asl.read_struct(g["stats"][sh.L_obs - 1], asl.AslStat)
    assert st.evaluated == 1 and st.n_rows == sh.L_obs
    ctx.close()
