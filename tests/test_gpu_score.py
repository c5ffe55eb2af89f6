"""GPU parity of asl_score_layer (Alg. 1 steps 5-8) against the float64 oracle on the same seeded
inputs: |gpu - oracle| <= 1e-5 + 2e-3 |oracle| element by element (bf16 in, fp32 accumulate)."""
import numpy as np
import pytest

import gpu_util as gu
from oracle import asl_oracle as orc
from paper_2601_07667_amd import asl, synth

pytestmark = pytest.mark.gpu


def _run_score(dev, L, flags=0, lse=None, scale=0.0):
    import torch
    sh = L.shape
    ctx = gu.ctx_for(sh)
    p = gu.params_of(sh, flags=flags, scale=scale)
    qd, kd = gu.to_dev(L.q_obs, sh.dtype, dev), gu.to_dev(L.k, sh.dtype, dev)
    P = torch.full((sh.Hk, sh.T), float("nan"), dtype=torch.float32, device=dev)
    s = torch.full((sh.T,), float("nan"), dtype=torch.float32, device=dev)
    lsed = None if lse is None else torch.from_numpy(lse.astype(np.float32)).to(dev)
    ctx.asl_score_layer(p, qd, kd, P, s, lse=lsed)
    out = P.cpu().numpy(), s.cpu().numpy()
    ctx.close()
    return out


def _small(Hq, Hk, d, N, W, S=7, dtype="bf16", seed=0):
    sh = synth.Shape(Hq=Hq, Hk=Hk, d=d, N=N, W=W, S=S, budget=W + 8, dtype=dtype)
    return synth.iid_layer(sh, seed, name=f"small-{Hq}-{Hk}-{d}-{N}-{W}-{dtype}")


def _compare(dev, L, flags=0, use_lse=False, scale=0.0):
    sh = L.shape
    sc = scale if scale > 0 else None
    P_ref, s_ref = orc.score_layer(L.q_obs, L.k, sh.W, sh.S, sc)
    lse = orc.row_lse(L.q_obs, L.k, sh.W, sc) if use_lse else None
    P, s = _run_score(dev, L, flags=flags, lse=lse, scale=scale)
    gu.assert_scores_close(P, P_ref, f"{L.name} P")
    gu.assert_scores_close(s, s_ref, f"{L.name} s")
    return P, s


def test_config1_f32_and_bf16(gpu_device):
    L = synth.config_layer(1)                                   # fp32 storage: plain-FMA kernels
    _compare(gpu_device, L)
    sh = synth.shape_of(1)
    sh.dtype = "bf16"                                           # bf16-rounded copy: MFMA kernels, d = 64
    Lb = synth.iid_layer(sh, synth.BASE_SEED + 1, name="C1-bf16")
    P, s = _compare(gpu_device, Lb)
    Pg, sg = _compare(gpu_device, Lb, flags=asl.ASL_FLAG_GENERIC_SCORE)     # on-GPU cross-check
    np.testing.assert_allclose(P, Pg, rtol=1e-4, atol=1e-7)


# several tiles and a ragged tail; row counts that do not fill a 32-row block; d = 64 and 128;
# M = 224 (seven heads per group) and M = 256 (W = 64)
@pytest.mark.parametrize("Hq,Hk,d,N,W", [
    (4, 2, 128, 1000, 16), (3, 1, 64, 333, 5), (8, 2, 128, 4096 + 77, 32), (7, 1, 128, 2500, 32),
    (4, 1, 128, 3000, 64), (2, 2, 64, 130, 1), (4, 4, 128, 129, 128), (8, 8, 128, 40, 33)])
def test_small_shapes(gpu_device, Hq, Hk, d, N, W):
    L = _small(Hq, Hk, d, N, W, seed=N)
    _compare(gpu_device, L)


@pytest.mark.parametrize("N", [64 * 5 + 16, 64 * 5 + 15, 64 * 5 + 17, 64 * 6 + 32, 64 * 40 + 1])
def test_key_counts_around_tile_edges(gpu_device, N):
    """N - W one below / at / one above a multiple of the 64-key tile; several chunks per head."""
    _compare(gpu_device, _small(4, 2, 128, N, 16, seed=N))
    _compare(gpu_device, _small(4, 2, 128, N, 16, seed=N + 1), use_lse=True)


@pytest.mark.parametrize("d,dtype", [(96, "bf16"), (256, "bf16"), (80, "f32")])
def test_other_head_dims_take_the_plain_kernels(gpu_device, d, dtype):
    """Head dimensions outside {64, 128} are scored by the plain-FMA kernels."""
    _compare(gpu_device, _small(4, 2, d, 700, 8, dtype=dtype, seed=d))


def test_random_shapes(gpu_device):
    """Sixteen seeded random shapes: group sizes 1-8, windows 1-64 (M = G*W up to 256, so both the
    one-block and the two-block wavefront layouts and every wavefront count occur), d in {64, 128},
    sequence lengths that are not multiples of anything, pooling kernels 1-15."""
    rng = np.random.default_rng(20260128)
    done = 0
    while done < 16:
        G = int(rng.integers(1, 9))
        W = int(rng.integers(1, 65))
        if G * W > 256:
            continue
        Hk = int(rng.integers(1, 4))
        d = int(rng.choice([64, 128]))
        N = W + int(rng.integers(1, 3000))
        S = int(rng.choice([1, 3, 7, 15]))
        print(f"case {done}: Hq={G * Hk} Hk={Hk} d={d} N={N} W={W} S={S} (M={G * W})", flush=True)
        _compare(gpu_device, _small(G * Hk, Hk, d, N, W, S=S, seed=1000 + done), use_lse=bool(done % 2))
        done += 1


def test_lse_supplied_mode_and_scale(gpu_device):
    L = _small(8, 2, 128, 5000, 32, seed=3)
    P1, s1 = _compare(gpu_device, L)
    P2, s2 = _compare(gpu_device, L, use_lse=True)              # single pass over K
    np.testing.assert_allclose(P1, P2, rtol=1e-4, atol=1e-7)
    _compare(gpu_device, L, scale=0.05)
    Lf = _small(4, 2, 64, 700, 16, dtype="f32", seed=4)
    _compare(gpu_device, Lf, use_lse=True)


def test_pool_kernel_one_and_large(gpu_device):
    _compare(gpu_device, _small(4, 2, 128, 900, 16, S=1, seed=5))
    _compare(gpu_device, _small(4, 2, 128, 900, 16, S=31, seed=6))


def test_strided_k(gpu_device):
    """K as a slice of a fused [Hk, N, 2d] buffer (token stride 2d)."""
    import torch
    L = _small(8, 2, 128, 3000, 32, seed=7)
    sh = L.shape
    ctx = gu.ctx_for(sh)
    kd = gu.to_dev(L.k, "bf16", gpu_device)
    wide = torch.zeros((sh.Hk, sh.N, 2 * sh.d), dtype=torch.bfloat16, device=gpu_device)
    wide[:, :, sh.d:] = kd
    p = asl.make_params(sh.Hq, sh.Hk, sh.d, sh.N, sh.W, sh.S, sh.budget,
                        k_strides=(sh.N * 2 * sh.d, 2 * sh.d))
    P = torch.empty((sh.Hk, sh.T), dtype=torch.float32, device=gpu_device)
    s = torch.empty((sh.T,), dtype=torch.float32, device=gpu_device)
    ctx.asl_score_layer(p, gu.to_dev(L.q_obs, "bf16", gpu_device), wide[:, :, sh.d:], P, s)
    P_ref, s_ref = orc.score_layer(L.q_obs, L.k, sh.W, sh.S)
    gu.assert_scores_close(P.cpu().numpy(), P_ref, "strided P")
    gu.assert_scores_close(s.cpu().numpy(), s_ref, "strided s")
    ctx.close()


def test_heavy_tailed_keys(gpu_device):
    """Per-token lognormal key scale: logits of a few hundred, exercises the running maximum."""
    sh = synth.Shape(Hq=8, Hk=2, d=128, N=6000, W=64, S=7, budget=512)
    L = synth.needle_layer(sh, 11, 16, synth.needle_gain_strong(sh), heavy_tail=True, name="heavy")
    _compare(gpu_device, L)


def test_config2_full(gpu_device):
    L = synth.config_layer(2)
    P, s = _compare(gpu_device, L)
    P2, s2 = _run_score(gpu_device, L)                          # determinism: bit-identical rerun
    assert np.array_equal(P, P2) and np.array_equal(s, s2)


def test_config3_full_128k(gpu_device):
    L = synth.config_layer(3)
    _compare(gpu_device, L)
    gu.report_margins(L.name)


def test_config3_lse_supplied_128k(gpu_device):
    """The one-pass mode at the size the benchmark times it: the rows' log-sum-exp comes from the
    oracle (float64, rounded to fp32), K is streamed once."""
    L = synth.config_layer(3)
    L.name += "-lse"
    _compare(gpu_device, L, use_lse=True)
    gu.report_margins(L.name)


def _window_lse(dev, L, flags=0):
    import torch
    sh = L.shape
    ctx = gu.ctx_for(sh)
    p = gu.params_of(sh, flags=flags)
    qd, kd = gu.to_dev(L.q_obs, sh.dtype, dev), gu.to_dev(L.k, sh.dtype, dev)
    lse = torch.full((sh.Hq, sh.W), float("nan"), dtype=torch.float32, device=dev)
    ctx.asl_window_lse(p, qd, kd, lse)
    P0 = torch.empty((sh.Hk, sh.T), dtype=torch.float32, device=dev)
    s0 = torch.empty((sh.T,), dtype=torch.float32, device=dev)
    P1, s1 = torch.empty_like(P0), torch.empty_like(s0)
    ctx.asl_score_layer(p, qd, kd, P0, s0)                       # self-contained: two passes over K
    ctx.asl_score_layer(p, qd, kd, P1, s1, lse=lse)              # with the library's own log-sum-exp
    torch.cuda.synchronize()
    ctx.close()
    return lse.cpu().numpy().astype(np.float64), (P0, s0), (P1, s1)


@pytest.mark.parametrize("case", ["small-d64", "ragged-rows", "w64", "f32-plain", "heavy-tail", "c2"])
def test_window_lse_matches_oracle_and_hands_back_exactly(gpu_device, case):
    """asl_window_lse against the oracle's log-sum-exp of the masked, scaled logits (fp32 accumulation
    of a sum of N positive terms: 1e-5 absolute + 2e-6 relative on a logarithm), and the hand-off:
    scoring with these values supplied equals the self-contained call up to the rounding of the
    natural-log <-> base-2 conversion of the normaliser (one ulp of a number near 20 in the exponent:
    a few 1e-6 relative on every score)."""
    import torch
    if case == "small-d64":
        L = _small(4, 2, 64, 700, 16, seed=21)
    elif case == "ragged-rows":
        L = _small(7, 1, 128, 2500, 32, seed=22)                 # 224 query rows per KV head
    elif case == "w64":
        L = _small(8, 2, 128, 4096 + 77, 64, seed=23)
    elif case == "f32-plain":
        L = _small(4, 2, 64, 700, 16, dtype="f32", seed=24)
    elif case == "heavy-tail":
        sh = synth.Shape(Hq=8, Hk=2, d=128, N=6000, W=64, S=7, budget=512)
        L = synth.needle_layer(sh, 11, 16, synth.needle_gain_strong(sh), heavy_tail=True, name="heavy")
    else:
        L = synth.config_layer(2)
    sh = L.shape
    lse, (P0, s0), (P1, s1) = _window_lse(gpu_device, L)
    ref = orc.row_lse(L.q_obs, L.k, sh.W)
    err = np.abs(lse - ref)
    assert np.all(err <= 1e-5 + 2e-6 * np.abs(ref)), f"{case}: worst lse error {err.max()}"
    for a, b in ((P0, P1), (s0, s1)):
        a, b = a.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(a - b) <= 1e-5 * np.abs(a) + 1e-12), f"{case}: hand-back differs by {np.abs(a / b - 1).max()}"


def test_config5_full_256k(gpu_device):
    L = synth.config_layer(5)
    _compare(gpu_device, L)
    gu.report_margins(L.name)


# The 28-layer model's head geometry (App. B.3: 4 KV heads, 7 query heads per group) at the paper's
# long contexts: 224 query rows per KV head at window 32, 448 at window 64.
@pytest.mark.parametrize("N,W,budget", [(131072, 32, 8192), (262144, 64, 8192)])
def test_second_model_geometry_full_size(gpu_device, N, W, budget):
    sh = synth.Shape(Hq=28, Hk=4, d=128, N=N, W=W, S=7, budget=budget, L_min=9)
    L = synth.needle_layer(sh, 91 + W, 64, synth.needle_gain_strong(sh), name=f"qwen-like-N{N}-W{W}")
    print(f"score {L.name}", flush=True)
    _compare(gpu_device, L)
    gu.report_margins(L.name)


@pytest.mark.parametrize("Hq,Hk,W", [(5, 1, 64), (6, 1, 64), (16, 2, 64), (12, 1, 32), (7, 1, 48)])
def test_row_counts_up_to_512(gpu_device, Hq, Hk, W):
    """G*W = 320, 384, 512, 384, 336 query rows per KV head: five to eight wavefronts of two 32-row
    blocks, with and without padded rows."""
    _compare(gpu_device, _small(Hq, Hk, 128, 3000 + 13 * Hq, W, seed=30 + Hq))
    _compare(gpu_device, _small(Hq, Hk, 64, 1500 + 7 * Hq, W, seed=40 + Hq))


@pytest.mark.parametrize("Hq,Hk,W,N,reps", [(32, 8, 32, 131072, 300), (16, 4, 64, 65536, 200), (8, 4, 32, 40000, 200),
                                            (14, 2, 32, 50000, 200)])
def test_scoring_is_reproducible(gpu_device, Hq, Hk, W, N, reps):
    """The same call on the same inputs gives the same bits every time (all reductions have a fixed
    order), with another key tensor scored in between.  Regression test: a missing wait for the LDS
    writes of pass 2's column partials once made one 32-key sub-tile differ in a few runs per hundred."""
    import torch
    dev = gpu_device
    torch.manual_seed(Hq * 1000 + W)
    ctx = asl.Asl(N, Hk, Hq * W)
    p = asl.make_params(Hq, Hk, 128, N, W, 7, 2048)
    q = torch.randn(Hq, W, 128, device=dev).to(torch.bfloat16)
    k = torch.randn(Hk, N, 128, device=dev).to(torch.bfloat16)
    other = torch.randn(Hk, N, 128, device=dev).to(torch.bfloat16)
    P = torch.empty(Hk, N - W, dtype=torch.float32, device=dev)
    s = torch.empty(N - W, dtype=torch.float32, device=dev)
    ctx.asl_score_layer(p, q, k, P, s)
    P0, s0 = P.clone(), s.clone()
    for i in range(reps):
        if i % 3 == 0:
            ctx.asl_score_layer(p, q, other, P, s)
        P.fill_(-1.0)
        s.fill_(-1.0)
        ctx.asl_score_layer(p, q, k, P, s)
        if not (torch.equal(P, P0) and torch.equal(s, s0)):
            d = torch.nonzero(P != P0)
            raise AssertionError(f"run {i} differs from run 0 at {d.shape[0]} places of P, KV heads "
                                 f"{sorted(set(d[:, 0].tolist()))}, keys {int(d[:, 1].min())}..{int(d[:, 1].max())}")
    ctx.close()
