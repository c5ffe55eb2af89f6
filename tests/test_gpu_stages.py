"""Stage-isolated GPU parity: each libasl kernel is fed the oracle-side input of its stage
(cast to the kernel's input dtype) and compared with the oracle's output for that stage.
Integer outputs (ranks, statistic integers, top-k indices, gathered bytes) must be bit-exact."""
import ctypes as C

import numpy as np
import pytest

from oracle import asl_oracle as orc
from paper_2601_07667_amd import asl, synth
import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(gpu_device):
    c = asl.Asl(262144, 8, 32 * 64)
    yield c
    assert c.asl_device_fault() == 0, "a workgroup gave up waiting for its peers during this module"
    c.close()


def _torch():
    import torch
    return torch


# ----------------------------------------------------------------------------- pool
@pytest.mark.parametrize("rows,T,S", [(1, 1, 1), (2, 5, 7), (8, 496, 7), (3, 1000, 1), (8, 32736, 7),
                                      (2, 777, 129), (8, 131040, 7)])
def test_pool(ctx, gpu_device, rows, T, S):
    torch = _torch()
    rng = np.random.default_rng(rows * 7 + T)
    u = rng.random((rows, T), dtype=np.float32)
    ud = torch.from_numpy(u).to(gpu_device)
    p = torch.empty_like(ud)
    s = torch.empty(T, dtype=torch.float32, device=gpu_device)
    ctx.asl_pool(ud, rows, T, S, p, s)
    ref = orc.avg_pool1d(u.astype(np.float64), S)
    np.testing.assert_allclose(p.cpu().numpy(), ref, rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(s.cpu().numpy(), ref.sum(axis=0), rtol=4e-6, atol=1e-7)


# ----------------------------------------------------------------------------- rank
def _rank_case(ctx, dev, s: np.ndarray):
    torch = _torch()
    T = s.shape[0]
    sd = torch.from_numpy(s).to(dev)
    out = torch.full((T,), -1, dtype=torch.int32, device=dev)
    ctx.asl_rank(sd, T, out)
    np.testing.assert_array_equal(out.cpu().numpy().astype(np.int64), orc.rank_desc(s.astype(np.float64)))


@pytest.mark.parametrize("T", [1, 2, 63, 64, 65, 2047, 2048, 2049, 5000, 32736, 131040, 262080])
def test_rank_random_with_ties(ctx, gpu_device, T):
    rng = np.random.default_rng(T)
    s = rng.standard_normal(T).astype(np.float32)
    if T > 10:
        s[rng.integers(0, T, T // 4)] = s[rng.integers(0, T, T // 4)]     # exact ties
        s[rng.integers(0, T, T // 8)] = 0.0
        s[rng.integers(0, T, T // 8)] = -0.0                               # -0 ties with +0
    _rank_case(ctx, gpu_device, s)


@pytest.mark.parametrize("T", [524288, 524289, 700001])
def test_rank_beyond_the_small_tile_limit(gpu_device, T):
    """Above 256 tiles of 2048 the sort switches to tiles of 8192 elements: the last size that still uses
    the small tiles, the first that does not, and a ragged larger one."""
    torch = _torch()
    c = asl.Asl(T, 1, 32)
    rng = np.random.default_rng(T)
    s = np.round(rng.standard_normal(T), 2).astype(np.float32)        # heavy ties
    sd = torch.from_numpy(s).to(gpu_device)
    out = torch.full((T,), -1, dtype=torch.int32, device=gpu_device)
    c.asl_rank(sd, T, out)
    np.testing.assert_array_equal(out.cpu().numpy().astype(np.int64), orc.rank_desc(s.astype(np.float64)))
    assert c.asl_device_fault() == 0
    c.close()


def test_rank_special(ctx, gpu_device):
    T = 5000
    _rank_case(ctx, gpu_device, np.ones(T, dtype=np.float32))                               # all equal
    _rank_case(ctx, gpu_device, np.arange(T, dtype=np.float32))                             # increasing
    _rank_case(ctx, gpu_device, -np.arange(T, dtype=np.float32))                            # decreasing
    _rank_case(ctx, gpu_device, np.exp(np.random.default_rng(1).normal(0, 3, T)).astype(np.float32))
    tiny = (np.random.default_rng(2).random(T) * 1e-40).astype(np.float32)                  # denormals
    _rank_case(ctx, gpu_device, tiny)


def test_rank_is_deterministic(ctx, gpu_device):
    torch = _torch()
    T = 131040
    s = torch.from_numpy(np.random.default_rng(3).random(T, dtype=np.float32)).to(gpu_device)
    a = torch.empty(T, dtype=torch.int32, device=gpu_device)
    b = torch.empty(T, dtype=torch.int32, device=gpu_device)
    ctx.asl_rank(s, T, a)
    ctx.asl_rank(s, T, b)
    assert torch.equal(a, b)


@pytest.mark.parametrize("T", [2048 * 3 - 1, 2048 * 3, 2048 * 3 + 1, 4095, 4096, 4097, 64 * 33 + 7])
def test_rank_and_select_at_tile_boundaries(ctx, gpu_device, T):
    """Sizes one below, at and one above multiples of the sort tile (2048) and the select tile (4096)."""
    rng = np.random.default_rng(T)
    s = np.round(rng.standard_normal(T), 2).astype(np.float32)            # heavy ties
    _rank_case(ctx, gpu_device, s)
    for budget in (9, T // 3 + 8, T + 8):                                   # k = 1, ~T/3, T
        _select_case(ctx, gpu_device, np.stack([s, -s]), budget, 8)


# ----------------------------------------------------------------------------- statistic
def _stat_case(ctx, dev, R: np.ndarray, l_obs: int, k: int, tau: float, layer_idx: int,
               init_var=None):
    """Place the rows of R (oldest first) in the ring as the library expects and run asl_rankvar."""
    torch = _torch()
    n, T = R.shape
    ring = np.full((l_obs, T), 10**9, dtype=np.int32)                 # poison unused rows
    for j in range(n):
        layer = layer_idx - (n - 1) + j
        ring[layer % l_obs] = R[j]
    ringd = torch.from_numpy(ring).to(dev)
    state = asl.new_state(dev)
    asl.write_state(state, init_var=init_var or 0.0, init_set=int(init_var is not None),
                    n_valid_rows=n, last_layer=layer_idx)
    out = asl.new_stat(dev)
    ctx.asl_rankvar(ringd, l_obs, T, layer_idx, 0, k, tau, state, out)
    return asl.read_struct(out, asl.AslStat), asl.read_struct(state, asl.AslState)


@pytest.mark.parametrize("n,l_obs,T,k", [(2, 8, 100, 10), (8, 8, 5000, 300), (5, 8, 32736, 992),
                                         (8, 8, 131040, 2016), (3, 3, 1000, 1000), (8, 8, 262080, 4032),
                                         # more rows than one load batch holds; rings that wrap part-way
                                         (12, 12, 3001, 200), (9, 16, 70001, 500), (17, 24, 131073, 640),
                                         (64, 64, 2500, 100)])
def test_rankvar_exact(ctx, gpu_device, n, l_obs, T, k):
    rng = np.random.default_rng(n + T)
    base = rng.standard_normal(T)
    R = np.stack([orc.rank_desc(base + 0.5 * rng.standard_normal(T)) for _ in range(n)])
    ref = orc.rank_variance(R, k)
    st, state = _stat_case(ctx, gpu_device, R, l_obs, k, tau=0.3, layer_idx=37)
    assert st.evaluated == 1 and st.n_rows == n
    assert st.numerator == ref.numerator and st.union_size == ref.union_size
    assert st.var_top == ref.var_top                                   # same integer, same single division
    assert st.rel_var == 1.0 and st.selected == 0                      # first evaluation: relative variance 1
    assert state.init_set == 1 and state.init_var == ref.var_top and state.n_valid_rows == n
    # second evaluation against a given init_var: decision and release of the ring
    st2, state2 = _stat_case(ctx, gpu_device, R, l_obs, k, tau=0.3, layer_idx=37, init_var=ref.var_top * 4)
    assert st2.rel_var == ref.var_top / (ref.var_top * 4) and st2.selected == 1
    assert state2.n_valid_rows == 0 and state2.init_var == ref.var_top * 4


def test_rankvar_guards_and_degenerate(ctx, gpu_device):
    torch = _torch()
    T = 300
    R = np.stack([np.arange(T), np.arange(T)])
    st, state = _stat_case(ctx, gpu_device, R[:1], 8, 10, 0.3, layer_idx=12)          # one row only
    assert st.evaluated == 0 and st.selected == 0 and state.init_set == 0
    st, state = _stat_case(ctx, gpu_device, R, 8, 10, 0.3, layer_idx=12)              # identical rows
    assert st.evaluated == 1 and st.var_top == 0.0 and np.isnan(st.rel_var) and st.selected == 0
    assert state.init_set == 1 and state.init_var == 0.0
    st, _ = _stat_case(ctx, gpu_device, np.stack([np.arange(T), np.arange(T)[::-1]]), 8, 10, 0.3,
                       layer_idx=13, init_var=0.0)
    assert np.isinf(st.rel_var) and st.selected == 0
    # layer below L_min: nothing evaluated, state untouched
    ring = torch.zeros((8, T), dtype=torch.int32, device=gpu_device)
    state = asl.new_state(gpu_device)
    asl.write_state(state, n_valid_rows=5, last_layer=4)
    out = asl.new_stat(gpu_device)
    ctx.asl_rankvar(ring, 8, T, 4, 10, 10, 0.3, state, out)
    assert asl.read_struct(out, asl.AslStat).evaluated == 0
    assert asl.read_struct(state, asl.AslState).n_valid_rows == 5


# ----------------------------------------------------------------------------- select
def _select_case(ctx, dev, scores: np.ndarray, budget: int, W: int):
    torch = _torch()
    rows, T = scores.shape
    N = T + W
    p = asl.make_params(rows, rows, 64, N, W, 7, budget)
    k = min(budget, N) - W
    sd = torch.from_numpy(scores).to(dev)
    out = torch.full((rows, k + W), -7, dtype=torch.int32, device=dev)
    ctx.asl_select_topk(p, sd, rows, out)
    ref = orc.select_indices(scores.astype(np.float64), k, W)
    np.testing.assert_array_equal(out.cpu().numpy().astype(np.int64), ref)


@pytest.mark.parametrize("rows,T,budget,W", [(1, 10, 6, 2), (2, 496, 128, 16), (8, 32736, 2048, 32),
                                             (8, 131040, 2048, 32), (1, 131040, 2048, 32),
                                             (8, 262080, 4096, 64), (3, 4097, 5000, 8), (2, 9000, 33, 32)])
def test_select_random_with_ties(ctx, gpu_device, rows, T, budget, W):
    rng = np.random.default_rng(T + rows)
    s = rng.random((rows, T), dtype=np.float32)
    if T > 100:
        s = np.round(s, 3).astype(np.float32)           # many exact ties around the threshold
    _select_case(ctx, gpu_device, s, budget, W)


def test_rank_select_pool_random_shapes(ctx, gpu_device):
    """Forty seeded random cases: sizes, budgets, window widths, tie densities and value ranges drawn at
    random (positive-only scores, mixed signs, a few distinct values, tiny magnitudes)."""
    rng = np.random.default_rng(20260127)
    for case in range(40):
        T = int(rng.integers(1, 9000))
        rows = int(rng.integers(1, 4))
        W = int(rng.integers(1, 40))
        budget = W + int(rng.integers(1, T + 20))
        kind = case % 4
        if kind == 0:
            s = rng.random((rows, T)).astype(np.float32)                          # positive, few ties
        elif kind == 1:
            s = np.round(rng.standard_normal((rows, T)), 1).astype(np.float32)     # mixed signs, heavy ties
        elif kind == 2:
            s = rng.integers(0, 3, (rows, T)).astype(np.float32)                   # three distinct values
        else:
            s = (rng.random((rows, T)) * 1e-30).astype(np.float32)                 # tiny magnitudes / denormals
        print(f"case {case}: T={T} rows={rows} W={W} budget={budget} kind={kind}", flush=True)
        _rank_case(ctx, gpu_device, s[0])
        _select_case(ctx, gpu_device, s, budget, W)


@pytest.mark.parametrize("rows,T,budget", [(96, 100000, 1056), (96, 100001, 1056), (300, 9000, 532),
                                           (128, 131040, 2080), (130, 100001, 1056), (256, 20000, 8192),
                                           (129, 70000, 35000), (128, 5, 4), (140, 4096, 33)])
def test_select_many_rows(gpu_device, rows, T, budget):
    """96 rows x 25 tiles: the tile count from which the filter stage runs as many small workgroups
    (a few rows take one round of large ones); with T a multiple of four the rows are read four scores
    per load, with T = 100001 one at a time.  300 rows: more than the candidate buffers hold at once,
    so the three launches run twice.  Further: 128 full-size rows, a budget of 8192 on many rows, a
    budget of half the row (the candidates overflow: selection from the whole row), rows of five
    tokens, rows of exactly one tile."""
    W = 32 if T > 100 else 2
    rng = np.random.default_rng(rows + T)
    s = np.round(rng.random((rows, T), dtype=np.float32), 4).astype(np.float32)
    c = asl.Asl(T + W, rows, rows * W)
    try:
        _select_case(c, gpu_device, s, budget, W)
        assert c.asl_device_fault() == 0
    finally:
        c.close()


def test_select_many_hard_rows(gpu_device):
    """Many rows at once whose sampled bound is useless or whose candidates overflow (top tokens
    clustered at either end or inside one tile, a few distinct values, all equal, sorted either way,
    negative scores), several of each kind in one call, beside ordinary rows."""
    rng = np.random.default_rng(77)
    rows, T, W, budget = 144, 70000, 32, 2048
    s = rng.random((rows, T), dtype=np.float32)
    for r in range(rows):
        kind = r % 9
        if kind == 1:
            s[r, :3000] += 10.0
        elif kind == 2:
            s[r, -3000:] += 10.0
        elif kind == 3:
            s[r] = rng.integers(0, 4, T).astype(np.float32)
        elif kind == 4:
            s[r] = 0.25
        elif kind == 5:
            s[r] = np.sort(s[r])[::-1]
        elif kind == 6:
            s[r] = np.sort(s[r])
        elif kind == 7:
            s[r, 16384:20480] = 5.0 + rng.random(4096, dtype=np.float32)
        elif kind == 8:
            s[r] = -s[r] - 1.0
    c = asl.Asl(T + W, rows, rows * W)
    try:
        _select_case(c, gpu_device, np.ascontiguousarray(s), budget, W)
        _select_case(c, gpu_device, np.ascontiguousarray(s), W + 1, W)             # k = 1
        _select_case(c, gpu_device, np.ascontiguousarray(s[:, :3000]), 4000, W)    # budget >= N: keep all
        assert c.asl_device_fault() == 0
    finally:
        c.close()


@pytest.mark.parametrize("rows", [3, 130])
def test_select_around_zero(gpu_device, rows):
    """Scores drawn from a few values on both sides of zero (+0, -0, denormals of either sign, small
    and large magnitudes), so that for one budget or another the threshold falls on each of them:
    -0 and +0 tie (lower index first), denormals do not count as zero, negative scores order by
    magnitude downwards (the filter decides on the scores' bits: every sign and zero case matters)."""
    rng = np.random.default_rng(rows)
    T, W = 20000, 16
    vals = np.array([0.0, -0.0, 1e-40, -1e-40, 1e-45, -1e-45, 1.0, -1.0, 3e38, -3e38, 1e-20, -1e-20], dtype=np.float32)
    s = vals[rng.integers(0, len(vals), (rows, T))]
    assert np.signbit(s).any() and (s == 0).any()
    c = asl.Asl(T + W, rows, rows * W)
    try:
        for k in (1, 900, 1700, 2500, 3400, 5000, 8400, 10000, 12000, 15000, 19999):
            _select_case(c, gpu_device, s, k + W, W)
        assert c.asl_device_fault() == 0
    finally:
        c.close()


def test_select_special(ctx, gpu_device):
    T, W = 6000, 16
    _select_case(ctx, gpu_device, np.ones((2, T), dtype=np.float32), 100, W)               # all equal: first k
    _select_case(ctx, gpu_device, np.zeros((1, T), dtype=np.float32), 100, W)
    s = np.random.default_rng(5).standard_normal((2, T)).astype(np.float32)                 # negatives
    _select_case(ctx, gpu_device, s, 1000, W)
    _select_case(ctx, gpu_device, s, T + W + 50, W)                                         # budget >= N: keep all


@pytest.mark.parametrize("kind", ["clustered-front", "clustered-back", "few-values", "half-kept", "all-equal-large",
                                  "sorted-desc", "sorted-asc", "one-outlier-tile"])
def test_select_when_the_sampled_bound_does_not_help(ctx, gpu_device, kind):
    """Inputs on which the top-k's sampled bound is useless or its candidate buffers overflow, so the
    finishing kernel selects from the whole row: every top token inside one 4096-token tile (the tile's
    2048-slot segment overflows), a handful of distinct values (tens of thousands of keys tie with the
    bound), half the row kept (the candidates exceed what one workgroup holds), monotone rows."""
    rng = np.random.default_rng(len(kind) * 31 + ord(kind[0]))
    T, W = 70000, 32
    budget = 2048
    s = rng.random((3, T), dtype=np.float32)
    if kind == "clustered-front":
        s[:, :3000] += 10.0
    elif kind == "clustered-back":
        s[:, -3000:] += 10.0
    elif kind == "few-values":
        s = rng.integers(0, 4, (3, T)).astype(np.float32)
    elif kind == "half-kept":
        budget = T // 2
    elif kind == "all-equal-large":
        s[:] = 0.25
    elif kind == "sorted-desc":
        s = np.sort(s, axis=1)[:, ::-1].copy()
    elif kind == "sorted-asc":
        s = np.sort(s, axis=1)
    elif kind == "one-outlier-tile":
        s[1, 8192:12288] = 5.0 + rng.random(4096, dtype=np.float32)      # exactly one tile holds the whole top-k
    _select_case(ctx, gpu_device, np.ascontiguousarray(s), budget, W)


# ----------------------------------------------------------------------------- gather
@pytest.mark.parametrize("cfg", [1, 2])
def test_gather_bit_exact(ctx, gpu_device, cfg):
    torch = _torch()
    L = synth.config_layer(cfg)
    sh = L.shape
    p = gu.params_of(sh)
    kd, vd = gu.to_dev(L.k, sh.dtype, gpu_device), gu.to_dev(L.v, sh.dtype, gpu_device)
    rng = np.random.default_rng(cfg)
    n_idx = sh.k + sh.W
    idx = np.stack([np.sort(rng.choice(sh.N, n_idx, replace=False)) for _ in range(sh.Hk)]).astype(np.int32)
    for idx_rows, I in ((sh.Hk, idx), (1, idx[:1])):
        Id = torch.from_numpy(I).to(gpu_device)
        ko = torch.zeros((sh.Hk, n_idx, sh.d), dtype=kd.dtype, device=gpu_device)
        vo = torch.zeros_like(ko)
        ctx.asl_gather_kv(p, kd, vd, Id, idx_rows, n_idx, ko, vo)
        kr, vr = orc.gather_kv(L.k, L.v, I if idx_rows > 1 else I[0])
        assert np.array_equal(ko.float().cpu().numpy(), kr)            # bf16/f32 values are exact in fp32
        assert np.array_equal(vo.float().cpu().numpy(), vr)
    # identity index = plain copy; strided K (token stride 2d) reads the right rows
    Id = torch.arange(sh.N, dtype=torch.int32, device=gpu_device)
    ko = torch.zeros_like(kd)
    ctx.asl_gather_kv(p, kd, None, Id, 1, sh.N, ko, None)
    assert torch.equal(ko, kd)
    wide = torch.zeros((sh.Hk, sh.N, 2 * sh.d), dtype=kd.dtype, device=gpu_device)
    wide[:, :, :sh.d] = kd
    p2 = asl.make_params(sh.Hq, sh.Hk, sh.d, sh.N, sh.W, sh.S, sh.budget, dtype=p.dtype,
                         k_strides=(sh.N * 2 * sh.d, 2 * sh.d))
    ko.zero_()
    ctx.asl_gather_kv(p2, wide, None, Id, 1, sh.N, ko, None)
    assert torch.equal(ko, kd)


def test_gather_empty_and_f32(ctx, gpu_device):
    torch = _torch()
    sh = synth.shape_of(1)                                   # fp32 storage, d = 64
    L = synth.config_layer(1)
    p = gu.params_of(sh)
    kd, vd = gu.to_dev(L.k, "f32", gpu_device), gu.to_dev(L.v, "f32", gpu_device)
    ko = torch.full((sh.Hk, 4, sh.d), 7.0, device=gpu_device)
    vo = torch.full_like(ko, 7.0)
    I = torch.tensor([[3, 0, 511, 3]], dtype=torch.int32, device=gpu_device)     # repeats allowed
    ctx.asl_gather_kv(p, kd, vd, I, 1, 0, ko, vo)                                  # n_idx = 0: nothing written
    assert torch.all(ko == 7.0) and torch.all(vo == 7.0)
    ctx.asl_gather_kv(p, kd, vd, I, 1, 4, ko, vo)
    assert np.array_equal(ko.cpu().numpy(), L.k[:, [3, 0, 511, 3], :])
    assert np.array_equal(vo.cpu().numpy(), L.v[:, [3, 0, 511, 3], :])


# ----------------------------------------------------------------------------- errors
def test_argument_errors(ctx, gpu_device):
    torch = _torch()
    sh = synth.shape_of(1)
    good = gu.params_of(sh)
    t = torch.zeros(16, device=gpu_device)

    def expect(status, fn):
        with pytest.raises(asl.AslError) as e:
            fn()
        assert e.value.status == status, str(e.value)

    def with_(**kw):
        p = gu.params_of(sh)
        for a, b in kw.items():
            setattr(p, a, b)
        return p

    sc = lambda p: ctx.asl_score_layer(p, t, t, t, t)
    expect(asl.ASL_EINVAL, lambda: sc(with_(n_q_heads=3)))               # Hq % Hk
    expect(asl.ASL_EINVAL, lambda: sc(with_(window=0)))
    expect(asl.ASL_EINVAL, lambda: sc(with_(window=sh.N)))               # W < N
    expect(asl.ASL_EINVAL, lambda: sc(with_(pool_kernel=4)))             # even S
    expect(asl.ASL_EINVAL, lambda: sc(with_(budget=sh.W)))               # k <= 0
    expect(asl.ASL_EUNSUPPORTED, lambda: sc(with_(dtype=5)))
    expect(asl.ASL_EINVAL, lambda: sc(with_(flags=64)))                  # unknown flag bit
    expect(asl.ASL_ENOMEM, lambda: sc(with_(seq_len=1 << 20)))           # beyond the context limits
    expect(asl.ASL_EINVAL, lambda: ctx.asl_score_layer(good, None, t, t, t))
    expect(asl.ASL_EINVAL, lambda: ctx.asl_rank(t, 0, t))
    expect(asl.ASL_EINVAL, lambda: ctx.asl_pool(t, 1, 16, 2, t))
    expect(asl.ASL_EINVAL, lambda: ctx.asl_gather_kv(good, t, None, t, 3, 4, t, None))   # idx_rows not 1/Hk
    expect(asl.ASL_EINVAL, lambda: ctx.asl_rankvar(t, 1, 16, 0, 0, 4, 0.3, t, t))        # L_obs < 2
    expect(asl.ASL_EUNSUPPORTED, lambda: ctx.asl_rankvar(t, 64, 2_000_000, 0, 0, 4, 0.3, t, t))
    # a shape without an MFMA scoring kernel (d = 96) at a size the plain kernels are not meant for
    big = asl.Asl(1 << 20, 1, 64 * 128)
    pb = asl.make_params(64, 1, 96, 1 << 20, 128, 7, 4096)
    expect(asl.ASL_EUNSUPPORTED, lambda: big.asl_score_layer(pb, t, t, t, t))
    expect(asl.ASL_EUNSUPPORTED, lambda: big.asl_window_lse(pb, t, t, t))
    big.close()
    # ranking more tokens than one launch can hold
    expect(asl.ASL_ENOMEM, lambda: ctx.asl_rank(t, 1 << 22, t))
    h = C.c_void_p()
    assert ctx.lib.asl_create(C.byref(h), 0, 1, 8, 8) == asl.ASL_EINVAL
    assert ctx.lib.asl_create(C.byref(h), 99, 1024, 8, 8) == asl.ASL_EHIP


def test_stat_written_straight_to_pinned_host_memory(ctx, gpu_device):
    """The decision record may live in page-locked host memory: the statistic kernel writes it there
    and the host reads it after a stream synchronisation, with no copy of its own."""
    import torch
    T, l_obs, k = 5000, 4, 300
    rng = np.random.default_rng(5)
    ring = torch.zeros((l_obs, T), dtype=torch.int32, device=gpu_device)
    state = asl.new_state(gpu_device)
    stat_dev = asl.new_stat(gpu_device)
    stat_host = torch.zeros(stat_dev.numel(), dtype=torch.uint8).pin_memory()
    p = asl.make_params(4, 2, 64, T + 8, 8, 7, k + 8)
    for layer in range(l_obs + 2):
        s = torch.from_numpy(rng.standard_normal(T).astype(np.float32)).to(gpu_device)
        st2 = state.clone()
        ctx.asl_rank_stat(p, s, layer, 0, l_obs, 0.0, ring.clone(), st2, stat_dev)
        ctx.asl_rank_stat(p, s, layer, 0, l_obs, 0.0, ring, state, stat_host)
        torch.cuda.synchronize()
        assert bytes(stat_host.numpy().tobytes()) == bytes(stat_dev.cpu().numpy().tobytes())
    assert asl.AslStat.from_buffer_copy(bytes(stat_host.numpy().tobytes())).evaluated == 1
