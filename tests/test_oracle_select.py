"""Pins for the oracle's ranking, statistic, decision, top-k and gather steps
(Alg. 1 steps 9-12, Alg. 2, Sec. 4.1 top(L) / var_top / relative-variance equations)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import asl_oracle as orc
from paper_2601_07667_amd import synth


# ----------------------------------------------------------------------------- RankDesc
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_rank_matches_counting_definition(seed):
    rng = np.random.default_rng(seed)
    s = rng.standard_normal(200)
    s[rng.integers(0, 200, 40)] = s[rng.integers(0, 200, 40)]   # plant ties
    s = np.round(s, 1)                                            # and many more ties
    r = orc.rank_desc(s)
    np.testing.assert_array_equal(r, orc.rank_desc_bruteforce(s))
    assert sorted(r.tolist()) == list(range(200))                 # a permutation


def test_rank_special_inputs():
    T = 64
    np.testing.assert_array_equal(orc.rank_desc(np.ones(T)), np.arange(T))              # all equal
    np.testing.assert_array_equal(orc.rank_desc(-np.arange(T, dtype=float)), np.arange(T))   # decreasing
    np.testing.assert_array_equal(orc.rank_desc(np.arange(T, dtype=float)), T - 1 - np.arange(T))
    # the largest score gets rank 0
    s = np.array([0.1, 5.0, 0.3, 5.0])
    np.testing.assert_array_equal(orc.rank_desc(s), [3, 0, 2, 1])


# ----------------------------------------------------------------------------- k
def test_budget_k_identity():
    """Alg. 1 step 9 and Alg. 2 step 6 give the same k."""
    for budget in (1, 17, 128, 2048, 10**6):
        for N in (18, 512, 4096):
            for W in (1, 16, 17):
                if W < N:
                    assert orc.budget_k(budget, N, W) == min(budget - W, N - W)


# ----------------------------------------------------------------------------- union + variance
def _brute_rank_variance(R, k):
    """Explicit per-row top-k (argsort), Python set union, exact rationals."""
    n, T = R.shape
    union = set()
    for l in range(n):
        union |= set(np.argsort(R[l], kind="stable")[:k].tolist())
    tot = Fraction(0)
    for t in sorted(union):
        col = [int(x) for x in R[:, t]]
        mean = Fraction(sum(col), n)
        tot += sum((Fraction(c) - mean) ** 2 for c in col) / n
    return tot / len(union), len(union)


@pytest.mark.parametrize("n,T,k", [(2, 30, 5), (8, 100, 13), (3, 64, 64), (5, 50, 1)])
def test_rank_variance_matches_bruteforce(n, T, k):
    rng = np.random.default_rng(n * 1000 + T)
    R = np.stack([rng.permutation(T) for _ in range(n)])
    st = orc.rank_variance(R, k)
    v, m = _brute_rank_variance(R, k)
    assert st.union_size == m and st.n_rows == n
    assert Fraction(st.numerator, n * n * m) == v                 # exact
    assert abs(st.var_top - float(v)) <= 1e-15 * float(v)
    assert k <= m <= min(T, k * n)                                # App. B.1: m <= k * L_obs


def test_rank_variance_closed_forms():
    T = 101
    r0 = np.random.default_rng(4).permutation(T)
    # identical rows -> zero variance
    st = orc.rank_variance(np.stack([r0] * 4), 10)
    assert st.numerator == 0 and st.var_top == 0.0
    # two rows, second the reversal of the first, everything in the union:
    # per-token variance ((2r-(T-1))/2)^2, mean over a permutation = (T^2-1)/12
    st = orc.rank_variance(np.stack([r0, T - 1 - r0]), T)
    assert st.union_size == T
    assert Fraction(st.numerator, 4 * T) == Fraction(T * T - 1, 12)
    # shift invariance (0- vs 1-based ranks) of the variance
    R = np.stack([np.random.default_rng(s).permutation(T) for s in range(5)])
    a = orc.rank_variance(R, T)
    s1 = (R + 1).sum(0)
    s2 = ((R + 1) ** 2).sum(0)
    assert a.numerator == int((5 * s2 - s1 * s1).sum())


def test_rank_variance_statistical():
    """n independent uniform permutations, whole set in the union:
    E[population variance] = (n-1)/n * (T^2-1)/12."""
    T, n = 400, 8
    rng = np.random.default_rng(7)
    vals = [orc.rank_variance(np.stack([rng.permutation(T) for _ in range(n)]), T).var_top
            for _ in range(20)]
    expect = (n - 1) / n * (T * T - 1) / 12
    assert abs(np.mean(vals) / expect - 1) < 0.02


def test_union_uses_every_row():
    """A token that is top-k only in an old row still enters the union."""
    T = 10
    new = np.arange(T)
    old = np.arange(T)[::-1].copy()
    st = orc.rank_variance(np.stack([old, new]), 2)
    assert st.union_size == 4                                      # {0,1} from new, {8,9} from old


# ----------------------------------------------------------------------------- Alg. 2 driver
def _run_sweep(scores_per_layer, budget, W, L_min, L_obs, tau):
    st = orc.SelectState.new(L_obs)
    out = []
    for l, s in enumerate(scores_per_layer):
        st.push(l, orc.rank_desc(s))
        d = orc.select_tokens(st, l, budget, W, L_min, tau)
        out.append(d)
        if d.selected:
            break
    return out


def test_select_tokens_basics():
    T, W, budget = 300, 8, 40
    z = synth.sweep_latents(T, 32)
    scores = [synth.sweep_scores(z[l]) for l in range(32)]
    out = _run_sweep(scores, budget, W, L_min=10, L_obs=8, tau=0.5)
    for l, d in enumerate(out):
        if l < 10:
            assert not d.evaluated and d.select_idx is None       # guard layer < L_min
    assert out[10].evaluated and out[10].rel_var == 1.0           # relative variance at L_min is 1
    assert out[10].n_rows == 8
    last = out[-1]
    assert last.selected and 10 < len(out) - 1 <= 31
    idx = last.select_idx
    k = min(budget - W, T)
    assert len(idx) == k + W == min(budget, T + W)
    assert np.all(np.diff(idx) > 0)                                # sorted, unique
    np.testing.assert_array_equal(idx[-W:], np.arange(T, T + W))  # window tokens present
    # J_last equals the top-k of the last layer's scores
    np.testing.assert_array_equal(idx[:k], orc.topk_indices(scores[len(out) - 1], k))


def test_tau_grid_monotone():
    """Larger tau selects at an earlier-or-equal layer (Sec. 5.6 ablation grid)."""
    T, W, budget = 500, 8, 60
    z = synth.sweep_latents(T, 32)
    scores = [synth.sweep_scores(z[l]) for l in range(32)]
    layers = []
    for tau in (0.2, 0.3, 0.4, 0.5, 0.6):
        out = _run_sweep(scores, budget, W, 10, 8, tau)
        layers.append(len(out) - 1 if out[-1].selected else 99)
    assert layers == sorted(layers, reverse=True)
    assert layers[-1] < 99


def test_decision_invariant_to_variance_normaliser():
    """Sample (1/(n-1)) instead of population (1/n) variance rescales var_top by a constant,
    so the relative variance is unchanged."""
    T, n, k = 200, 8, 25
    rng = np.random.default_rng(3)
    Ra = np.stack([rng.permutation(T) for _ in range(n)])
    base = rng.permutation(T)
    Rb = np.stack([np.argsort(np.argsort(base + rng.normal(0, 20, T))) for _ in range(n)])
    a, b = orc.rank_variance(Ra, k), orc.rank_variance(Rb, k)
    rel_pop = b.var_top / a.var_top

    def sample(R):
        u = (R < k).any(axis=0)
        return R[:, u].var(axis=0, ddof=1).mean()
    rel_smp = sample(Rb) / sample(Ra)
    assert abs(rel_pop / rel_smp - 1) < 1e-12
    assert abs(a.var_top - Ra[:, (Ra < k).any(0)].var(axis=0).mean()) < 1e-9 * a.var_top


def test_degenerate_init_var_zero_never_selects():
    T, W = 50, 4
    st = orc.SelectState.new(3)
    r = np.arange(T)
    for l in range(3):
        st.push(l, r)
    d = orc.select_tokens(st, 2, 20, W, L_min=2, tau=0.3)
    assert d.evaluated and not d.selected and np.isnan(d.rel_var) and st.init_var == 0.0
    st.push(3, r[::-1].copy())
    d = orc.select_tokens(st, 3, 20, W, L_min=2, tau=0.3)
    assert not d.selected and np.isinf(d.rel_var)


def test_fewer_than_two_rows_not_evaluated():
    st = orc.SelectState.new(8)
    st.push(0, np.arange(10))
    d = orc.select_tokens(st, 0, 6, 2, L_min=0, tau=0.3)
    assert not d.evaluated and st.init_var is None


def test_cache_released_after_selection():
    """Alg. 2 step 13: the selection empties the rank cache; the next layer's push starts from a
    single row, which is not evaluated (fewer than two rows) and leaves init_var untouched."""
    T, W, budget = 120, 4, 24
    rng = np.random.default_rng(11)
    st = orc.SelectState.new(4)
    base = rng.permutation(T)
    st.push(0, rng.permutation(T))
    st.push(1, rng.permutation(T))
    d = orc.select_tokens(st, 1, budget, W, L_min=1, tau=0.3)     # first evaluation: rel = 1, no selection
    assert d.evaluated and not d.selected and d.rel_var == 1.0 and len(st.rows) == 2
    init = st.init_var
    for l in (2, 3, 4, 5):                                         # identical rows: variance collapses to 0
        st.push(l, base)
        d = orc.select_tokens(st, l, budget, W, L_min=1, tau=0.3)
        if d.selected:
            break
    assert d.selected and l == 5 and d.var_top == 0.0              # the 4-row window holds 4 equal rows
    assert st.rows == [] and st.init_var == init                   # step 13: cache cleared, init_var kept
    k = budget - W
    np.testing.assert_array_equal(d.select_idx[:k], np.sort(np.argsort(base, kind="stable")[:k]))
    st.push(6, rng.permutation(T))
    d = orc.select_tokens(st, 6, budget, W, L_min=1, tau=0.3)
    assert len(st.rows) == 1 and not d.evaluated and d.n_rows == 1 and d.select_idx is None
    assert st.init_var == init


@pytest.mark.parametrize("rows_available", [2, 3, 5])
def test_partial_window_uses_the_rows_available(rows_available):
    """Evaluation at L_min with 2 <= rows < L_obs rows in the cache: n is the number of rows
    held, and var_top is the brute-force mean variance over those rows only."""
    T, W, budget, L_obs = 90, 6, 20, 8
    rng = np.random.default_rng(20 + rows_available)
    st = orc.SelectState.new(L_obs)
    R = [rng.permutation(T) for _ in range(rows_available)]
    for l, r in enumerate(R):
        st.push(l, r)
    d = orc.select_tokens(st, rows_available - 1, budget, W, L_min=rows_available - 1, tau=0.3)
    assert d.evaluated and d.n_rows == rows_available and d.rel_var == 1.0
    want, m = _brute_rank_variance(np.stack(R), budget - W)
    assert d.union_size == m
    assert abs(d.var_top - float(want)) <= 1e-12 * float(want)
    # one more row: the window grows by one (still below L_obs) and the divisor stays init_var
    st.push(rows_available, rng.permutation(T))
    d2 = orc.select_tokens(st, rows_available, budget, W, L_min=rows_available - 1, tau=0.0)
    assert d2.n_rows == rows_available + 1
    want2, _ = _brute_rank_variance(np.stack([r for _, r in st.rows]), budget - W)
    assert abs(d2.rel_var - float(want2 / want)) <= 1e-12 * float(want2 / want)


# ----------------------------------------------------------------------------- top-k, gather
def test_topk_exhaustive_small():
    """All score vectors over a 3-letter alphabet of length 6, every k: compare with the
    definition via explicit (score desc, index asc) sort."""
    import itertools
    for vals in itertools.product([0.0, 1.0, 2.0], repeat=6):
        s = np.array(vals)
        order = sorted(range(6), key=lambda t: (-s[t], t))
        for k in range(0, 7):
            np.testing.assert_array_equal(orc.topk_indices(s, k), sorted(order[:k]))
    s = np.random.default_rng(0).standard_normal(40)
    np.testing.assert_array_equal(orc.topk_indices(s, 40), np.arange(40))   # k = T keeps everything
    # consistent with RankDesc: top-k == {rank < k}
    r = orc.rank_desc(s)
    np.testing.assert_array_equal(orc.topk_indices(s, 7), np.nonzero(r < 7)[0])


def test_select_indices_rows_and_window():
    rng = np.random.default_rng(5)
    P = rng.random((3, 30))
    I = orc.select_indices(P, 5, 4)
    assert I.shape == (3, 9)
    for g in range(3):
        np.testing.assert_array_equal(I[g, 5:], [30, 31, 32, 33])
        np.testing.assert_array_equal(I[g, :5], orc.topk_indices(P[g], 5))


def test_gather_matches_element_loop():
    """Alg. 1 step 12 element by element: out[g, i, c] = k[g, idx[g or shared, i], c], with
    repeated and unsorted indices and per-head rows that differ from each other."""
    rng = np.random.default_rng(6)
    k = rng.standard_normal((3, 20, 4))
    v = rng.standard_normal((3, 20, 4))
    idx = np.array([[1, 5, 19, 5], [0, 2, 3, 0], [9, 8, 7, 19]])
    ko, vo = orc.gather_kv(k, v, idx)
    assert ko.shape == vo.shape == (3, 4, 4)
    for g in range(3):
        for i in range(4):
            for c in range(4):
                assert ko[g, i, c] == k[g, idx[g, i], c]
                assert vo[g, i, c] == v[g, idx[g, i], c]
    shared = np.array([4, 2, 4])                                   # one index row for every head
    ko, vo = orc.gather_kv(k, v, shared)
    assert ko.shape == (3, 3, 4)
    for g in range(3):
        for i in range(3):
            for c in range(4):
                assert ko[g, i, c] == k[g, shared[i], c]
                assert vo[g, i, c] == v[g, shared[i], c]
    ko, vo = orc.gather_kv(k, v, np.arange(20))                    # identity selection
    np.testing.assert_array_equal(ko, k)
    np.testing.assert_array_equal(vo, v)
    ko[0, 0, 0] = 99.0                                             # a copy, not a view
    assert k[0, 0, 0] != 99.0


def test_propagate_tokens_is_row_selection():
    rng = np.random.default_rng(8)
    hidden = rng.standard_normal((30, 5))
    idx = np.array([0, 3, 4, 17, 28, 29])
    out = orc.propagate_tokens(hidden, idx)
    assert out.shape == (6, 5)
    for i, t in enumerate(idx):
        for c in range(5):
            assert out[i, c] == hidden[t, c]
    out[0, 0] = 99.0                                               # a copy, not a view
    assert hidden[0, 0] != 99.0


def test_get_ranks_whole_on_config1():
    L = synth.config_layer(1)
    sh = L.shape
    out = orc.get_ranks(L.q_obs, L.k, L.v, sh.W, sh.S, sh.budget)
    assert out["k"] == 112 and out["I"].shape == (sh.Hk, 128)
    assert out["K"].shape == (sh.Hk, 128, sh.d)
    np.testing.assert_array_equal(out["rank"], orc.rank_desc_bruteforce(out["s"]))
    for g in range(sh.Hk):
        np.testing.assert_array_equal(out["K"][g], L.k[g][out["I"][g]])


# ----------------------------------------------------------------------------- paper's stated hyper-parameters
def test_paper_hyperparameters_fixture():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_hyperparameters.txt")
    vals = {}
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) == 2:
            vals[line[0]] = float(line[1])
    sh = synth.shape_of(3)
    assert (sh.W, sh.S, sh.budget, sh.L_obs, sh.tau) == (
        vals["window"], vals["pool_kernel"], vals["budget"], vals["L_obs"], vals["tau"])
    assert sh.L_min == vals["L_min_32"] == 32 // 3 and vals["L_min_28"] == 28 // 3
    assert (sh.Hk, sh.d) == (vals["kv_heads"], vals["head_dim"])
    assert sh.k == 2016 and sh.T == 131040
