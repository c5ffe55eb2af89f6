"""CPU oracle for the ASL per-layer token-importance pass.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy implementation of what the paper's GetRanks (Alg. 1) and
SelectTokens (Alg. 2) compute, in the paper's step order and notation.  It exists to check
the HIP library; it shares no code with it and nothing in the product path may import it
(only tests, the smoke check and the benchmark's cpu_baseline leg do).

The method is defined by its steps (a heuristic statistic), so each function is the
corresponding step written out; library primitives (matmul, exp, stable argsort) serve as
steps, with no blocking or fusion.  Every function cites the passage it follows.

Readings taken where the paper is silent or inconsistent (each also pinned or shown
immaterial in the tests):
  * ranks and the token selection use the all-head score  s = sum over KV heads of P
    (Sec. 4.1 "scores" equation; Alg. 2 treats rank_cache[l] as one length-T vector);
    the per-KV-head P is used for the per-head TopK / KV compression of Alg. 1;
  * the layer window is the L_obs rows  layer-L_obs+1 .. layer  of Alg. 2 (the main text's
    L-L_obs .. L would be L_obs+1 rows);
  * variance is the population variance (1/n) of the raw 0-based integer ranks; the
    relative variance, hence the decision, does not depend on 1/n vs 1/(n-1) nor on the
    rank base;
  * RankDesc / TopK ties: the lower token index wins (stable descending order);
  * AvgPool1D pads with zeros and always divides by S; the padding boundary is the end of
    the past-only vector U (window columns are never pulled in); S is odd;
  * TopK output and select_idx are in ascending token order, window indices last.

Pins: every function here is pinned by tests/test_oracle_*.py (closed forms, brute force,
textbook routines, invariants).  The paper prints no worked numerical example (its figure
of the variance computation is an image), so fidelity to the authors' own code on the
readings above is unpinned; parity of each function with its definition is pinned.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


# --------------------------------------------------------------------------- Alg. 1, scoring
def window_logits(q_h: np.ndarray, k_g: np.ndarray, scale: float) -> np.ndarray:
    """Alg. 1 step 5 (inside the softmax): scaled window-query x all-key logits plus the causal
    mask on the last W x W block.  q_h [W,d] (the last W queries of one head), k_g [N,d]
    (all keys of its KV head).  Returns l [W,N]; masked entries are -inf.
    Key T+j (T = N-W) is visible to window row i iff j <= i; past keys are never masked."""
    q_h = np.asarray(q_h, dtype=np.float64)
    k_g = np.asarray(k_g, dtype=np.float64)
    W, N = q_h.shape[0], k_g.shape[0]
    T = N - W
    l = (q_h @ k_g.T) * scale
    i = np.arange(W)[:, None]
    j = np.arange(W)[None, :]
    l[:, T:][j > i] = -np.inf
    return l


def softmax_rows(l: np.ndarray) -> np.ndarray:
    """Alg. 1 step 5: row softmax over all N key columns."""
    m = l.max(axis=1, keepdims=True)
    e = np.exp(l - m)
    return e / e.sum(axis=1, keepdims=True)


def window_attention(q_h: np.ndarray, k_g: np.ndarray, scale: float) -> np.ndarray:
    """Alg. 1 step 5 / Sec. 4.1 PA equation (before pooling): A [W,N] for one query head."""
    return softmax_rows(window_logits(q_h, k_g, scale))


def past_column_sum(A: np.ndarray, W: int) -> np.ndarray:
    """Alg. 1 step 6: U[j] = sum over the W window rows of A[t, j], past columns j < N-W only."""
    T = A.shape[1] - W
    return A[:, :T].sum(axis=0)


def avg_pool1d(U: np.ndarray, S: int) -> np.ndarray:
    """Alg. 1 step 7: AvgPool1D(kernel S, stride 1, pad floor(S/2)) along the last axis,
    zero padding counted in the divisor.  S odd so the length is preserved."""
    if S < 1 or S % 2 == 0:
        raise ValueError("pool kernel S must be odd and >= 1")
    U = np.asarray(U, dtype=np.float64)
    T = U.shape[-1]
    h = S // 2
    out = np.zeros_like(U)
    for delta in range(-h, h + 1):
        lo, hi = max(0, -delta), min(T, T - delta)      # j with 0 <= j+delta < T
        if hi > lo:
            out[..., lo:hi] += U[..., lo + delta:hi + delta]
    return out / S


def score_layer(q_obs: np.ndarray, k: np.ndarray, W: int, S: int,
                scale: Optional[float] = None):
    """Alg. 1 steps 5-8 and the Sec. 4.1 "scores" equation.
    q_obs [Hq,W,d], k [Hk,N,d].  Returns (P [Hk,T], s [T]):
    P = group sums of the pooled per-head column sums, s = sum of P over the KV heads."""
    q_obs = np.asarray(q_obs, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    Hq, Wq, d = q_obs.shape
    Hk, N, _ = k.shape
    assert Wq == W and Hq % Hk == 0 and 1 <= W < N
    G = Hq // Hk
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    T = N - W
    P = np.zeros((Hk, T))
    for h in range(Hq):                                  # one [W,N] tile at a time
        A = window_attention(q_obs[h], k[h // G], scale)           # step 5
        U = past_column_sum(A, W)                                   # step 6
        V = avg_pool1d(U, S)                                        # step 7
        P[h // G] += V                                              # step 8 (sum over G)
    s = P.sum(axis=0)                                    # Sec. 4.1: sum over groups and heads
    return P, s


def row_lse(q_obs: np.ndarray, k: np.ndarray, W: int, scale: Optional[float] = None) -> np.ndarray:
    """Natural-log-sum-exp of each window row's masked, scaled logits: lse [Hq,W].
    (What a prefill attention kernel of the same layer would hand over; Alg. 1 step 5's
    softmax normaliser.)"""
    q_obs = np.asarray(q_obs, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    Hq, _, d = q_obs.shape
    G = Hq // k.shape[0]
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((Hq, W))
    for h in range(Hq):
        l = window_logits(q_obs[h], k[h // G], scale)
        m = l.max(axis=1)
        out[h] = m + np.log(np.exp(l - m[:, None]).sum(axis=1))
    return out


# --------------------------------------------------------------------------- ranks, top-k
def rank_desc(s: np.ndarray) -> np.ndarray:
    """Alg. 1 step 11, RankDesc: rank[t] = #{t': s[t'] > s[t]} + #{t' < t: s[t'] == s[t]}
    (0-based; position of t in the stable descending order).  Returns int64 [T]."""
    s = np.asarray(s)
    order = np.argsort(-s, kind="stable")                # descending, ties by lower index
    rank = np.empty(s.shape[0], dtype=np.int64)
    rank[order] = np.arange(s.shape[0], dtype=np.int64)
    return rank


def rank_desc_bruteforce(s: np.ndarray) -> np.ndarray:
    """The counting definition of RankDesc, O(T^2); for small T only."""
    s = np.asarray(s)
    T = s.shape[0]
    rank = np.zeros(T, dtype=np.int64)
    for t in range(T):
        c = 0
        for u in range(T):
            if s[u] > s[t] or (s[u] == s[t] and u < t):
                c += 1
        rank[t] = c
    return rank


def budget_k(budget: int, N: int, W: int) -> int:
    """Alg. 1 step 9: k = min(KV_budget, N_q) - W   (equal to Alg. 2 step 6: min(budget-W, T))."""
    return min(budget, N) - W


def topk_indices(scores: np.ndarray, k: int) -> np.ndarray:
    """TopK of Alg. 1 step 10 on one row: the indices of the k largest scores, ties to the
    lower index, returned in ascending index order."""
    scores = np.asarray(scores)
    order = np.argsort(-scores, kind="stable")
    return np.sort(order[:k]).astype(np.int64)


def select_indices(scores: np.ndarray, k: int, W: int) -> np.ndarray:
    """Alg. 1 step 10 / Alg. 2 steps 11-12: Concat(TopK(row, k), I_w) with I_w = {T..T+W-1}.
    scores [rows,T] or [T].  Returns int64 [rows, k+W] (or [k+W])."""
    scores = np.asarray(scores)
    one = scores.ndim == 1
    rows = scores[None, :] if one else scores
    T = rows.shape[1]
    I_w = np.arange(T, T + W, dtype=np.int64)
    out = np.stack([np.concatenate([topk_indices(r, k), I_w]) for r in rows])
    return out[0] if one else out


def gather_kv(k: np.ndarray, v: np.ndarray, idx: np.ndarray):
    """Alg. 1 step 12: K[I], V[I].  k, v [Hk,N,d]; idx [Hk,n] (per KV head) or [n] (shared)."""
    idx = np.asarray(idx)
    Hk = k.shape[0]
    if idx.ndim == 1:
        return k[:, idx, :].copy(), v[:, idx, :].copy()
    return (np.stack([k[g, idx[g], :] for g in range(Hk)]),
            np.stack([v[g, idx[g], :] for g in range(Hk)]))


def propagate_tokens(hidden: np.ndarray, select_idx: np.ndarray) -> np.ndarray:
    """Sec. 4.2 "Prefilling": once the selection layer is determined, only the selected tokens'
    hidden states go on to the deeper layers.  hidden [N, D]; select_idx from Alg. 2."""
    return np.asarray(hidden)[np.asarray(select_idx)].copy()


# --------------------------------------------------------------------------- Alg. 2, statistic
@dataclass
class RankStat:
    numerator: int        # sum over the union of  n * sum_l R^2 - (sum_l R)^2  (exact integer)
    union_size: int       # |top(L)|
    n_rows: int           # number of stacked rank rows n
    var_top: float        # numerator / (n^2 * union_size)


def rank_variance(R: np.ndarray, k: int) -> RankStat:
    """Alg. 2 steps 6-9 and the Sec. 4.1 top(L) / var_top equations.
    R [n,T] stacked rank rows (each a permutation of 0..T-1).  The union is the set of tokens
    that are among the k smallest ranks of at least one row (ranks are a permutation, so that
    is  R[l,t] < k  for some l).  var_top is the mean over the union of the population variance
    of each token's n ranks; the numerator is kept as an exact integer and divided once."""
    R = np.asarray(R, dtype=np.int64)
    n, T = R.shape
    in_union = (R < k).any(axis=0)                        # steps 6-8: TopKIndices + Unique
    Ru = R[:, in_union]
    s1 = Ru.sum(axis=0)
    s2 = (Ru * Ru).sum(axis=0)
    num = int(sum(int(n) * int(b) - int(a) * int(a) for a, b in zip(s1.tolist(), s2.tolist())))
    m = int(in_union.sum())
    var_top = float(num) / float(n * n * m) if m > 0 else float("nan")
    return RankStat(num, m, n, var_top)


@dataclass
class SelectState:
    """Cross-layer state of Alg. 2: the rank cache (last L_obs rows) and init_var."""
    L_obs: int
    rows: list            # list of (layer_idx, rank vector), newest last
    init_var: Optional[float] = None

    @classmethod
    def new(cls, L_obs: int) -> "SelectState":
        return cls(L_obs=L_obs, rows=[], init_var=None)

    def push(self, layer_idx: int, rank: np.ndarray) -> None:
        self.rows.append((layer_idx, np.asarray(rank, dtype=np.int64)))
        if len(self.rows) > self.L_obs:
            self.rows.pop(0)


@dataclass
class Decision:
    evaluated: bool
    selected: bool
    var_top: float
    rel_var: float
    union_size: int
    n_rows: int
    select_idx: Optional[np.ndarray]


def select_tokens(state: SelectState, layer_idx: int, budget: int, W: int,
                  L_min: int, tau: float) -> Decision:
    """Alg. 2 (SelectTokens) on the rank cache held in ``state`` (whose newest row is this
    layer's).  Before L_min, or with fewer than two rows, nothing is evaluated.  The first
    evaluation sets init_var; relative variance = var_top / init_var; the layer is the
    selection layer iff that is strictly below tau (IEEE comparison: NaN/inf never select).
    On selection select_idx = ascending {t: current rank < k} followed by T..T+W-1 and the
    cache is cleared."""
    none = Decision(False, False, float("nan"), float("nan"), 0, len(state.rows), None)
    if layer_idx < L_min or len(state.rows) < 2:
        return none
    R = np.stack([r for _, r in state.rows])              # step 5: Stack
    T = R.shape[1]
    k = min(budget - W, T)                                # step 6
    st = rank_variance(R, k)                              # steps 7-9
    if state.init_var is None:
        state.init_var = st.var_top
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = float(np.float64(st.var_top) / np.float64(state.init_var))
    selected = bool(rel < tau)                            # step 10
    idx = None
    if selected:
        J_last = np.nonzero(R[-1] < k)[0].astype(np.int64)            # k smallest ranks of the last row
        idx = np.concatenate([J_last, np.arange(T, T + W, dtype=np.int64)])   # steps 11-12
        state.rows.clear()                                # step 13
    return Decision(True, selected, st.var_top, rel, st.union_size, st.n_rows, idx)


# --------------------------------------------------------------------------- Alg. 1, whole
def get_ranks(q_obs, k, v, W: int, S: int, budget: int, scale: Optional[float] = None):
    """Alg. 1 (GetRanks) for one layer.  Returns a dict with P, s, rank (RankDesc of s),
    I (per-KV-head Concat(TopK(P,k), I_w)) and the compressed K[I], V[I]."""
    P, s = score_layer(q_obs, k, W, S, scale)
    N = np.asarray(k).shape[1]
    kk = budget_k(budget, N, W)
    I = select_indices(P, kk, W)
    rank = rank_desc(s)
    Kc, Vc = gather_kv(np.asarray(k), np.asarray(v), I)
    return {"P": P, "s": s, "rank": rank, "I": I, "K": Kc, "V": Vc, "k": kk}
