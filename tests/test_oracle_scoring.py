"""Pins for the oracle's scoring steps (Alg. 1 steps 5-8, Sec. 4.1 PA / scores equations).

Each test checks the oracle against something that is not the oracle: a closed form, an
invariant, a textbook/library routine, or a pure-Python brute force on a tiny input.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle import asl_oracle as orc
from paper_2601_07667_amd import synth


def _tiny(seed=0, Hq=4, Hk=2, d=8, N=24, W=4):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((Hq, W, d)), rng.standard_normal((Hk, N, d)), rng.standard_normal((Hk, N, d))


# ----------------------------------------------------------------------------- brute force
def _brute_score_layer(q, k, W, S, scale):
    """Triple loops in pure Python, written from the equations: logits, mask, softmax,
    column sum over window rows, zero-padded mean over S neighbours, sum over the group."""
    Hq, _, d = q.shape
    Hk, N, _ = k.shape
    G = Hq // Hk
    T = N - W
    P = [[0.0] * T for _ in range(Hk)]
    for h in range(Hq):
        g = h // G
        U = [0.0] * T
        for i in range(W):
            row = []
            for j in range(N):
                if j >= T and (j - T) > i:
                    row.append(None)
                else:
                    row.append(scale * sum(q[h, i, c] * k[g, j, c] for c in range(d)))
            mx = max(x for x in row if x is not None)
            ex = [0.0 if x is None else math.exp(x - mx) for x in row]
            Z = sum(ex)
            for j in range(T):
                U[j] += ex[j] / Z
        for j in range(T):
            acc = 0.0
            for dlt in range(-(S // 2), S // 2 + 1):
                if 0 <= j + dlt < T:
                    acc += U[j + dlt]
            P[g][j] += acc / S
    s = [sum(P[g][j] for g in range(Hk)) for j in range(T)]
    return np.array(P), np.array(s)


@pytest.mark.parametrize("S", [1, 3, 7])
def test_score_layer_matches_bruteforce(S):
    q, k, _ = _tiny(seed=S)
    W = q.shape[1]
    scale = 1.0 / math.sqrt(q.shape[2])
    P, s = orc.score_layer(q, k, W, S, scale)
    Pb, sb = _brute_score_layer(q, k, W, S, scale)
    np.testing.assert_allclose(P, Pb, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(s, sb, rtol=1e-12, atol=1e-15)


# ----------------------------------------------------------------------------- softmax invariants
def test_rows_sum_to_one_and_mask_structure():
    q, k, _ = _tiny(seed=3, N=40, W=6)
    W, N = 6, 40
    T = N - W
    for h in range(q.shape[0]):
        A = orc.window_attention(q[h], k[h // 2], 0.3)
        np.testing.assert_allclose(A.sum(axis=1), 1.0, rtol=0, atol=1e-12)
        blk = A[:, T:]
        for i in range(W):
            assert np.all(blk[i, i + 1:] == 0.0)          # masked entries exactly zero
            assert np.count_nonzero(blk[i]) == i + 1      # row i sees i+1 window keys
        assert np.all(A[:, :T] > 0)                       # past keys never masked
        # total mass: past column sums + window column sums = W
        assert abs(orc.past_column_sum(A, W).sum() + blk.sum() - W) < 1e-12


def test_unmasked_part_is_library_softmax():
    """Row W-1 sees every key, so it must equal a library softmax of q.k/sqrt(d)."""
    q, k, _ = _tiny(seed=5, N=50, W=5, d=16)
    scale = 1.0 / 4.0
    A = orc.window_attention(q[1], k[0], scale)
    ref = scipy.special.softmax(np.einsum("c,jc->j", q[1, -1], k[0]) * scale)
    np.testing.assert_allclose(A[-1], ref, rtol=1e-12, atol=0)
    # row 0 sees past keys and window key 0 only
    l0 = np.einsum("c,jc->j", q[1, 0], k[0, :46]) * scale
    np.testing.assert_allclose(A[0, :46], scipy.special.softmax(l0), rtol=1e-12, atol=0)


def test_zero_queries_closed_form():
    """Q_obs = 0: window row i is uniform over its T+i+1 visible keys, so
    U[h,j] = sum_i 1/(T+i+1); with S=1, P = G*U and s = Hq*U."""
    Hq, Hk, d, N, W = 6, 2, 8, 37, 5
    T = N - W
    rng = np.random.default_rng(1)
    k = rng.standard_normal((Hk, N, d))
    q = np.zeros((Hq, W, d))
    P, s = orc.score_layer(q, k, W, 1, 0.5)
    u = sum(1.0 / (T + i + 1) for i in range(W))
    np.testing.assert_allclose(P, (Hq // Hk) * u, rtol=1e-13)
    np.testing.assert_allclose(s, Hq * u, rtol=1e-13)


def test_operand_orientation_and_scale():
    """One dominant key: a query aligned with key j0 (and no other) puts nearly all mass on
    j0 -- fails if Q/K were transposed, the scale dropped, or the sign flipped."""
    d, N, W = 8, 20, 2
    k = np.zeros((1, N, d))
    for j in range(N):
        k[0, j, j % d] = 1.0 if j != 7 else 0.0
    k[0, 7, :] = 0.0
    k[0, 7, 3] = 50.0
    q = np.zeros((1, W, d))
    q[0, :, 3] = 1.0
    A = orc.window_attention(q[0], k[0], 1.0)
    assert np.all(A[:, 7] > 0.999)
    A_small = orc.window_attention(q[0], k[0], 0.01)      # scale matters
    assert np.all(A_small[:, 7] < 0.2)


def test_lse_is_log_of_row_normaliser():
    q, k, _ = _tiny(seed=9, N=30, W=4)
    scale = 0.4
    lse = orc.row_lse(q, k, 4, scale)
    for h in range(q.shape[0]):
        l = orc.window_logits(q[h], k[h // 2], scale)
        A = orc.window_attention(q[h], k[h // 2], scale)
        with np.errstate(divide="ignore"):
            np.testing.assert_allclose(np.exp(l - lse[h][:, None]), A, rtol=1e-12, atol=0)


# ----------------------------------------------------------------------------- pooling
def test_pool_identity_constant_impulse_convolve():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(53)
    np.testing.assert_array_equal(orc.avg_pool1d(x, 1), x)
    c = 3.5 * np.ones(20)
    p = orc.avg_pool1d(c, 7)
    np.testing.assert_allclose(p[3:-3], 3.5, rtol=1e-15)
    np.testing.assert_allclose(p[:3], [3.5 * 4 / 7, 3.5 * 5 / 7, 3.5 * 6 / 7], rtol=1e-15)
    np.testing.assert_allclose(p[-3:][::-1], [3.5 * 4 / 7, 3.5 * 5 / 7, 3.5 * 6 / 7], rtol=1e-15)
    imp = np.zeros(31)
    imp[10] = 1.0
    box = np.zeros(31)
    box[7:14] = 1.0 / 7
    np.testing.assert_allclose(orc.avg_pool1d(imp, 7), box, rtol=1e-15, atol=0)
    for S in (3, 5, 7, 9):
        np.testing.assert_allclose(orc.avg_pool1d(x, S), np.convolve(x, np.ones(S) / S, "same"),
                                   rtol=1e-12, atol=1e-15)
    with pytest.raises(ValueError):
        orc.avg_pool1d(x, 4)


def test_pool_shorter_than_kernel():
    x = np.array([1.0, 2.0, 4.0])
    np.testing.assert_allclose(orc.avg_pool1d(x, 7), np.full(3, 7.0 / 7), rtol=1e-15)
    np.testing.assert_allclose(orc.avg_pool1d(x, 3), [3 / 3, 7 / 3, 6 / 3], rtol=1e-15)


def test_pool_and_sums_commute():
    """Pool-then-group-sum (Alg. 1 order) equals group-sum-then-pool (all linear)."""
    q, k, _ = _tiny(seed=11, N=64, W=8)
    W, S, scale = 8, 7, 0.35
    P, s = orc.score_layer(q, k, W, S, scale)
    G = q.shape[0] // k.shape[0]
    for g in range(k.shape[0]):
        Usum = sum(orc.past_column_sum(orc.window_attention(q[h], k[g], scale), W)
                   for h in range(g * G, (g + 1) * G))
        np.testing.assert_allclose(orc.avg_pool1d(Usum, S), P[g], rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(P.sum(axis=0), s, rtol=1e-15)


# ----------------------------------------------------------------------------- permutations
def test_past_key_permutation_equivariance():
    q, k, _ = _tiny(seed=13, N=48, W=6)
    W, N = 6, 48
    T = N - W
    rng = np.random.default_rng(0)
    pi = rng.permutation(T)
    kp = k.copy()
    kp[:, :T] = k[:, pi]                                   # new position j holds old key pi[j]
    P, s = orc.score_layer(q, k, W, 1, 0.3)
    Pp, sp = orc.score_layer(q, kp, W, 1, 0.3)
    np.testing.assert_allclose(Pp, P[:, pi], rtol=1e-12)
    np.testing.assert_allclose(sp, s[pi], rtol=1e-12)
    kk = 10
    top = set(orc.topk_indices(s, kk).tolist())
    topp = set(pi[orc.topk_indices(sp, kk)].tolist())      # map back to old positions
    assert top == topp


def test_head_permutations():
    q, k, _ = _tiny(seed=17, Hq=8, Hk=2, N=40, W=5)
    W, S = 5, 7
    P, s = orc.score_layer(q, k, W, S, 0.3)
    q2 = q.copy()
    q2[0:4] = q[[2, 0, 3, 1]]                              # permute heads inside group 0
    P2, s2 = orc.score_layer(q2, k, W, S, 0.3)
    np.testing.assert_allclose(P2, P, rtol=1e-12)
    np.testing.assert_allclose(s2, s, rtol=1e-12)
    q3 = np.concatenate([q[4:], q[:4]])                    # swap the two groups with their KV heads
    k3 = k[::-1].copy()
    P3, s3 = orc.score_layer(q3, k3, W, S, 0.3)
    np.testing.assert_allclose(P3, P[::-1], rtol=1e-12)
    np.testing.assert_allclose(s3, s, rtol=1e-12)


def test_window_row_permutation_is_not_an_invariance():
    """The causal block ties window row i to key T+i: reversing the rows changes the result."""
    q, k, _ = _tiny(seed=19, N=30, W=6)
    P, _ = orc.score_layer(q, k, 6, 1, 0.5)
    P2, _ = orc.score_layer(q[:, ::-1].copy(), k, 6, 1, 0.5)
    assert np.max(np.abs(P - P2) / np.abs(P)) > 1e-3


# ----------------------------------------------------------------------------- default scale, tiny config
def test_default_scale_and_config1_mass():
    L = synth.config_layer(1)
    sh = L.shape
    P, s = orc.score_layer(L.q_obs, L.k, sh.W, sh.S)       # scale defaults to 1/sqrt(d)
    P2, _ = orc.score_layer(L.q_obs, L.k, sh.W, sh.S, 1.0 / math.sqrt(sh.d))
    np.testing.assert_array_equal(P, P2)
    assert P.shape == (sh.Hk, sh.T) and s.shape == (sh.T,)
    # pooling with zero padding loses only edge mass; total past mass < Hq*W
    assert 0 < s.sum() < sh.Hq * sh.W
