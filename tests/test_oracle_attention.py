"""Pins of the oracle's attention and consistency score (CPU only).

Each test checks the oracle against something other than itself: explicit
scalar loops, PyTorch's float64 attention routine, or a closed form.
"""
import math

import numpy as np
import pytest
import torch

from oracle import pyr_oracle as orc


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def brute_probs(q, k, scale):
    """A[h][i][j] by scalar loops: softmax over j <= i of scale * <q_i, k_j>, kv head = h // g."""
    S, Hq, d = q.shape
    g = Hq // k.shape[1]
    A = [[[0.0] * S for _ in range(S)] for _ in range(Hq)]
    for h in range(Hq):
        for i in range(S):
            logits = []
            for j in range(i + 1):
                acc = 0.0
                for c in range(d):
                    acc += q[i, h, c] * k[j, h // g, c]
                logits.append(scale * acc)
            mx = max(logits)
            ex = [math.exp(x - mx) for x in logits]
            den = sum(ex)
            for j in range(i + 1):
                A[h][i][j] = ex[j] / den
    return A


@pytest.mark.parametrize("S,Hq,Hkv,d", [(1, 1, 1, 4), (7, 2, 2, 4), (13, 4, 2, 8), (16, 6, 1, 5)])
def test_attention_matches_scalar_loops(S, Hq, Hkv, d):
    q, k, v = _rand((S, Hq, d), 1), _rand((S, Hkv, d), 2), _rand((S, Hkv, d), 3)
    scale = 1.0 / math.sqrt(d)
    A = brute_probs(q, k, scale)
    g = Hq // Hkv
    out, P = orc.attention_rows(q, k, v, np.arange(S))
    for h in range(Hq):
        for i in range(S):
            for j in range(S):
                assert abs(P[h, i, j] - A[h][i][j]) < 1e-14
            for c in range(d):
                ref = sum(A[h][i][j] * v[j, h // g, c] for j in range(i + 1))
                assert abs(out[i, h, c] - ref) < 1e-13


def test_attention_row_subset_equals_full():
    S, Hq, Hkv, d = 33, 4, 2, 8
    q, k, v = _rand((S, Hq, d), 4), _rand((S, Hkv, d), 5), _rand((S, Hkv, d), 6)
    full = orc.causal_attention(q, k, v)
    rows = np.array([0, 5, 31, 32])
    sub, _ = orc.attention_rows(q, k, v, rows)
    np.testing.assert_allclose(sub, full[rows], rtol=0, atol=1e-14)


@pytest.mark.parametrize("Hq,Hkv,d,S", [(4, 4, 16, 50), (8, 2, 32, 77)])
def test_attention_matches_library_routine(Hq, Hkv, d, S):
    """PyTorch's scaled_dot_product_attention in float64 with is_causal=True is
    the textbook operation; grouped heads are expanded by explicit repetition."""
    q, k, v = _rand((S, Hq, d), 7), _rand((S, Hkv, d), 8), _rand((S, Hkv, d), 9)
    g = Hq // Hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, g, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, g, axis=1)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    out = orc.causal_attention(q, k, v)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)


def test_custom_scale_is_used():
    S, H, d = 9, 2, 4
    q, k, v = _rand((S, H, d), 10), _rand((S, H, d), 11), _rand((S, H, d), 12)
    A = brute_probs(q, k, 0.37)
    _, P = orc.attention_rows(q, k, v, np.arange(S), scale=0.37)
    assert abs(P[1, 8, 3] - A[1][8][3]) < 1e-14
    # a non-positive scale selects the default 1/sqrt(d)
    _, P0 = orc.attention_rows(q, k, v, np.arange(S), scale=0.0)
    _, P1 = orc.attention_rows(q, k, v, np.arange(S), scale=0.5)
    np.testing.assert_allclose(P0, P1, atol=1e-15)


def test_rows_sum_to_one_and_first_row_copies_v0():
    S, Hq, Hkv, d = 40, 4, 2, 8
    q, k, v = _rand((S, Hq, d), 13), _rand((S, Hkv, d), 14), _rand((S, Hkv, d), 15)
    out, P = orc.attention_rows(q, k, v, np.arange(S))
    np.testing.assert_allclose(P.sum(axis=2), 1.0, atol=1e-14)
    assert np.all(P >= 0.0)
    assert np.all(np.triu(P[0], 1) == 0.0)          # nothing above the diagonal
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], v[0, h // 2], atol=1e-15)


def test_zero_keys_give_prefix_means_and_harmonic_scores():
    """K = 0 makes every causal row uniform: out[i] = mean(v[0..i]) and
    score[t] = 1/L * sum_{i >= max(t, S-L)} 1/(i+1)."""
    S, H, d, L = 37, 3, 4, 6
    q, v = _rand((S, H, d), 16), _rand((S, H, d), 17)
    k = np.zeros((S, H, d))
    out = orc.causal_attention(q, k, v)
    pref = np.cumsum(v, axis=0) / np.arange(1, S + 1)[:, None, None]
    np.testing.assert_allclose(out, pref, atol=1e-13)
    score = orc.consistency_score(q, k, L)
    ref = np.array([sum(1.0 / (i + 1) for i in range(max(t, S - L), S)) / L for t in range(S)])
    np.testing.assert_allclose(score, ref, atol=1e-15)


def test_constant_values_give_constant_output():
    S, H, d = 21, 2, 4
    q, k = _rand((S, H, d), 18), _rand((S, H, d), 19)
    v = np.tile(np.array([1.5, -2.0, 0.25, 3.0]), (S, H, 1))
    out = orc.causal_attention(q, k, v)
    np.testing.assert_allclose(out, v, atol=1e-14)


@pytest.mark.parametrize("S,L", [(12, 4), (12, 12), (5, 9), (1, 3)])
def test_score_matches_scalar_loops_and_sums_to_one(S, L):
    Hq, Hkv, d = 4, 2, 4
    q, k = _rand((S, Hq, d), 20), _rand((S, Hkv, d), 21)
    A = brute_probs(q, k, 1.0 / math.sqrt(d))
    Le = min(L, S)
    ref = [sum(A[h][i][t] for h in range(Hq) for i in range(S - Le, S)) / (Hq * Le) for t in range(S)]
    score = orc.consistency_score(q, k, L)
    np.testing.assert_allclose(score, ref, atol=1e-14)
    assert abs(score.sum() - 1.0) < 1e-13
    assert np.all(score >= 0)


def test_score_ignores_rows_before_the_window():
    """Changing a query outside the last L rows must not move the score; changing one inside must."""
    S, H, d, L = 20, 2, 4, 5
    q, k = _rand((S, H, d), 22), _rand((S, H, d), 23)
    base = orc.consistency_score(q, k, L)
    q2 = q.copy(); q2[S - L - 1] += 3.0
    np.testing.assert_array_equal(orc.consistency_score(q2, k, L), base)
    q3 = q.copy(); q3[S - L] += 3.0
    assert np.abs(orc.consistency_score(q3, k, L) - base).max() > 1e-3


# ---- weighted recent rows (Section 4.1, prefill phase: larger weights for more recent rows)

@pytest.mark.parametrize("S,L", [(12, 4), (9, 9), (5, 9), (1, 3)])
def test_weighted_score_matches_scalar_loops(S, L):
    Hq, Hkv, d = 4, 2, 4
    q, k = _rand((S, Hq, d), 30), _rand((S, Hkv, d), 31)
    rw = np.random.default_rng(32).uniform(0.1, 2.0, L)
    A = brute_probs(q, k, 1.0 / math.sqrt(d))
    Le = min(L, S)
    used = [rw[L - Le + r] for r in range(Le)]          # the most recent row takes the last weight
    ref = [sum(used[r] * A[h][S - Le + r][t] for h in range(Hq) for r in range(Le)) / (Hq * sum(used)) for t in range(S)]
    score = orc.consistency_score(q, k, L, row_weights=rw)
    np.testing.assert_allclose(score, ref, atol=1e-14)
    assert abs(score.sum() - 1.0) < 1e-13


def test_weighted_score_special_cases():
    S, H, d, L = 24, 3, 8, 6
    q, k = _rand((S, H, d), 33), _rand((S, H, d), 34)
    uniform = orc.consistency_score(q, k, L)
    # equal weights of any size are the plain average
    np.testing.assert_allclose(orc.consistency_score(q, k, L, row_weights=np.full(L, 3.7)), uniform, atol=1e-15)
    # all weight on one row: the head-mean of that row of the softmax
    for r in (0, 2, L - 1):
        onehot = np.zeros(L); onehot[r] = 5.0
        _, P = orc.attention_rows(q, k, k, [S - L + r])
        np.testing.assert_allclose(orc.consistency_score(q, k, L, row_weights=onehot), P[:, 0, :].mean(axis=0), atol=1e-15)
    # un-normalised sums are additive in the weights
    a, b = np.array([1.0, 0, 2, 0, 0.5, 0]), np.array([0, 3.0, 0, 1, 0, 4])
    sa, sb, sab = (orc.consistency_score(q, k, L, row_weights=x) for x in (a, b, a + b))
    np.testing.assert_allclose(sab * (a + b).sum(), sa * a.sum() + sb * b.sum(), atol=1e-14)
    # more weight on the last row moves the score towards that row's distribution
    _, P = orc.attention_rows(q, k, k, [S - 1])
    last = P[:, 0, :].mean(axis=0)
    ramp = orc.consistency_score(q, k, L, row_weights=np.arange(1, L + 1))
    assert np.abs(ramp - last).sum() < np.abs(uniform - last).sum()


def test_weighted_score_rejects_bad_weights():
    q, k = _rand((8, 2, 4), 35), _rand((8, 2, 4), 36)
    for bad in (np.ones(3), -np.ones(4), np.array([1, np.nan, 1, 1]), np.zeros(4)):
        with pytest.raises(ValueError):
            orc.consistency_score(q, k, 4, row_weights=bad)
    # a short sequence only needs a positive weight among the rows it uses
    orc.consistency_score(q[:2], k[:2], 4, row_weights=np.array([0, 0, 0, 1.0]))
    with pytest.raises(ValueError):
        orc.consistency_score(q[:2], k[:2], 4, row_weights=np.array([1.0, 1, 0, 0]))
