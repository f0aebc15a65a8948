"""Pins for the selection half of the CPU checker (votes, pool, top-k).

The paper states only the goal (keep s < n tokens chosen at prefill, Section 3
"KV Pruning") and that the last 32 tokens are retained (Appendix B); the
scoring rule is this build's reading.  These tests tie each step to something
other than the checker: library routines (scipy softmax, scipy maximum
filter, numpy lexsort), special cases with a textbook answer, brute force on
tiny inputs and invariants.
"""
import itertools

import numpy as np
import pytest
from scipy.ndimage import maximum_filter1d
from scipy.special import softmax

from paper_2412_12706_amd import synth


def _f64(a):
    return a.astype(np.float64)


def votes_by_library(q_obs, k, sm_scale):
    """Same quantity from dense masked matrices and scipy's softmax."""
    B, Hq, W, D = q_obs.shape
    _, Hkv, L, _ = k.shape
    P, Gq = L - W, Hq // Hkv
    out = np.zeros((B, Hkv, P))
    mask = np.full((W, L), -np.inf)
    for i in range(W):
        mask[i, : P + i + 1] = 0.0
    for b in range(B):
        for h in range(Hq):
            logits = sm_scale * _f64(q_obs[b, h]) @ _f64(k[b, h // Gq]).T + mask
            out[b, h // Gq] += softmax(logits, axis=1)[:, :P].sum(axis=0)
    return out


@pytest.mark.parametrize("shape", [(1, 4, 2, 40, 8, 64), (2, 2, 2, 33, 5, 64), (1, 8, 2, 70, 1, 128)])
def test_votes_match_library_softmax(orc, shape):
    B, Hq, Hkv, L, W, D = shape
    q_obs, k, _ = synth.prompt_host(B, Hq, Hkv, L, W, D, config=90)
    got = orc.window_votes(q_obs, k, 0.17)
    ref = votes_by_library(q_obs, k, 0.17)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-15)


def test_vote_mass_bounded_by_rows(orc):
    # each window row distributes probability 1 over prefix + visible window keys
    q_obs, k, _ = synth.prompt_host(1, 4, 2, 64, 8, 64, config=91)
    vote = orc.window_votes(q_obs, k, 0.1)
    assert np.all(vote >= 0)
    assert np.all(vote.sum(-1) < 2 * 8)          # Gq*W, strict: window keys take mass
    # push the window keys far away from every query: they lose all mass
    k2 = k.copy()
    k2[:, :, -8:, :] = 0
    q2 = q_obs.copy()
    vote2 = orc.window_votes(q2, k2 * np.float16(1.0), 0.1)
    assert np.all(vote2.sum(-1) <= 16 + 1e-9)


def test_head_permutation_inside_group_leaves_votes(orc):
    q_obs, k, _ = synth.prompt_host(1, 8, 2, 48, 4, 64, config=92)
    perm = [2, 0, 3, 1, 5, 4, 7, 6]               # permutes within each group of 4
    a = orc.window_votes(q_obs, k, 0.2)
    b = orc.window_votes(q_obs[:, perm], k, 0.2)
    np.testing.assert_allclose(a, b, rtol=1e-13)


@pytest.mark.parametrize("pool", [1, 3, 7, 9])
def test_pool_matches_scipy_maximum_filter(orc, pool):
    rng = np.random.default_rng(pool)
    x = rng.random((5, 37))
    got = orc.max_pool(x, pool)
    ref = maximum_filter1d(x, size=pool, axis=1, mode="constant", cval=-np.inf)
    assert np.array_equal(got, ref)


def test_pool_rejects_even_kernel(orc):
    with pytest.raises(ValueError):
        orc.max_pool(np.zeros((1, 8)), 4)


def test_topk_matches_lexsort_with_ties(orc):
    rng = np.random.default_rng(3)
    for trial in range(50):
        P = int(rng.integers(1, 60))
        x = rng.integers(0, 6, P).astype(np.float64)      # many exact ties
        k = int(rng.integers(0, P + 1))
        order = np.lexsort((np.arange(P), -x))            # score desc, then index asc
        ref = np.sort(order[:k]).astype(np.int32)
        assert np.array_equal(orc.topk(x, k), ref)


def test_topk_brute_force_subsets(orc):
    # the chosen set maximises the score sum and, among maximisers, is the
    # lexicographically smallest index set at the boundary score
    rng = np.random.default_rng(4)
    for trial in range(20):
        P, k = 9, int(rng.integers(1, 9))
        x = rng.integers(0, 4, P).astype(np.float64)
        got = orc.topk(x, k)
        best = max(itertools.combinations(range(P), k), key=lambda s: (sum(x[list(s)]), [-i for i in s]))
        assert sum(x[got]) == sum(x[list(best)])
        thr = min(x[got])
        outside = [j for j in range(P) if j not in set(got)]
        assert all(x[j] <= thr for j in outside)
        tied_out = [j for j in outside if x[j] == thr]
        tied_in = [j for j in got if x[j] == thr]
        assert not tied_out or max(tied_in) < min(tied_out)


def test_budget_covering_prefix_is_identity(orc):
    B, Hq, Hkv, L, W, D = 1, 4, 2, 96, 32, 64
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=93)
    for budget in (64, 100, 10**6):
        _, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=budget, bits=4, G=32, sm_scale=0.1)
        assert idx.shape == (B, Hkv, 64)
        assert np.array_equal(idx, np.broadcast_to(np.arange(64, dtype=np.int32), idx.shape))


def test_single_row_no_pool_is_topk_of_raw_logits(orc):
    # W=1, pool=1, Gq=1: softmax is monotone, so the survivors are the keys
    # with the largest q.k, computed here with a plain matmul and a sort
    B, H, L, W, D, kk = 1, 2, 129, 1, 64, 32
    q_obs, k, v = synth.prompt_host(B, H, H, L, W, D, config=94)
    _, idx, _ = orc.compress(q_obs, k, v, window=W, pool=1, budget=kk, bits=4, G=32, sm_scale=0.09)
    for h in range(H):
        logits = _f64(k[0, h, : L - 1]) @ _f64(q_obs[0, h, 0])
        ref = np.sort(np.argsort(-logits, kind="stable")[:kk])
        assert np.array_equal(idx[0, h], ref)


def test_planted_needle_and_its_pool_neighbours_survive(orc):
    B, Hq, Hkv, L, W, D = 1, 4, 1, 160, 32, 64
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=95)
    u = np.where(np.arange(D) % 2 == 0, 1.0, -1.0)             # a direction every window query leans to
    q_obs = (_f64(q_obs) + u).astype(np.float16)
    k[0, 0, 77] = (1.5 * u).astype(np.float16)                 # the one prefix key aligned with it
    _, idx, pooled = orc.compress(q_obs, k, v, window=W, pool=7, budget=32, bits=4, G=32, sm_scale=1 / np.sqrt(D))
    assert pooled[0, 0].argmax() in range(74, 81)
    assert set(range(74, 81)) <= set(idx[0, 0].tolist())


def test_indices_ascending_unique_in_prefix_and_scale_invariant(orc):
    B, Hq, Hkv, L, W, D = 2, 4, 2, 200, 8, 64
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=96)
    _, idx, pooled = orc.compress(q_obs, k, v, window=W, pool=7, budget=64, bits=4, G=32, sm_scale=0.1)
    assert np.all(np.diff(idx, axis=-1) > 0) and idx.min() >= 0 and idx.max() < L - W
    for b in range(B):
        for g in range(Hkv):
            assert np.array_equal(orc.topk(pooled[b, g] * 3.5, 64), idx[b, g])   # positive scaling keeps order
            # every survivor scores at least as high as every discarded token
            keep = np.zeros(L - W, bool)
            keep[idx[b, g]] = True
            assert pooled[b, g][keep].min() >= pooled[b, g][~keep].max()


def test_pool_happens_after_group_sum_not_before(orc):
    # the reading fixed for this build: sum votes over the group's heads and
    # window rows, then pool once.  Pooling per head first gives other scores.
    q_obs, k, v = synth.prompt_host(1, 4, 1, 120, 8, 64, config=97)
    _, _, pooled = orc.compress(q_obs, k, v, window=8, pool=7, budget=32, bits=4, G=32, sm_scale=0.3)
    lib_votes = votes_by_library(q_obs, k, 0.3)
    ref = maximum_filter1d(lib_votes, size=7, axis=2, mode="constant", cval=-np.inf)
    np.testing.assert_allclose(pooled, ref, rtol=1e-12)
