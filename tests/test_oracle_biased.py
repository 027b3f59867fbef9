"""Pins for the oracle's score-biased selection (the variant of paper Sec. 3.3.1 in which the batch score is
added to the router logits).  The paper gives it in one sentence and no numbers, so it is pinned by what that
sentence and the surrounding text fix: gamma = 0 is the unchanged top-k, the top-ranked expert always stays, only
experts the batch already invokes are used, the bias redone in exact rational arithmetic, a limit case with a
closed form (gamma so large that the bias decides), and an exhaustive search over subsets on tiny batches.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as wl


def _topk(z, k):
    T, N = z.shape
    out = np.zeros((T, k), np.int32)
    for t in range(T):
        out[t] = np.lexsort((np.arange(N), -z[t].astype(np.float64)))[:k]
    return out


CASES = [(16, 8, 2), (8, 8, 2), (32, 60, 4), (64, 64, 6), (40, 128, 8), (5, 6, 3), (2, 4, 2), (33, 17, 5), (7, 9, 1)]
PRESETS = [(2.0, 2), (4.0, 1), (1.0, 3), (0.5, 6)]


@pytest.mark.parametrize("T,N,k", CASES)
@pytest.mark.parametrize("alpha,beta", PRESETS)
def test_gamma_zero_and_bypass_leave_the_selection_alone(T, N, k, alpha, beta):
    z = wl.make_logits(T, N, seed=T + N)
    idx = _topk(z, k)
    ref = oracle.topk(z, k)
    for gamma, enable in ((0.0, 1), (3.0, 0)):
        a = oracle.affinity_bin_biased(z, idx, alpha, beta, gamma, enable)
        assert np.array_equal(a["new_idx"], idx)
        np.testing.assert_allclose(a["new_gate"], ref["gate"], rtol=1e-12)
        assert np.array_equal(a["cnt_after"], a["cnt_before"]) and a["num_active"][0] == a["num_active"][1]
    one = oracle.affinity_bin_biased(z[:1], idx[:1], alpha, beta, 5.0, 1)      # a single token is bypassed
    assert np.array_equal(one["new_idx"], idx[:1])


@pytest.mark.parametrize("T,N,k", CASES)
@pytest.mark.parametrize("gamma", [0.25, 1.0, 4.0])
def test_invariants(T, N, k, gamma):
    z = wl.make_logits(T, N, seed=3 * T + N, tail_frac=0.1)
    idx = _topk(z, k)
    a = oracle.affinity_bin_biased(z, idx, 2.0, 2, gamma)
    b = oracle.affinity_bin(z, idx, 2.0, 2)                      # histogram and counts are those of the main method
    assert np.array_equal(a["bin_hist"], b["bin_hist"]) and np.array_equal(a["cnt_before"], b["cnt_before"])
    U = set(np.flatnonzero(a["cnt_before"]).tolist())
    for t in range(T):
        sel = a["new_idx"][t].tolist()
        assert sel[0] == idx[t, 0]                               # the top-ranked expert always stays
        assert len(set(sel)) == k and set(sel) <= U              # k distinct experts the batch already invokes
    np.testing.assert_allclose(a["new_gate"].sum(1), 1.0, rtol=1e-12)
    assert a["num_active"][1] <= a["num_active"][0] == len(U)
    assert np.array_equal(np.bincount(a["new_idx"].ravel(), minlength=N), a["cnt_after"])
    # gates are the softmax over the ORIGINAL logits of the selection
    zs = np.take_along_axis(z.astype(np.float64), a["new_idx"], axis=1)
    g = np.exp(zs - zs.max(1, keepdims=True))
    np.testing.assert_allclose(a["new_gate"], g / g.sum(1, keepdims=True), rtol=1e-12)


@pytest.mark.parametrize("T,N,k,beta", [(16, 8, 2, 2), (33, 17, 5, 3), (64, 64, 6, 1), (12, 20, 4, 6)])
def test_bias_in_exact_rational_arithmetic(T, N, k, beta):
    z = wl.make_logits(T, N, seed=T * N)
    idx = _topk(z, k)
    gamma = 0.75
    a = oracle.affinity_bin_biased(z, idx, 1.5, beta, gamma)
    for e in range(N):
        score = sum(int(a["bin_hist"][e, j]) * T ** (beta - 1 - j) for j in range(beta))      # Python big integers
        s = np.float32(float(Fraction(score, T ** beta)))          # correctly rounded fp64 quotient, then fp32
        assert a["bias"][e] == np.float32(gamma) * s
        assert 0.0 <= a["bias"][e] <= gamma


@pytest.mark.parametrize("T,N,k", [(16, 8, 3), (33, 17, 5), (20, 60, 4)])
def test_large_gamma_limit_takes_the_best_scored_experts(T, N, k):
    """With gamma far above the logit range the bias decides: the other k-1 slots are the invoked experts of
    largest score (equal fp32 biases fall back to the larger logit, then the lower index)."""
    z = wl.make_logits(T, N, seed=7 * T + N)
    idx = _topk(z, k)
    a = oracle.affinity_bin_biased(z, idx, 2.0, 2, 1.0e6)
    U = np.flatnonzero(a["cnt_before"])
    for t in range(T):
        cand = [e for e in U if e != idx[t, 0]]
        key = sorted(cand, key=lambda e: (-np.float32(z[t, e] + a["bias"][e]), e))
        assert a["new_idx"][t, 1:].tolist() == key[:k - 1]
        got = sorted(a["bias"][a["new_idx"][t, 1:]].tolist(), reverse=True)
        best = sorted(a["bias"][cand].tolist(), reverse=True)[:k - 1]
        assert got == pytest.approx(best, abs=2.0 * np.spacing(np.float32(1.0e6)))        # the k-1 largest biases


def test_exhaustive_subsets_on_tiny_batches():
    """The k-1 experts chosen maximise the sum of biased logits over all (k-1)-subsets of the allowed experts."""
    rng = np.random.default_rng(11)
    for trial in range(200):
        T, N, k = int(rng.integers(2, 6)), int(rng.integers(3, 8)), int(rng.integers(2, 4))
        if k > N:
            continue
        z = rng.standard_normal((T, N)).astype(np.float32)
        idx = _topk(z, k)
        gamma = float(rng.choice([0.3, 1.0, 2.5]))
        a = oracle.affinity_bin_biased(z, idx, 2.0, 2, gamma)
        U = np.flatnonzero(a["cnt_before"]).tolist()
        for t in range(T):
            zb = (z[t] + a["bias"]).astype(np.float32)
            cand = [e for e in U if e != idx[t, 0]]
            best = max(itertools.combinations(cand, k - 1), key=lambda c: sum(float(zb[e]) for e in c))
            chosen = a["new_idx"][t, 1:].tolist()
            assert sum(float(zb[e]) for e in chosen) == pytest.approx(sum(float(zb[e]) for e in best), abs=1e-6)
            assert all(zb[chosen[i]] >= zb[chosen[i + 1]] for i in range(k - 2))        # descending biased logit


def test_bias_pulls_low_affinity_slots_onto_popular_experts():
    """Sec. 3.3.1: experts preferred by many high-conviction tokens gain, so the batch touches fewer experts."""
    z = wl.make_logits(64, 64, seed=5, zipf_s=1.0)
    idx = _topk(z, 6)
    before = oracle.affinity_bin_biased(z, idx, 2.0, 2, 0.0)["num_active"][1]
    mid = oracle.affinity_bin_biased(z, idx, 2.0, 2, 1.0)["num_active"][1]
    big = oracle.affinity_bin_biased(z, idx, 2.0, 2, 8.0)["num_active"][1]
    assert big <= mid <= before and big < before


def test_argument_errors():
    z = wl.make_logits(4, 6, seed=1)
    idx = _topk(z, 2)
    with pytest.raises(oracle.OracleError):
        oracle.affinity_bin_biased(z, idx, 2.0, 2, -1.0)
    with pytest.raises(oracle.OracleError):
        oracle.affinity_bin_biased(z, idx, 2.0, 0, 1.0)
    bad = idx.copy()
    bad[0, 1] = bad[0, 0]
    with pytest.raises(oracle.OracleError):
        oracle.affinity_bin_biased(z, bad, 2.0, 2, 1.0)
