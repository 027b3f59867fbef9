"""Pins of the oracle's sigmoid-gated router (paper Sec. 3.2.1, last case: routers that do not use softmax).

The paper fixes one thing for such routers: the bins come from differences of the pre-sigmoid scores, i.e. of the
logits, so everything up to the remap is the softmax path unchanged.  The gate formula (selected sigmoid scores over
their sum) is this build's reading; it is pinned here against closed forms and a library logistic function, and
against the properties that tell it from a softmax over the selection.
"""
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import expit

import oracle
import workloads as wl


def test_closed_forms():
    # sigmoid(ln 3) = 3/4, sigmoid(-ln 3) = 1/4, sigmoid(0) = 1/2
    l3 = np.float32(np.log(3.0))
    z = np.array([[l3, -l3, 0.0, -50.0]], np.float32)
    r = oracle.topk_sigmoid(z, 3)
    assert r["idx"].tolist() == [[0, 2, 1]]
    s = [expit(float(l3)), 0.5, expit(float(-l3))]                # the fp32 logit is not exactly ln 3
    np.testing.assert_allclose(r["gate"][0], np.array(s) / sum(s), rtol=1e-15)
    np.testing.assert_allclose(r["gate"][0], [float(Fraction(3, 6)), float(Fraction(2, 6)), float(Fraction(1, 6))], rtol=1e-7)
    np.testing.assert_allclose(r["ssum"][0], 1.5, rtol=1e-7)
    # all logits zero: every score 1/2, gates 1/k, picks by index
    r = oracle.topk_sigmoid(np.zeros((2, 6), np.float32), 4)
    assert r["idx"].tolist() == [[0, 1, 2, 3]] * 2
    np.testing.assert_array_equal(r["gate"], np.full((2, 4), 0.25))
    np.testing.assert_array_equal(r["ssum"], [2.0, 2.0])


@pytest.mark.parametrize("T,N,k,seed", [(1, 8, 2, 0), (16, 8, 2, 1), (33, 60, 4, 2), (64, 128, 8, 3), (7, 256, 16, 4)])
def test_against_a_library_logistic_function(T, N, k, seed):
    z = wl.make_logits(T, N, seed=seed, quantum=[None, 0.25][seed % 2])
    r = oracle.topk_sigmoid(z, k)
    # the selection is the softmax router's: the sigmoid is increasing, ties go to the lower index
    assert np.array_equal(r["idx"], oracle.topk(z, k)["idx"])
    order = np.argsort(-z.astype(np.float64), axis=1, kind="stable")[:, :k]
    assert np.array_equal(r["idx"], order)
    s = expit(np.take_along_axis(z.astype(np.float64), order, axis=1))
    np.testing.assert_allclose(r["gate"], s / s.sum(1, keepdims=True), rtol=1e-13)
    np.testing.assert_allclose(r["ssum"], s.sum(1), rtol=1e-13)
    np.testing.assert_allclose(r["gate"].sum(1), 1.0, rtol=1e-14)
    assert np.all(np.diff(r["gate"], axis=1) <= 0)               # gates follow the logits' order


def test_what_tells_it_from_softmax():
    # softmax gates over the selection depend on logit differences only; sigmoid gates do not: a shift of all logits
    # moves them towards 1/k (large positive: every score near 1) or towards the softmax ratio (large negative:
    # sigmoid(z) ~ exp(z))
    z = np.array([[2.0, 0.0, -1.0]], np.float32)
    soft = oracle.topk(z, 2)["gate"][0]
    np.testing.assert_allclose(soft, [1 / (1 + np.exp(-2.0)), 1 / (1 + np.exp(2.0))], rtol=1e-15)
    sig = oracle.topk_sigmoid(z, 2)["gate"][0]
    np.testing.assert_allclose(sig, [expit(2.0) / (expit(2.0) + 0.5), 0.5 / (expit(2.0) + 0.5)], rtol=1e-15)
    assert abs(sig[0] - soft[0]) > 0.2
    up = oracle.topk_sigmoid(z + np.float32(30.0), 2)["gate"][0]
    np.testing.assert_allclose(up, [0.5, 0.5], atol=1e-12)
    down = oracle.topk_sigmoid(z - np.float32(40.0), 2)["gate"][0]
    np.testing.assert_allclose(down, soft, rtol=1e-12)           # far in the negative tail the two agree
    assert np.all(np.isfinite(oracle.topk_sigmoid(z - np.float32(700.0), 2)["gate"]))   # no overflow in exp(-z)


def test_gates_of_a_given_selection_and_errors():
    z = wl.make_logits(9, 12, seed=5)
    rng = np.random.default_rng(0)
    idx = np.stack([rng.permutation(12)[:5] for _ in range(9)]).astype(np.int32)
    g, ssum = oracle.sigmoid_gates(z, idx)
    s = expit(np.take_along_axis(z.astype(np.float64), idx, axis=1))
    np.testing.assert_allclose(g, s / s.sum(1, keepdims=True), rtol=1e-13)
    np.testing.assert_allclose(ssum, s.sum(1), rtol=1e-13)
    bad = idx.copy()
    bad[3, 2] = 12
    with pytest.raises(oracle.OracleError):
        oracle.sigmoid_gates(z, bad)
    with pytest.raises(oracle.OracleError):
        oracle.topk_sigmoid(z, 13)


@pytest.mark.parametrize("T,N,k,alpha,beta", [(16, 8, 2, 2.0, 2), (40, 60, 4, 4.0, 1), (64, 128, 8, 1.0, 3)])
def test_binning_is_the_softmax_path_with_other_gates(T, N, k, alpha, beta):
    z = wl.make_logits(T, N, seed=T + N)
    idx = oracle.topk_sigmoid(z, k)["idx"]
    a, b = oracle.affinity_bin(z, idx, alpha, beta), oracle.affinity_bin_sigmoid(z, idx, alpha, beta)
    for key in ("new_idx", "cnt_before", "cnt_after", "bin_hist", "num_active", "q", "score", "active"):
        assert np.array_equal(a[key], b[key]), key               # logit differences only: nothing else moves
    s = expit(np.take_along_axis(z.astype(np.float64), b["new_idx"], axis=1))
    np.testing.assert_allclose(b["new_gate"], s / s.sum(1, keepdims=True), rtol=1e-13)
    assert not np.allclose(a["new_gate"], b["new_gate"])
