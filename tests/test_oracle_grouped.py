"""Pins of the oracle's group-limited router (paper Sec. 1 names expert grouping among the architectures to cover and
gives no rule for it).

The reading (groups of consecutive experts, group score = largest logit, a token stays inside its topk_group best
groups, also after the remap) is this build's own.  What pins its implementation: hand-worked cases, a numpy statement
of the mask, the special cases that are the ungrouped method, and the reduction of the whole grouped remap to the
ungrouped one on logits whose forbidden entries are pushed far down.
"""
import numpy as np
import pytest
from scipy.special import softmax

import oracle
import workloads as wl


def _numpy_allowed(z, n_group, topk_group):
    T, N = z.shape
    gs = N // n_group
    gmax = z.reshape(T, n_group, gs).max(axis=2)
    order = np.argsort(-gmax.astype(np.float64), axis=1, kind="stable")[:, :topk_group]
    allow = np.zeros((T, n_group), np.uint8)
    np.put_along_axis(allow, order, 1, axis=1)
    return np.repeat(allow, gs, axis=1)


def test_hand_worked_selection():
    # groups {0,1} {2,3} {4,5}: group scores 1, 5, 4.5 -> groups 1 and 2; top-2 inside them = experts 2 and 4
    z = np.array([[1.0, 0.0, 5.0, -1.0, 4.5, 4.0]], np.float32)
    assert oracle.group_allowed(z, 3, 2).tolist() == [[0, 0, 1, 1, 1, 1]]
    r = oracle.topk_grouped(z, 2, 3, 2)
    assert r["idx"].tolist() == [[2, 4]]
    # one group only: the best expert of the whole token decides, and the second pick is its neighbour, not expert 4
    assert oracle.topk_grouped(z, 2, 3, 1)["idx"].tolist() == [[2, 3]]
    # equal group scores go to the lower group
    z = np.array([[2.0, 0.0, 1.0, 2.0, 2.0, -3.0]], np.float32)
    assert oracle.group_allowed(z, 3, 2).tolist() == [[1, 1, 1, 1, 0, 0]]
    assert oracle.topk_grouped(z, 3, 3, 2)["idx"].tolist() == [[0, 3, 2]]
    # the third output is the share of the softmax over ALL experts, forbidden ones included
    p = softmax(z.astype(np.float64), axis=1)[0]
    np.testing.assert_allclose(oracle.topk_grouped(z, 3, 3, 2)["third"][0], p[0] + p[3] + p[2], rtol=1e-14)


@pytest.mark.parametrize("T,N,k,G,tg,seed", [(9, 16, 3, 4, 2, 0), (33, 64, 6, 8, 3, 1), (20, 160, 6, 8, 3, 2),
                                             (17, 256, 8, 8, 4, 3), (5, 60, 4, 3, 2, 4), (12, 48, 5, 48, 7, 5)])
def test_mask_and_selection_against_numpy(T, N, k, G, tg, seed):
    z = wl.make_logits(T, N, seed=seed, quantum=[None, 0.5][seed % 2])
    allow = oracle.group_allowed(z, G, tg)
    assert np.array_equal(allow, _numpy_allowed(z, G, tg))
    assert (allow.sum(axis=1) == tg * (N // G)).all()
    assert allow[np.arange(T), z.argmax(axis=1)].all()            # the group of the best expert is always in
    for gate_fn in (0, 1):
        r = oracle.topk_grouped(z, k, G, tg, gate_fn)
        # the ungrouped top-k of the logits with the forbidden experts pushed out of reach
        zm = np.where(allow != 0, z, np.float32(-1e30))
        ref = (oracle.topk_sigmoid if gate_fn else oracle.topk)(zm, k)
        assert np.array_equal(r["idx"], ref["idx"])
        np.testing.assert_allclose(r["gate"], ref["gate"], rtol=1e-13)
        if gate_fn == 0:
            p = softmax(z.astype(np.float64), axis=1)
            np.testing.assert_allclose(r["third"], np.take_along_axis(p, r["idx"], 1).sum(1), rtol=1e-12)
        else:
            np.testing.assert_allclose(r["third"], ref["ssum"], rtol=1e-13)


@pytest.mark.parametrize("G,tg", [(1, 1), (4, 4), (8, 8)])
def test_no_limit_is_the_ungrouped_method(G, tg):
    z = wl.make_logits(40, 64, seed=11, quantum=0.25)
    r = oracle.topk_grouped(z, 6, G, tg)
    ref = oracle.topk(z, 6)
    assert np.array_equal(r["idx"], ref["idx"])
    np.testing.assert_array_equal(r["gate"], ref["gate"])
    np.testing.assert_allclose(r["third"], ref["psum"], rtol=1e-14)
    a = oracle.affinity_bin_grouped(z, r["idx"], G, tg, 1.0, 2)
    b = oracle.affinity_bin(z, ref["idx"], 1.0, 2)
    for key in ("new_idx", "new_gate", "cnt_before", "cnt_after", "bin_hist", "num_active", "active"):
        np.testing.assert_array_equal(a[key], b[key])


def test_hand_worked_remap_keeps_a_token_inside_its_groups():
    # two groups of two, one group per token, k = 2, one bin of width 1.
    # token 0: experts 0 and 1, both in bin 0 -> nominates 0 and 1.  token 1: experts 2 (bin 0) and 3 (25 below the
    # top: out of range) -> nominates 2 only.  A = {0, 1, 2}.  Token 1 may only use {2, 3}: one member of A, so its
    # second slot keeps its own pick 3 (without groups it would move to expert 0).
    z = np.array([[5.0, 4.9, 0.0, 0.0], [0.0, 0.0, 5.0, -20.0]], np.float32)
    sel = oracle.topk_grouped(z, 2, 2, 1)["idx"]
    assert sel.tolist() == [[0, 1], [2, 3]]
    a = oracle.affinity_bin_grouped(z, sel, 2, 1, 1.0, 1)
    assert a["active"].tolist() == [1, 1, 1, 0]
    assert a["new_idx"].tolist() == [[0, 1], [2, 3]]
    assert a["bin_hist"][:, 0].tolist() == [1, 1, 1, 0]           # expert 0 gets no vote from token 1: not allowed there
    assert a["num_active"].tolist() == [4, 4]
    b = oracle.affinity_bin(z, sel, 1.0, 1)
    assert b["new_idx"].tolist() == [[0, 1], [2, 0]]
    assert b["bin_hist"][:, 0].tolist() == [1, 1, 1, 0]


@pytest.mark.parametrize("T,N,k,G,tg,alpha,beta,seed", [(24, 32, 4, 4, 2, 1.0, 2, 0), (64, 64, 6, 8, 3, 0.5, 3, 1),
                                                        (40, 160, 6, 8, 3, 1.0, 2, 2), (32, 256, 8, 8, 4, 1.0, 2, 3),
                                                        (100, 60, 4, 6, 2, 2.0, 2, 4), (16, 128, 8, 4, 1, 1.0, 1, 5)])
def test_grouped_remap_reduces_to_the_ungrouped_one_on_masked_logits(T, N, k, G, tg, alpha, beta, seed):
    z = wl.make_logits(T, N, seed=seed, quantum=[None, 0.25][seed % 2])
    allow = oracle.group_allowed(z, G, tg)
    sel = oracle.topk_grouped(z, k, G, tg)["idx"]
    a = oracle.affinity_bin_grouped(z, sel, G, tg, alpha, beta)
    # invariants of the reading
    assert np.take_along_axis(allow, a["new_idx"], 1).all()       # every token stays inside its groups
    assert all(len(set(row)) == k for row in a["new_idx"].tolist())
    assert a["cnt_after"].sum() == T * k and a["num_active"][1] <= a["num_active"][0]
    assert (a["cnt_before"][a["cnt_after"] > 0] > 0).all()        # only experts the batch already invoked
    # forbidden entries far below everything: bin beta (no vote, never nominated), never among a token's k best of
    # the active set unless the token runs short of allowed ones
    zm = np.where(allow != 0, z, np.float32(-1e4))
    b = oracle.affinity_bin(zm, sel, alpha, beta)
    np.testing.assert_array_equal(a["bin_hist"], b["bin_hist"])
    np.testing.assert_array_equal(a["cnt_before"], b["cnt_before"])
    np.testing.assert_array_equal(a["active"], b["active"])
    full = np.take_along_axis(allow, b["new_idx"], 1).all(axis=1)  # tokens whose groups held k active experts
    assert full.any()
    np.testing.assert_array_equal(a["new_idx"][full], b["new_idx"][full])
    np.testing.assert_allclose(a["new_gate"][full], b["new_gate"][full], rtol=1e-13)
    for t in np.nonzero(~full)[0]:
        # short tokens: the allowed part of the ungrouped answer first, then own picks in rank order
        keep = [e for e in b["new_idx"][t].tolist() if allow[t, e]]
        rest = [e for e in sel[t].tolist() if e not in keep]
        assert a["new_idx"][t].tolist() == (keep + rest)[:k]


def test_short_tokens_occur_and_keep_their_own_picks():
    # one group per token and a single narrow bin: tokens nominate little, so groups often hold fewer than k active experts
    z = wl.make_logits(48, 64, seed=9)
    sel = oracle.topk_grouped(z, 6, 8, 1)["idx"]
    a = oracle.affinity_bin_grouped(z, sel, 8, 1, 4.0, 1)
    kept = [(set(a["new_idx"][t].tolist()) - set(np.nonzero(a["active"])[0].tolist())) for t in range(48)]
    assert any(kept)                                              # the case is exercised
    for t, extra in enumerate(kept):
        assert extra <= set(sel[t].tolist())                      # what is outside A is the token's own pick


def test_bad_arguments():
    z = np.zeros((2, 12), np.float32)
    for G, tg, k in [(5, 2, 2), (4, 5, 2), (0, 1, 2), (4, 0, 2), (4, 1, 4)]:   # 12 % 5, tg > G, zeros, 1 * 3 < 4
        with pytest.raises(oracle.OracleError):
            oracle.topk_grouped(z, k, G, tg)
    # picks outside the token's groups are refused
    z = np.array([[3.0, 0.0, 1.0, 0.0]], np.float32)
    with pytest.raises(oracle.OracleError):
        oracle.affinity_bin_grouped(z, np.array([[0, 2]], np.int32), 2, 1, 1.0, 2)
