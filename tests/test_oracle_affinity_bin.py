"""Pins for the oracle's AffinityBinning / scoring / remapping (paper Secs. 3.2.1, 3.3.1, 3.4, 4).

The paper gives this part in prose only, so it is pinned by: the hand-worked example under
tests/golden/, the invariants the paper states, closed-form special cases, exact integer arithmetic
redone with Python big integers, and an exhaustive subset search on tiny batches.
"""
import itertools

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


def _run(z, k, alpha, beta, enable=1):
    idx = _topk(z, k)
    return idx, oracle.affinity_bin(z, idx, alpha, beta, enable)


CASES = [(16, 8, 2, 1.1, 0.0), (8, 8, 2, 1.1, 0.0), (32, 60, 4, 1.0, 0.0), (64, 64, 6, 0.9, 0.05),
         (128, 128, 8, 1.0, 0.0), (5, 6, 3, 1.0, 0.2), (2, 4, 2, 1.0, 0.0), (33, 17, 5, 1.0, 0.1)]
PRESETS = [(2.0, 2), (4.0, 1), (1.0, 3), (0.5, 6), (8.0, 2)]


# ---------------------------------------------------------------- worked example --------------------------------------

def test_worked_example(golden_w1):
    g = golden_w1
    z = np.array(g["logits"], np.float32)
    idx = np.array(g["topk_idx"], np.int32)
    assert np.array_equal(_topk(z, 2), idx)
    r = oracle.affinity_bin(z, idx, 1.0, 2, 1)
    assert np.array_equal(r["q"], np.minimum(np.array(g["q_floor"], np.int32), 2))
    assert np.array_equal(r["bin_hist"], np.array(g["bin_hist"], np.int32))
    assert [int(s) for s in r["score"]] == [int(v) for v in g["score"][0]]
    assert np.array_equal(r["active"], np.array(g["active_set"][0], np.int32))
    assert np.array_equal(r["cnt_before"], np.array(g["cnt_before"][0], np.int32))
    assert np.array_equal(r["new_idx"], np.array(g["new_idx"], np.int32))
    assert np.array_equal(r["cnt_after"], np.array(g["cnt_after"][0], np.int32))
    assert r["num_active"].tolist() == [int(g["num_active_before"][0][0]), int(g["num_active_after"][0][0])]
    np.testing.assert_allclose(r["new_gate"], np.array(g["gate_after"]), atol=6e-6)
    r_off = oracle.affinity_bin(z, idx, 1.0, 2, 0)
    np.testing.assert_allclose(r_off["new_gate"], np.array(g["gate_before"]), atol=6e-6)
    p = oracle.permute(r["new_idx"], 4)
    assert p["offsets"].tolist() == [int(v) for v in g["offsets"][0]]
    assert p["perm"].tolist() == [int(v) for v in g["perm"][0]]
    n = int(p["num_active"][0])
    assert p["active"][:n].tolist() == [int(v) for v in g["active_list"][0]]


# ---------------------------------------------------------------- exact integer parts ---------------------------------

@pytest.mark.parametrize("T,N,k,s,tail", CASES)
@pytest.mark.parametrize("alpha,beta", PRESETS)
def test_bins_histogram_and_score_are_exact(T, N, k, s, tail, alpha, beta):
    z = wl.make_logits(T, N, seed=T + N, zipf_s=s, tail_frac=tail)
    idx, r = _run(z, k, alpha, beta)
    # bins: one fp32 subtract, one fp32 multiply, floor, clamp -- redone with numpy float32 scalars
    d = (z.max(1, keepdims=True) - z).astype(np.float32)
    q_ref = np.minimum(np.floor(np.float32(alpha) * d), beta).astype(np.int32)
    assert np.array_equal(r["q"], q_ref)
    assert np.all(r["q"][np.arange(T), idx[:, 0]] == 0)                   # the top-1 sits in bin 0
    # bins never get better as the logit drops
    order = np.argsort(-z, axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(r["q"], order, 1), axis=1) >= 0)
    hist = np.stack([(q_ref == j).sum(0) for j in range(beta)], axis=1)
    assert np.array_equal(r["bin_hist"], hist)
    for e in range(N):
        s_int = sum(int(hist[e, j]) * T ** (beta - 1 - j) for j in range(beta))   # Python big ints
        assert int(r["score"][e]) == s_int
    assert np.all(r["bin_hist"].sum(1) <= T)
    top1_votes = np.bincount(idx[:, 0], minlength=N)
    assert np.all(r["bin_hist"][:, 0] >= top1_votes)
    assert np.array_equal(r["cnt_before"], np.bincount(idx.reshape(-1), minlength=N))


def test_score_weights_follow_base_T_exponent():
    # One token moving an expert from bin -1 to bin 0 raises its score by T^(beta-1) - T^(beta-2): the
    # batch size is the base and the bin value the exponent (Sec. 3.3.1).
    T, N, k, beta = 5, 3, 1, 3
    z = np.zeros((T, N), np.float32)
    z[:, 0] = 10.0
    z[:, 1] = 10.0 - 1.5          # bin 1 at alpha = 1
    z[:, 2] = 10.0 - 2.5          # bin 2
    _, r = _run(z, k, 1.0, beta)
    assert [int(v) for v in r["score"]] == [5 * 25, 5 * 5, 5 * 1]
    z[0, 1] = 10.0 - 0.5          # token 0 now holds expert 1 in bin 0
    _, r2 = _run(z, k, 1.0, beta)
    assert int(r2["score"][1]) - int(r["score"][1]) == 25 - 5
    z[:, 2] = 10.0 - 3.0          # exactly on the boundary of the last allowed bin: out of range, weight 0
    _, r3 = _run(z, k, 1.0, beta)
    assert int(r3["score"][2]) == 0 and np.all(r3["q"][:, 2] == beta)


# ---------------------------------------------------------------- invariants ------------------------------------------

@pytest.mark.parametrize("T,N,k,s,tail", CASES)
@pytest.mark.parametrize("alpha,beta", PRESETS)
def test_invariants(T, N, k, s, tail, alpha, beta):
    for seed in range(3):
        z = wl.make_logits(T, N, seed=seed * 100 + T, zipf_s=s, tail_frac=tail,
                           quantum=0.25 if seed == 2 else None)       # seed 2: many exact ties / boundary hits
        idx, r = _run(z, k, alpha, beta)
        new, q, A = r["new_idx"], r["q"], r["active"].astype(bool)
        U = r["cnt_before"] > 0
        # each token keeps exactly k distinct experts
        assert np.all((new >= 0) & (new < N))
        assert all(len(set(row)) == k for row in new.tolist())
        # remap onto experts the batch already activates: idx' within A within U
        assert np.all(A[new]) and np.all(U[A])
        assert A.sum() >= k
        # invoked experts never rise
        assert r["num_active"][1] <= r["num_active"][0] == U.sum()
        assert r["num_active"][1] == (r["cnt_after"] > 0).sum()
        # gates: positive, non-increasing, sum 1
        g = r["new_gate"]
        np.testing.assert_allclose(g.sum(1), 1.0, rtol=1e-12)
        assert np.all(g > 0) and np.all(np.diff(g, axis=1) <= 1e-15)
        # new selection is in descending logit order with ties to the lower index
        zsel = np.take_along_axis(z, new.astype(np.int64), 1)
        assert np.all(np.diff(zsel, axis=1) <= 0)
        tie = np.diff(zsel, axis=1) == 0
        assert np.all(np.diff(new, axis=1)[tie] > 0)
        # pair counts conserved
        assert r["cnt_before"].sum() == r["cnt_after"].sum() == T * k
        assert np.array_equal(r["cnt_after"], np.bincount(new.reshape(-1), minlength=N))
        # per in-range slot the new expert is in a bin at least as good as the old one
        q_old = np.take_along_axis(q, idx.astype(np.int64), 1)
        q_new = np.take_along_axis(q, new.astype(np.int64), 1)
        in_range = q_old < beta
        assert np.all(q_new[in_range] <= q_old[in_range])
        # a token whose top-1 is alone in bin 0 keeps it in first place
        alone = (q == 0).sum(1) == 1
        assert np.all(new[alone, 0] == idx[alone, 0])
        # unchanged selections keep bit-identical gates
        r_off = oracle.affinity_bin(z, idx, alpha, beta, 0)
        same = np.all(new == idx, axis=1)
        assert np.array_equal(g[same], r_off["new_gate"][same])
        # new selection = top-k by logit within A (independent of the oracle's own selection routine)
        zm = np.where(A[None, :], z.astype(np.float64), -np.inf)
        assert np.array_equal(new, _topk(zm, k))


@pytest.mark.parametrize("T,N,k", [(16, 8, 2), (24, 60, 4), (40, 64, 6)])
def test_token_order_does_not_matter(T, N, k):
    z = wl.make_logits(T, N, seed=7, tail_frac=0.1)
    idx, r = _run(z, k, 2.0, 2)
    perm = np.random.default_rng(3).permutation(T)
    idx_p, r_p = _run(z[perm], k, 2.0, 2)
    assert np.array_equal(r_p["active"], r["active"])
    assert np.array_equal(r_p["new_idx"], r["new_idx"][perm])
    assert np.array_equal(r_p["new_gate"], r["new_gate"][perm])
    assert np.array_equal(r_p["score"], r["score"])


# ---------------------------------------------------------------- closed forms ----------------------------------------

@pytest.mark.parametrize("T,N,k", [(16, 8, 2), (1, 8, 2), (32, 60, 4)])
def test_bypass_is_identity(T, N, k):
    z = wl.make_logits(T, N, seed=11)
    idx = _topk(z, k)
    for enable in ((0,) if T > 1 else (0, 1)):            # T = 1 is an identity even when enabled
        r = oracle.affinity_bin(z, idx, 4.0, 1, enable)
        assert np.array_equal(r["new_idx"], idx)
        assert np.array_equal(r["cnt_after"], r["cnt_before"])
        assert r["num_active"][0] == r["num_active"][1]
        e = np.exp(np.take_along_axis(z.astype(np.float64), idx.astype(np.int64), 1))
        np.testing.assert_allclose(r["new_gate"], e / e.sum(1, keepdims=True), rtol=1e-12)
        assert r["bin_hist"].sum() > 0                        # histogram is still produced


def test_alpha_zero_collapses_onto_lowest_indexed_active_experts():
    T, N, k = 20, 12, 3
    z = wl.make_logits(T, N, seed=5)
    idx, r = _run(z, k, 0.0, 2)
    assert np.all(r["q"] == 0)
    U = np.nonzero(r["cnt_before"])[0]
    A = np.nonzero(r["active"])[0]
    assert np.array_equal(A, U[:k])
    assert r["num_active"][1] == k


def test_identical_tokens_change_nothing():
    N, k = 10, 3
    z = np.tile(wl.make_logits(1, N, seed=2), (9, 1))
    idx, r = _run(z, k, 2.0, 2)
    assert np.array_equal(r["new_idx"], idx) and r["num_active"].tolist() == [k, k]


def test_very_fine_bins_keep_only_distinct_top1_then_fill():
    T, N, k = 12, 16, 4
    z = wl.make_logits(T, N, seed=8)
    idx, r = _run(z, k, 1.0e6, 1)
    top1 = set(idx[:, 0].tolist())
    A = set(np.nonzero(r["active"])[0].tolist())
    assert top1 <= A and len(A) == max(len(top1), k)
    assert np.array_equal(r["new_idx"][:, 0], idx[:, 0])
    if len(top1) < k:                                         # the fill takes the best-scoring remaining experts of U
        rest = sorted((e for e in np.nonzero(r["cnt_before"])[0] if e not in top1),
                      key=lambda e: (-int(r["score"][e]), e))
        assert A - top1 == set(rest[:k - len(top1)])


def test_fill_when_nominations_leave_fewer_than_k():
    # every token has the same confident top-1, and all second picks are out of range
    z = np.array([[9.0, 1.0, 0.0, 0.5], [9.0, 0.0, 1.0, 0.5], [9.0, 0.2, 1.0, 0.0]], np.float32)
    idx, r = _run(z, 2, 1.0, 2)
    assert r["score"].tolist() == [9, 0, 0, 0]                # 3 bin-0 votes * T, nothing else in range
    assert r["active"].tolist() == [1, 1, 0, 0]               # filled from U by score, tie -> lower index
    assert r["new_idx"].tolist() == [[0, 1], [0, 1], [0, 1]]


def test_picks_in_any_order_are_accepted():
    """The picks normally arrive in rank order (descending logit).  Rows in another order must not break anything: a
    slot whose candidates are all used nominates nothing, the active set stays inside the invoked experts and holds at
    least min(k, |U|) of them, and the new selection stays inside the active set."""
    # hand case: token 0 lists its worse pick first; slot 0 (pick 1, bin 1) nominates the best-scoring expert with
    # bin <= 1, which is expert 0; slot 1 (pick 0, bin 0) finds expert 0 used and no other expert in bin 0
    z = np.array([[4.0, 3.0, 0.0], [4.0, 3.0, 0.0]], np.float32)
    idx = np.array([[1, 0], [1, 0]], np.int32)
    r = oracle.affinity_bin(z, idx, 1.0, 2)
    assert r["active"].tolist() == [1, 1, 0] and r["new_idx"].tolist() == [[0, 1], [0, 1]]
    for seed in range(60):
        rng = np.random.default_rng(seed)
        T, N = int(rng.integers(2, 200)), int(rng.integers(2, 130))
        k = int(rng.integers(1, min(N, 16) + 1))
        z = wl.make_logits(T, N, seed=seed, quantum=[None, 0.25][seed % 2])
        idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
        r = oracle.affinity_bin(z, idx, float(rng.choice([0.5, 2.0, 4.0])), int(rng.integers(1, 5)))
        U, A = set(idx.ravel().tolist()), set(np.nonzero(r["active"])[0].tolist())
        assert A <= U and len(A) >= min(k, len(U))
        assert set(r["new_idx"].ravel().tolist()) <= A
        assert r["num_active"][1] <= r["num_active"][0] == len(U)


def test_errors():
    z = wl.make_logits(4, 4, seed=0)
    idx = _topk(z, 2)
    for kwargs, code in [(dict(alpha=1.0, beta=0), oracle.ERR_INVALID_ARG), (dict(alpha=-1.0, beta=2), oracle.ERR_INVALID_ARG),
                         (dict(alpha=float("nan"), beta=2), oracle.ERR_INVALID_ARG),
                         (dict(alpha=1.0, beta=7), oracle.ERR_UNSUPPORTED)]:
        with pytest.raises(oracle.OracleError) as ei:
            oracle.affinity_bin(z, idx, **kwargs)
        assert ei.value.code == code
    bad = idx.copy()
    bad[0, 1] = bad[0, 0]
    with pytest.raises(oracle.OracleError):
        oracle.affinity_bin(z, bad, 1.0, 2)
    with pytest.raises(oracle.OracleError) as ei:             # T^beta must stay below 2^62
        oracle.affinity_bin(wl.make_logits(2048, 4, seed=0), _topk(wl.make_logits(2048, 4, seed=0), 2), 1.0, 6)
    assert ei.value.code == oracle.ERR_UNSUPPORTED


# ---------------------------------------------------------------- exhaustive search on tiny batches -------------------

def _feasible(S, q, idx, beta, k):
    """A subset S of experts can serve the batch if it has at least k members and, for every token and every
    in-range slot i (1-based), at least i members in a bin at least as good as that slot's own pick."""
    if len(S) < k:
        return False
    S = list(S)
    for t in range(q.shape[0]):
        for i in range(idx.shape[1]):
            qi = q[t, idx[t, i]]
            if qi >= beta:
                break
            if sum(1 for e in S if q[t, e] <= qi) < i + 1:
                return False
    return True


@pytest.mark.parametrize("T,N,k", [(2, 4, 2), (3, 5, 2), (4, 6, 3), (4, 6, 2), (3, 6, 1)])
def test_active_set_is_feasible_and_near_minimal_on_tiny_batches(T, N, k):
    gaps = []
    for seed in range(40):
        z = wl.make_logits(T, N, seed=seed, quantum=0.5 if seed % 2 else None)
        for alpha, beta in [(1.0, 2), (2.0, 2), (4.0, 1), (0.5, 3)]:
            idx, r = _run(z, k, alpha, beta)
            q = r["q"]
            U = [e for e in range(N) if r["cnt_before"][e] > 0]
            A = [e for e in range(N) if r["active"][e]]
            assert _feasible(A, q, idx, beta, k)
            best = min(len(S) for n in range(k, len(U) + 1) for S in itertools.combinations(U, n)
                       if _feasible(S, q, idx, beta, k))
            assert best <= len(A) <= len(U)
            gaps.append(len(A) - best)
    # the slot-by-slot rule is greedy: it may exceed the minimum, but not by much on batches this small
    assert np.mean(gaps) < 0.5 and max(gaps) <= 2


# ---- the probability mass of a selection (the "top-k weight sums" of Sec. 4) ------------------------------------------

def test_selection_mass_is_the_share_of_the_full_softmax():
    """orc_selection_mass against a library softmax: sum of the selected probabilities; the router's own top-k gives
    orc_topk's psum; entries outside [0, N) are skipped; all experts selected gives 1."""
    from scipy.special import softmax
    rng = np.random.default_rng(5)
    for T, N, k in [(1, 4, 2), (9, 60, 4), (33, 128, 8)]:
        z = (rng.standard_normal((T, N)) * 3).astype(np.float32)
        p = softmax(z.astype(np.float64), axis=1)
        sel = np.stack([rng.choice(N, size=k, replace=False) for _ in range(T)]).astype(np.int32)
        np.testing.assert_allclose(oracle.selection_mass(z, sel), np.take_along_axis(p, sel, 1).sum(1), rtol=1e-12)
        tk = oracle.topk(z, k)
        np.testing.assert_allclose(oracle.selection_mass(z, tk["idx"]), tk["psum"], rtol=1e-12)
        bad = sel.copy()
        bad[:, 0] = -1
        np.testing.assert_allclose(oracle.selection_mass(z, bad), np.take_along_axis(p, sel[:, 1:], 1).sum(1), rtol=1e-12)
        every = np.tile(np.arange(N, dtype=np.int32), (T, 1))
        np.testing.assert_allclose(oracle.selection_mass(z, every), 1.0, rtol=1e-12)
    # a closed form: logits ln 1, ln 2, ln 3, ln 4 are probabilities 0.1 .. 0.4
    z = np.log(np.array([[1.0, 2.0, 3.0, 4.0]])).astype(np.float32)
    np.testing.assert_allclose(oracle.selection_mass(z, np.array([[3, 1]], np.int32)), [0.6], rtol=1e-6)


@pytest.mark.parametrize("preset", ["moderate", "aggressive"])
def test_remap_never_gains_probability_mass_and_keeps_it_where_nothing_moves(preset):
    """new_psum <= the mass of the router's own top-k (the top-k is the selection of largest mass), with equality
    exactly where the selection is unchanged; bypassed calls keep everything."""
    alpha, beta = wl.PRESETS[preset]
    for T, N, k, seed in [(8, 8, 2, 0), (32, 128, 8, 1), (64, 60, 4, 2), (256, 64, 6, 3)]:
        z = wl.make_logits(T, N, seed=seed, tail_frac=0.05)
        tk = oracle.topk(z, k)
        a = oracle.affinity_bin(z, tk["idx"], alpha, beta, 1)
        assert np.all(a["new_psum"] <= tk["psum"] * (1 + 1e-12))
        same = np.all(np.sort(a["new_idx"], 1) == np.sort(tk["idx"], 1), axis=1)
        np.testing.assert_allclose(a["new_psum"][same], tk["psum"][same], rtol=1e-12)
        assert np.all(a["new_psum"][~same] < tk["psum"][~same])
        off = oracle.affinity_bin(z, tk["idx"], alpha, beta, 0)
        np.testing.assert_allclose(off["new_psum"], tk["psum"], rtol=1e-12)


def test_rank0_retention_under_the_reading():
    """Sec. 3.3.1: high-confidence tokens always keep their top-ranked expert.  Under the reading implemented here a
    token keeps its top-1 whenever that expert is alone in the token's bin 0 (no other expert within 1/alpha of it); a
    token whose top-1 has company in bin 0 may be moved to the batch-preferred member of that bin, which is at most one
    bin width below.  Both halves, on router-like logits."""
    for preset in ("moderate", "aggressive"):
        alpha, beta = wl.PRESETS[preset]
        for T, N, k, seed in [(32, 128, 8, 0), (128, 64, 6, 1), (16, 8, 2, 2)]:
            z = wl.make_logits(T, N, seed=seed)
            tk = oracle.topk(z, k)
            a = oracle.affinity_bin(z, tk["idx"], alpha, beta, 1)
            top = tk["idx"][:, 0]
            alone = (a["q"] == 0).sum(1) == 1
            kept = (a["new_idx"] == top[:, None]).any(1)
            assert kept[alone].all()
            # a token that lost its top-1 got, as its best expert, one of the same bin: less than 1/alpha below
            lost = ~kept
            zt = np.take_along_axis(z, top[:, None], 1)[:, 0]
            zn = np.take_along_axis(z, a["new_idx"][:, :1], 1)[:, 0]
            assert np.all(zt[lost] - zn[lost] < 1.0 / alpha)
