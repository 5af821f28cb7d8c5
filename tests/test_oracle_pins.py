"""Pins for the float64 oracle: everything here checks the oracle against something
other than itself -- a library routine (numpy float64 matmul), exact integer
arithmetic, closed forms, and the invariants the paper's definitions fix.
None of these tests needs a GPU."""
import math

import numpy as np
import pytest

import oracle
from paper_2605_03110_amd import workloads as wl


# ----------------------------------------------------------------------------- helpers
def numpy_gram(X):
    """Independent statement of Section 2.1 with numpy's float64 matmul."""
    X = np.asarray(X, dtype=np.float64)
    n = np.linalg.norm(X, axis=1, keepdims=True)
    Xn = np.divide(X, n, out=np.zeros_like(X), where=n > 0)
    return Xn @ Xn.T


def exact_near(X_int, num, den):
    """near[s][t] <=> |cos(x_s, x_t)| >= num/den, decided in exact integer arithmetic:
    (x_s . x_t)^2 * den^2 >= num^2 * |x_s|^2 |x_t|^2.  Also returns the smallest relative
    distance of any pair from equality so callers can reject inputs a float64
    evaluation could not decide."""
    T = len(X_int)
    near = [[False] * T for _ in range(T)]
    margin = math.inf
    for s in range(T):
        for t in range(T):
            dot = sum(int(a) * int(b) for a, b in zip(X_int[s], X_int[t]))
            ns = sum(int(a) * int(a) for a in X_int[s])
            nt = sum(int(b) * int(b) for b in X_int[t])
            lhs = dot * dot * den * den
            rhs = num * num * ns * nt
            near[s][t] = lhs >= rhs
            if rhs > 0:
                margin = min(margin, abs(lhs - rhs) / rhs)
    return near, margin


def exact_full(near, T):
    return [t for t in range(T) if not any(near[s][t] for s in range(t))]


def exact_cascade(near, T, R, earlier_only):
    R = sorted(R)
    valid = [s for s in R if not any(near[sp][s] for sp in R if sp < s)]
    new = [t for t in range(T) if t not in R
           and not any(near[t][s] for s in valid if (s < t or not earlier_only))]
    idx = sorted(valid + new)
    removes = [s for s in R if s not in valid]
    ops = len(R) ** 2 + (T - len(R)) * len(valid)
    return idx, new, removes, ops


def integer_tokens(rng, T, d, n_base):
    """Integer vectors with a mix of near-parallel and unrelated pairs."""
    base = rng.integers(-9, 10, size=(n_base, d))
    base[np.all(base == 0, axis=1)] = 1
    rows = []
    for _ in range(T):
        b = base[rng.integers(0, n_base)]
        k = int(rng.integers(1, 4)) * (1 if rng.random() < 0.8 else -1)
        noise = rng.integers(-2, 3, size=d) * (rng.random(d) < 0.5)
        rows.append(k * 6 * b + noise)
    return np.array(rows, dtype=np.int64)


RATIONAL_TAUS = [((1, 10), (99, 100)), ((3, 10), (91, 100)), ((1, 2), (3, 4)), ((7, 10), (51, 100))]


# ----------------------------------------------------------------------------- Section 2.1
def test_gram_matches_numpy_float64_and_is_a_cosine_matrix():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((37, 53)) * rng.uniform(0.1, 30.0, size=(37, 1))
    G = oracle.gram(X)
    assert np.allclose(G, numpy_gram(X), atol=1e-13, rtol=0)
    assert np.allclose(G, G.T, atol=1e-15)
    assert np.allclose(np.diag(G), 1.0, atol=1e-14)
    assert np.max(np.abs(G)) <= 1.0 + 1e-14


def test_normalize_gives_unit_rows_and_reports_norms():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((9, 17)) * 5.0
    Xhat, norms = oracle.normalize(X)
    assert np.allclose(norms, np.linalg.norm(X, axis=1), rtol=1e-15)
    assert np.allclose(np.linalg.norm(Xhat, axis=1), 1.0, atol=1e-15)
    assert np.allclose(Xhat * norms[:, None], X, rtol=1e-14, atol=0)


def test_scale_invariance():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((40, 24))
    X[20:] = X[:20] + 0.01 * rng.standard_normal((20, 24))
    a = oracle.select_full(X, 0.3)
    b = oracle.select_full(X * rng.uniform(0.01, 100.0, size=(40, 1)), 0.3)
    assert np.array_equal(a["mask"], b["mask"])
    assert np.allclose(a["gamma"], b["gamma"], atol=1e-13)


# ----------------------------------------------------------------------------- Definition "Gram threshold"
def test_gamma_is_strictly_lower_triangular_max_of_abs_gram():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((61, 29))
    X[30:] = -X[:31] + 0.05 * rng.standard_normal((31, 29))      # negative correlations matter (|G|)
    res = oracle.select_full(X, 0.3)
    A = np.abs(numpy_gram(X))
    expect = np.array([A[:t, t].max() if t else 0.0 for t in range(61)])
    assert np.allclose(res["gamma"], expect, atol=1e-13)
    assert res["gamma"][0] == 0.0
    assert np.array_equal(res["mask"], (expect < 1 - 0.3 ** 2).astype(np.uint8))
    assert res["r"] == int(res["mask"].sum())


def test_exact_duplicates_leave_only_the_first():
    rng = np.random.default_rng(4)
    base = rng.standard_normal((5, 16))
    order = [0, 1, 0, 2, 1, 1, 3, 0, 4, 4, 2]
    X = base[order] * rng.uniform(0.5, 2.0, size=(len(order), 1))   # scaled copies are still duplicates
    res = oracle.select_full(X, 0.1)
    assert res["idx"].tolist() == [0, 1, 3, 6, 8]


def test_mutually_orthogonal_tokens_are_all_representative():
    Q, _ = np.linalg.qr(np.random.default_rng(5).standard_normal((32, 32)))
    res = oracle.select_full(Q[:20] * 3.0, 0.1)
    assert res["r"] == 20 and res["mask"].all()
    assert np.max(res["gamma"]) < 1e-14


def test_first_token_is_always_representative_and_sign_is_ignored():
    x = np.array([[1.0, 2.0, -3.0]])
    X = np.vstack([x, -x, 2 * x])
    res = oracle.select_full(X, 0.5)
    assert res["mask"].tolist() == [1, 0, 0]
    assert np.allclose(res["gamma"][1:], 1.0)


def test_zero_row_is_representative_and_covers_nobody():
    X = np.array([[0.0, 0.0], [1.0, 0.0], [0.0, 0.0], [1.0, 1e-9]])
    res = oracle.select_full(X, 0.1)
    assert res["mask"].tolist() == [1, 1, 1, 0]
    assert res["gamma"][2] == 0.0


@pytest.mark.parametrize("tau", [0.1, 0.3, 0.6])
def test_threshold_flips_exactly_at_chord_sqrt2_tau(tau):
    """cos >= 1 - tau^2  <=>  chord |xhat_s - xhat_t| <= sqrt(2) tau (proof of the
    depth-persistence proposition): build 2-D pairs from the chord length."""
    for delta, expect_rep in [(+1e-6, 1), (-1e-6, 0), (+1e-3, 1), (-1e-3, 0)]:
        chord = math.sqrt(2.0) * tau + delta              # longer chord -> smaller cosine -> representative
        theta = 2.0 * math.asin(chord / 2.0)
        X = np.array([[1.0, 0.0], [math.cos(theta), math.sin(theta)]]) * 7.0
        res = oracle.select_full(X, tau)
        assert res["mask"].tolist() == [1, expect_rep]
        assert abs(res["gamma"][1] - (1.0 - chord * chord / 2.0)) < 1e-12


def test_tie_at_threshold_is_redundant():
    # tau = 1/2 gives the threshold 0.75 exactly in binary; x = e_1 and y = (3,2,1,1,1) (|y| = 4) give
    # cos = 3/4 with every intermediate exactly representable, so gamma == threshold: strict "<" fails.
    X = np.array([[1.0, 0, 0, 0, 0], [3.0, 2, 1, 1, 1]])
    res = oracle.select_full(X, 0.5)
    assert res["gamma"][1] == 0.75
    assert res["mask"].tolist() == [1, 0]
    assert oracle.cascade_step(X, 0.5, [0])["idx"].tolist() == [0]


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("tau_q,thr_q", RATIONAL_TAUS)
def test_full_selection_agrees_with_exact_integer_brute_force(seed, tau_q, thr_q):
    rng = np.random.default_rng(100 + seed)
    T, d = 16, 6
    Xi = integer_tokens(rng, T, d, n_base=4)
    near, margin = exact_near(Xi.tolist(), *thr_q)
    if margin < 1e-9:
        pytest.skip("a pair sits on the threshold; float64 cannot be required to decide it")
    res = oracle.select_full(Xi.astype(np.float64), tau_q[0] / tau_q[1])
    assert res["idx"].tolist() == exact_full(near, T)
    assert res["gram_ops"] == T * T


def test_brute_force_inputs_exercise_both_decisions():
    """Guard for the brute-force pins: the integer inputs must contain both redundant
    and representative tokens, or the comparison would be vacuous."""
    seen = set()
    for seed in range(6):
        rng = np.random.default_rng(100 + seed)
        Xi = integer_tokens(rng, 16, 6, n_base=4)
        near, _ = exact_near(Xi.tolist(), 99, 100)
        r = len(exact_full(near, 16))
        assert 1 < r < 16
        seen.add(r)
    assert len(seen) > 1


def test_definition_and_greedy_reading_differ_exactly_on_chains():
    # a ~ b, b ~ c, a !~ c at threshold cos >= 0.91 (tau = 0.3): angles 0, 20, 40 degrees
    ang = np.deg2rad([0.0, 20.0, 40.0])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    assert math.cos(ang[1]) > 0.91 > math.cos(ang[2])
    assert oracle.select_full(X, 0.3)["mask"].tolist() == [1, 0, 0]              # Definition: c is covered by b
    assert oracle.select_full(X, 0.3, greedy=True)["mask"].tolist() == [1, 0, 1]  # greedy covering: c stays


def exact_greedy(near, T):
    """Section 2.5 in exact arithmetic: t is kept iff no earlier KEPT token is near it."""
    kept = []
    for t in range(T):
        if not any(near[s][t] for s in kept):
            kept.append(t)
    return kept


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("tau_q,thr_q", RATIONAL_TAUS)
def test_greedy_covering_agrees_with_exact_integer_brute_force(seed, tau_q, thr_q):
    rng = np.random.default_rng(300 + seed)
    T, d = 16, 5
    Xi = integer_tokens(rng, T, d, n_base=3)
    near, margin = exact_near(Xi.tolist(), *thr_q)
    if margin < 1e-9:
        pytest.skip("a pair sits on the threshold; float64 cannot be required to decide it")
    res = oracle.select_full(Xi.astype(np.float64), tau_q[0] / tau_q[1], greedy=True)
    assert res["idx"].tolist() == exact_greedy(near, T)


def test_greedy_covering_is_a_maximal_separated_set_and_contains_the_definitions_set():
    """Section 2.5's two properties, which hold for the greedy reading: representatives are pairwise below the
    threshold (separated), every other token is within the threshold of an earlier representative (covering).
    And every token the Definition keeps is kept by the greedy reading too (it compares with fewer tokens)."""
    rng = np.random.default_rng(5)
    differ = 0
    for trial in range(8):
        ang = np.sort(rng.uniform(0, np.pi, size=40))            # points on a half circle: many chains
        X = np.stack([np.cos(ang), np.sin(ang)], axis=1)[rng.permutation(40)]
        tau = 0.3
        thr = 1 - tau * tau
        G = np.abs(numpy_gram(X))
        g = oracle.select_full(X, tau, greedy=True)
        R = g["idx"].tolist()
        for i, a in enumerate(R):
            for b in R[:i]:
                assert G[a, b] < thr
        for t in range(40):
            if t not in R:
                assert any(G[t, s] >= thr for s in R if s < t)
        dfn = oracle.select_full(X, tau)["idx"].tolist()
        assert set(dfn) <= set(R)
        differ += set(dfn) != set(R)
    assert differ > 0                                             # the inputs do contain chains


def test_clustered_tokens_first_occurrence_of_each_centre_is_selected():
    w = wl.small(T=300, d=64, K=40, L=1, dtype="f32", seed=11)
    rng = np.random.default_rng(w.seed(0))
    # replay the generator's first two draws to learn the assignment (the module draws C then a)
    _ = rng.standard_normal((w.K, w.d), dtype=np.float32)
    a = rng.integers(0, w.K, size=w.T)
    X = wl.as_f64(wl.layer_list(w)[0])
    res = oracle.select_full(X, w.tau)
    first = sorted({int(c): t for t, c in reversed(list(enumerate(a)))}.values())
    assert res["idx"].tolist() == first
    assert res["r"] == len(set(a.tolist()))


def test_gamma_full_rows_matches_whole_selection():
    rng = np.random.default_rng(8)
    X = rng.standard_normal((50, 12))
    rows = [0, 1, 7, 49, 20]
    assert np.array_equal(oracle.gamma_full_rows(X, rows), oracle.select_full(X, 0.2)["gamma"][rows])


def test_force_overrides_only_the_named_tokens():
    rng = np.random.default_rng(9)
    X = rng.standard_normal((12, 5))
    free = oracle.select_full(X, 0.3)
    force = -np.ones(12, dtype=np.int8)
    force[3] = 1 - free["mask"][3]
    forced = oracle.select_full(X, 0.3, force=force)
    diff = np.flatnonzero(forced["mask"] != free["mask"])
    assert diff.tolist() == [3]
    assert np.array_equal(forced["gamma"], free["gamma"])


def test_argument_errors():
    X = np.ones((4, 3))
    for tau in (0.0, 1.0, -0.1, 1.5, float("nan")):
        with pytest.raises(ValueError):
            oracle.select_full(X, tau)
        with pytest.raises(ValueError):
            oracle.cascade_step(X, tau, [0])
    for prev in ([], [1, 1], [2, 1], [0, 4], [-1, 2], [0, 1, 2, 3, 3]):
        with pytest.raises(ValueError):
            oracle.cascade_step(X, 0.1, prev)


# ----------------------------------------------------------------------------- Algorithm 1
@pytest.mark.parametrize("earlier_only", [False, True])
@pytest.mark.parametrize("seed", range(3))
def test_cascade_agrees_with_exact_brute_force_for_every_inherited_subset(seed, earlier_only):
    rng = np.random.default_rng(200 + seed)
    T, d = 10, 5
    Xi = integer_tokens(rng, T, d, n_base=3)
    (tn, td), thr_q = RATIONAL_TAUS[seed % 2]
    near, margin = exact_near(Xi.tolist(), *thr_q)
    if margin < 1e-9:
        pytest.skip("a pair sits on the threshold")
    X = Xi.astype(np.float64)
    flags = oracle.CROSS_EARLIER_ONLY if earlier_only else 0
    n_changed = 0
    for bits in range(1, 2 ** T):
        R = [t for t in range(T) if bits >> t & 1]
        idx, new, removes, ops = exact_cascade(near, T, R, earlier_only)
        res = oracle.cascade_step(X, tn / td, R, flags=flags)
        assert res["idx"].tolist() == idx, R
        assert res["adds"].tolist() == new, R
        assert res["removes"].tolist() == removes, R
        assert res["gram_ops"] == ops, R
        n_changed += bool(new or removes)
    assert n_changed > 100            # the sweep is not vacuous


def test_cascade_sampled_subsets_T16():
    rng = np.random.default_rng(300)
    T, d = 16, 6
    Xi = integer_tokens(rng, T, d, n_base=4)
    near, margin = exact_near(Xi.tolist(), 91, 100)
    assert margin >= 1e-9
    for _ in range(400):
        R = sorted(rng.choice(T, size=int(rng.integers(1, T + 1)), replace=False).tolist())
        for eo in (False, True):
            idx, new, removes, ops = exact_cascade(near, T, R, eo)
            res = oracle.cascade_step(Xi.astype(np.float64), 0.3, R, flags=int(eo))
            assert (res["idx"].tolist(), res["adds"].tolist(), res["removes"].tolist(), res["gram_ops"]) == \
                   (idx, new, removes, ops)


def test_cascade_gamma_is_rep_max_for_inherited_and_cross_max_for_the_rest():
    rng = np.random.default_rng(12)
    T = 40
    X = rng.standard_normal((T, 9))
    X[25:] = X[:15] * 2.0 + 0.02 * rng.standard_normal((15, 9))
    R = sorted(rng.choice(T, size=14, replace=False).tolist())
    tau = 0.3
    res = oracle.cascade_step(X, tau, R)
    A = np.abs(numpy_gram(X))
    thr = 1 - tau * tau
    g_rep = {s: max([A[sp, s] for sp in R if sp < s], default=0.0) for s in R}
    valid = [s for s in R if g_rep[s] < thr]
    assert len(valid) < len(R)                       # some inherited token is removed, so the two maxima differ
    for t in range(T):
        want = g_rep[t] if t in R else max([A[t, s] for s in valid], default=0.0)
        assert abs(res["gamma"][t] - want) < 1e-13
        want_all = g_rep[t] if t in R else max(A[t, s] for s in R)
        assert abs(res["gamma_all"][t] - want_all) < 1e-13
    assert np.any(res["gamma_all"] > res["gamma"] + 1e-6)


def test_cascade_invariants_on_clustered_layers():
    w = wl.small(T=400, d=96, K=50, L=6, dtype="f32", seed=21, p=0.08)
    Xs = [wl.as_f64(x) for x in wl.layer_list(w)]
    R = oracle.select_full(Xs[0], w.tau)["idx"]
    total_changes = 0
    for X in Xs[1:]:
        for flags in (0, oracle.CROSS_EARLIER_ONLY):
            res = oracle.cascade_step(X, w.tau, R, flags=flags)
            full = oracle.select_full(X, w.tau)
            assert res["idx"][0] == R[0] == 0 or R[0] in res["idx"]           # smallest inherited index survives
            assert res["r_new"] == len(R) - len(res["removes"]) + len(res["adds"])
            assert set(res["removes"]) <= set(R.tolist())
            assert not (set(res["adds"]) & set(R.tolist()))
            assert np.all(np.diff(res["idx"]) > 0)
            r_valid = len(R) - len(res["removes"])
            assert res["gram_ops"] == len(R) ** 2 + (w.T - len(R)) * r_valid
            missing = set(full["idx"].tolist()) - set(res["idx"].tolist())
            if flags:   # strict superset (superset proposition, with the comparison set restricted to earlier tokens)
                assert not missing
            else:       # as printed: a missing independent representative duplicates a LATER cascade representative
                A = np.abs(numpy_gram(X))
                for t in missing:
                    later = [s for s in res["idx"] if s > t and A[t, s] >= 1 - w.tau ** 2]
                    assert later
        res = oracle.cascade_step(X, w.tau, R)
        total_changes += len(res["adds"]) + len(res["removes"])
        R = res["idx"]
    assert total_changes > 0


def test_cascade_from_the_same_layers_full_selection_changes_nothing_on_cliques():
    w = wl.small(T=256, d=48, K=30, L=1, dtype="f32", seed=31)
    X = wl.as_f64(wl.layer_list(w)[0])
    full = oracle.select_full(X, w.tau)
    res = oracle.cascade_step(X, w.tau, full["idx"])
    assert res["idx"].tolist() == full["idx"].tolist()
    assert len(res["adds"]) == 0 and len(res["removes"]) == 0
    assert res["gram_ops"] == w.T * full["r"]                 # eq. (6): r^2 + (T-r) r = T r when nothing is removed


def test_cascade_on_a_chain_adds_exactly_the_uncovered_tail():
    ang = np.deg2rad([0.0, 20.0, 40.0])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    full = oracle.select_full(X, 0.3)
    assert full["idx"].tolist() == [0]
    res = oracle.cascade_step(X, 0.3, full["idx"])
    assert res["adds"].tolist() == [2] and res["removes"].tolist() == [] and res["idx"].tolist() == [0, 2]


def test_cascade_removed_representative_still_counts_against_later_ones_and_is_not_readded():
    # inherited {0,1,2}: 1 duplicates 0, 2 duplicates 1 only through the chain 0~1~2 with 0 !~ 2.
    ang = np.deg2rad([0.0, 20.0, 40.0, 90.0])
    X = np.stack([np.cos(ang), np.sin(ang)], axis=1)
    res = oracle.cascade_step(X, 0.3, [0, 1, 2])
    assert res["removes"].tolist() == [1, 2]          # step 4 maxes over all inherited, also the removed token 1
    assert res["adds"].tolist() == [3]                # token 3 is orthogonal to token 0
    assert res["idx"].tolist() == [0, 3]              # token 2 is uncovered but was inherited: not reconsidered
    assert res["gram_ops"] == 9 + 1 * 1


def test_cascade_unordered_and_earlier_only_cross_step_differ_on_a_later_duplicate():
    # token 0 unrelated, token 1 = non-inherited duplicate of the LATER inherited token 2
    X = np.array([[1.0, 0, 0], [0, 1.0, 0], [0, 1.0, 1e-6]])
    a = oracle.cascade_step(X, 0.1, [0, 2])
    b = oracle.cascade_step(X, 0.1, [0, 2], flags=oracle.CROSS_EARLIER_ONLY)
    assert a["idx"].tolist() == [0, 2] and a["adds"].tolist() == []
    assert b["idx"].tolist() == [0, 1, 2] and b["adds"].tolist() == [1]


def test_cascade_extreme_set_sizes():
    rng = np.random.default_rng(13)
    X = rng.standard_normal((20, 30))
    X[10:] = X[:10]
    one = oracle.cascade_step(X, 0.1, [0])                      # r = 1: only the copy of token 0 is covered
    assert one["idx"].tolist() == [t for t in range(20) if t != 10] and one["removes"].tolist() == []
    assert one["gram_ops"] == 1 + 19
    every = oracle.cascade_step(X, 0.1, list(range(20)))        # r = T: the cross step is empty
    assert every["idx"].tolist() == list(range(10)) and every["removes"].tolist() == list(range(10, 20))
    assert every["gram_ops"] == 400


# ----------------------------------------------------------------------------- Section 2.3: nearest representative
def exact_argmax_sets(X_int, R):
    """For every token the set of members of R that maximise cos^2 = (x_t . x_s)^2 / (|x_t|^2 |x_s|^2), compared as
    exact fractions by cross-multiplication of Python ints (no floating point), and the smallest relative gap between
    the best and the runner-up so callers can reject inputs float64 could not rank."""
    T = len(X_int)
    sq = [sum(int(a) * int(a) for a in row) for row in X_int]
    out, gap = [], math.inf
    for t in range(T):
        cand = []
        for s in R:
            dot = sum(int(a) * int(b) for a, b in zip(X_int[t], X_int[s]))
            cand.append((dot * dot, sq[s], s))              # cos^2 up to the common factor 1 / |x_t|^2
        best = cand[0]
        for c in cand[1:]:
            if c[0] * best[1] > best[0] * c[1]:
                best = c
        winners = [c[2] for c in cand if c[0] * best[1] == best[0] * c[1]]
        for c in cand:
            if c[2] not in winners and best[0] > 0:
                gap = min(gap, (best[0] * c[1] - c[0] * best[1]) / (best[0] * c[1]))
        out.append(winners)
    return out, gap


@pytest.mark.parametrize("seed", range(6))
def test_assignment_agrees_with_exact_integer_argmax(seed):
    rng = np.random.default_rng(400 + seed)
    T, d = 18, 5
    Xi = integer_tokens(rng, T, d, n_base=4)
    R = sorted(rng.choice(T, size=int(rng.integers(1, 8)), replace=False).tolist())
    winners, gap = exact_argmax_sets(Xi.tolist(), R)
    if gap < 1e-9:
        pytest.skip("a runner-up too close to the maximum for float64 to rank")
    res = oracle.assign_nearest(Xi.astype(np.float64), R)
    for t in range(T):
        if t in R:
            assert res["assign"][t] == t and res["corr"][t] == 1.0
        else:
            assert res["assign"][t] == min(winners[t])       # smallest token id among exact ties (e.g. +x and -x)
            s = int(res["assign"][t])
            dot = sum(int(a) * int(b) for a, b in zip(Xi[t], Xi[s]))
            cos = abs(dot) / math.sqrt(sum(int(a) ** 2 for a in Xi[t]) * sum(int(b) ** 2 for b in Xi[s]))
            assert res["corr"][t] == pytest.approx(cos, abs=1e-12)


def test_assignment_matches_numpy_argmax_of_abs_gram():
    rng = np.random.default_rng(77)
    X = rng.standard_normal((120, 24))
    R = sorted(rng.choice(120, size=17, replace=False).tolist())
    G = np.abs(numpy_gram(X))[:, R]                          # independent float64 matmul
    res = oracle.assign_nearest(X, R)
    others = [t for t in range(120) if t not in R]
    assert res["assign"][others].tolist() == [R[j] for j in G[others].argmax(axis=1)]
    assert np.allclose(res["corr"][others], G[others].max(axis=1), atol=1e-13)
    assert res["assign"][R].tolist() == R


def test_assignment_sign_and_later_representatives_count():
    # token 1 = -token 3 (|G| = 1 with a LATER member of R), token 2 nearer to 0 than to 3
    X = np.array([[1.0, 0, 0], [0, -2.0, 0], [0.9, 0.1, 0], [0, 1.0, 0], [0, 0, 1.0]])
    res = oracle.assign_nearest(X, [0, 3])
    assert res["assign"].tolist() == [0, 3, 0, 3, 0]          # token 4 is orthogonal to both: smallest id among ties
    assert res["corr"][1] == pytest.approx(1.0) and res["corr"][4] == 0.0


def test_assignment_on_clustered_tokens_is_the_own_clusters_representative():
    w = wl.small(T=300, d=64, K=40, L=1, dtype="f32", seed=11)
    rng = np.random.default_rng(w.seed(0))
    _ = rng.standard_normal((w.K, w.d), dtype=np.float32)    # replay the generator: centres, then the assignment
    a = rng.integers(0, w.K, size=w.T)
    X = wl.as_f64(wl.layer_list(w)[0])
    full = oracle.select_full(X, w.tau)
    res = oracle.assign_nearest(X, full["idx"])
    first = {}
    for t, c in enumerate(a):
        first.setdefault(int(c), t)
    assert res["assign"].tolist() == [first[int(c)] for c in a]
    redundant = full["mask"] == 0
    assert (res["corr"][redundant] >= 1.0 - w.tau ** 2).all()  # a covered token is within the threshold of its own


def test_assignment_rejects_bad_sets():
    X = np.eye(4)
    for bad in ([], [2, 1], [1, 1], [0, 4], [-1]):
        with pytest.raises(ValueError):
            oracle.assign_nearest(X, bad)


# ----------------------------------------------------------------------------- eq. (1): attention on the representatives
def numpy_attention(Q, K, V, H, R, assign, causal=False):
    """Independent statement of eq. (1) with numpy / scipy routines (float64 matmul, scipy's softmax)."""
    from scipy.special import softmax
    T, D = Q.shape
    dh = D // H
    R = np.asarray(R)
    O = np.empty((len(R), D))
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        S = Q[R][:, c] @ K[R][:, c].T / math.sqrt(dh)
        if causal:
            S = np.where(np.arange(len(R))[None, :] <= np.arange(len(R))[:, None], S, -np.inf)
        O[:, c] = softmax(S, axis=1) @ V[R][:, c]
    return O[np.searchsorted(R, assign)]


@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_numpy_and_scipy_softmax(causal):
    rng = np.random.default_rng(31)
    T, H, dh = 90, 3, 8
    Q, K, V = (rng.standard_normal((T, H * dh)) for _ in range(3))
    X = rng.standard_normal((T, 16))
    R = sorted(rng.choice(T, size=23, replace=False).tolist())
    assign = oracle.assign_nearest(X, R)["assign"]
    out = oracle.attention_compressed(Q, K, V, H, R, assign, flags=oracle.ATTN_CAUSAL if causal else 0)
    assert np.allclose(out, numpy_attention(Q, K, V, H, R, assign, causal), rtol=0, atol=1e-12)
    for t in range(T):                                       # a token carries its representative's row, unchanged
        assert np.array_equal(out[t], out[assign[t]])


def test_attention_closed_forms():
    rng = np.random.default_rng(32)
    T, H, dh = 40, 2, 6
    Q, V = rng.standard_normal((T, H * dh)), rng.standard_normal((T, H * dh))
    R = [1, 5, 6, 20, 33]
    assign = np.array([R[t % len(R)] for t in range(T)], dtype=np.int32)
    assign[R] = R
    # identical keys: every score in a row is equal -> uniform weights -> the mean of the value rows
    K = np.tile(rng.standard_normal((1, H * dh)), (T, 1))
    out = oracle.attention_compressed(Q, K, V, H, R, assign)
    assert np.allclose(out[R], np.tile(V[R].mean(axis=0), (len(R), 1)), atol=1e-12)
    # adding one vector to every key shifts each row of scores by a constant: softmax does not move
    K2 = rng.standard_normal((T, H * dh))
    a = oracle.attention_compressed(Q, K2, V, H, R, assign)
    b = oracle.attention_compressed(Q, K2 + rng.standard_normal((1, H * dh)), V, H, R, assign)
    assert np.allclose(a, b, atol=1e-10)
    # one key dominating: the output approaches that key's value row; scores are divided by sqrt(d_h)
    K3 = np.zeros((T, H * dh)); Q3 = np.zeros((T, H * dh))
    Q3[:, 0] = 1.0; Q3[:, dh] = 1.0
    K3[R[2], 0] = 80.0 * math.sqrt(dh); K3[R[2], dh] = 80.0 * math.sqrt(dh)
    out3 = oracle.attention_compressed(Q3, K3, V, H, R, assign)
    assert np.allclose(out3[R], np.tile(V[R[2]], (len(R), 1)), atol=1e-9)
    K3[R[2], 0] = math.log(3.0) * math.sqrt(dh); K3[R[2], dh] = 0.0   # head 0: weights 3 : 1 : 1 : 1 : 1
    out4 = oracle.attention_compressed(Q3, K3, V, H, R, assign)
    w = np.ones(len(R)); w[2] = 3.0
    assert np.allclose(out4[R[0], :dh], (w / w.sum()) @ V[R][:, :dh], atol=1e-12)
    assert np.allclose(out4[R[0], dh:], V[R][:, dh:].mean(axis=0), atol=1e-12)
    # a single representative: everybody gets its value row; causal: the first representative sees only itself
    one = oracle.attention_compressed(Q, K2, V, H, [7], np.full(T, 7, dtype=np.int32))
    assert np.array_equal(one, np.tile(V[7], (T, 1)))
    c = oracle.attention_compressed(Q, K2, V, H, R, assign, flags=oracle.ATTN_CAUSAL)
    assert np.allclose(c[R[0]], V[R[0]], atol=1e-15)
    assert (out.min(axis=0) >= V[R].min(axis=0) - 1e-12).all() and (out.max(axis=0) <= V[R].max(axis=0) + 1e-12).all()


def test_attention_rejects_bad_input():
    Q = np.zeros((6, 4))
    good = np.array([0, 0, 2, 2, 2, 0], dtype=np.int32)
    oracle.attention_compressed(Q, Q, Q, 2, [0, 2], good)
    for R, a in (([2, 0], good), ([0, 2], np.array([0, 1, 2, 2, 2, 0], dtype=np.int32)), ([0, 9], good)):
        with pytest.raises(ValueError):
            oracle.attention_compressed(Q, Q, Q, 2, R, a)
    with pytest.raises(ValueError):
        oracle.attention_compressed(Q, Q, Q, 3, [0, 2], good)       # 4 columns do not split into 3 heads


# ----------------------------------------------------------------------------- Section 8.1 (adaptive threshold)
def test_adapt_tau_closed_forms():
    m = oracle.metrics
    assert m.adapt_tau(0.2, 0.25, 0.0, 0.1, 0.05, 0.5) == 0.2                    # no gain: fixed
    assert m.adapt_tau(0.2, 0.1, 0.5, 0.1, 0.05, 0.5) == 0.2                     # on target: fixed
    assert m.adapt_tau(0.25, 0.0, 0.5, 0.5, 0.05, 0.9) == 0.5                    # stable set: tighter (tau up by 0.25)
    assert m.adapt_tau(0.5, 1.0, 0.25, 0.0, 0.05, 0.9) == 0.25                   # evolving set: looser (tau down)
    assert m.adapt_tau(0.25, 0.0, 4.0, 0.5, 0.05, 0.75) == 0.75                  # clipped above
    assert m.adapt_tau(0.25, 2.0, 4.0, 0.5, 0.125, 0.75) == 0.125                # clipped below
    # low turnover gives the larger tau, i.e. the lower threshold 1 - tau^2: fewer representatives
    lo, hi = m.adapt_tau(0.2, 0.0, 0.3, 0.2, 0.01, 0.9), m.adapt_tau(0.2, 0.6, 0.3, 0.2, 0.01, 0.9)
    assert lo > 0.2 > hi and 1 - lo * lo < 1 - hi * hi


def test_adaptive_layer_loop_with_zero_gain_is_the_fixed_loop_and_follows_the_turnover_otherwise():
    w = wl.small(T=300, d=64, K=40, L=6, dtype="f32", seed=19, p=0.15)
    Xs = [wl.as_f64(x) for x in wl.layer_list(w)]
    taus, res = oracle.cascade_layers_adaptive(Xs, w.tau, 0.0, 0.1, 0.01, 0.9)
    t32 = float(np.float32(w.tau))
    assert taus == [t32] * w.L
    prev = oracle.select_full(Xs[0], t32)["idx"]
    assert res[0]["idx"].tolist() == prev.tolist()
    for l in range(1, w.L):
        step = oracle.cascade_step(Xs[l], t32, prev)
        assert res[l]["idx"].tolist() == step["idx"].tolist()
        prev = step["idx"]
    # with a gain: layers 0 and 1 use tau0, every later tau is the rule applied to the previous step's own counts
    taus, res = oracle.cascade_layers_adaptive(Xs, w.tau, 0.05, 0.8, 0.02, 0.6)
    assert taus[0] == taus[1] == t32
    prev_r = len(res[0]["idx"])
    for l in range(1, w.L - 1):
        eta = (len(res[l]["adds"]) + len(res[l]["removes"])) / prev_r
        assert taus[l + 1] == min(max(taus[l] + 0.05 * (0.8 - eta), 0.02), 0.6)
        prev_r = len(res[l]["idx"])
    assert len(set(taus)) > 2                                                    # the threshold really moved
    # identical layers: no turnover at all, so tau climbs by kappa * eta_target per layer until it is clipped
    taus, res = oracle.cascade_layers_adaptive([Xs[0]] * 5, 0.25, 0.5, 0.25, 0.05, 0.5)
    assert taus == [0.25, 0.25, 0.375, 0.5, 0.5]
    assert all(len(r["removes"]) == 0 for r in res[1:3])
