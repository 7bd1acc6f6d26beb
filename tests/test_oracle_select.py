"""Pins for the oracle's selection step (token choice, expert choice, slots): CPU only."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from conftest import load_golden

TCR, ECR, BIDIR = 0, 1, 2


def kept_sets(slot_token, counts):
    return [list(slot_token[e, :counts[e]]) for e in range(slot_token.shape[0])]


def check_permutation_tables(T, E, C, slot_of, slot_token, counts):
    assert slot_of.shape == (T, E) and slot_token.shape == (E, C) and counts.shape == (E,)
    assert int((slot_of >= 0).sum()) == int(counts.sum())
    for e in range(E):
        n = counts[e]
        assert 0 <= n <= C
        row = slot_token[e]
        assert np.all(row[n:] == -1)
        assert np.all(np.diff(row[:n]) > 0)                      # ascending token order, no duplicates
        assert np.all(slot_of[row[:n], e] == np.arange(n))
        col = slot_of[:, e]
        assert int((col >= 0).sum()) == n


def test_worked_example(oracle):
    g = load_golden("select_worked_example.json")
    S = np.array(g["score"], np.float32)
    C = g["capacity"]
    for kname, k in (("k1", 1), ("k2", 2)):
        for mname, mode in (("tcr", TCR), ("bidir", BIDIR)):
            topk, slot_of, slot_token, counts = oracle.select(S, k, C, mode)
            assert topk.tolist() == g[kname]["topk"]
            assert [list(map(int, s)) for s in kept_sets(slot_token, counts)] == g[kname][mname]["kept"]
            check_permutation_tables(6, 3, C, slot_of, slot_token, counts)
    for k in (1, 2, 3):
        _, slot_of, slot_token, counts = oracle.select(S, k, C, ECR)
        assert [list(map(int, s)) for s in kept_sets(slot_token, counts)] == g["ecr"]["kept"]


def _scores(rng, T, E, levels=None):
    if levels:                                                   # many exact ties
        return (rng.integers(-levels, levels + 1, size=(T, E)) / levels).astype(np.float32)
    return rng.uniform(-1, 1, size=(T, E)).astype(np.float32)


def _best_subset(cands, n, key):
    """Brute force: the size-n subset with the largest exact score sum; among
    equal sums the lexicographically smallest index tuple."""
    best, best_sum = None, None
    for sub in itertools.combinations(cands, n):                 # generated in lexicographic order
        s = sum((Fraction(float(key(i))) for i in sub), Fraction(0))
        if best is None or s > best_sum:
            best, best_sum = sub, s
    return list(best) if best is not None else []


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("levels", [None, 3])
def test_brute_force_small(oracle, seed, levels):
    rng = np.random.default_rng(100 + seed)
    T, E = int(rng.integers(5, 13)), int(rng.integers(2, 5))
    k = int(rng.integers(1, E + 1))
    C = int(rng.integers(1, T + 2))
    S = _scores(rng, T, E, levels)
    # token choice by enumeration
    choice = []
    for t in range(T):
        sub = _best_subset(range(E), k, lambda e: S[t, e])
        choice.append(sorted(sub, key=lambda e: (-S[t, e], e)))
    for mode in (TCR, BIDIR, ECR):
        topk, slot_of, slot_token, counts = oracle.select(S, k, C, mode)
        check_permutation_tables(T, E, C, slot_of, slot_token, counts)
        if mode != ECR:
            assert topk.tolist() == choice
        for e in range(E):
            cands = list(range(T)) if mode == ECR else [t for t in range(T) if e in choice[t]]
            n = min(C, len(cands))
            if mode == TCR:
                expect = cands[:n]
            else:
                expect = sorted(_best_subset(cands, n, lambda t: S[t, e]))
            assert list(slot_token[e, :counts[e]]) == expect, (mode, e)


@pytest.mark.parametrize("levels", [None, 5])
def test_invariants_medium(oracle, levels):
    rng = np.random.default_rng(7)
    T, E, k, C = 700, 9, 3, 150
    S = _scores(rng, T, E, levels)
    order = np.lexsort((np.arange(E)[None, :].repeat(T, 0), -S.astype(np.float64)), axis=1)   # score desc, idx asc
    chose = np.zeros((T, E), bool)
    np.put_along_axis(chose, order[:, :k], True, axis=1)
    res = {m: oracle.select(S, k, C, m) for m in (TCR, ECR, BIDIR)}
    for m, (topk, slot_of, slot_token, counts) in res.items():
        check_permutation_tables(T, E, C, slot_of, slot_token, counts)
        kept = slot_of >= 0
        if m != ECR:
            np.testing.assert_array_equal(topk, order[:, :k])
            assert np.all(kept <= chose)                          # kept only where chosen
            assert np.all(kept.sum(1) <= k)
            np.testing.assert_array_equal(counts, np.minimum(C, chose.sum(0)))
        else:
            assert np.all(counts == min(C, T))
        if m == TCR:
            for e in range(E):
                np.testing.assert_array_equal(slot_token[e, :counts[e]], np.flatnonzero(chose[:, e])[:C])
        else:
            # exchange property: no unkept candidate ranks before a kept one
            for e in range(E):
                cand = np.ones(T, bool) if m == ECR else chose[:, e]
                kk = np.flatnonzero(kept[:, e])
                uu = np.flatnonzero(cand & ~kept[:, e])
                if len(kk) and len(uu):
                    worst_kept = max(kk, key=lambda t: (-S[t, e], t))
                    best_unkept = min(uu, key=lambda t: (-S[t, e], t))
                    assert (-S[worst_kept, e], worst_kept) < (-S[best_unkept, e], best_unkept)
    # BIDIR subset of TCR candidates, ECR/BIDIR equal when every token lists every expert
    _, so_b, st_b, c_b = oracle.select(S, E, C, BIDIR)
    _, so_e, st_e, c_e = oracle.select(S, E, C, ECR)
    np.testing.assert_array_equal(so_b, so_e)
    np.testing.assert_array_equal(st_b, st_e)
    # capacity >= T: nothing is dropped, TCR == BIDIR == all choosers
    _, so_t, _, c_t = oracle.select(S, k, T + 3, TCR)
    _, so_b, _, c_b = oracle.select(S, k, T + 3, BIDIR)
    np.testing.assert_array_equal(so_t, so_b)
    np.testing.assert_array_equal(so_t >= 0, chose)
    np.testing.assert_array_equal(c_t, chose.sum(0))


def test_negative_zero_ties_by_index(oracle):
    S = np.array([[0.0, -0.0], [-0.0, 0.0], [0.0, 0.0]], np.float32)
    topk, _, slot_token, counts = oracle.select(S, 1, 2, TCR)
    assert topk[:, 0].tolist() == [0, 0, 0]
    _, _, st, c = oracle.select(S, 1, 2, ECR)
    assert st.tolist() == [[0, 1], [0, 1]]


def test_tcr_keep_rate_is_binomial(oracle):
    """Proof of the Theorem, part 1: under isotropic tokens and top-1 choice the
    number of earlier tokens on the same expert is Binomial(k-1, 1/n), so the
    token at (1-based) position k is kept with probability P(Bin(k-1,1/n) < C)."""
    rng = np.random.default_rng(11)
    T, n, C, trials = 48, 4, 6, 3000
    kept = np.zeros(T)
    for _ in range(trials):
        S = rng.uniform(-1, 1, size=(T, n)).astype(np.float32)
        _, slot_of, _, _ = oracle.select(S, 1, C, TCR)
        kept += (slot_of >= 0).any(1)
    rate = kept / trials
    for pos in (1, 6, 7, 16, 24, 32, 48):
        p = stats.binom.cdf(C - 1, pos - 1, 1.0 / n)
        sigma = max(np.sqrt(p * (1 - p) / trials), 1e-9)
        assert abs(rate[pos - 1] - p) <= 4.5 * sigma + 1e-12, (pos, rate[pos - 1], p)


def test_ecr_success_is_binomial_tail(oracle):
    """Proof of the Theorem, part 2: expert i keeps a given token iff at most
    C-1 other tokens score higher; with i.i.d. continuous scores the number of
    higher-scoring tokens is uniform on {0..s-1}, so P(kept) = C/s."""
    rng = np.random.default_rng(12)
    T, n, C, trials = 40, 3, 7, 3000
    hit = 0
    for _ in range(trials):
        S = rng.uniform(-1, 1, size=(T, n)).astype(np.float32)
        _, slot_of, _, _ = oracle.select(S, 1, C, ECR)
        hit += slot_of[17, 1] >= 0
        higher = int((S[:, 1] > S[17, 1]).sum())
        assert (slot_of[17, 1] >= 0) == (higher <= C - 1)
    p = C / T
    assert abs(hit / trials - p) < 4.5 * np.sqrt(p * (1 - p) / trials)


def test_rejects_bad_arguments(oracle):
    S = np.zeros((4, 3), np.float32)
    with pytest.raises(RuntimeError):
        oracle.select(S, 4, 2, TCR)          # k > E
    with pytest.raises(RuntimeError):
        oracle.select(S, 1, 0, TCR)          # capacity < 1
    # ECR ignores k
    oracle.select(S, 7, 2, ECR)


# ---------------------------------------------------------------------------------------
# adaptive token count: "l is determined by a threshold of the sum of affinity scores"
# ---------------------------------------------------------------------------------------
def _fixed(s):
    """round(clamp(s, -1, 1) * 2^30), ties to even: sums of these integers are order-independent."""
    return int(np.rint(np.float64(min(1.0, max(-1.0, float(s)))) * 2.0 ** 30))


def _adaptive_brute(S, e, cands, C, thr):
    """Independent statement: sort by (score desc, index asc); l = first prefix whose fixed-point
    affinity sum reaches the threshold, all candidates if the positive affinities never do."""
    order = sorted(cands, key=lambda t: (-float(S[t, e]), t))
    need = int(np.rint(np.float64(np.float32(thr)) * 2.0 ** 30))
    run, ell = 0, len(order)
    for m, t in enumerate(order):
        if not S[t, e] > 0:
            break
        run += _fixed(S[t, e])
        if run >= need:
            ell = m + 1
            break
    return sorted(order[:min(C, ell)])


def test_adaptive_worked_example(oracle):
    g = load_golden("select_worked_example.json")
    S = np.array(g["score"], np.float32)
    # ECR, capacity 6 (never binding), threshold 1.6:
    #   expert 0: .9 + .8 = 1.7 >= 1.6 -> 2 tokens; expert 1: .7 + .6 + .5 = 1.8 -> 3 tokens (ties .5/.5: token 3 first)
    #   expert 2: .5 + .4 + .3 + .2 + .1 = 1.5 never reaches 1.6 -> all 6
    _, _, st, c = oracle.select_adaptive(S, 1, 6, ECR, 1.6)
    assert c.tolist() == [2, 3, 6]
    assert st[0, :2].tolist() == [0, 1] and st[1, :3].tolist() == [1, 2, 3]
    # the capacity still binds: with C = 2 expert 1 and 2 keep two
    _, _, st, c = oracle.select_adaptive(S, 1, 2, ECR, 1.6)
    assert c.tolist() == [2, 2, 2]
    # threshold off or unreachable: the plain selection; tiny threshold: one token each
    for thr in (0.0, -1.0):
        np.testing.assert_array_equal(oracle.select_adaptive(S, 2, 2, BIDIR, thr)[1], oracle.select(S, 2, 2, BIDIR)[1])
    assert oracle.select_adaptive(S, 1, 6, ECR, 0.05)[3].tolist() == [1, 1, 1]
    # token choice keeps by position: the threshold does not apply
    np.testing.assert_array_equal(oracle.select_adaptive(S, 2, 2, TCR, 0.3)[1], oracle.select(S, 2, 2, TCR)[1])


def test_adaptive_threshold_reached_exactly(oracle):
    """"Reaches the threshold" is >=, pinned with dyadic affinities whose sums are exact in every arithmetic:
    expert 0 sees 0.5, 0.25, 0.125, 0.0625 (descending): the prefix sums are 0.5, 0.75, 0.875, 0.9375."""
    S = np.array([[0.5], [0.25], [0.125], [0.0625], [-0.5]], np.float32)
    step = 2.0 ** -20                                   # far above the 2^-30 quantum, exact in fp32 next to 0.75
    for thr, want in ((0.75, 2),                        # 0.5 + 0.25 == 0.75: the second token completes the prefix
                      (0.75 - step, 2),                 # just below: still two (0.5 alone is not enough)
                      (0.75 + step, 3),                 # just above: the third token is needed
                      (0.5, 1), (0.5 + step, 2), (0.9375, 4),
                      (0.9375 + step, 5)):              # the positive affinities never get there: all five candidates
        counts = oracle.select_adaptive(S, 1, 5, ECR, np.float32(thr))[3]
        assert counts.tolist() == [want], (thr, counts)
    # same sums with the order of the tokens reversed: the cut is a property of the sorted candidates
    counts = oracle.select_adaptive(S[::-1].copy(), 1, 5, ECR, np.float32(0.75))[3]
    assert counts.tolist() == [2]
    # the kept tokens are the highest ones, and ties (two tokens at 0.25) go to the lower index
    S2 = np.array([[0.25], [0.5], [0.25], [0.125]], np.float32)
    _, _, st, c = oracle.select_adaptive(S2, 1, 4, ECR, np.float32(0.75))
    assert c.tolist() == [2] and sorted(st[0, :2].tolist()) == [0, 1]


@pytest.mark.parametrize("seed", range(6))
def test_adaptive_fixed_point_cut_is_the_double_precision_cut(oracle, seed):
    """The oracle sums round(s * 2^30) in integers so that a parallel sum gives the same cut.  What the paper's
    sentence describes is the running sum of the affinities themselves: computed here in float64 over the sorted
    candidates, it must give the same token count, except when it passes within T * 2^-30 of the threshold
    (the most the T roundings can move the sum)."""
    rng = np.random.default_rng(900 + seed)
    T, E = 400, 3
    S = rng.uniform(-1, 1, size=(T, E)).astype(np.float32)
    C = T
    checked = 0
    for thr in rng.uniform(0.5, 60.0, size=12).astype(np.float32):
        counts = oracle.select_adaptive(S, 1, C, ECR, thr)[3]
        for e in range(E):
            col = np.sort(S[:, e].astype(np.float64))[::-1]
            run = np.cumsum(np.where(col > 0, col, 0.0))
            hit = np.flatnonzero((run >= np.float64(thr)) & (col > 0))
            ell = int(hit[0]) + 1 if hit.size else T
            near = np.min(np.abs(run[: int((col > 0).sum())] - np.float64(thr))) <= T * 2.0 ** -30
            if not near:
                assert counts[e] == min(C, ell), (thr, e, counts[e], ell)
                checked += 1
    assert checked >= 30                                # the exception is rare: nearly every case is compared


@pytest.mark.parametrize("seed", range(8))
def test_adaptive_brute_force(oracle, seed):
    rng = np.random.default_rng(300 + seed)
    T, E = int(rng.integers(5, 40)), int(rng.integers(2, 6))
    k = int(rng.integers(1, E + 1))
    C = int(rng.integers(1, T + 2))
    S = _scores(rng, T, E, 4 if seed % 2 else None)
    thr = float(rng.uniform(0.2, 3.0))
    order = np.lexsort((np.arange(E)[None, :].repeat(T, 0), -S.astype(np.float64)), axis=1)
    chose = np.zeros((T, E), bool)
    np.put_along_axis(chose, order[:, :k], True, axis=1)
    for mode in (ECR, BIDIR):
        _, slot_of, slot_token, counts = oracle.select_adaptive(S, k, C, mode, thr)
        check_permutation_tables(T, E, C, slot_of, slot_token, counts)
        plain = oracle.select(S, k, C, mode)[1] >= 0
        assert np.all((slot_of >= 0) <= plain)                   # a prefix of what the capacity alone would keep
        for e in range(E):
            cands = list(range(T)) if mode == ECR else list(np.flatnonzero(chose[:, e]))
            assert list(slot_token[e, :counts[e]]) == _adaptive_brute(S, e, cands, C, thr), (mode, e)


# ---------------------------------------------------------------------------------------
# variant readings: rank-major token choice, strict intersection of the two pure phases
# ---------------------------------------------------------------------------------------
TCR_RANK, STRICT = 3, 4


def test_variants_worked_example(oracle):
    g = load_golden("select_worked_example.json")
    S = np.array(g["score"], np.float32)
    C = g["capacity"]
    for kname, k in (("k1", 1), ("k2", 2)):
        for mname, mode in (("tcr_rank", TCR_RANK), ("strict", STRICT)):
            topk, slot_of, slot_token, counts = oracle.select(S, k, C, mode)
            assert topk.tolist() == g[kname]["topk"]
            assert [list(map(int, s)) for s in kept_sets(slot_token, counts)] == g[kname][mname]["kept"], (kname, mname)
            check_permutation_tables(6, 3, C, slot_of, slot_token, counts)


def _rank_major_sequential(topk, E, C):
    """The classic sequential statement: walk the choice ranks in turn, inside a rank the tokens in
    order; a choice is granted while the expert still has room."""
    T, k = topk.shape
    used = [0] * E
    kept = [[] for _ in range(E)]
    for r in range(k):
        for t in range(T):
            e = int(topk[t, r])
            if used[e] < C:
                used[e] += 1
                kept[e].append(t)
    return [sorted(s) for s in kept]


@pytest.mark.parametrize("seed", range(10))
def test_variants_brute_force(oracle, seed):
    rng = np.random.default_rng(500 + seed)
    T, E = int(rng.integers(5, 60)), int(rng.integers(2, 7))
    k = int(rng.integers(1, E + 1))
    C = int(rng.integers(1, T + 2))
    S = _scores(rng, T, E, 3 if seed % 2 else None)
    topk, slot_of, slot_token, counts = oracle.select(S, k, C, TCR_RANK)
    check_permutation_tables(T, E, C, slot_of, slot_token, counts)
    assert [list(map(int, s)) for s in kept_sets(slot_token, counts)] == _rank_major_sequential(topk, E, C)
    # strict: choosers (Eq. 5) intersected with the top-min(C, T) of all tokens under (score desc, index asc)
    topk2, slot_of, slot_token, counts = oracle.select(S, k, C, STRICT)
    np.testing.assert_array_equal(topk2, topk)
    check_permutation_tables(T, E, C, slot_of, slot_token, counts)
    for e in range(E):
        top = set(sorted(range(T), key=lambda t: (-float(S[t, e]), t))[:min(C, T)])
        want = sorted(t for t in range(T) if e in topk[t] and t in top)
        assert list(map(int, slot_token[e, :counts[e]])) == want


def test_variants_reduce_to_the_plain_modes(oracle):
    rng = np.random.default_rng(77)
    T, E, C = 50, 5, 7
    S = _scores(rng, T, E)
    # one choice per token: rank-major priority is the position priority
    for a, b in zip(oracle.select(S, 1, C, TCR_RANK), oracle.select(S, 1, C, TCR)):
        np.testing.assert_array_equal(a, b)
    # every token lists every expert: the intersection is pure expert choice
    for a, b in zip(oracle.select(S, E, C, STRICT)[1:], oracle.select(S, E, C, ECR)[1:]):
        np.testing.assert_array_equal(a, b)
    # capacity never binds: both variants keep every chooser, like Eq. 6
    for mode in (TCR_RANK, STRICT):
        for a, b in zip(oracle.select(S, 2, T, mode), oracle.select(S, 2, T, BIDIR)):
            np.testing.assert_array_equal(a, b)
    # strict is a subset of Eq. 6's keep set
    strict, bidir = oracle.select(S, 2, C, STRICT)[1], oracle.select(S, 2, C, BIDIR)[1]
    assert np.all((strict < 0) | (bidir >= 0))
    with pytest.raises(RuntimeError):
        oracle.select_adaptive(S, 2, C, STRICT, 0.5)     # the affinity-sum threshold is not defined for it
