"""Pins for the CPU oracle: every check here compares it with something other than
its own formulas -- values the paper prints, closed forms, exact rational
arithmetic, brute-force enumeration, independent re-implementations of textbook
routines, library log-softmax / autograd, finite differences."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import dppo_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ advantages
@pytest.mark.parametrize("ddof", [0, 1])
def test_advantages_sum_to_zero_and_unit_scale(ddof):
    rng = np.random.default_rng(1)
    r = rng.normal(size=(7, 9))
    A = O.group_advantages(r, ddof=ddof, eps=0.0)
    assert np.abs(A.sum(axis=1)).max() < 1e-12 * 9
    # (Eq. 2) with eps = 0 the normalised values have sum of squares G - ddof
    assert np.allclose((A ** 2).sum(axis=1), 9 - ddof, rtol=1e-12)
    # against the library definition
    ref = (r - r.mean(axis=1, keepdims=True)) / r.std(axis=1, ddof=ddof, keepdims=True)
    assert np.allclose(A, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("G,ddof", [(4, 1), (8, 1), (8, 0), (16, 1), (5, 0)])
def test_binary_reward_closed_form(G, ddof):
    # k ones of G: p = k/G, sigma = sqrt(p(1-p) G/(G-ddof)), A_one = (1-p)/sigma, A_zero = -p/sigma,
    # mean|A| = 2p(1-p)/sigma, so the candidates are the majority class (all if balanced/constant).
    for k in range(G + 1):
        r = np.zeros((1, G), dtype=np.float32)
        r[0, :k] = 1.0
        A = O.group_advantages(r, ddof=ddof, eps=0.0) if 0 < k < G else O.group_advantages(r, ddof=ddof)
        cand = O.completion_candidates(r)[0]
        if k in (0, G):
            assert np.all(A == 0.0) and cand.all()
            continue
        p = k / G
        sigma = math.sqrt(p * (1 - p) * G / (G - ddof))
        assert np.allclose(A[0, :k], (1 - p) / sigma, rtol=1e-12)
        assert np.allclose(A[0, k:], -p / sigma, rtol=1e-12)
        sel = O.select(r, None, None, None, 0.0, 0.0, ddof=ddof, eps=0.0)
        assert math.isclose(sel["mean_abs_adv"][0], 2 * p * (1 - p) / sigma, rel_tol=1e-12)
        if 2 * k == G:
            assert cand.all()
        elif 2 * k > G:
            assert cand[:k].all() and not cand[k:].any()
        else:
            assert cand[k:].all() and not cand[:k].any()


def test_candidates_match_exact_rational_inequality():
    # Eq. 15 decided in exact arithmetic on integer rewards: |r_i - mu| <= mean_j |r_j - mu|
    rng = np.random.default_rng(7)
    for _ in range(300):
        G = int(rng.integers(2, 17))
        r = rng.integers(0, 4, size=G)
        mu = Fraction(int(r.sum()), G)
        dev = [abs(Fraction(int(x)) - mu) for x in r]
        thr = sum(dev, Fraction(0)) / G
        want = np.array([d <= thr for d in dev])
        got = O.completion_candidates(r[None, :].astype(np.float32))[0]
        assert np.array_equal(got, want), (r, got, want)


def test_candidates_agree_with_float_advantages_away_from_ties():
    rng = np.random.default_rng(3)
    r = rng.normal(size=(200, 8)).astype(np.float32)
    A = O.group_advantages(r)
    thr = np.abs(A).mean(axis=1, keepdims=True)
    margin = np.abs(np.abs(A) - thr)
    cand = O.completion_candidates(r)
    clear = margin > 1e-6
    assert np.array_equal(cand[clear], (np.abs(A) <= thr)[clear])


# ---------------------------------------------------------- prompt candidates
def test_prompt_candidates_rank_and_ties():
    hist = np.array([0.5, 0.0, 0.5, 0.0, 0.9, 0.0, 0.1], dtype=np.float32)
    inB = O.prompt_candidates(hist, 0.5)          # floor(3.5) = 3 lowest: the three zeros
    assert inB.tolist() == [False, True, False, True, False, True, False]
    hist = np.zeros(6, dtype=np.float32)          # all tied: lowest indices first
    assert O.prompt_candidates(hist, 0.5).tolist() == [True, True, True, False, False, False]
    rng = np.random.default_rng(0)
    h = rng.random(31).astype(np.float32)
    inB = O.prompt_candidates(h, 0.5)
    assert inB.sum() == 15 and h[inB].max() <= h[~inB].min()


# -------------------------------------------------------------------- weights
def test_no_pruning_recovers_plain_grpo_weights():
    rng = np.random.default_rng(2)
    r = (rng.random((6, 5)) < 0.5).astype(np.float32)
    for kw in (dict(hist=None, u_prompt=None, u_comp=None, r_q=0.5, r_o=0.5),
               dict(hist=rng.random(6), u_prompt=rng.random(6), u_comp=rng.random((6, 5)), r_q=0.0, r_o=0.0)):
        s = O.select(r, kw["hist"], kw["u_prompt"], kw["u_comp"], kw["r_q"], kw["r_o"])
        assert s["keep_prompt"].all() and s["keep_comp"].all()
        assert np.all(s["gamma_q"] == 1.0) and np.all(s["gamma_o"] == 1.0)
        assert np.allclose(s["coef"], 1.0 / 30, rtol=1e-15)


def _golden_factor_rows():
    rows = []
    with open(os.path.join(GOLDEN, "thm_d1_variance_factor.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                b, r, rel, v = line.split()
                rows.append((float(b), float(r), rel, float(v)))
    return rows


@pytest.mark.parametrize("beta,r_q,rel,value", _golden_factor_rows())
def test_prompt_weights_reproduce_printed_variance_factor(beta, r_q, rel, value):
    # 200 prompts, bottom half candidates, exactly r_q*100 of them pruned (uniforms chosen so):
    # the mean of gamma_q^2 over retained prompts is the paper's factor (App. D.3).
    Q, G = 200, 2
    hist = np.arange(Q, dtype=np.float32)
    n_prune = int(round(r_q * beta * Q))
    u_prompt = np.ones(Q, dtype=np.float32) * 0.999
    u_prompt[:n_prune] = 0.0
    rewards = np.zeros((Q, G), dtype=np.float32)
    s = O.select(rewards, hist, u_prompt, None, r_q, 0.0, bottom_frac=beta)
    kept = s["keep_prompt"].astype(bool)
    assert kept.sum() == Q - n_prune
    got = float((s["gamma_q"][kept] ** 2).mean())
    closed = (1 - beta * r_q) * (1 - (1 - beta) * r_q) / (1 - r_q)
    assert math.isclose(got, closed, rel_tol=1e-6)    # r_q goes through float32
    if rel == "le":
        assert got <= value and got > value - 0.02
    else:
        assert abs(got - value) < 5e-4


def _enumerate_masks(rewards, hist, r_q, r_o, bottom_frac=0.5):
    """All joint prune masks with their probabilities, realised through the uniforms."""
    Q, G = rewards.shape
    inB = O.prompt_candidates(hist, bottom_frac) if hist is not None else np.zeros(Q, bool)
    cand = O.completion_candidates(rewards)
    pb = [k for k in range(Q) if inB[k]]
    cb = [(k, i) for k in range(Q) for i in range(G) if cand[k, i]]
    for bits_q in itertools.product([0, 1], repeat=len(pb)):
        for bits_o in itertools.product([0, 1], repeat=len(cb)):
            up = np.full(Q, 0.999, dtype=np.float32)
            uc = np.full((Q, G), 0.999, dtype=np.float32)
            prob = 1.0
            for b, k in zip(bits_q, pb):
                if b:
                    up[k] = 0.0
                prob *= r_q if b else (1 - r_q)
            for b, (k, i) in zip(bits_o, cb):
                if b:
                    uc[k, i] = 0.0
                prob *= r_o if b else (1 - r_o)
            yield prob, up, uc


@pytest.mark.parametrize("Q,G,seed", [(2, 3, 0), (3, 3, 1), (2, 4, 2), (3, 2, 3)])
def test_expected_weight_is_unpruned_weight(Q, G, seed):
    # Eq. 9, 12, 13 in the discrete setting: averaging coef over every prune mask,
    # weighted by its probability, gives each completion the plain GRPO weight 1/(QG).
    rng = np.random.default_rng(seed)
    rewards = (rng.random((Q, G)) < 0.5).astype(np.float32)
    hist = rng.random(Q).astype(np.float32)
    r_q, r_o = 0.5, 0.25
    acc = np.zeros((Q, G))
    ptot = 0.0
    for prob, up, uc in _enumerate_masks(rewards, hist, r_q, r_o):
        acc += prob * O.select(rewards, hist, up, uc, r_q, r_o)["coef"]
        ptot += prob
    assert math.isclose(ptot, 1.0, rel_tol=1e-12)
    assert np.allclose(acc, 1.0 / (Q * G), rtol=1e-12)


def test_weights_equal_horvitz_thompson_form():
    rng = np.random.default_rng(5)
    Q, G = 10, 6
    rewards = (rng.random((Q, G)) < 0.4).astype(np.float32)
    s = O.select(rewards, rng.random(Q), rng.random(Q), rng.random((Q, G)), 0.5, 0.5)
    kept = s["keep_comp"].astype(bool)
    ht = 1.0 / (Q * G * (1 - s["P_q"][:, None]) * (1 - s["P_o"]))
    assert np.allclose(s["coef"][kept], ht[kept], rtol=1e-12)
    assert np.all(s["coef"][~kept] == 0.0)
    assert not kept[~s["keep_prompt"].astype(bool)].any()
    assert s["counts"][0] == s["keep_prompt"].sum()
    assert np.array_equal(s["counts"][1:], kept.sum(axis=1))


# ------------------------------------------------- fixed-count pruning, history
def test_fixed_prune_count_floor_with_float32_rates():
    assert O.fixed_prune_count(0.9, 10) == 9          # float32(0.9) * 10 is just below 9
    assert O.fixed_prune_count(0.5, 3) == 1 and O.fixed_prune_count(0.5, 1) == 0
    assert O.fixed_prune_count(0.7, 100) == 70 and O.fixed_prune_count(0.0, 5) == 0
    assert O.fixed_prune_count(0.999999, 4) == 3      # someone always survives
    assert O.fixed_prune_count(0.5, 0) == 0


def _enumerate_fixed_subsets(rewards, hist, r_q, r_o):
    """Every equally likely outcome of fixed-count pruning, realised through the uniforms."""
    Q, G = rewards.shape
    inB = O.prompt_candidates(hist, 0.5)
    cand = O.completion_candidates(rewards)
    B = [k for k in range(Q) if inB[k]]
    m_q = O.fixed_prune_count(r_q, len(B))
    groups = [[i for i in range(G) if cand[k, i]] for k in range(Q)]
    m_o = [O.fixed_prune_count(r_o, len(g)) for g in groups]
    choices = [list(itertools.combinations(B, m_q))] + \
              [list(itertools.combinations(groups[k], m_o[k])) for k in range(Q)]
    n_total = 1
    for c in choices:
        n_total *= len(c)
    for combo in itertools.product(*choices):
        up = np.full(Q, 0.9, dtype=np.float32)
        uc = np.full((Q, G), 0.9, dtype=np.float32)
        for k in combo[0]:
            up[k] = 0.1
        for k in range(Q):
            for i in combo[1 + k]:
                uc[k, i] = 0.1
        yield 1.0 / n_total, up, uc, (m_q, m_o)


@pytest.mark.parametrize("Q,G,r_q,r_o,seed", [(4, 3, 0.5, 0.5, 0), (4, 4, 0.75, 0.4, 1), (2, 5, 0.5, 0.7, 2)])
def test_fixed_count_pruning_counts_and_unbiased_weights(Q, G, r_q, r_o, seed):
    rng = np.random.default_rng(seed)
    rewards = (rng.random((Q, G)) < 0.5).astype(np.float32)
    hist = rng.random(Q).astype(np.float32)
    acc = np.zeros((Q, G))
    acc_nominal = np.zeros((Q, G))
    for prob, up, uc, (m_q, m_o) in _enumerate_fixed_subsets(rewards, hist, r_q, r_o):
        s = O.select(rewards, hist, up, uc, r_q, r_o, fixed_count=True)
        assert Q - s["keep_prompt"].sum() == m_q                    # exactly floor(r |B|) prompts go
        for k in range(Q):
            if s["keep_prompt"][k]:
                assert G - s["keep_comp"][k].sum() == m_o[k]        # and floor(r |C_k|) completions
            else:
                assert s["keep_comp"][k].sum() == 0
        acc += prob * s["coef"]
        acc_nominal += prob * O.select(rewards, hist, up, uc, r_q, r_o, fixed_count=True, realised_rate=False)["coef"]
    # with the realised rate in Eq. 18 the expected weight is the plain GRPO weight, exactly
    assert np.allclose(acc, 1.0 / (Q * G), rtol=1e-12)
    # with the nominal rate it is so only where r * n is an integer
    inB = O.prompt_candidates(hist, 0.5)
    cand = O.completion_candidates(rewards)
    nB = int(inB.sum())
    for k in range(Q):
        nC = int(cand[k].sum())
        exact_q = (not inB[k]) or abs(r_q * nB - round(r_q * nB)) < 1e-9
        for i in range(G):
            exact_o = (not cand[k, i]) or abs(r_o * nC - round(r_o * nC)) < 1e-6
            if exact_q and exact_o:
                assert math.isclose(acc_nominal[k, i], 1.0 / (Q * G), rel_tol=1e-6)


def test_fixed_count_picks_smallest_uniforms_ties_to_lower_index():
    rewards = np.array([[1, 0, 0, 0, 0, 0]], dtype=np.float32)      # five zeros are the candidates
    uc = np.array([[0.0, 0.5, 0.2, 0.2, 0.9, 0.1]], dtype=np.float32)
    s = O.select(rewards, None, None, uc, 0.0, 0.6, fixed_count=True)   # floor(0.6 * 5) = 3 pruned
    assert s["keep_comp"].tolist() == [[1, 1, 0, 0, 1, 0]]          # 0.1, then the tie 0.2/0.2: both go
    s = O.select(rewards, None, None, uc, 0.0, 0.4, fixed_count=True)   # 2 pruned: 0.1 and the first 0.2
    assert s["keep_comp"].tolist() == [[1, 1, 0, 1, 1, 0]]
    assert math.isclose(s["gamma_o"][0, 1], (4 / 6) / (1 - 2 / 5), rel_tol=1e-12)
    assert s["gamma_o"][0, 0] == 4 / 6                               # never a candidate: P = 0


def test_history_update_carries_pruned_prompts_forward():
    table = np.array([0.0, 0.3, 0.0, 0.8, 0.5], dtype=np.float32)
    out = O.history_update(table, [3, 0, 4], [1, 0, 1], [0.25, 0.9, 0.0])
    assert out.tolist() == [0.0, np.float32(0.3), 0.0, 0.25, 0.0]   # prompt 0 was pruned: unchanged
    assert table[3] == np.float32(0.8)                              # input untouched


# -------------------------------------------------------------------- packing
def _next_fit(lens, cap):
    rows, cur, rem = [], [], cap
    for j, l in enumerate(lens):
        if l > rem:
            rows.append(cur)
            cur, rem = [], cap
        cur.append(j)
        rem -= l
    if cur:
        rows.append(cur)
    return rows


def _first_fit(lens, cap):
    rows, rems = [], []
    for j, l in enumerate(lens):
        for b in range(len(rows)):
            if l <= rems[b]:
                rows[b].append(j)
                rems[b] -= l
                break
        else:
            rows.append([j])
            rems.append(cap - l)
    return rows


def _window_restart_scan(lens, cap, n_win):
    """Second statement of Sec. 4.3: after every placement rescan the pool from its oldest item."""
    n = len(lens)
    pool = list(range(min(n_win, n)))
    nxt = len(pool)
    rows = []
    while pool:
        row, rem = [], cap
        while True:
            hit = next((j for j in pool if lens[j] <= rem), None)
            if hit is None:
                break
            row.append(hit)
            rem -= lens[hit]
            pool.remove(hit)
            if nxt < n:
                pool.append(nxt)
                nxt += 1
        rows.append(row)
    return rows


def _rows_of(p):
    return [p["order"][p["row_ptr"][r]:p["row_ptr"][r + 1]].tolist() for r in range(p["n_rows"])]


def test_pack_hand_worked_cases():
    ones = np.ones(5, dtype=np.int64)
    p = O.pack(ones, np.array([5, 4, 3, 6, 2]) - 1, None, 10, 2)
    assert p["order"].tolist() == [0, 1, 2, 3, 4] and p["row_ptr"].tolist() == [0, 2, 4, 5]
    p = O.pack(ones, np.array([7, 5, 3, 4, 2]) - 1, None, 10, 3)
    assert p["order"].tolist() == [0, 2, 1, 3, 4] and p["row_ptr"].tolist() == [0, 2, 4, 5]
    # offsets: prompt 2 + completion 3 starting at 0, then prompt 1 + completion 2
    p = O.pack(np.array([2, 1]), np.array([3, 2]), None, 16, 4)
    assert p["cu_seqlens"].tolist() == [0, 5, 8] and p["loss_cu"].tolist() == [0, 3, 5]
    assert p["loss_pos"].tolist() == [1, 2, 3, 5, 6]


def test_pack_invariants_and_reductions():
    rng = np.random.default_rng(11)
    for trial in range(200):
        n = int(rng.integers(1, 40))
        cap = int(rng.integers(8, 64))
        pl = rng.integers(1, cap // 2 + 1, size=n)
        cl = rng.integers(1, cap - pl + 1)
        lens = (pl + cl).tolist()
        for n_win in (1, 2, 5, n, n + 7):
            p = O.pack(pl, cl, None, cap, n_win)
            rows = _rows_of(p)
            assert sorted(p["order"].tolist()) == list(range(n))
            assert all(sum(lens[j] for j in row) <= cap for row in rows)
            assert p["T"] == sum(lens) == p["cu_seqlens"][-1]
            assert p["N"] == int(cl.sum()) == p["loss_cu"][-1] == len(p["loss_pos"])
            assert p["n_rows"] >= math.ceil(sum(lens) / cap)
            assert rows == _window_restart_scan(lens, cap, n_win)
            if n_win == 1:
                assert rows == _next_fit(lens, cap)
            if n_win >= n:
                assert rows == _first_fit(lens, cap)
            # loss positions: inside their sequence, and the next position is a completion token
            for s, j in enumerate(p["order"]):
                a, b = p["loss_cu"][s], p["loss_cu"][s + 1]
                lp = p["loss_pos"][a:b]
                assert b - a == cl[j]
                assert lp[0] == p["cu_seqlens"][s] + pl[j] - 1
                assert lp[-1] == p["cu_seqlens"][s + 1] - 2
                assert np.all(np.diff(lp) == 1)


def test_pack_equal_lengths_and_keep_mask():
    p = O.pack(np.full(23, 3), np.full(23, 4), None, 30, 6)
    assert p["n_rows"] == math.ceil(23 / (30 // 7))
    keep = np.array([1, 0, 1, 1, 0, 1], dtype=np.uint8)
    pl = np.array([2, 9, 3, 4, 9, 5])
    cl = np.array([2, 9, 2, 2, 9, 2])
    p = O.pack(pl, cl, keep, 10, 2)
    q = O.pack(pl[keep == 1], cl[keep == 1], None, 10, 2)
    assert p["order"].tolist() == np.flatnonzero(keep)[q["order"]].tolist()
    assert p["cu_seqlens"].tolist() == q["cu_seqlens"].tolist()
    assert p["S"] == 4
    with pytest.raises(ValueError):
        O.pack(np.array([6]), np.array([6]), None, 10, 2)


def _window_best_fit(lens, cap, n_win):
    """Best-fit reading without an explicit pool: after p placements the pool is the set of unplaced
    items among the first n_win + p of the stream; take the longest that fits, oldest among equals."""
    n = len(lens)
    placed = [False] * n
    n_placed, rows = 0, []
    while n_placed < n:
        row, rem = [], cap
        while True:
            visible = [j for j in range(min(n, n_win + n_placed)) if not placed[j] and lens[j] <= rem]
            if not visible:
                break
            j = sorted(visible, key=lambda t: (-lens[t], t))[0]
            placed[j] = True
            n_placed += 1
            row.append(j)
            rem -= lens[j]
        rows.append(row)
    return rows


def test_pack_best_fit_policy():
    ones = np.ones(5, dtype=np.int64)
    # pool {4,6,3}: take 6, refill 5, take 4 (row full); then 5, 3, 2
    p = O.pack(ones, np.array([4, 6, 3, 5, 2]) - 1, None, 10, 3, policy="best_fit")
    assert p["order"].tolist() == [1, 0, 3, 2, 4] and p["row_ptr"].tolist() == [0, 2, 5]
    # a case where the two readings differ in the number of rows
    lens = np.array([5, 4, 6, 5])
    ff = O.pack(ones[:4], lens - 1, None, 10, 4)
    bf = O.pack(ones[:4], lens - 1, None, 10, 4, policy="best_fit")
    assert _rows_of(ff) == [[0, 1], [2], [3]] and _rows_of(bf) == [[2, 1], [0, 3]]
    assert ff["density"] == pytest.approx(20 / 30) and bf["density"] == 1.0
    rng = np.random.default_rng(23)
    for trial in range(200):
        n = int(rng.integers(1, 40))
        cap = int(rng.integers(8, 64))
        pl = rng.integers(1, cap // 2 + 1, size=n)
        cl = rng.integers(1, cap - pl + 1)
        lens = (pl + cl).tolist()
        for n_win in (1, 2, 5, n, n + 7):
            p = O.pack(pl, cl, None, cap, n_win, policy="best_fit")
            rows = _rows_of(p)
            assert sorted(p["order"].tolist()) == list(range(n))
            assert all(sum(lens[j] for j in row) <= cap for row in rows)
            assert rows == _window_best_fit(lens, cap, n_win)
            if n_win == 1:
                assert rows == _next_fit(lens, cap)
            if n_win >= n:
                # every row opens with the longest item still unplaced
                left = set(range(n))
                for row in rows:
                    assert lens[row[0]] == max(lens[j] for j in left)
                    left -= set(row)
            assert p["density"] == pytest.approx(sum(lens) / (p["n_rows"] * cap))
    with pytest.raises(ValueError):
        O.pack(ones, ones, None, 10, 2, policy="worst_fit")


def test_pack_prompts_alone_with_longest_item_as_capacity():
    # Sec. 4.3: prompts are packed before any rollout, L_max = the longest sample
    pl = np.array([3, 9, 4, 2, 5, 9, 1])
    for policy in ("first_fit", "best_fit"):
        p = O.pack(pl, None, None, None, 3, policy=policy)
        assert p["capacity"] == 9 and p["N"] == 0 and len(p["loss_pos"]) == 0
        assert p["loss_cu"].tolist() == [0] * 8
        assert p["T"] == 33 and sorted(p["order"].tolist()) == list(range(7))
        assert np.array_equal(np.diff(p["cu_seqlens"]), pl[p["order"]])
    # first fit, window 3, worked by hand (items fetched during a scan are still visited by it):
    p = O.pack(pl, None, None, None, 3)
    #   row 0: pool (3,9,4): 3 -> fetch 2: pool (9,4,2): 9 no, 4 (rem 2) -> fetch 5: 2 (rem 0) -> fetch 9
    #   row 1: pool (9,5,9): 9 (rem 0) -> fetch 1
    #   row 2: pool (5,9,1): 5 (rem 4), 9 no, 1 (rem 3)
    #   row 3: pool (9): 9
    assert _rows_of(p) == [[0, 2, 3], [1], [4, 6], [5]]
    assert p["density"] == pytest.approx(33 / 36)
    # completions may not be empty when they are given
    with pytest.raises(ValueError):
        O.pack(pl, np.zeros(7, dtype=np.int64), None, 16, 3)
    # keep mask decides which items define L_max
    p = O.pack(pl, None, np.array([1, 0, 1, 1, 1, 0, 1], dtype=np.uint8), 0, 2)
    assert p["capacity"] == 5 and p["S"] == 5


# ------------------------------------------------------------------ log-probs
def _tiny_head(seed, N=11, D=8, V=16):
    rng = np.random.default_rng(seed)
    H = rng.normal(size=(N + 3, D))
    W = rng.normal(size=(V, D)) * 0.5
    ids = rng.integers(0, V, size=N + 3)
    loss_pos = np.array([0, 1, 2, 4, 5, 6, 7, 9, 10, 11, 12][:N]) if N <= 11 else np.arange(N)
    return H, W, ids, loss_pos


def test_logprob_special_cases():
    H, W, ids, lp = _tiny_head(0)
    V = W.shape[0]
    logp, lse = O.token_logprob(H, np.zeros_like(W), ids, lp)
    assert np.allclose(logp, -math.log(V), rtol=1e-14) and np.allclose(lse, math.log(V))
    logp, _ = O.token_logprob(H, np.tile(W[:1], (V, 1)), ids, lp)
    assert np.allclose(logp, -math.log(V), rtol=1e-12)
    # a constant added to every logit of a row does not change log-probs
    base, _ = O.token_logprob(H, W, ids, lp)
    H1 = np.concatenate([H, np.ones((H.shape[0], 1))], axis=1)
    W1 = np.concatenate([W, np.full((V, 1), 3.7)], axis=1)
    shifted, lse1 = O.token_logprob(H1, W1, ids, lp)
    assert np.allclose(base, shifted, rtol=1e-12, atol=1e-12)
    # probabilities of a row sum to one
    Z = H1[lp] @ W1.T
    assert np.allclose(np.exp(Z - lse1[:, None]).sum(axis=1), 1.0, rtol=1e-12)


def test_logprob_matches_library_log_softmax():
    import torch
    H, W, ids, lp = _tiny_head(1)
    logp, lse = O.token_logprob(H, W, ids, lp)
    Ht, Wt = torch.tensor(H), torch.tensor(W)
    lsm = torch.log_softmax(Ht[torch.tensor(lp)] @ Wt.T, dim=-1)
    y = torch.tensor(ids[lp + 1]).long()
    want = lsm.gather(1, y[:, None])[:, 0].numpy()
    assert np.allclose(logp, want, rtol=1e-12, atol=1e-12)
    # identity indexing form
    logp2, _ = O.token_logprob(H[lp], W, ids[lp + 1], None)
    assert np.allclose(logp, logp2, rtol=0, atol=0)


# ------------------------------------------------------------ loss and grads
def _loss_case(seed, clip_noise=0.3):
    rng = np.random.default_rng(seed)
    pl = np.array([2, 3, 1, 2])
    cl = np.array([3, 1, 4, 2])
    p = O.pack(pl, cl, None, 12, 2)
    T, N = p["T"], p["N"]
    D, V = 6, 13
    H = rng.normal(size=(T, D))
    W = rng.normal(size=(V, D)) * 0.7
    ids = rng.integers(0, V, size=T)
    base, _ = O.token_logprob(H, W, ids, p["loss_pos"])
    old = base + rng.normal(0, clip_noise, size=N)
    ref = base + rng.normal(0, 0.2, size=N)
    adv = np.array([1.3, -0.7, 0.4, -1.1])
    coef = np.array([0.1, 0.4, 0.25, 0.3])
    return p, H, W, ids, old, ref, adv, coef


def test_coincident_policies_give_unit_ratio_zero_kl():
    p, H, W, ids, _, _, adv, coef = _loss_case(0)
    base, _ = O.token_logprob(H, W, ids, p["loss_pos"])
    out = O.loss_fwd_bwd(H, W, ids, p["loss_pos"], p["loss_cu"], adv, coef, base, base)
    assert np.allclose(out["seq_loss"], -adv, rtol=1e-12)
    assert math.isclose(out["loss"], -float(coef @ adv), rel_tol=1e-12)
    assert out["mean_kl"] == 0.0 and out["clip_frac"] == 0.0
    # plain GRPO weights and full groups: the loss vanishes because advantages sum to zero
    r = np.array([[1, 0, 0, 1], [0, 0, 1, 0]], dtype=np.float32)
    s = O.select(r, None, None, None, 0.0, 0.0)
    rng = np.random.default_rng(4)
    pl, cl = np.repeat([2, 3], 4), rng.integers(1, 5, size=8)
    pk = O.pack(pl, cl, None, 16, 3)
    Hh = rng.normal(size=(pk["T"], 5)); Ww = rng.normal(size=(9, 5)); ii = rng.integers(0, 9, pk["T"])
    b, _ = O.token_logprob(Hh, Ww, ii, pk["loss_pos"])
    out = O.loss_fwd_bwd(Hh, Ww, ii, pk["loss_pos"], pk["loss_cu"],
                         s["adv"].reshape(-1)[pk["order"]], s["coef"].reshape(-1)[pk["order"]], b, b)
    assert abs(out["loss"]) < 1e-12


def test_loss_and_grads_match_autograd():
    import torch
    p, H, W, ids, old, ref, adv, coef = _loss_case(1)
    out = O.loss_fwd_bwd(H, W, ids, p["loss_pos"], p["loss_cu"], adv, coef, old, ref, 0.2, 0.25, 0.04)
    assert out["clip_frac"] > 0.0          # the case does exercise clipping
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    lp = torch.tensor(p["loss_pos"]).long()
    y = torch.tensor(ids[p["loss_pos"] + 1]).long()
    logp = torch.log_softmax(Ht[lp] @ Wt.T, dim=-1).gather(1, y[:, None])[:, 0]
    total = torch.zeros((), dtype=torch.float64)
    for s in range(4):
        a, b = int(p["loss_cu"][s]), int(p["loss_cu"][s + 1])
        rho = torch.exp(logp[a:b] - torch.tensor(old[a:b]))
        sur = torch.minimum(rho * adv[s], torch.clamp(rho, 0.8, 1.25) * adv[s])
        rh = torch.exp(torch.tensor(ref[a:b]) - logp[a:b])
        kl = rh - torch.log(rh) - 1
        total = total + coef[s] * (-(sur) + 0.04 * kl).mean()
    total.backward()
    assert math.isclose(out["loss"], float(total.detach()), rel_tol=1e-12)
    assert np.allclose(out["dH"], Ht.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_gradient_finite_differences_and_invariants():
    p, H, W, ids, old, ref, adv, coef = _loss_case(2, clip_noise=0.05)
    f = lambda Hx, Wx: O.loss_fwd_bwd(Hx, Wx, ids, p["loss_pos"], p["loss_cu"], adv, coef, old, ref)
    out = f(H, W)
    rng = np.random.default_rng(9)
    h = 1e-6
    for _ in range(12):
        t, d = int(rng.integers(H.shape[0])), int(rng.integers(H.shape[1]))
        Hp, Hm = H.copy(), H.copy(); Hp[t, d] += h; Hm[t, d] -= h
        fd = (f(Hp, W)["loss"] - f(Hm, W)["loss"]) / (2 * h)
        assert abs(fd - out["dH"][t, d]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9
        v, d = int(rng.integers(W.shape[0])), int(rng.integers(W.shape[1]))
        Wp, Wm = W.copy(), W.copy(); Wp[v, d] += h; Wm[v, d] -= h
        fd = (f(H, Wp)["loss"] - f(H, Wm)["loss"]) / (2 * h)
        assert abs(fd - out["dW"][v, d]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9
    # softmax gradients sum to zero over the vocabulary
    assert np.abs(out["dW"].sum(axis=0)).max() < 1e-13
    # rows that predict nothing get no gradient
    mask = np.ones(H.shape[0], bool); mask[p["loss_pos"]] = False
    assert np.all(out["dH"][mask] == 0.0) and np.abs(out["dH"][~mask]).min() > 0
    # identical vocabulary rows: log-probs do not depend on H
    Wc = np.tile(W[:1], (W.shape[0], 1))
    assert np.abs(f(H, Wc)["dH"]).max() < 1e-13


def test_expected_loss_and_gradients_are_unbiased_over_all_masks():
    # Eq. 13 for the full Eq. 1 loss: sum over prune masks of P(mask) * {L, dH, dW}(mask)
    # equals the unpruned GRPO values; each mask runs select -> pack -> loss from scratch.
    rng = np.random.default_rng(21)
    Q, G, D, V = 2, 3, 5, 9
    rewards = np.array([[1, 1, 1], [0, 1, 0]], dtype=np.float32)   # a constant group can be pruned whole
    hist = np.array([0.3, 0.1], dtype=np.float32)
    pl = np.repeat(rng.integers(1, 4, size=Q), G)
    cl = rng.integers(1, 5, size=Q * G)
    seqH = [rng.normal(size=(pl[j] + cl[j], D)) for j in range(Q * G)]
    seqI = [rng.integers(0, V, size=pl[j] + cl[j]) for j in range(Q * G)]
    W = rng.normal(size=(V, D)) * 0.6
    seq_old = [rng.normal(0, 0.1, size=cl[j]) for j in range(Q * G)]
    seq_ref = [rng.normal(0, 0.1, size=cl[j]) for j in range(Q * G)]
    r_q, r_o = 0.5, 0.375          # exactly representable in float32

    def run(up, uc, rq, ro):
        s = O.select(rewards, hist, up, uc, rq, ro)
        keep = s["keep_comp"].reshape(-1)
        dHs = [np.zeros_like(h) for h in seqH]
        if keep.sum() == 0:
            return 0.0, dHs, np.zeros_like(W)
        pk = O.pack(pl, cl, keep, 16, 2)
        od = pk["order"]
        H = np.concatenate([seqH[j] for j in od]); ids = np.concatenate([seqI[j] for j in od])
        base, _ = O.token_logprob(H, W, ids, pk["loss_pos"])
        old = base + np.concatenate([seq_old[j] for j in od])
        ref = base + np.concatenate([seq_ref[j] for j in od])
        out = O.loss_fwd_bwd(H, W, ids, pk["loss_pos"], pk["loss_cu"],
                             s["adv"].reshape(-1)[od], s["coef"].reshape(-1)[od], old, ref)
        for si, j in enumerate(od):
            dHs[j] = out["dH"][pk["cu_seqlens"][si]:pk["cu_seqlens"][si + 1]]
        return out["loss"], dHs, out["dW"]

    L0, dH0, dW0 = run(None, None, 0.0, 0.0)
    EL, EdH, EdW = 0.0, [np.zeros_like(h) for h in seqH], np.zeros_like(W)
    n_masks = 0
    saw_empty_group = False
    for prob, up, uc in _enumerate_masks(rewards, hist, r_q, r_o):
        L, dHs, dW = run(up, uc, r_q, r_o)
        EL += prob * L
        EdW += prob * dW
        for j in range(Q * G):
            EdH[j] += prob * dHs[j]
        n_masks += 1
        s = O.select(rewards, hist, up, uc, r_q, r_o)
        saw_empty_group |= bool((s["counts"][1:][s["keep_prompt"] == 1] == 0).any())
    assert n_masks >= 32 and saw_empty_group
    assert math.isclose(EL, L0, rel_tol=1e-10)
    assert np.allclose(EdW, dW0, rtol=1e-9, atol=1e-13)
    for j in range(Q * G):
        assert np.allclose(EdH[j], dH0[j], rtol=1e-9, atol=1e-13)


# ------------------------------------------- objective variants (sequence ratio, token normalisation)
VARIANTS = [("token", "seq_mean"), ("token", "token_sum"), ("sequence", "seq_mean"), ("sequence", "token_sum")]


@pytest.mark.parametrize("ratio_level,aggregation", VARIANTS)
def test_variant_loss_and_grads_match_autograd(ratio_level, aggregation):
    import torch
    p, H, W, ids, old, ref, adv, coef = _loss_case(5, clip_noise=0.4)
    lo, hi, beta = 0.2, 0.28, 0.04
    out = O.loss_fwd_bwd(H, W, ids, p["loss_pos"], p["loss_cu"], adv, coef, old, ref, lo, hi, beta,
                         ratio_level=ratio_level, aggregation=aggregation)
    assert 0.0 < out["clip_frac"] < 1.0
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    lp = torch.tensor(p["loss_pos"]).long()
    y = torch.tensor(ids[p["loss_pos"] + 1]).long()
    logp = torch.log_softmax(Ht[lp] @ Wt.T, dim=-1).gather(1, y[:, None])[:, 0]
    total = torch.zeros((), dtype=torch.float64)
    for s in range(4):
        a, b = int(p["loss_cu"][s]), int(p["loss_cu"][s + 1])
        d = logp[a:b] - torch.tensor(old[a:b])
        rho = torch.exp(d.mean()).expand(b - a) if ratio_level == "sequence" else torch.exp(d)
        sur = torch.minimum(rho * adv[s], torch.clamp(rho, 1 - lo, 1 + hi) * adv[s])
        rh = torch.exp(torch.tensor(ref[a:b]) - logp[a:b])
        per_tok = -sur + beta * (rh - torch.log(rh) - 1)
        total = total + coef[s] * (per_tok.mean() if aggregation == "seq_mean" else per_tok.sum())
    total.backward()
    assert math.isclose(out["loss"], float(total.detach()), rel_tol=1e-12)
    assert np.allclose(out["dH"], Ht.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_sequence_ratio_is_the_geometric_mean_of_token_ratios():
    from fractions import Fraction
    # log-ratios that are exact binary fractions: exp(mean) = (prod of token ratios)^(1/C)
    cu = np.array([0, 3, 4, 8])
    d = np.array([0.5, -0.25, 0.125, 0.75, -0.5, 0.25, 0.0, -0.125])
    logp = -np.arange(1, 9) * 0.5
    old = logp - d
    adv = np.array([1.0, -2.0, 0.5])
    term, dterm, ell, kl, away = O.sequence_terms(logp, old, logp, cu, adv, 0.3, 0.3, 0.0, "sequence", "seq_mean")
    for s in range(3):
        a, b = cu[s], cu[s + 1]
        geo = math.prod(math.exp(x) for x in d[a:b]) ** (1.0 / (b - a))
        want = -min(geo * adv[s], min(max(geo, 0.7), 1.3) * adv[s])
        assert math.isclose(term[s], want, rel_tol=1e-12)
        assert np.all(ell[a:b] == ell[a])           # every token of a sequence carries the same term
    # sequence 1: ratio exp(0.75) = 2.117 > 1.3 with A < 0: not clipped away (the min keeps the unclipped branch)
    assert not away[3] and dterm[3] == -adv[1] * math.exp(0.75)
    # sequence 0: ratio exp(0.125) inside the interval; sequence 2: exp(-0.09375), inside too
    assert not away[:3].any() and not away[4:].any()
    # a sequence whose ratio leaves the interval on the penalised side gets no gradient
    term, dterm, _, _, away = O.sequence_terms(logp, old, logp, cu, -adv, 0.3, 0.3, 0.0, "sequence", "seq_mean")
    assert away[3] and dterm[3] == 0.0 and math.isclose(term[1], -(1.3 * 2.0), rel_tol=1e-12)


def test_variants_reduce_to_eq1_in_their_special_cases():
    rng = np.random.default_rng(8)
    # (a) one-token completions: a sequence ratio is its token ratio
    cu = np.arange(0, 8)
    logp, old, ref = -rng.random(7), -rng.random(7), -rng.random(7)
    adv = rng.normal(size=7)
    base = O.sequence_terms(logp, old, ref, cu, adv, 0.2, 0.2, 0.04, "token", "seq_mean")
    for rl, ag in VARIANTS[1:]:
        other = O.sequence_terms(logp, old, ref, cu, adv, 0.2, 0.2, 0.04, rl, ag)
        for x, y in zip(base, other):
            assert np.allclose(x, y, rtol=1e-14, atol=0)
    # (b) equal lengths C: the token sum is C times the token mean, for both ratio levels
    cu = np.arange(0, 13, 4)
    logp, old, ref = -rng.random(12), -rng.random(12), -rng.random(12)
    adv = rng.normal(size=3)
    for rl in ("token", "sequence"):
        m = O.sequence_terms(logp, old, ref, cu, adv, 0.2, 0.2, 0.04, rl, "seq_mean")
        t = O.sequence_terms(logp, old, ref, cu, adv, 0.2, 0.2, 0.04, rl, "token_sum")
        assert np.allclose(t[0], 4 * m[0], rtol=1e-14) and np.allclose(t[1], 4 * m[1], rtol=1e-14)
    # (c) coincident policies: ratio 1 at either level, term = -A (mean) or -A |o| (sum)
    cu = np.array([0, 2, 7])
    lp = -rng.random(7)
    for rl in ("token", "sequence"):
        term, dterm, _, kl, away = O.sequence_terms(lp, lp, lp, cu, np.array([0.5, -1.5]), 0.2, 0.2, 0.04, rl, "token_sum")
        assert np.allclose(term, [-0.5 * 2, 1.5 * 5], rtol=1e-14) and not away.any() and np.all(kl == 0)
        assert np.allclose(dterm, np.repeat([-0.5, 1.5], [2, 5]), rtol=1e-14)
    with pytest.raises(ValueError):
        O.sequence_terms(lp, lp, lp, cu, np.zeros(2), 0.2, 0.2, 0.0, "word", "seq_mean")


def test_token_norm_coef_makes_the_token_level_objective_unbiased():
    # unpruned: sum_i coef'_i sum_t l = (1/Q) sum_q (1 / tokens of the group) sum_{i,t} l
    rng = np.random.default_rng(31)
    Q, G = 2, 3
    cl = rng.integers(1, 6, size=(Q, G))
    tok_loss = [[rng.normal(size=cl[q, i]) for i in range(G)] for q in range(Q)]
    direct = np.mean([sum(x.sum() for x in tok_loss[q]) / cl[q].sum() for q in range(Q)])
    rewards = np.array([[1, 1, 1], [0, 1, 0]], dtype=np.float32)
    hist = np.array([0.3, 0.1], dtype=np.float32)
    s0 = O.select(rewards, None, None, None, 0.0, 0.0)
    c0 = O.token_norm_coef(s0["coef"], cl)
    assert math.isclose(sum(c0[q, i] * tok_loss[q][i].sum() for q in range(Q) for i in range(G)), direct, rel_tol=1e-12)
    # pruned: the expectation over all masks is the same number (lengths of pruned completions still count)
    r_q, r_o = 0.5, 0.375
    E = 0.0
    for prob, up, uc in _enumerate_masks(rewards, hist, r_q, r_o):
        s = O.select(rewards, hist, up, uc, r_q, r_o)
        c = O.token_norm_coef(s["coef"], cl)
        E += prob * sum(c[q, i] * tok_loss[q][i].sum() for q in range(Q) for i in range(G))
    assert math.isclose(E, direct, rel_tol=1e-10)


# ---------------------------------------------------------------- variance of the estimator (App. D)
def _direct_two_stage_variance(g, Pq, Po):
    """Var of gamma(q) gamma(o,q) g(q,o) by its definition: enumerate every (q, o) with its probability
    under the pruned densities."""
    Q, G = g.shape
    wq = (1 - Pq) / (1 - Pq).sum()
    m1 = m2 = 0.0
    for q in range(Q):
        wo = (1 - Po[q]) / (1 - Po[q]).sum()
        gam_q = (1 - Pq).mean() / (1 - Pq[q])
        for o in range(G):
            x = gam_q * ((1 - Po[q]).mean() / (1 - Po[q, o])) * g[q, o]
            m1 += wq[q] * wo[o] * x
            m2 += wq[q] * wo[o] * x * x
    return m1, m2 - m1 * m1


def test_variance_terms_match_the_definition_and_the_unpruned_case():
    rng = np.random.default_rng(41)
    Q, G = 5, 4
    g = rng.normal(size=(Q, G))
    # no pruning: weights are 1, every term is a plain population variance, and the law of total
    # variance makes the total the variance of g over all (q, o)
    v = O.variance_terms(g, np.zeros(Q), np.zeros((Q, G)))
    assert np.allclose(v["var_o"], g.var(axis=1), rtol=1e-12) and np.allclose(v["var_O"], g.var(axis=1), rtol=1e-12)
    assert math.isclose(v["egamma2"], 1.0, rel_tol=1e-15)
    assert math.isclose(v["total"], g.var(), rel_tol=1e-12) and math.isclose(v["bound"], g.var(), rel_tol=1e-12)
    # pruning: the decomposition equals the variance computed from the definition, and the estimator is unbiased
    Pq = np.array([0.5, 0.0, 0.5, 0.0, 0.0])
    Po = np.where(rng.random((Q, G)) < 0.5, 0.375, 0.0)
    v = O.variance_terms(g, Pq, Po)
    mean, var = _direct_two_stage_variance(g, Pq, Po)
    assert math.isclose(mean, g.mean(), rel_tol=1e-12)
    assert math.isclose(v["total"], var, rel_tol=1e-11)
    # prompt-level factor: bottom half pruned with r_q gives the closed form of Theorem D.1
    for r in (0.3, 0.7, 0.9):
        Pq = np.array([r] * 3 + [0.0] * 3)
        e = O.variance_terms(rng.normal(size=(6, 2)), Pq, np.zeros((6, 2)))["egamma2"]
        assert math.isclose(e, (1 - 0.5 * r) * (1 - 0.5 * r) / (1 - r), rel_tol=1e-12)


def test_variance_bound_holds_under_its_conditions_and_can_fail_without_them():
    rng = np.random.default_rng(43)
    Q, G = 6, 8
    Pq = np.array([0.7] * 3 + [0.0] * 3)
    Po = np.zeros((Q, G)); Po[:, :5] = 0.7
    # candidates carry small components (the paper's premise: low |A| means small gradient)
    g = rng.normal(size=(Q, G)); g[:, :5] *= 0.05; g[:3] *= 0.05
    v = O.variance_terms(g, Pq, Po)
    assert v["cond_o"].all() and v["cond_q"]
    assert np.all(v["var_o"] <= v["var_O"] + 1e-15)               # Eq. (completion-level bound)
    assert v["term1"] <= v["var_Q"] + 1e-15                       # Eq. (prompt-level bound)
    assert v["total"] <= v["bound"] + 1e-15                       # Theorem D.1
    # the reverse rule (prune the LARGE components) violates the conditions and the bound
    g2 = rng.normal(size=(Q, G)); g2[:, 5:] *= 0.05
    w = O.variance_terms(g2, np.zeros(Q), Po)
    assert not w["cond_o"].any() and np.all(w["var_o"] > w["var_O"]) and w["total"] > w["bound"]


def test_variance_terms_agree_with_sampling():
    # Monte-Carlo over the two-stage pruned sampling: mean g (unbiased) and the predicted variance
    rng = np.random.default_rng(47)
    Q, G = 4, 6
    g = rng.normal(size=(Q, G))
    Pq = np.array([0.5, 0.5, 0.0, 0.0])
    Po = np.zeros((Q, G)); Po[:, ::2] = 0.5
    v = O.variance_terms(g, Pq, Po)
    n = 400000
    qs = rng.choice(Q, size=n, p=(1 - Pq) / (1 - Pq).sum())
    cdf = np.cumsum((1 - Po) / (1 - Po).sum(axis=1, keepdims=True), axis=1)
    os_ = (rng.random(n)[:, None] > cdf[qs]).sum(axis=1)
    x = ((1 - Pq).mean() / (1 - Pq[qs])) * ((1 - Po).mean(axis=1)[qs] / (1 - Po[qs, os_])) * g[qs, os_]
    se = x.std() / math.sqrt(n)
    assert abs(x.mean() - g.mean()) < 5 * se
    assert abs(x.var() - v["total"]) < 0.02 * v["total"]
