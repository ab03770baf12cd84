"""Pins of the oracle's functions beyond the core pass: the other low-margin indicators of
Sec. 3.3 (probability ratio, fixed logit margin; Eq. 5-6), the committed sequence V_out of Alg. 1
with the cache rows that stay, the threshold sweep of the ablation in Sec. 4, and the
distributions of the top-2 statistics (appendix histogram figure).  CPU only.

Each test checks the oracle against something other than itself: a hand-worked example, a closed
form, a library routine (scipy softmax, numpy histogram / argmax), brute force, or an invariant.
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import softmax

from oracle import mars_ref as R

LR, PR, GAP = R.IND_LOGIT_RATIO, R.IND_PROB_RATIO, R.IND_LOGIT_GAP


def f32(a):
    return np.asarray(a, dtype=np.float32)


def run(z, tok, par, theta, T, u=None, q=None, indicator=LR):
    z = f32(z)
    if z.ndim == 2:
        z = z[None]
    tok = np.asarray(tok, np.int32).reshape(z.shape[0], -1)
    par = np.asarray(par, np.int32).reshape(z.shape[0], -1)
    if u is not None:
        u = f32(u).reshape(z.shape[0], -1)
    if q is not None:
        q = f32(q)
        if q.ndim == 2:
            q = q[None]
    return R.verify(z, tok, par, theta, T, u, q, indicator)


# ----------------------------------------------------------------------------- indicators, by hand
# One row z = (10, 9.5, 1): v(1) = 0, v(2) = 1, r = 0.95, Delta = 0.5,
# p2/p1 = exp(-0.5) = 0.60653 at T = 1 (and in greedy mode), exp(-1) = 0.36788 at T = 0.5.
# A chain root -> node 1 whose draft token is the runner-up (1): accepted iff the test passes;
# on rejection the greedy correction is v(1) = 0.
X_Z = [[10, 9.5, 1], [3, 2, 1]]
X_PAR = [-1, 0]


@pytest.mark.parametrize("indicator,theta,relaxed", [
    (LR, 0.9, True), (LR, 0.951, False), (LR, 0.96, False),
    (PR, 0.9, False), (PR, 0.61, False), (PR, 0.60, True), (PR, 0.3, True),
    (GAP, 0.6, True), (GAP, 0.5, False), (GAP, 0.25, False), (GAP, 0.5000001, True),
])
def test_indicator_worked_example_greedy(indicator, theta, relaxed):
    o = run(X_Z, [0, 1], X_PAR, theta, 0.0, indicator=indicator)
    st = o["stats"][0, 0]
    assert (st["id1"], st["id2"]) == (0, 1)
    assert st["ratio"] == pytest.approx(0.95, rel=1e-12)
    assert st["gap"] == 0.5
    assert st["prob_ratio"] == pytest.approx(math.exp(-0.5), rel=1e-14)
    assert bool(st["relax_ok"]) == relaxed and bool(st["relax_ok64"]) == relaxed
    assert o["accept_len"][0] == (1 if relaxed else 0)
    assert o["bonus_token"][0] == (0 if relaxed else 0)  # row1's v(1) = 0 as well as row0's
    assert int(o["decision"][0, 1]) == (2 if relaxed else 0)


def test_probability_ratio_uses_the_sampling_temperature():
    # T = 0.5: p2/p1 = exp(-0.5/0.5) = 0.36788; the runner-up draft is a deterministic accept
    # for theta = 0.36 and goes through Eq. 1 (u = 0.999 rejects: p(1) is about 0.27) for theta = 0.37.
    u = [0.0, 0.999, 0.5]
    lo = run(X_Z, [0, 1], X_PAR, 0.36, 0.5, u=u, indicator=PR)
    hi = run(X_Z, [0, 1], X_PAR, 0.37, 0.5, u=u, indicator=PR)
    assert lo["stats"][0, 0]["prob_ratio"] == pytest.approx(math.exp(-1.0), rel=1e-14)
    assert int(lo["decision"][0, 1]) == 2 and lo["accept_len"][0] == 1
    assert hi["accept_len"][0] == 0 and int(hi["decision"][0, 1]) == 0


def test_probability_ratio_equals_scipy_softmax_ratio():
    rng = np.random.default_rng(5)
    z = f32(rng.normal(0, 3, size=(3, 7, 50)))
    for T in (0.0, 0.5, 1.0, 2.0):
        st = R.row_stats(z, 0.5, T, PR)
        p = softmax(z.astype(np.float64) / (T if T > 0 else 1.0), axis=-1)
        ps = np.sort(p, axis=-1)
        want = ps[..., -2] / ps[..., -1]
        np.testing.assert_allclose(st["prob_ratio"], want, rtol=1e-12)
        assert np.array_equal(st["relax_ok64"].astype(bool), want > np.float64(np.float32(0.5)))
        far = np.abs(want - 0.5) > 1e-4
        assert np.array_equal(st["relax_ok"][far], st["relax_ok64"][far])


def test_margin_and_ratio_relations_eq5_eq6():
    # Eq. 5: r = 1 - Delta / z(1).  Eq. 6: r > theta  <=>  Delta < (1 - theta) z(1) on the positive domain,
    # i.e. the ratio test at theta is the fixed-margin test with a per-row threshold (1 - theta) z(1).
    rng = np.random.default_rng(6)
    z = f32(rng.normal(0, 3, size=(400, 1, 24)) + 6.0)
    theta = 0.8
    ratio = R.row_stats(z, theta, 0.0, LR)[:, 0]
    np.testing.assert_allclose(ratio["ratio"], 1.0 - ratio["gap"] / ratio["z1"], rtol=0, atol=1e-13)
    delta = f32((1.0 - np.float64(np.float32(theta))) * ratio["z1"])  # per-request threshold of the margin test
    gap = R.row_stats(z, delta, 0.0, GAP)[:, 0]
    clear = (ratio["z1"] > 0) & (np.abs(ratio["ratio"] - theta) > 1e-5)
    assert clear.sum() > 300
    assert np.array_equal(ratio["relax_ok"][clear], gap["relax_ok"][clear])
    assert 0 < ratio["relax_ok"][clear].sum() < clear.sum()


def test_scale_changes_probability_ratio_and_margin_but_not_logit_ratio():
    # Sec. 3.3: the logit ratio ignores the global scale of z; p2/p1 is squared and Delta doubled by z -> 2z.
    rng = np.random.default_rng(7)
    z = f32(rng.normal(2, 3, size=(2, 5, 40)))
    a = R.row_stats(z, 0.9, 1.0, LR)
    b = R.row_stats(f32(2.0 * z), 0.9, 1.0, LR)
    assert np.array_equal(a["ratio"], b["ratio"])
    np.testing.assert_allclose(b["prob_ratio"], a["prob_ratio"] ** 2, rtol=1e-12)
    assert np.array_equal(b["gap"], 2.0 * a["gap"])


def test_only_the_logit_ratio_needs_the_positive_domain():
    z = [[-1.0, -1.25, -5.0], [1, 0, 0]]
    assert run(z, [0, 1], X_PAR, 0.5, 0.0, indicator=LR)["accept_len"][0] == 0      # r = 1.25 but z(1) < 0
    assert run(z, [0, 1], X_PAR, 0.5, 0.0, indicator=GAP)["accept_len"][0] == 1     # Delta = 0.25 < 0.5
    assert run(z, [0, 1], X_PAR, 0.5, 0.0, indicator=PR)["accept_len"][0] == 1      # exp(-0.25) = 0.78 > 0.5


def test_margin_decision_is_one_fp32_subtraction():
    # z1 = 1 + 2^-23, z2 = 2^-24 (both fp32): exact Delta = 1 + 2^-24, which rounds to 1.0 (ties to even).
    # fp32 decision against delta = 1 + 2^-23: 1.0 < delta -> relax; and against delta = 1.0: not (1.0 < 1.0).
    z1, z2 = np.float32(1.0) + np.float32(2.0 ** -23), np.float32(2.0 ** -24)
    z = [[z1, z2, -4.0], [1, 0, 0]]
    st = run(z, [0, 1], X_PAR, 1.0, 0.0, indicator=GAP)["stats"][0, 0]
    assert st["gap"] == 1.0 + 2.0 ** -24
    assert st["relax_ok"] == 0 and st["relax_ok64"] == 0
    st = run(z, [0, 1], X_PAR, np.float32(1.0) + np.float32(2.0 ** -23), 0.0, indicator=GAP)["stats"][0, 0]
    assert st["relax_ok"] == 1 and st["relax_ok64"] == 1


def tree_depths(par):
    d = [0] * len(par)
    for i in range(1, len(par)):
        d[i] = d[par[i]] + 1
    return d


def greedy_bruteforce(z, tok, par, theta, indicator, T):
    """The three-way test of Sec. 3.4 with the low-margin predicate swapped, along every root path."""
    N = len(par)
    d = tree_depths(par)

    def low_margin(z1, z2):
        if indicator == LR:
            return z1 > 0 and z2 / z1 > theta
        if indicator == PR:
            return math.exp(-(z1 - z2) / (T if T > 0 else 1.0)) > theta
        return z1 - z2 < theta

    def edge_ok(k):
        row = z[par[k]].astype(np.float64)
        order = sorted(range(len(row)), key=lambda v: (-row[v], v))
        v1, v2 = order[0], order[1]
        if tok[k] == v1:
            return 1
        return 2 if tok[k] == v2 and low_margin(row[v1], row[v2]) else 0

    best, best_path = 0, []
    for n in range(1, N):
        path, k, ok = [], n, True
        while k != 0:
            path.append(k)
            ok = ok and edge_ok(k) != 0
            k = par[k]
        if ok and d[n] > d[best]:
            best, best_path = n, path[::-1]
    row = z[best]
    return best_path, min(range(len(row)), key=lambda v: (-row[v], v)), [edge_ok(k) for k in best_path]


ALL_TREES_4 = [[-1, 0, 0, 0], [-1, 0, 0, 1], [-1, 0, 0, 2], [-1, 0, 1, 0], [-1, 0, 1, 1], [-1, 0, 1, 2]]


@pytest.mark.parametrize("indicator,thetas", [(PR, (0.2, 0.5)), (GAP, (0.75, 1.5, 2.5))])
def test_bruteforce_greedy_other_indicators(indicator, thetas):
    rng = np.random.default_rng(80 + indicator)
    V, N = 3, 4
    grid = np.array([-2.0, 8.0, 9.0, 10.0], np.float32)  # gaps 0, 1, 2, 10, 11, 12; p2/p1 = e^-gap
    n = 0
    for par in ALL_TREES_4:
        for trial in range(8):
            z = grid[rng.integers(len(grid), size=(N, V))]
            for toks in itertools.product(range(V), repeat=N - 1):
                tok = [0] + list(toks)
                for theta in thetas:
                    o = run(z, tok, par, theta, 0.0, indicator=indicator)
                    path, bonus, codes = greedy_bruteforce(z, tok, par, theta, indicator, 0.0)
                    assert o["accept_len"][0] == len(path)
                    assert o["path_idx"][0][:len(path)].tolist() == path
                    assert o["bonus_token"][0] == bonus
                    assert [int(o["decision"][0][k]) for k in path] == codes
                    n += 1
    assert n == len(ALL_TREES_4) * 8 * 27 * len(thetas)


def test_indicator_that_never_fires_is_strict_verification():
    # theta >= 1 for the probability ratio (p2/p1 <= 1) and delta <= 0 for the margin (Delta >= 0) can never
    # relax; the pass must then equal the logit-ratio pass at theta > 1 in both modes.
    rng = np.random.default_rng(9)
    B, N, V = 3, 6, 12
    z = f32(rng.normal(0, 2, size=(B, N, V)))
    par = np.tile(np.array([-1, 0, 0, 1, 1, 3], np.int32), (B, 1))
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    u = f32(rng.random((B, N + 1)))
    for T in (0.0, 1.0):
        base = R.verify(z, tok, par, 2.0, T, u, None, LR)
        for ind, th in ((PR, 1.0), (GAP, 0.0), (GAP, -1.0)):
            o = R.verify(z, tok, par, th, T, u, None, ind)
            for key in ("accept_len", "path_idx", "bonus_token", "decision", "accept_mask"):
                assert np.array_equal(o[key], base[key]), (T, ind, key)


# ----------------------------------------------------------------------------- committed sequence
# Alg. 1 on the chain of the core worked example (V = 5, three drafts 2, 0, 3): node 1 relaxed, node 2
# exact, node 3 rejected with correction v(1) of row 2 = 2.  V_out = (2, 0, 2); the cache keeps the
# rows of the root and of nodes 1 and 2.
W1_Z = [[1, 10, 9.5, 2, -3], [8, 1, 0, 5, 2], [2, 3, 20, 14, 1], [0, 0, 0, 7, 1]]
W1_PAR = [-1, 0, 1, 2]


def test_commit_worked_example_chain():
    o = run(W1_Z, [4, 2, 0, 3], W1_PAR, 0.9, 0.0)
    c = R.commit([[4, 2, 0, 3]], o["accept_len"], o["path_idx"], o["bonus_token"])
    assert c["out_tokens"].tolist() == [[2, 0, 2, -1]]
    assert c["out_len"].tolist() == [3]
    assert c["keep_offsets"].tolist() == [0, 3]
    assert c["keep_rows"].tolist() == [0, 1, 2, -1]


def test_commit_tree_batch_by_hand():
    # Two requests, N = 5.  Request 0 accepted path 2 -> 4 (tokens 7, 9), bonus 11.  Request 1 nothing
    # accepted, correction token 5.  Rows are numbered b*N + node.
    tok = [[0, 6, 7, 8, 9], [0, 1, 2, 3, 4]]
    c = R.commit(tok, [2, 0], [[2, 4, -1, -1, -1], [-1, -1, -1, -1, -1]], [11, 5])
    assert c["out_tokens"].tolist() == [[7, 9, 11, -1, -1], [5, -1, -1, -1, -1]]
    assert c["out_len"].tolist() == [3, 1]
    assert c["keep_offsets"].tolist() == [0, 3, 4]
    assert c["keep_rows"].tolist() == [0, 2, 4, 5] + [-1] * 6


def test_commit_full_acceptance_has_k_plus_one_tokens():
    c = R.commit([[0, 3, 4]], [2], [[1, 2, -1]], [9])
    assert c["out_tokens"].tolist() == [[3, 4, 9]] and c["out_len"].tolist() == [3]
    assert c["keep_rows"].tolist() == [0, 1, 2]


def test_commit_strict_greedy_chain_is_the_targets_own_continuation():
    # With theta > 1 every committed token, accepted or corrected, is the arg-max of the row it was
    # checked against, so V_out is the target's greedy continuation along the chain (numpy argmax).
    rng = np.random.default_rng(10)
    B, N, V = 40, 7, 6
    z = f32(rng.normal(0, 2, size=(B, N, V)))
    par = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    top = z.argmax(-1)
    tok = np.zeros((B, N), np.int32)
    tok[:, 1:] = np.where(rng.random((B, N - 1)) < 0.7, top[:, :-1], rng.integers(0, V, size=(B, N - 1)))
    o = R.verify(z, tok, par, 2.0, 0.0)
    c = R.commit(tok, o["accept_len"], o["path_idx"], o["bonus_token"])
    assert 1 < c["out_len"].mean() < N
    for b in range(B):
        L = c["out_len"][b]
        assert c["out_tokens"][b, :L].tolist() == top[b, :L].tolist()
        assert (c["out_tokens"][b, L:] == -1).all()


def test_commit_keep_rows_against_mask():
    # The kept rows are exactly the rows flagged in accept_mask (root included), in request-major order;
    # on a path node indices increase with depth, so path order is index order.
    rng = np.random.default_rng(11)
    B, N, V = 9, 12, 8
    z = f32(rng.normal(0, 2, size=(B, N, V)))
    par = np.zeros((B, N), np.int32)
    par[:, 0] = -1
    for b in range(B):
        for i in range(1, N):
            par[b, i] = rng.integers(0, i)
    top = z.argmax(-1)
    tok = np.zeros((B, N), np.int32)
    for b in range(B):
        for i in range(1, N):
            tok[b, i] = top[b, par[b, i]] if rng.random() < 0.8 else rng.integers(0, V)
    u = f32(rng.random((B, N + 1)))
    for T in (0.0, 1.0):
        o = R.verify(z, tok, par, 0.9, T, u)
        c = R.commit(tok, o["accept_len"], o["path_idx"], o["bonus_token"])
        flat = np.flatnonzero(o["accept_mask"].reshape(-1))
        total = c["keep_offsets"][-1]
        assert total == len(flat) == int(o["accept_len"].sum()) + B
        assert c["keep_rows"][:total].tolist() == flat.tolist()
        assert (c["keep_rows"][total:] == -1).all()
        assert np.array_equal(np.diff(c["keep_offsets"]), c["out_len"])
        assert np.array_equal(c["out_len"], o["accept_len"] + 1)


def test_commit_rejects_impossible_lengths():
    with pytest.raises(ValueError):
        R.commit([[0, 1]], [2], [[1, -1]], [0])


# ----------------------------------------------------------------------------- threshold sweep
def test_sweep_rows_equal_single_runs_and_shrink_with_theta():
    rng = np.random.default_rng(12)
    B, N, V = 6, 8, 16
    z = f32(rng.normal(0, 1, size=(B, N, V)) + 8.0)       # top-2 ratios near 1: theta matters
    par = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    order = np.argsort(-z, axis=-1, kind="stable")
    tok = np.zeros((B, N), np.int32)
    tok[:, 1:] = order[:, :-1, 1]                           # every draft is the runner-up of its parent's row
    thetas = f32(np.tile(np.array([0.84, 0.88, 0.92, 0.96, 1.5])[:, None], (1, B)))
    sw = R.verify_sweep(z, tok, par, thetas, 0.0)
    assert sw["accept_len"].shape == (5, B)
    one = R.verify(z, tok, par, thetas[2], 0.0)
    assert np.array_equal(sw["accept_len"][2], one["accept_len"])
    assert np.array_equal(sw["path_idx"][2], one["path_idx"])
    assert (np.diff(sw["accept_len"], axis=0) <= 0).all()   # fewer relaxations as theta rises
    assert (sw["accept_len"][-1] == 0).all()                # strict: a runner-up is never accepted
    assert sw["accept_len"][0].sum() > 0


# ----------------------------------------------------------------------------- distributions of the statistics
def test_margin_stats_rows_by_hand():
    # rows: (10, 9.5, 1) -> r 0.95, p2/p1 e^-0.5;  (4, 1, 0) -> 0.25, e^-3;  (-1, -2, -3) -> z1 < 0;
    # (0, -1, -2) -> z1 = 0.  Cells of width 0.1 on [0, 1) for both ratios, width 5 on [0, 20) for z1.
    z = f32([[[10, 9.5, 1], [4, 1, 0], [-1, -2, -3], [0, -1, -2]]])
    m = R.margin_stats(z, 0.9, 1.0, ((0, 20), (0, 1), (0, 1)), (4, 10, 10))
    assert m["rows"]["z1"].tolist() == [[10, 4, -1, 0]]
    np.testing.assert_allclose(m["rows"]["ratio"][0, :2], [0.95, 0.25], rtol=1e-15)
    np.testing.assert_allclose(m["rows"]["prob_ratio"][0], np.exp([-0.5, -3.0, -1.0, -1.0]), rtol=1e-15)
    assert m["hist_z1"].tolist() == [1, 2, 0, 1, 0, 0]         # -1 below; 0 and 4 in [0,5); 10 in [10,15)
    assert m["hist_ratio"].tolist() == [0, 0, 0, 1, 0, 0, 0, 0, 0, 0, 1, 0]   # only the two rows with z1 > 0
    assert m["hist_prob"].tolist() == [0, 1, 0, 0, 2, 0, 0, 1, 0, 0, 0, 0]    # .0498 | .3679 x2 | .6065
    assert m["summary"].tolist() == [4, 1, 2, 1]               # rows, z1 < 0, z1 <= 0, low margin at theta
    # a tie: p2/p1 = 1 sits on the upper end of [0, 1) and is counted above it
    m = R.margin_stats(f32([[[3, 3, 0]]]), 0.9, 1.0, ((0, 20), (0, 1), (0, 1)), (4, 10, 10))
    assert m["hist_prob"][-1] == 1 and m["hist_ratio"][-1] == 1 and m["edge_dist"][0, 0] == 0.0


@pytest.mark.parametrize("T", [0.0, 0.7])
def test_margin_stats_equal_numpy_histogram(T):
    rng = np.random.default_rng(13)
    B, N, V = 8, 25, 300
    z = f32(rng.normal(0, 3, size=(B, N, V)))
    z[0, :5] -= 20.0                                           # a few rows with a negative top-1
    ranges, bins = ((-5, 25), (0.5, 1.0), (0.0, 1.0)), (30, 25, 20)
    m = R.margin_stats(z, 0.9, T, ranges, bins)
    s = np.sort(z.astype(np.float64), axis=-1)
    z1, z2 = s[..., -1].ravel(), s[..., -2].ravel()
    pr = np.exp(-(z1 - z2) / (float(np.float32(T)) if T > 0 else 1.0))   # the temperature is an fp32 scalar
    pos = z1 > 0

    def clear(x, lo, hi, nb, tol=1e-6):                        # samples that are not on a cell boundary
        t = (x - lo) * nb / (hi - lo)
        return np.abs(t - np.rint(t)) > tol

    for name, x, (lo, hi), nb in (("hist_z1", z1, ranges[0], bins[0]), ("hist_ratio", (z2 / z1)[pos], ranges[1], bins[1]),
                                  ("hist_prob", pr, ranges[2], bins[2])):
        assert clear(x, lo, hi, nb).all()
        inner, _ = np.histogram(x, bins=nb, range=(lo, hi))
        inner[-1] -= (x == hi).sum()                           # numpy closes the last cell; here [lo, hi) is half open
        want = np.concatenate([[(x < lo).sum()], inner, [(x >= hi).sum()]])
        assert m[name].tolist() == want.tolist(), name
        assert m[name].sum() == len(x)
    assert m["summary"].tolist() == [B * N, int((z1 < 0).sum()), int((z1 <= 0).sum()),
                                     int((pos & (z2 / np.where(pos, z1, 1) > np.float64(np.float32(0.9)))).sum())]
    assert m["summary"][1] >= 5
    np.testing.assert_allclose(m["edge_dist"].ravel(),
                               np.abs(pr * bins[2] - np.rint(pr * bins[2])), atol=1e-9)
