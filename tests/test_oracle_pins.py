"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU or the HIP library.  The checkers in this file are
written independently of oracle/mars_ref.c (numpy sorting, explicit path enumeration,
a textbook speculative-sampling routine), so that a dropped term, a wrong sign or index,
or a transposed operand in the oracle fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp
from scipy.stats import chi2

from oracle import mars_ref as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f32(a):
    return np.asarray(a, dtype=np.float32)


def run(z, tok, par, theta, T, u=None, q=None):
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
    return R.verify(z, tok, par, theta, T, u, q)


# ----------------------------------------------------------------------------- hand-worked examples
# W1 (Alg. 1 on a chain, V=5, three drafts).  Rows and their top-2 by inspection:
#   row0 = (1, 10, 9.5, 2, -3): v(1)=1, v(2)=2, r = 9.5/10 = 0.95
#   row1 = (8, 1, 0, 5, 2)    : v(1)=0, v(2)=3, r = 5/8   = 0.625
#   row2 = (2, 3, 20, 14, 1)  : v(1)=2, v(2)=3, r = 14/20 = 0.70
#   row3 = (0, 0, 0, 7, 1)    : v(1)=3
# drafts (2, 0, 3): node 1 is the runner-up of row0 with 0.95 > 0.9 -> relaxed accept;
# node 2 equals v(1) of row1 -> exact; node 3 is the runner-up of row2 but 0.70 <= 0.9 -> reject,
# emit v(1) of row2 = 2.  Committed: 2, 0, 2 (tau = 3).
W1_Z = [[1, 10, 9.5, 2, -3], [8, 1, 0, 5, 2], [2, 3, 20, 14, 1], [0, 0, 0, 7, 1]]
W1_PAR = [-1, 0, 1, 2]


def test_w1_greedy_chain_relaxed_then_exact_then_reject():
    o = run(W1_Z, [0, 2, 0, 3], W1_PAR, 0.9, 0.0)
    assert o["accept_len"].tolist() == [2]
    assert o["path_idx"].tolist() == [[1, 2, -1, -1]]
    assert o["accept_mask"].tolist() == [[1, 1, 1, 0]]
    assert o["decision"].tolist() == [[0, 2, 1, 0]]
    assert o["bonus_token"].tolist() == [2]
    st = o["stats"][0]
    assert st["id1"].tolist() == [1, 0, 2, 3] and st["id2"].tolist()[:3] == [2, 3, 3]
    np.testing.assert_allclose(st["ratio"][:3], [0.95, 0.625, 0.70], rtol=1e-12)


def test_w1_theta_above_one_is_strict():
    o = run(W1_Z, [0, 2, 0, 3], W1_PAR, 1.5, 0.0)
    assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [1]
    assert o["decision"].sum() == 0


def test_w1_all_accepted_gives_bonus_and_tau_k_plus_1():
    # third draft = v(1) of row2: everything accepted, bonus = v(1) of row3, tau = K+1 = 4
    o = run(W1_Z, [0, 2, 0, 2], W1_PAR, 0.9, 0.0)
    assert o["accept_len"].tolist() == [3] and o["bonus_token"].tolist() == [3]
    assert o["path_idx"].tolist() == [[1, 2, 3, -1]]


def test_w2_paper_fig2_ratios():
    lines = [l.split() for l in open(os.path.join(GOLDEN, "fig2_ratios.txt")) if l.strip() and l[0] != "#"]
    theta = float(lines[0][1])
    for r, outcome in lines[1:]:
        r = float(r)
        z = [[10.0, 10.0 * r, 1.0], [1.0, 2.0, 3.0]]
        o = run(z, [0, 1], [-1, 0], theta, 0.0)  # the draft token is the runner-up (id 1)
        if outcome == "accept":
            assert o["accept_len"].tolist() == [1] and o["decision"][0, 1] == 2
            assert o["bonus_token"].tolist() == [2]
        else:
            assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [0]  # top-1 emitted


# W3: greedy tree, the longest path runs through a relaxed branch.
#   parents (-1,0,0,1,2,4); row0 = (0,20,19,1,2,3): v(1)=1, v(2)=2, r=0.95; tok1=1 (exact), tok2=2 (relaxed)
#   row1 = (9,1,2,3,4,5): top-2 ids (0,5); tok3 = 3 -> rejected
#   row2 = (1,2,3,4,10,5): v(1)=4; tok4 = 4 exact.   row4 = (7,1,1,1,1,1): v(1)=0; tok5 = 0 exact
#   row5 = (1,1,8,1,1,1): v(1)=2 -> bonus.   Deepest accepted node: 5 (depth 3) via 2,4,5.
W3_Z = [[0, 20, 19, 1, 2, 3], [9, 1, 2, 3, 4, 5], [1, 2, 3, 4, 10, 5], [5, 4, 3, 2, 1, 0],
        [7, 1, 1, 1, 1, 1], [1, 1, 8, 1, 1, 1]]
W3_PAR = [-1, 0, 0, 1, 2, 4]
W3_TOK = [0, 1, 2, 3, 4, 0]


def test_w3_greedy_tree_longest_path_through_relaxed_branch():
    o = run(W3_Z, W3_TOK, W3_PAR, 0.9, 0.0)
    assert o["accept_len"].tolist() == [3]
    assert o["path_idx"][0].tolist() == [2, 4, 5, -1, -1, -1]
    assert o["accept_mask"][0].tolist() == [1, 0, 1, 0, 1, 1]
    assert o["decision"][0].tolist() == [0, 0, 2, 0, 1, 1]
    assert o["bonus_token"].tolist() == [2]
    o = run(W3_Z, W3_TOK, W3_PAR, 1.5, 0.0)  # strict: only node 1 survives
    assert o["accept_len"].tolist() == [1] and o["path_idx"][0, 0] == 1
    assert o["bonus_token"].tolist() == [0]  # v(1) of row1


def test_w3_depth_tie_goes_to_lowest_node():
    o = run(W3_Z[:3], W3_TOK[:3], W3_PAR[:3], 0.9, 0.0)
    assert o["accept_len"].tolist() == [1] and o["path_idx"][0, 0] == 1
    assert o["bonus_token"].tolist() == [0]


# W4: sampling, one-hot q, V=3, T=1.  z_root = ln(6,3,1) -> p = (0.6,0.3,0.1); r = ln3/ln6 = 0.613: no relaxation.
#   child 1: token 1, u=0.5 >= 0.3 -> reject; residual (0.6,0,0.1)/0.7 = (6/7, 0, 1/7)
#   child 2: token 2, u=0.1 < 1/7 -> accept (code 3).  Row 2 = ln(1,3,1) -> p = (0.2,0.6,0.2), CDF (0.2,0.8,1.0)
#   u_bonus = 0.75 -> token 1.
def test_w4_sampling_one_hot_two_siblings():
    z = np.log(np.array([[6, 3, 1], [1, 1, 1], [1, 3, 1]], np.float64))
    o = run(z, [0, 1, 2], [-1, 0, 0], 0.9, 1.0, u=[0, 0.5, 0.1, 0.75])
    assert o["accept_len"].tolist() == [1] and o["path_idx"][0].tolist() == [2, -1, -1]
    assert o["decision"][0].tolist() == [0, 0, 3] and o["bonus_token"].tolist() == [1]
    d = o["diag"][0]
    assert d["residual_passes"] == 1 and d["last_node"] == 2
    assert abs(d["last_residual_norm"] - 0.7) < 1e-6
    assert abs(d["min_accept_margin"] - (1 / 7 - 0.1)) < 1e-6
    assert abs(d["bonus_prob"] - 0.6) < 1e-6
    # variant: u_2 = 0.2 >= 1/7 -> both rejected; f = (1,0,0): token 0 whatever the last uniform is
    for ub in (0.0, 0.3, 0.999):
        o = run(z, [0, 1, 2], [-1, 0, 0], 0.9, 1.0, u=[0, 0.5, 0.2, ub])
        assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [0]
        assert abs(o["diag"][0]["last_residual_norm"] - 6 / 7) < 1e-6


# W5: dense q on a chain.  p = (0.5,0.3,0.2), q = (0.2,0.6,0.2).
#   token 1: a = 0.3/0.6 = 0.5; u = 0.6 -> reject; max(0,p-q) = (0.3,0,0), Z = 0.3 -> token 0
#   token 0: a = min(1, 0.5/0.2) = 1 -> accept for any u
def test_w5_dense_q_chain():
    z = np.log(np.array([[0.5, 0.3, 0.2], [0.2, 0.3, 0.5]]))
    q = np.array([[0.2, 0.6, 0.2], [1 / 3, 1 / 3, 1 / 3]])
    o = run(z, [0, 1], [-1, 0], 2.0, 1.0, u=[0, 0.6, 0.9], q=q)
    assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [0]
    assert abs(o["diag"][0]["last_residual_norm"] - 0.3) < 1e-6
    assert abs(o["diag"][0]["min_accept_margin"] - 0.1) < 1e-6
    o = run(z, [0, 0], [-1, 0], 2.0, 1.0, u=[0, 0.999, 0.6], q=q)
    assert o["accept_len"].tolist() == [1] and o["decision"][0, 1] == 3
    assert o["bonus_token"].tolist() == [2]  # row 1: CDF (0.2, 0.5, 1.0), u = 0.6 -> token 2


#   two dense siblings: p = (0.4,0.35,0.25), q = (0.1,0.3,0.6)
#   A (token 2): a = 0.25/0.6 = 0.41667 -> rejected with u = 0.5; g = (0.3,0.05,0), Z1 = 0.35, f1 = (6/7,1/7,0)
#   B (token 1): a = (1/7)/0.3 = 0.47619 -> rejected with u = 0.9; g = (6/7-0.1, 0, 0), Z2 = 0.757143 -> token 0
def test_w5_two_dense_siblings():
    z = np.log(np.array([[0.4, 0.35, 0.25], [1, 1, 1], [1, 1, 1]], np.float64))
    q = np.array([[0.1, 0.3, 0.6], [1 / 3] * 3, [1 / 3] * 3])
    o = run(z, [0, 2, 1], [-1, 0, 0], 2.0, 1.0, u=[0, 0.5, 0.9, 0.3], q=q)
    d = o["diag"][0]
    assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [0]
    assert d["residual_passes"] == 2
    assert abs(d["last_residual_norm"] - (6 / 7 - 0.1)) < 1e-6
    assert abs(d["min_accept_margin"] - min(0.5 - 0.25 / 0.6, 0.9 - (1 / 7) / 0.3)) < 1e-6
    # B accepted when its uniform is below 0.47619
    o = run(z, [0, 2, 1], [-1, 0, 0], 2.0, 1.0, u=[0, 0.5, 0.47, 0.3], q=q)
    assert o["accept_len"].tolist() == [1] and o["path_idx"][0, 0] == 2


# W6: relaxation under sampling.  z = (10, 9.5, 0), T = 1, draft = runner-up, u = 0.999.
#   theta = 0.9: r = 0.95 -> accepted (code 2) whatever u is.
#   theta = 2  : p(1) = e^-0.5 / (1 + e^-0.5 + e^-10) = 0.377530 -> rejected;
#                one-hot residual (0.999955, 0, 0.000045) -> token 0 for u = 0.5
def test_w6_relaxation_in_sampling_mode():
    z = [[10, 9.5, 0], [0, 1, 2]]
    o = run(z, [0, 1], [-1, 0], 0.9, 1.0, u=[0, 0.999, 0.5])
    assert o["accept_len"].tolist() == [1] and o["decision"][0, 1] == 2
    o = run(z, [0, 1], [-1, 0], 2.0, 1.0, u=[0, 0.999, 0.5])
    assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [0]
    S = 1 + math.exp(-0.5) + math.exp(-10)
    assert abs(o["stats"][0, 0]["sum_exp"] - S) < 1e-12
    assert abs(o["diag"][0]["min_accept_margin"] - (0.999 - math.exp(-0.5) / S)) < 1e-6
    assert abs(o["diag"][0]["bonus_prob"] - (1 / S) / (1 - math.exp(-0.5) / S)) < 1e-9
    # the top-1 draft is NOT an automatic accept when sampling: p(0) = 0.62244 < u
    o = run(z, [0, 0], [-1, 0], 0.9, 1.0, u=[0, 0.7, 0.5])
    assert o["accept_len"].tolist() == [0]
    o = run(z, [0, 0], [-1, 0], 0.9, 1.0, u=[0, 0.6, 0.5])
    assert o["accept_len"].tolist() == [1] and o["decision"][0, 1] == 3


def test_temperature_scales_logits_in_softmax():
    # z = (2,1,0), T = 0.5: S = 1 + e^-2 + e^-4 = 1.153651, p = (0.866813, 0.117310, 0.015876)
    st = R.row_stats(f32([[[2, 1, 0]]]), 0.9, 0.5)[0, 0]
    assert abs(st["sum_exp"] - (1 + math.exp(-2) + math.exp(-4))) < 1e-12
    assert abs(1 / st["sum_exp"] - 0.866813) < 1e-6
    z = [[2, 1, 0], [0, 0, 0]]
    # accept token 1 iff u < 0.117310
    assert run(z, [0, 1], [-1, 0], 2.0, 0.5, u=[0, 0.1172, 0.5])["accept_len"].tolist() == [1]
    assert run(z, [0, 1], [-1, 0], 2.0, 0.5, u=[0, 0.1174, 0.5])["accept_len"].tolist() == [0]


# ----------------------------------------------------------------------------- storage types, ties, domain
def test_bf16_widening_known_bit_patterns():
    # 0x3F80 = 1.0, 0x4049 = 3.140625, 0xC000 = -2.0, 0x41A0 = 20.0, 0xFF80 = -inf
    bits = np.array([[[0x3F80, 0x4049, 0xC000, 0x41A0, 0xFF80]]], np.uint16)
    st = R.row_stats(bits, 0.5, 1.0)[0, 0]
    assert (st["z1"], st["id1"], st["z2"], st["id2"]) == (20.0, 3, 3.140625, 1)
    S = 1 + math.exp(3.140625 - 20) + math.exp(1 - 20) + math.exp(-2 - 20) + 0.0
    assert abs(st["sum_exp"] - S) < 1e-15


def test_ties_value_desc_index_asc():
    st = R.row_stats(f32([[[3, 7, 7, 1, 7], [5, 2, 4, 4, 1], [1, 1, 1, 1, 1]]]), 0.9, 0.0)[0]
    assert st["id1"].tolist() == [1, 0, 0] and st["id2"].tolist() == [2, 2, 1]
    assert st["z2"].tolist() == [7, 4, 1] and st["ratio"][0] == 1.0 and st["relax_ok"][0] == 1


def test_no_relaxation_outside_positive_domain():
    # z1 < 0: the raw ratio is > 1 but relaxation is off (Sec. 3.3 assumes positive top logits);
    # z1 == 0 likewise; z2 < 0 < z1 gives a negative ratio.
    st = R.row_stats(f32([[[-1, -1.05, -9], [0, -1, -2], [4, -3.9, -8]]]), 0.9, 0.0)[0]
    assert st["relax_ok"].tolist() == [0, 0, 0] and st["relax_ok64"].tolist() == [0, 0, 0]
    o = run([[-1, -1.05, -9], [1, 2, 3]], [0, 1], [-1, 0], 0.9, 0.0)
    assert o["accept_len"].tolist() == [0] and o["bonus_token"].tolist() == [0]


def test_masked_tokens_minus_inf():
    z = f32([[[-np.inf, 2.0, -np.inf, 1.0], [0, 0, 0, 0]]])
    o = R.verify(z, np.array([[0, 3]], np.int32), np.array([[-1, 0]], np.int32), 0.4, 1.0,
                 f32([[0, 0.2, 0.9]]))
    st = o["stats"][0, 0]
    assert (st["id1"], st["id2"]) == (1, 3) and st["relax_ok"] == 1
    assert abs(st["sum_exp"] - (1 + math.exp(-1))) < 1e-12
    assert o["decision"][0, 1] == 2


def test_request_status_and_fallback():
    z = f32([[[1, 5, 2], [3, 1, 0], [0, 0, 9]]])
    bad_tree = R.verify(z, np.array([[0, 1, 0]], np.int32), np.array([[-1, 1, 0]], np.int32), 0.9, 0.0)
    assert bad_tree["request_status"].tolist() == [1]
    assert bad_tree["accept_len"].tolist() == [0] and bad_tree["bonus_token"].tolist() == [1]
    assert bad_tree["path_idx"][0].tolist() == [-1, -1, -1] and bad_tree["accept_mask"][0].tolist() == [1, 0, 0]
    bad_root = R.verify(z, np.array([[0, 1, 0]], np.int32), np.array([[0, 0, 1]], np.int32), 0.9, 0.0)
    assert bad_root["request_status"].tolist() == [1]
    bad_tok = R.verify(z, np.array([[0, 3, 0]], np.int32), np.array([[-1, 0, 1]], np.int32), 0.9, 0.0)
    assert bad_tok["request_status"].tolist() == [2] and bad_tok["bonus_token"].tolist() == [1]
    neg_tok = R.verify(z, np.array([[-7, -1, 0]], np.int32), np.array([[-1, 0, 1]], np.int32), 0.9, 0.0)
    assert neg_tok["request_status"].tolist() == [2]  # the root token itself is never read
    with pytest.raises(ValueError):
        R.verify(z, np.zeros((1, 3), np.int32), np.array([[-1, 0, 1]], np.int32), 0.9, -1.0)
    with pytest.raises(ValueError):
        R.verify(z, np.zeros((1, 3), np.int32), np.array([[-1, 0, 1]], np.int32), 0.9, 1.0, None)


# ----------------------------------------------------------------------------- library special cases
def random_logits(rng, shape, ties=False):
    z = (rng.standard_normal(shape) * 3).astype(np.float32)
    if ties:
        z = np.round(z * 2) / 2  # a coarse grid: many exact ties
    return z.astype(np.float32)


@pytest.mark.parametrize("ties", [False, True])
def test_row_stats_equal_numpy_sort_and_scipy_logsumexp(ties):
    rng = np.random.default_rng(11)
    B, N, V = 3, 5, 257
    z = random_logits(rng, (B, N, V), ties)
    T = float(np.float32(0.7))  # the temperature crosses the boundary as an fp32 scalar
    st = R.row_stats(z, 0.9, T)
    for b in range(B):
        for i in range(N):
            row = z[b, i].astype(np.float64)
            order = np.lexsort((np.arange(V), -row))  # value descending, index ascending
            assert st[b, i]["id1"] == order[0] and st[b, i]["id2"] == order[1]
            assert st[b, i]["z1"] == row[order[0]] and st[b, i]["z2"] == row[order[1]]
            lse = logsumexp(row / T)
            assert abs(math.log(st[b, i]["sum_exp"]) + row[order[0]] / T - lse) < 1e-12


def test_ratio_test_equals_adaptive_margin_form():
    # Eq. 6: for z1 > 0, r > theta  <=>  z1 - z2 < (1 - theta) * z1.  Checked in fp64 on rows whose
    # ratio is at least 1e-4 away from theta, where the fp32 decision must agree too.
    rng = np.random.default_rng(5)
    V = 64
    z = random_logits(rng, (1, 4000, V))
    z[0, :, 0] = rng.uniform(5, 30, 4000).astype(np.float32)
    z[0, :, 1] = (z[0, :, 0] * rng.uniform(0.8, 1.0, 4000)).astype(np.float32)
    for theta in (0.85, 0.9, 0.95):
        st = R.row_stats(z, theta, 0.0)[0]
        th = float(np.float32(theta))
        z1, z2 = st["z1"], st["z2"]
        far = (z1 > 0) & (np.abs(z2 / z1 - th) >= 1e-4)
        margin_form = (z1 - z2) < (1.0 - th) * z1
        assert far.sum() > 3000
        assert np.array_equal(st["relax_ok64"][far] == 1, margin_form[far])
        assert np.array_equal(st["relax_ok"][far], st["relax_ok64"][far])
        assert 0.2 < st["relax_ok"].mean() < 0.8


def test_fp32_ratio_decision_at_the_boundary():
    # 18/20 rounds to 0.9f in fp32, which is not greater than theta = 0.9f; in fp64, 0.9 > (double)0.9f.
    st = R.row_stats(f32([[[20, 18, 0]]]), 0.9, 0.0)[0, 0]
    assert st["relax_ok"] == 0 and st["relax_ok64"] == 1


# ----------------------------------------------------------------------------- theta > 1: the standard rules
def tree_depths(par):
    d = np.zeros(len(par), int)
    for i in range(1, len(par)):
        d[i] = d[par[i]] + 1
    return d


def strict_greedy_reference(z, tok, par):
    """Plain arg-max matching on a tree: enumerate every node's root path, keep those whose
    every edge carries the arg-max of the parent's row, take the deepest (lowest index on ties)."""
    N = len(par)
    d = tree_depths(par)
    best, best_path = 0, []
    for n in range(1, N):
        path, k, ok = [], n, True
        while k != 0:
            path.append(k)
            ok &= tok[k] == int(np.argmax(z[par[k]]))
            k = par[k]
        if ok and d[n] > d[best]:
            best, best_path = n, path[::-1]
    return best_path, int(np.argmax(z[best]))


def random_tree(rng, N, max_children=3):
    par = [-1]
    for i in range(1, N):
        while True:
            p = int(rng.integers(i))
            if par.count(p) < max_children:
                break
        par.append(p)
    return par


def test_theta_above_one_greedy_equals_argmax_matching():
    rng = np.random.default_rng(21)
    for trial in range(200):
        N, V = int(rng.integers(2, 12)), int(rng.integers(2, 9))
        par = random_tree(rng, N)
        z = random_logits(rng, (N, V), ties=trial % 2 == 0)
        tok = [0] + [int(np.argmax(z[par[i]])) if rng.random() < 0.7 else int(rng.integers(V)) for i in range(1, N)]
        o = run(z, tok, par, 1.01, 0.0)
        path, bonus = strict_greedy_reference(z, tok, par)
        assert o["accept_len"][0] == len(path)
        assert o["path_idx"][0][:len(path)].tolist() == path and (o["path_idx"][0][len(path):] == -1).all()
        assert o["bonus_token"][0] == bonus
        assert set(np.unique(o["decision"])) <= {0, 1}


def textbook_speculative_sampling(z, q, tok, u, T):
    """Chain speculative sampling as in the cited rejection-sampling scheme: accept x_i with
    probability min(1, p_i(x)/q_i(x)); at the first rejection draw from norm(max(0, p - q));
    if all are accepted draw from the last row.  Draws use inverse CDF in index order."""
    K = len(tok) - 1
    accepted = 0
    for i in range(1, K + 1):
        p = np.exp(z[i - 1].astype(np.float64) / T)
        p /= p.sum()
        x = tok[i]
        if u[i] < min(1.0, p[x] / q[i - 1][x]):
            accepted += 1
            continue
        res = np.maximum(p - q[i - 1], 0)
        res /= res.sum()
        cdf = np.cumsum(res)
        return accepted, int(np.searchsorted(cdf, u[K + 1] * cdf[-1], side="right"))
    p = np.exp(z[K].astype(np.float64) / T)
    p /= p.sum()
    cdf = np.cumsum(p)
    return accepted, int(np.searchsorted(cdf, u[K + 1] * cdf[-1], side="right"))


def test_theta_above_one_sampling_chain_equals_textbook():
    rng = np.random.default_rng(33)
    checked = 0
    for trial in range(300):
        K, V = int(rng.integers(1, 6)), int(rng.integers(2, 10))
        T = float(rng.choice([0.5, 1.0, 1.3]))
        z = random_logits(rng, (K + 1, V))
        q = rng.dirichlet(np.ones(V), size=K + 1).astype(np.float32)
        qn = q.astype(np.float64) / q.astype(np.float64).sum(axis=1, keepdims=True)
        tok = [0] + [int(rng.choice(V, p=qn[i - 1])) for i in range(1, K + 1)]
        u = rng.random(K + 2).astype(np.float32)
        o = run(z, tok, list(range(-1, K)), 1.5, T, u=u, q=q)
        d = o["diag"][0]
        if d["min_accept_margin"] < 1e-6 or d["min_cdf_margin"] < 1e-6:
            continue  # a uniform within rounding of a threshold: either answer is legitimate
        acc, token = textbook_speculative_sampling(z, q.astype(np.float64), tok, u.astype(np.float64), T)
        assert o["accept_len"][0] == acc and o["bonus_token"][0] == token
        assert set(np.unique(o["decision"])) <= {0, 3}
        checked += 1
    assert checked > 250


# ----------------------------------------------------------------------------- brute force on tiny vocabularies
def mars_greedy_bruteforce(z, tok, par, theta):
    """Alg. 1's three-way test applied edge by edge along every root path, top-2 by sorting."""
    N = len(par)
    d = tree_depths(par)

    def edge_ok(k):
        row = z[par[k]].astype(np.float64)
        order = sorted(range(len(row)), key=lambda v: (-row[v], v))
        v1, v2 = order[0], order[1]
        if tok[k] == v1:
            return 1
        z1, z2 = np.float32(row[v1]), np.float32(row[v2])
        if tok[k] == v2 and z1 > 0 and np.float32(z2 / z1) > np.float32(theta):
            return 2
        return 0

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


def test_bruteforce_greedy_all_token_assignments_tiny_vocab():
    rng = np.random.default_rng(8)
    V, N = 3, 4
    grid = np.array([-2.0, 8.0, 9.0, 10.0], np.float32)  # ratios 0.8, 0.9, 0.888.., 1.0, negatives
    n = 0
    for par in ALL_TREES_4:
        for trial in range(12):
            z = grid[rng.integers(len(grid), size=(N, V))]
            for toks in itertools.product(range(V), repeat=N - 1):
                tok = [0] + list(toks)
                for theta in (0.85, 0.9, 1.2):
                    o = run(z, tok, par, theta, 0.0)
                    path, bonus, codes = mars_greedy_bruteforce(z, tok, par, theta)
                    assert o["accept_len"][0] == len(path)
                    assert o["path_idx"][0][:len(path)].tolist() == path
                    assert o["bonus_token"][0] == bonus
                    assert [int(o["decision"][0][k]) for k in path] == codes
                    n += 1
    assert n == len(ALL_TREES_4) * 12 * 27 * 3


def sampling_walk_reference(z, q, tok, par, u, theta, T):
    """Independent recursive statement of the sampling-mode walk (numpy, fp64)."""
    N, V = z.shape

    def softmax(row):
        e = np.exp((row.astype(np.float64) - row.max()) / T)
        return e / e.sum()

    def top2(row):
        order = np.lexsort((np.arange(V), -row.astype(np.float64)))
        return order[0], order[1]

    def descend(c, path):
        f = softmax(z[c])
        v1, v2 = top2(z[c])
        z1, z2 = z[c][v1], z[c][v2]
        relax = z1 > 0 and np.float32(z2) / np.float32(z1) > np.float32(theta)
        for k in [k for k in range(N) if par[k] == c]:
            x = tok[k]
            if x == v2 and relax:
                return descend(k, path + [(k, 2)])
            qk = q[c] if q is not None else np.eye(V)[x]
            if f[x] > 0 and (qk[x] <= 0 or u[k] < min(1.0, f[x] / qk[x])):
                return descend(k, path + [(k, 3)])
            g = np.maximum(f - qk, 0.0)
            if g.sum() > 0:
                f = g / g.sum()
        cdf = np.cumsum(f)
        return path, int(np.searchsorted(cdf, u[N] * cdf[-1], side="right"))

    return descend(0, [])


@pytest.mark.parametrize("dense", [False, True])
def test_bruteforce_sampling_uniform_grid_tiny_vocab(dense):
    rng = np.random.default_rng(77 + dense)
    checked = 0
    for par in ALL_TREES_4 + [[-1, 0, 0, 1, 1], [-1, 0, 1, 1, 2]]:
        N = len(par)
        for trial in range(6):
            V = int(rng.integers(2, 6))
            z = (rng.integers(0, 7, size=(N, V)) * 0.5 + 7).astype(np.float32)  # ratios straddle 0.9
            q = rng.dirichlet(np.ones(V) * 2, size=N).astype(np.float32) if dense else None
            for toks in itertools.islice(itertools.product(range(V), repeat=N - 1), 0, None, 3):
                tok = [0] + list(toks)
                for ugrid in itertools.product((0.05, 0.35, 0.65, 0.95), repeat=2):
                    u = np.array([0] + [ugrid[(i * 7 + trial) % 2] for i in range(1, N)] + [ugrid[1]], np.float32)
                    u[1:] = (u[1:] + rng.uniform(-0.04, 0.04, N)).astype(np.float32)
                    for theta, T in ((0.9, 1.0), (0.9, 0.6), (1.5, 1.0)):
                        o = run(z, tok, par, theta, T, u=u, q=q)
                        d = o["diag"][0]
                        if min(d["min_accept_margin"], d["min_cdf_margin"]) < 1e-9:
                            continue
                        path, token = sampling_walk_reference(z, None if q is None else q.astype(np.float64),
                                                              tok, par, u.astype(np.float64), theta, T)
                        assert o["accept_len"][0] == len(path)
                        assert o["path_idx"][0][:len(path)].tolist() == [k for k, _ in path]
                        assert [int(o["decision"][0][k]) for k, _ in path] == [c for _, c in path]
                        assert o["bonus_token"][0] == token
                        checked += 1
    assert checked > 5000


# ----------------------------------------------------------------------------- statistical check (strict sampling is lossless)
def chi_square_ok(counts, probs, alpha=0.001):
    n = counts.sum()
    exp = probs * n
    keep = exp > 5
    stat = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    return stat < chi2.ppf(1 - alpha, int(keep.sum()) - 1), stat


@pytest.mark.parametrize("m", [1, 2, 3])
def test_strict_sampling_reproduces_target_distribution_dense_q(m):
    """Root + m children drawn i.i.d. from q; theta = 2 (no relaxation).  The first committed token
    (the accepted child's token, else the resampled one) must follow p = softmax(z_root / T)."""
    rng = np.random.default_rng(100 + m)
    V, T, trials = 8, 0.8, 200_000
    z_root = rng.normal(0, 2, V).astype(np.float32)
    p = np.exp(z_root.astype(np.float64) / T)
    p /= p.sum()
    q = rng.dirichlet(np.ones(V)).astype(np.float32)
    N = m + 1
    z = np.zeros((trials, N, V), np.float32)
    z[:, 0] = z_root
    z[:, 1:] = rng.normal(0, 2, (1, m, V)).astype(np.float32)
    dq = np.zeros((trials, N, V), np.float32)
    dq[:, :] = q
    tok = np.zeros((trials, N), np.int32)
    qq = q.astype(np.float64) / q.astype(np.float64).sum()
    tok[:, 1:] = rng.choice(V, size=(trials, m), p=qq)
    par = np.tile(np.array([-1] + [0] * m, np.int32), (trials, 1))
    u = rng.random((trials, N + 1)).astype(np.float32)
    o = R.verify(z, tok, par, 2.0, T, u, dq)
    first = np.where(o["accept_len"] > 0, tok[np.arange(trials), np.maximum(o["path_idx"][:, 0], 0)],
                     o["bonus_token"])
    ok, stat = chi_square_ok(np.bincount(first, minlength=V).astype(np.float64), p)
    assert ok, stat
    # a biased variant must be detectable by this test: accepting always (ignoring Eq. 1) follows q, not p
    always = tok[:, 1]
    bad_ok, _ = chi_square_ok(np.bincount(always, minlength=V).astype(np.float64), p)
    assert not bad_ok


def test_strict_sampling_reproduces_target_distribution_one_hot_and_depth_two():
    """Deterministic drafts (draft_probs = NULL): children are the 3 most likely tokens under a
    fixed proposal; the walk must still commit tokens distributed as the target, at depth 1 and,
    conditionally on the first token, at depth 2."""
    rng = np.random.default_rng(4242)
    V, T, trials = 8, 1.0, 300_000
    rows = rng.normal(0, 1.5, (5, V)).astype(np.float32)  # root, 3 children, 1 grandchild under node 1
    soft = lambda r: np.exp(r.astype(np.float64) / T) / np.exp(r.astype(np.float64) / T).sum()
    kids = np.argsort(-rows[0])[[1, 0, 3]]  # distinct tokens, an arbitrary fixed order
    gk = int(np.argsort(-rows[1])[0])
    par = np.array([-1, 0, 0, 0, 1], np.int32)
    tok = np.array([0, kids[0], kids[1], kids[2], gk], np.int32)
    z = np.broadcast_to(rows, (trials, 5, V)).copy()
    u = rng.random((trials, 6)).astype(np.float32)
    o = R.verify(z, np.tile(tok, (trials, 1)), np.tile(par, (trials, 1)), 2.0, T, u, None)
    first = np.where(o["accept_len"] > 0, tok[np.maximum(o["path_idx"][:, 0], 0)], o["bonus_token"])
    ok, stat = chi_square_ok(np.bincount(first, minlength=V).astype(np.float64), soft(rows[0]))
    assert ok, stat
    # second committed token given that node 1 was accepted follows softmax(row 1)
    sel = o["path_idx"][:, 0] == 1
    second = np.where(o["accept_len"][sel] > 1, gk, o["bonus_token"][sel])
    ok, stat = chi_square_ok(np.bincount(second, minlength=V).astype(np.float64), soft(rows[1]))
    assert ok, stat
    # and given node 2 (a leaf) it follows softmax(row 2)
    sel = o["path_idx"][:, 0] == 2
    ok, stat = chi_square_ok(np.bincount(o["bonus_token"][sel], minlength=V).astype(np.float64), soft(rows[2]))
    assert ok, stat


def test_relaxation_makes_sampling_lossy_in_the_stated_way():
    """With theta = 0.9 and a low-margin root row, a runner-up draft is always accepted: the
    committed-token distribution moves mass to the runner-up by exactly the rejected share."""
    rng = np.random.default_rng(9)
    V, trials = 6, 100_000
    row = np.array([10.0, 9.6, 3, 2, 1, 0], np.float32)
    z = np.zeros((trials, 2, V), np.float32)
    z[:, 0] = row
    tok = np.tile(np.array([0, 1], np.int32), (trials, 1))
    par = np.tile(np.array([-1, 0], np.int32), (trials, 1))
    u = rng.random((trials, 3)).astype(np.float32)
    o = R.verify(z, tok, par, 0.9, 1.0, u, None)
    assert (o["accept_len"] == 1).all() and (o["decision"][:, 1] == 2).all()


# ----------------------------------------------------------------------------- invariances and bounds
def greedy_case(rng, B, N, V, chain, ties=False):
    z = random_logits(rng, (B, N, V), ties)
    z[:, :, 0] = rng.uniform(10, 30, (B, N)).astype(np.float32)
    z[:, :, 1] = (z[:, :, 0] * rng.uniform(0.8, 1.0, (B, N))).astype(np.float32)
    perm = rng.permuted(np.tile(np.arange(V), (B * N, 1)), axis=1).reshape(B, N, V)
    z = np.take_along_axis(z, perm, axis=2)
    par = np.array([list(range(-1, N - 1)) if chain else random_tree(rng, N) for _ in range(B)], np.int32)
    order = np.argsort(-z, axis=2, kind="stable")
    tok = np.zeros((B, N), np.int32)
    for b in range(B):
        for i in range(1, N):
            c = rng.random()
            tok[b, i] = order[b, par[b, i], 0] if c < 0.6 else order[b, par[b, i], 1] if c < 0.9 else rng.integers(V)
    return z, tok, par


def test_accept_len_monotone_in_theta_for_chains():
    rng = np.random.default_rng(3)
    z, tok, par = greedy_case(rng, 64, 8, 50, chain=True)
    prev = None
    for theta in (0.82, 0.86, 0.9, 0.94, 0.98, 1.1):
        L = R.verify(z, tok, par, theta, 0.0)["accept_len"]
        if prev is not None:
            assert (L <= prev).all()
        prev = L
    assert prev.mean() < R.verify(z, tok, par, 0.82, 0.0)["accept_len"].mean()


def test_scale_invariance_power_of_two():
    rng = np.random.default_rng(4)
    z, tok, par = greedy_case(rng, 32, 9, 40, chain=False)
    a = R.verify(z, tok, par, 0.9, 0.0)
    for s in (0.25, 8.0):
        b = R.verify((z * np.float32(s)).astype(np.float32), tok, par, 0.9, 0.0)
        for k in ("accept_len", "path_idx", "bonus_token", "decision", "accept_mask"):
            assert np.array_equal(a[k], b[k])


def test_vocabulary_permutation_equivariance():
    rng = np.random.default_rng(6)
    z, tok, par = greedy_case(rng, 16, 7, 30, chain=False)
    a = R.verify(z, tok, par, 0.9, 0.0)
    perm = rng.permutation(30)           # new id of old token v is perm[v]
    z2 = np.empty_like(z)
    z2[:, :, perm] = z
    b = R.verify(z2, perm[tok].astype(np.int32), par, 0.9, 0.0)
    assert np.array_equal(a["accept_len"], b["accept_len"]) and np.array_equal(a["path_idx"], b["path_idx"])
    assert np.array_equal(perm[a["bonus_token"]], b["bonus_token"])


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_output_structure_bounds(T):
    rng = np.random.default_rng(12)
    B, N, V = 40, 12, 20
    z, tok, par = greedy_case(rng, B, N, V, chain=False, ties=True)
    u = rng.random((B, N + 1)).astype(np.float32)
    o = R.verify(z, tok, par, 0.9, T, u if T > 0 else None)
    for b in range(B):
        d = tree_depths(par[b])
        L = int(o["accept_len"][b])
        assert 0 <= L <= d.max() <= N - 1
        path = o["path_idx"][b]
        assert (path[L:] == -1).all()
        prev = 0
        for depth, n in enumerate(path[:L], start=1):
            assert par[b][n] == prev and d[n] == depth
            prev = int(n)
        mask = np.zeros(N, np.uint8)
        mask[0] = 1
        mask[path[:L]] = 1
        assert np.array_equal(mask, o["accept_mask"][b])
        assert ((o["decision"][b] > 0) == (mask > 0))[1:].all() and o["decision"][b][0] == 0
        assert 0 <= o["bonus_token"][b] < V


def test_threads_do_not_change_results():
    rng = np.random.default_rng(2)
    z, tok, par = greedy_case(rng, 24, 6, 300, chain=False)
    u = rng.random((24, 7)).astype(np.float32)
    R.set_threads(1)
    a = R.verify(z, tok, par, 0.9, 0.9, u)
    R.set_threads(4)
    b = R.verify(z, tok, par, 0.9, 0.9, u)
    R.set_threads(1)
    for k in a:
        assert np.array_equal(a[k], b[k])
