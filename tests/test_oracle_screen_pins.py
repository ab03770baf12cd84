"""Pins of what decides which inputs the parity tests see: the oracle's decision-margin diagnostics
(distance of a uniform to its acceptance probability, distance of the final draw to a CDF step, size of
the residual normalisers, where the first small one is met) and the screening of uniforms built on them;
and of the tolerance the parity tests grant the residual normaliser.  CPU only."""
import math
from types import SimpleNamespace

import numpy as np
import pytest

from oracle import mars_ref as R
from oracle import screen


def f32(a):
    return np.asarray(a, dtype=np.float32)


def run(z, tok, par, theta, T, u, q=None):
    z = f32(z)[None]
    q = None if q is None else f32(q)[None]
    return R.verify(z, np.asarray(tok, np.int32)[None], np.asarray(par, np.int32)[None], theta, T, f32(u)[None], q)


# ----------------------------------------------------------------------------- diagnostics, by hand
def test_cdf_margin_and_normalisers_of_the_one_hot_example():
    # Root p = (0.6, 0.3, 0.1), two children with a one-hot draft (the worked example W4 of the oracle pins):
    # child 1 (token 1) rejected by u = 0.5 -> Z = 1 - 0.3 = 0.7; child 2 (token 2) accepted: 0.1 < 1/7.
    # Row of node 2: p = (0.2, 0.6, 0.2), CDF steps at 0.2, 0.8, 1.0; the draw u = 0.75 falls in [0.2, 0.8):
    # 0.55 above the step below, 0.05 below the step above -> margin 0.05.
    z = np.log(np.array([[6, 3, 1], [1, 1, 1], [1, 3, 1]], np.float64))
    d = run(z, [0, 1, 2], [-1, 0, 0], 0.9, 1.0, [0, 0.5, 0.1, 0.75])["diag"][0]
    assert abs(d["min_cdf_margin"] - 0.05) < 1e-6
    assert abs(d["min_norm"] - 0.7) < 1e-6
    assert abs(d["min_accept_margin"] - min(0.5 - 0.3, 1 / 7 - 0.1)) < 1e-6
    assert d["small_norm_plen"] == -1 and d["small_norm_node"] == -1
    # the draw moved to 0.21: 0.01 above the step at 0.2
    d = run(z, [0, 1, 2], [-1, 0, 0], 0.9, 1.0, [0, 0.5, 0.1, 0.21])["diag"][0]
    assert abs(d["min_cdf_margin"] - 0.01) < 1e-6
    # first token of the row: the lower "step" is 0
    d = run(z, [0, 1, 2], [-1, 0, 0], 0.9, 1.0, [0, 0.5, 0.1, 0.15])["diag"][0]
    assert abs(d["min_cdf_margin"] - 0.05) < 1e-6          # min(0.15 - 0, 0.2 - 0.15)


def test_smallest_normaliser_of_two_dense_siblings():
    # p = (0.4, 0.35, 0.25), q = (0.1, 0.3, 0.6), both children rejected (example W5 of the oracle pins):
    # Z1 = 0.3 + 0.05 = 0.35, then f = (6/7, 1/7, 0) and Z2 = 6/7 - 0.1 = 0.757: the smallest is 0.35,
    # the last 0.757.  Final f = (1, 0, 0): the draw u = 0.3 is 0.3 above 0 and 0.7 below 1.
    z = np.log(np.array([[0.4, 0.35, 0.25], [1, 1, 1], [1, 1, 1]], np.float64))
    q = np.array([[0.1, 0.3, 0.6], [1 / 3] * 3, [1 / 3] * 3])
    d = run(z, [0, 2, 1], [-1, 0, 0], 2.0, 1.0, [0, 0.5, 0.9, 0.3], q)["diag"][0]
    assert abs(d["min_norm"] - 0.35) < 1e-6
    assert abs(d["last_residual_norm"] - (6 / 7 - 0.1)) < 1e-6
    assert abs(d["min_cdf_margin"] - 0.3) < 1e-6
    assert d["small_norm_plen"] == -1


def test_where_the_first_small_normaliser_is_met():
    # Chain root -> 1 -> 2.  Root: p = (0.5, 0.3, 0.2), q = (0.2, 0.6, 0.2), token 0: a = 1, accepted.
    # Node 1: p = (0.98, 0.01, 0.01), q = (0.985, 0.005, 0.01), token 0: a = 0.98/0.985 = 0.99492, rejected by
    # u = 0.999; max(0, p - q) = (0, 0.005, 0): Z = 0.005, below the floor of 0.02, met with one draft accepted
    # while the children of node 1 were tried.
    z = np.log(np.array([[0.5, 0.3, 0.2], [0.98, 0.01, 0.01], [1, 1, 1]], np.float64))
    q = np.array([[0.2, 0.6, 0.2], [0.985, 0.005, 0.01], [1 / 3] * 3])
    R.set_norm_floor(2e-2)
    o = run(z, [0, 0, 0], [-1, 0, 1], 2.0, 1.0, [0, 0.3, 0.999, 0.5], q)
    d = o["diag"][0]
    assert o["accept_len"].tolist() == [1] and o["bonus_token"].tolist() == [1]
    assert abs(d["min_norm"] - 0.005) < 1e-6
    assert d["small_norm_plen"] == 1 and d["small_norm_node"] == 1
    # a lower floor: nothing to report; the results are the same
    R.set_norm_floor(1e-3)
    o2 = run(z, [0, 0, 0], [-1, 0, 1], 2.0, 1.0, [0, 0.3, 0.999, 0.5], q)
    assert o2["diag"][0]["small_norm_plen"] == -1 and o2["bonus_token"].tolist() == [1]
    R.set_norm_floor(2e-2)
    assert R.get_norm_floor() == 2e-2


# ----------------------------------------------------------------------------- screening
def tiny_workload():
    """Three requests over three tokens, each a root with two children (dense draft distribution).
    Request 0: its first uniform sits 2e-6 from the acceptance probability 0.5 -> must be drawn again.
    Request 1: every margin is wide -> must be left alone.
    Request 2: the first child's token has probability 0 under the target (a masked entry), so it is
    rejected whatever is drawn, and the residual mass is 0.005: no draw avoids the small normaliser."""
    ninf = -np.inf
    z = np.zeros((3, 3, 3), np.float32)
    z[0] = np.log(np.array([[0.5, 0.3, 0.2], [1, 1, 1], [1, 2, 1]], np.float64))
    z[1] = z[0]
    z[2] = np.array([np.log([0.99, 0.01, 1.0]), [0, 0, 0], [0, 0, 0]], np.float64)
    z[2, 0, 2] = ninf                                   # p = (0.99, 0.01, 0)
    q = np.zeros((3, 3, 3), np.float32)
    q[0] = q[1] = np.array([[0.2, 0.6, 0.2], [1 / 3] * 3, [1 / 3] * 3])
    q[2] = np.array([[0.985, 0.01, 0.005], [1 / 3] * 3, [1 / 3] * 3])
    tok = np.array([[0, 1, 0], [0, 1, 0], [0, 2, 1]], np.int32)
    par = np.tile(np.array([-1, 0, 0], np.int32), (3, 1))
    u = np.array([[0, 0.500002, 0.3, 0.6], [0, 0.9, 0.3, 0.45], [0, 0.5, 0.999, 0.5]], np.float32)
    return SimpleNamespace(logits=z, draft_tokens=tok, tree_parent=par, theta=np.full(3, 2.0, np.float32),
                           temperature=1.0, uniforms=u, draft_probs=q)


def test_screening_redraws_what_is_too_close_and_nothing_else():
    w = tiny_workload()
    before = w.uniforms.copy()
    first = R.verify(w.logits, w.draft_tokens, w.tree_parent, w.theta, 1.0, w.uniforms, w.draft_probs)
    assert first["diag"]["min_accept_margin"][0] < 1e-5 and first["diag"]["min_accept_margin"][1] > 1e-2
    ref = screen.screen_uniforms(w, allow_small_norm=True, norm_rounds=5)
    assert not np.array_equal(w.uniforms[0], before[0])          # request 0 drawn again
    assert np.array_equal(w.uniforms[1], before[1])              # request 1 untouched
    assert ref["clean"].tolist() == [True, True, False]          # request 2, and only it, is flagged
    d = ref["diag"]
    assert (d["min_accept_margin"] >= 1e-4).all() and (d["min_cdf_margin"] >= 1e-4).all()
    assert d["min_norm"][0] >= 2e-2 and d["min_norm"][1] >= 2e-2
    assert abs(d["min_norm"][2] - 0.005) < 1e-6 and d["small_norm_plen"][2] == 0 and d["small_norm_node"][2] == 0
    # what is returned is the oracle's output for the uniforms that are left in the workload
    again = R.verify(w.logits, w.draft_tokens, w.tree_parent, w.theta, 1.0, w.uniforms, w.draft_probs)
    for key in ("accept_len", "bonus_token", "path_idx", "accept_mask", "decision"):
        assert np.array_equal(ref[key], again[key]), key
    assert np.array_equal(ref["diag"]["min_accept_margin"], again["diag"]["min_accept_margin"])


def test_screening_refuses_a_small_normaliser_unless_told_otherwise():
    w = tiny_workload()
    with pytest.raises(RuntimeError, match="normaliser"):
        screen.screen_uniforms(w, norm_rounds=5)
    w = tiny_workload()
    w.logits, w.draft_tokens, w.tree_parent = w.logits[:2], w.draft_tokens[:2], w.tree_parent[:2]
    w.theta, w.uniforms, w.draft_probs = w.theta[:2], w.uniforms[:2], w.draft_probs[:2]
    assert screen.screen_uniforms(w)["clean"].all()              # without request 2 nothing is flagged


def test_screening_is_a_no_op_in_greedy_mode():
    w = tiny_workload()
    w.temperature = 0.0
    before = w.uniforms.copy()
    ref = screen.screen_uniforms(w)
    assert np.array_equal(w.uniforms, before) and ref["clean"].all()


# ----------------------------------------------------------------------------- the tolerance of Z
def test_an_fp32_residual_normaliser_is_off_by_an_absolute_amount_not_a_relative_one():
    # Z = sum max(0, f - q) is a difference of two probability masses of order 1.  An fp32 evaluation of
    # f(v) = exp2((z_v - z1) c) / S carries a few ulp of relative error in every f(v), part of it common to
    # all v (the rounded scale c, the sum S from the row reduction: about 3e-7 measured against this oracle).
    # Emulated here in float32 with numpy on rows whose draft distribution hugs the target (so that Z is
    # small): the error of Z stays below 1e-6 in absolute terms whatever Z is, while relative to Z it grows
    # like 1/Z and passes 1e-5 once Z is a few per cent.  That is the tolerance the parity tests use for the
    # normaliser (rel 1e-5 plus 1e-6 absolute) and the reason why inputs are screened to Z >= 2e-2 before
    # acceptance decisions behind a rejection are compared (error of the next acceptance probability
    # <= 1e-6 / 2e-2 = 5e-5, half the guard band of 1e-4).
    rng = np.random.default_rng(7)
    V, T = 8192, 0.7
    c64 = math.log2(math.e) / T
    worst_abs, rel_at = 0.0, {}
    for target_z in (2e-1, 2e-2, 3e-3):
        for trial in range(4):
            z = np.round(rng.normal(0, 3, V) * 128) / 128          # exactly representable in float32
            z[rng.integers(V)] = 20.0
            z1 = z.max()
            e64 = np.exp2((z - z1) * c64)
            S64 = e64.sum()
            p = e64 / S64
            # q: the target with mass target_z moved from the tokens above the median to those below
            up = p > np.median(p)
            q = p.copy()
            q[up] *= 1 - target_z / p[up].sum()
            q[~up] *= 1 + target_z / p[~up].sum()
            q32 = q.astype(np.float32)
            Z64 = np.maximum(p - q32.astype(np.float64), 0).sum()
            for eps_s in (-3e-7, 3e-7):                             # error of the sum from the row reduction
                arg = ((z - z1).astype(np.float32) * np.float32(c64)).astype(np.float32)
                f32_ = (np.exp2(arg).astype(np.float32) * np.float32(1.0 / (S64 * (1 + eps_s)))).astype(np.float32)
                Z32 = float(np.maximum(f32_ - q32, np.float32(0)).astype(np.float64).sum())
                worst_abs = max(worst_abs, abs(Z32 - Z64))
                rel_at[target_z] = max(rel_at.get(target_z, 0.0), abs(Z32 - Z64) / Z64)
    assert worst_abs < 1e-6, worst_abs
    assert rel_at[2e-1] < 1e-5                     # a well-conditioned normaliser meets the relative bar alone
    assert rel_at[3e-3] > 1e-5                     # a small one cannot, in any fp32 evaluation of f
    assert worst_abs / 2e-2 < 5e-5                 # and at the screening floor the knock-on error is half the guard band
