"""Pins of the LM-head oracle (Eq. 2 followed by the greedy pass) and of its input generator.

The oracle is pinned to things other than itself: exact rational arithmetic, torch's own
float32 -> bfloat16 conversion, hand-worked values and special cases with an obvious answer.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from mars_inputs.lmhead import LMHEAD_CONFIGS, make_lmhead_workload
from oracle import lmhead_ref, mars_ref


def bits_of(x):
    """bf16 bit patterns of values that are exactly representable."""
    b = np.asarray(x, np.float32).view(np.uint32)
    assert np.all((b & 0xFFFF) == 0)
    return (b >> 16).astype(np.uint16)


# ---------------------------------------------------------------- rounding to bf16
def test_round_matches_torch_on_float32_values():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 7,
                        rng.standard_normal(2000).astype(np.float32) * 1e-3,
                        np.float32([0.0, 1.0, -1.0, 3.0e38, 1.0e-30])])
    v, bits = lmhead_ref.bf16_round(x.astype(np.float64))
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(v, ref.to(torch.float64).numpy())
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())


def test_round_ties_go_to_even_and_doubles_are_rounded_once():
    one = 1.0
    ulp = 2.0 ** -7                               # spacing of bf16 in [1, 2)
    cases = [(one + ulp / 2, one),                # tie: 1.0 has an even significand
             (one + 3 * ulp / 2, one + 2 * ulp),  # tie: up to the even neighbour
             (one + ulp / 2 + 2.0 ** -40, one + ulp),   # just above the tie: float32 first would lose the 2^-40
             (one + ulp / 2 - 2.0 ** -40, one),
             (-(one + ulp / 2 + 2.0 ** -40), -(one + ulp)),
             (255.5, 256.0), (254.5, 254.0), (0.75 + 2.0 ** -9, 0.75)]
    for x, want in cases:
        v, bits = lmhead_ref.bf16_round(np.float64([x]))
        assert v[0] == want, (x, v[0], want)
        assert lmhead_ref.bf16_widen(bits)[0] == want
    # the trap this pins: rounding through float32 first gives the other answer for the third case
    assert float(torch.tensor([one + ulp / 2 + 2.0 ** -40], dtype=torch.float64).to(torch.float32).to(torch.bfloat16)) == one


def test_widen_is_exact():
    rng = np.random.default_rng(2)
    bits = rng.integers(0, 1 << 16, 5000).astype(np.uint16)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]     # leave out inf / nan
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(lmhead_ref.bf16_widen(bits), ref)


# ---------------------------------------------------------------- Eq. 2
def test_logits_against_exact_rational_arithmetic():
    rng = np.random.default_rng(3)
    R, H, V = 3, 7, 5
    hb = lmhead_ref.bf16_round(rng.standard_normal((R, H)) * 2)[1]
    wb = lmhead_ref.bf16_round(rng.standard_normal((V, H)))[1]
    h, w = lmhead_ref.bf16_widen(hb), lmhead_ref.bf16_widen(wb)
    z = lmhead_ref.logits_exact(hb, wb, chunk=2)
    zr, _ = lmhead_ref.bf16_round(z)
    for r in range(R):
        for v in range(V):
            exact = sum(Fraction(float(h[r, k])) * Fraction(float(w[v, k])) for k in range(H))
            assert abs(Fraction(float(z[r, v])) - exact) <= abs(exact) * Fraction(1, 10 ** 14) + Fraction(1, 10 ** 300)
            # nearest bf16 value to the exact rational, by search over the two neighbours of the result
            got = Fraction(float(zr[r, v]))
            step = Fraction(2) ** (np.frexp(float(zr[r, v]))[1] - 8)
            assert abs(exact - got) <= step / 2


def test_logits_are_transposed_the_right_way():
    # W = selected rows of the identity: logit v of row r is h[r, pick[v]]
    rng = np.random.default_rng(4)
    H = 8
    hb = lmhead_ref.bf16_round(rng.standard_normal((5, H)))[1]
    pick = np.array([3, 0, 7, 7, 1, 2])
    w = np.zeros((pick.size, H), np.float32)
    w[np.arange(pick.size), pick] = 1.0
    z = lmhead_ref.logits_exact(hb, bits_of(w))
    assert np.array_equal(z, lmhead_ref.bf16_widen(hb)[:, pick])


def test_hand_worked_chain():
    # H = 2, V = 4.  W rows: (1,0), (0,1), (1,1), (-1,0).  theta = 0.9, greedy, chain of three drafts.
    #  node 0: h = (10, 9.5)  -> z = (10, 9.5, 19.5, -10): top-1 = 2, top-2 = 0, ratio 10/19.5 = 0.51
    #  node 1: h = (8, 7.5)   -> z = (8, 7.5, 15.5, -8):   top-1 = 2, top-2 = 0
    #  node 2: h = (20, -19)  -> z = (20, -19, 1, -20):    top-1 = 0, top-2 = 2, ratio 0.05
    #  node 3: h = (4, -3.75) -> z = (4, -3.75, .25, -4)
    # drafts: node 1 carries token 2 (exact match with row 0), node 2 token 0 (runner-up of row 1,
    # ratio 8/15.5 = 0.516 < theta: rejected).  Accepted length 1, correction = top-1 of row 1 = 2.
    w = bits_of(np.float32([[1, 0], [0, 1], [1, 1], [-1, 0]]))
    h = bits_of(np.float32([[[10, 9.5], [8, 7.5], [20, -19], [4, -3.75]]]))
    tok = np.int32([[0, 2, 0, 0]])
    par = np.int32([[-1, 0, 1, 2]])
    out = lmhead_ref.lmhead_verify(h, w, tok, par, 0.9)
    assert np.array_equal(lmhead_ref.bf16_widen(out["logits_bits"])[0, 0], [10, 9.5, 19.5, -10])
    assert out["accept_len"][0] == 1 and out["bonus_token"][0] == 2
    assert list(out["path_idx"][0]) == [1, -1, -1, -1]
    # with theta = 0.5 the runner-up of row 1 passes (0.516 > 0.5), then token 0 = top-1 of row 2:
    out = lmhead_ref.lmhead_verify(h, w, tok, par, 0.5)
    assert out["accept_len"][0] == 3 and out["bonus_token"][0] == 0
    assert list(out["decision"][0]) == [0, 1, 2, 1]


def test_rounding_moves_a_logit_before_the_top2_are_taken():
    # the exact logits 1 + 3/512 and 1 + 2.25/512 are different, but both lie above the boundary
    # 1 + 2/512 and round to 1 + 1/128: the top-2 are taken from the rounded values (a tie, lower index first).
    h = bits_of(np.float32([[[1.0, 2.0 ** -7]]]))
    # W rows (a, b) give z = a + b / 128
    w = bits_of(np.float32([[1.0, 0.75], [1.0, 0.5625], [0.5, 0.0]]))
    out = lmhead_ref.lmhead_verify(h, w, np.int32([[0]]), np.int32([[-1]]), 0.9)
    z = lmhead_ref.bf16_widen(out["logits_bits"])[0, 0]
    assert list(z) == [1 + 2.0 ** -7, 1 + 2.0 ** -7, 0.5]
    st = out["stats"][0, 0]
    assert (st["id1"], st["id2"]) == (0, 1) and st["z1"] == st["z2"]   # equal after rounding: lower index first


def test_clearance_measures_the_distance_to_the_boundary():
    base = np.full(16, -5.0)
    for eps, want in [(2.0 ** -20, 2.0 ** -20), (-(2.0 ** -16), 2.0 ** -16)]:
        row = base.copy()
        row[3] = 1.0
        row[9] = 1.0 + 2.0 ** -8 + eps          # boundary of [1, 1 + 2^-7] is 1 + 2^-8
        got = lmhead_ref.rounding_clearance(row)
        assert got == pytest.approx(want / (1.0 + 2.0 ** -8), rel=1e-3)
    row = base.copy()
    row[3], row[9] = 1.0, 1.0 + 2.0 ** -7        # both on the grid: half a step from any boundary
    assert lmhead_ref.rounding_clearance(row) == pytest.approx(0.5 / 129, rel=1e-9)
    # an entry far below the runner-up does not count, one just below it does
    row = base.copy()
    row[3], row[9], row[5] = 2.0, 1.5, 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert lmhead_ref.rounding_clearance(row) > 1e-3
    m, e = np.frexp(1.5 * (1 - 2.0 ** -7))       # just under the runner-up: inside the window ...
    row[5] = np.ldexp((np.floor(m * 256) + 0.5) / 256 + 2.0 ** -30, e)   # ... and 2^-30 above a boundary
    assert lmhead_ref.rounding_clearance(row) < 1e-6


# ---------------------------------------------------------------- the generator
def small(seed=0, **kw):
    spec = dict(LMHEAD_CONFIGS["small"])
    spec.update(kw)
    return make_lmhead_workload(spec.pop("name"), seed=seed, **spec)


def test_generator_is_seeded_and_planted_rows_are_low_margin_rows():
    a, b = small(seed=5), small(seed=5)
    assert np.array_equal(a.hidden, b.hidden) and np.array_equal(a.weight, b.weight)
    assert np.array_equal(a.draft_tokens, b.draft_tokens)
    assert not np.array_equal(a.hidden, small(seed=6).hidden)
    out = lmhead_ref.lmhead_verify(a.hidden, a.weight, a.draft_tokens, a.tree_parent, a.theta)
    st = out["stats"]
    pl = a.planted
    has = pl[..., 0] >= 0
    assert 0.3 < has.mean() < 0.9
    assert (st["id1"][has] == pl[..., 0][has]).mean() > 0.95
    assert np.all(st["z1"][has] > 18.0)
    ratio = st["ratio"][has]
    assert ratio.min() > 0.7 and ratio.max() <= 1.0
    z = lmhead_ref.bf16_widen(out["logits_bits"]).reshape(-1, a.V)
    assert 2.5 < z.std() < 3.5                   # background like N(0, 3^2)
    assert out["accept_len"].max() >= 1


def test_redraw_changes_only_the_chosen_rows_and_their_columns():
    a, b = small(seed=7), small(seed=7)
    rows = [2, 11]
    b.redraw_rows(rows, 1)
    hid_a, hid_b = a.hidden.reshape(a.rows, a.H), b.hidden.reshape(b.rows, b.H)
    same = np.all(hid_a == hid_b, axis=1)
    assert list(np.nonzero(~same)[0]) == rows
    wrows = np.nonzero(np.any(a.weight != b.weight, axis=1))[0]
    allowed = set(int(x) for x in a.planted.reshape(-1, 2)[rows].reshape(-1) if x >= 0)
    assert set(int(x) for x in wrows) <= allowed


def test_screening_leaves_every_row_clear():
    w = small(seed=8)
    out = lmhead_ref.screen_lmhead(w, clearance=2e-3)    # a wide band, so that some rows have to move
    assert out["clearance"].min() >= 2e-3
    again = lmhead_ref.lmhead_verify(w.hidden, w.weight, w.draft_tokens, w.tree_parent, w.theta)
    assert np.array_equal(again["exact"], out["exact"])   # the incremental update equals a fresh product
    assert np.array_equal(again["accept_len"], out["accept_len"])
    ratio, z1 = out["stats"]["ratio"], out["stats"]["z1"]
    assert np.all((np.abs(ratio - w.theta[:, None]) >= 1e-4) | (z1 <= 0))


def test_screening_a_sub_batch_describes_those_requests():
    w = small(seed=9, B=6)
    sub = lmhead_ref.screen_lmhead(w, clearance=1e-3, requests=[4, 1])
    assert sub["clearance"].min() >= 1e-3 and sub["accept_len"].shape == (2,)
    full = lmhead_ref.lmhead_verify(w.hidden, w.weight, w.draft_tokens, w.tree_parent, w.theta)   # after the redraws
    for key in ("accept_len", "bonus_token", "path_idx", "decision"):
        assert np.array_equal(sub[key], full[key][[4, 1]]), key
    assert np.array_equal(sub["stats"]["id1"], full["stats"]["id1"][[4, 1]])
    assert np.array_equal(sub["exact"], full["exact"].reshape(6, w.N, w.V)[[4, 1]].reshape(-1, w.V))


def test_generator_rejects_a_vocabulary_too_small_for_its_rows():
    with pytest.raises(ValueError):
        make_lmhead_workload("x", B=2, N=5, H=64, V=20, tree={"kind": "chain"})


# ---------------------------------------------------------------- sampling mode from hidden states
def test_hand_worked_sampling_chain():
    # H = 2, V = 3, temperature 1/ln 2, so that exp(z/T) = 2^z.  W rows: (2,0), (1,0), (0,3).
    #  node 0: h = (1, 0) -> z = (2, 1, 0): weights 4, 2, 1, p = (4/7, 2/7, 1/7)
    #  node 1: h = (0, 1) -> z = (0, 0, 3): weights 1, 1, 8, p = (0.1, 0.1, 0.8)
    # Node 1 carries token 1 (one-hot draft): accepted with probability p(1) = 2/7 = 0.2857.
    #  u1 = 0.2: accepted; the bonus token comes from row 1: u = 0.15 falls in [0.1, 0.2) -> token 1.
    #  u1 = 0.3: rejected; residual = p without token 1 = (4/5, 0, 1/5); u = 0.9 > 0.8 -> token 2.
    T = np.float32(1.0 / np.log(2.0))
    w = bits_of(np.float32([[2, 0], [1, 0], [0, 3]]))
    h = bits_of(np.float32([[[1, 0], [0, 1]]]))
    tok, par = np.int32([[0, 1]]), np.int32([[-1, 0]])
    out = lmhead_ref.lmhead_verify_sampling(h, w, tok, par, 2.0, T, np.float32([[0, 0.2, 0.15]]))
    assert np.array_equal(lmhead_ref.bf16_widen(out["logits_bits"])[0], [[2, 1, 0], [0, 0, 3]])
    assert out["accept_len"][0] == 1 and out["bonus_token"][0] == 1
    assert abs(out["stats"]["sum_exp"][0, 0] - 7 / 4) < 1e-6 and abs(out["stats"]["sum_exp"][0, 1] - 10 / 8) < 1e-6
    out = lmhead_ref.lmhead_verify_sampling(h, w, tok, par, 2.0, T, np.float32([[0, 0.3, 0.9]]))
    assert out["accept_len"][0] == 0 and out["bonus_token"][0] == 2
    assert abs(out["diag"]["last_residual_norm"][0] - 5 / 7) < 1e-6
    # the same logits handed to the logits oracle directly give the same walk (the composition adds nothing)
    direct = mars_ref.verify(bits_of(np.float32([[[2, 1, 0], [0, 0, 3]]])), tok, par, 2.0, T, np.float32([[0, 0.3, 0.9]]))
    assert direct["bonus_token"][0] == 2 and direct["accept_len"][0] == 0


def test_lattice_workloads_have_exact_fp32_sums_in_any_order():
    # Hidden states on a grid of 2^-5, weights on a grid of 2^-10: every product is a multiple of 2^-15, and
    # with the magnitudes of a (row, entry) pair's products adding up to less than 512 every partial sum in
    # any order is a multiple of 2^-15 below 2^9, i.e. an fp32 number: fp32 accumulation is exact.
    w = make_lmhead_workload("lat", B=2, N=9, H=256, V=2048, tree={"kind": "chain"}, lattice=True, temperature=0.8,
                             dense_q=True, seed=3)
    h = lmhead_ref.bf16_widen(w.hidden).reshape(-1, w.H)
    W = lmhead_ref.bf16_widen(w.weight)
    assert np.all(h * 32 == np.rint(h * 32)) and np.abs(h).max() < 8
    assert np.all(W * 1024 == np.rint(W * 1024)) and np.abs(W).max() < 0.25
    assert (np.abs(h) @ np.abs(W).T).max() < 512
    exact = lmhead_ref.logits_exact(w.hidden.reshape(-1, w.H), w.weight)
    for order in (np.arange(w.H), np.random.default_rng(0).permutation(w.H), np.arange(w.H)[::-1]):
        acc = np.zeros(exact.shape, np.float32)
        for k in order:
            acc = (acc + h[:, k:k + 1].astype(np.float32) * W[:, k].astype(np.float32)[None, :]).astype(np.float32)
        assert np.array_equal(acc.astype(np.float64), exact)
    # planted rows still carry a low-margin pair, and the sampling inputs are there
    assert w.uniforms.shape == (2, 10) and w.draft_probs.shape == (2, 9, 2048)
    assert np.allclose(w.draft_probs.sum(axis=2), 1.0, atol=1e-5)
    out = lmhead_ref.lmhead_verify_sampling(w.hidden, w.weight, w.draft_tokens, w.tree_parent, w.theta, w.temperature,
                                            w.uniforms, w.draft_probs)
    assert out["stats"]["relax_ok"].sum() >= 3
    # redrawing a row keeps it on the lattice
    w.redraw_rows([4], 1)
    h2 = lmhead_ref.bf16_widen(w.hidden).reshape(-1, w.H)
    assert np.all(h2 * 32 == np.rint(h2 * 32))
    W2 = lmhead_ref.bf16_widen(w.weight)
    assert np.all(W2 * 1024 == np.rint(W2 * 1024))


def test_the_bound_on_the_products_holds_at_the_full_shape():
    # rows and columns sampled from the H = 4096 shape the benchmark runs: background pairs about 125, planted at most 30
    spec = dict(LMHEAD_CONFIGS["small"]); spec.pop("name")
    spec.update(H=4096, V=6000)
    w = make_lmhead_workload("lat4096", lattice=True, temperature=1.0, seed=5, **spec)
    h = np.abs(lmhead_ref.bf16_widen(w.hidden).reshape(-1, w.H))
    W = np.abs(lmhead_ref.bf16_widen(w.weight))
    assert (h @ W.T).max() < 512
