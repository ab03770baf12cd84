"""Helpers of the GPU parity tests: run one workload through the HIP library (via the C ABI
binding) and through the CPU oracle, and compare element by element.

Bar: decisions, lengths, paths, tokens, indices and the top-2 logit values are bit-exact;
fp32 statistics (sum-exp, bonus probability) agree within rel 1e-5.  The residual normaliser
Z = sum max(0, f - q) is a difference of probability masses of order 1: each f(v) is an fp32
number with a few ulp of relative error, so Z carries an absolute error of up to about
8 ulp(1) ~ 1e-6 however small it is; its tolerance is rel 1e-5 plus that absolute floor.
"""
import sys

import numpy as np
import torch

from oracle import mars_ref, screen
from paper_2601_15498_amd import binding as M

REL_TOL = 1e-5
RESIDUAL_ABS_TOL = 1e-6


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_device(w):
    dev = torch.device("cuda:0")
    d = {
        "logits": torch.from_numpy(w.logits).to(dev),
        "draft_tokens": torch.from_numpy(np.ascontiguousarray(w.draft_tokens, dtype=np.int32)).to(dev),
        "tree_parent": torch.from_numpy(np.ascontiguousarray(w.tree_parent, dtype=np.int32)).to(dev),
        "theta": torch.from_numpy(np.ascontiguousarray(w.theta, dtype=np.float32)).to(dev),
        "uniforms": None if w.uniforms is None else torch.from_numpy(w.uniforms).to(dev),
        "draft_probs": None if w.draft_probs is None else torch.from_numpy(w.draft_probs).to(dev),
    }
    return d


def run_gpu(w, dev_tensors=None):
    d = dev_tensors or to_device(w)
    out = M.mars_verify(d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], w.temperature,
                        d["uniforms"], d["draft_probs"])
    torch.cuda.synchronize()
    return out


def assert_stats_match(stats_gpu, ref_stats, sampling, label=""):
    s = {k: v.cpu().numpy() for k, v in M.unpack_stats(stats_gpu).items()}
    r = ref_stats.reshape(-1)
    for key in ("id1", "id2", "relax_ok"):
        bad = np.nonzero(s[key] != r[key])[0]
        assert bad.size == 0, f"{label}: {key} differs at rows {bad[:8]}: gpu {s[key][bad[:8]]} ref {r[key][bad[:8]]}"
    for key in ("z1", "z2"):
        bad = np.nonzero(s[key].astype(np.float64) != r[key])[0]
        assert bad.size == 0, f"{label}: {key} differs at rows {bad[:8]}"
    if sampling:
        rel = np.abs(s["sum_exp"].astype(np.float64) - r["sum_exp"]) / r["sum_exp"]
        assert rel.max() <= REL_TOL, f"{label}: sum_exp rel err {rel.max():.3e} at row {rel.argmax()}"
        return float(rel.max())
    assert (s["sum_exp"] == 0).all()
    return 0.0


def bonus_prob_floor(ref_diag):
    """Absolute tolerance of bonus_prob = f(token) / sum f.  After a rejection f(token) is a residual
    max(0, f - q) / Z (Sec. 2.3): a difference of two probabilities whose absolute error is that of its
    operands (about RESIDUAL_ABS_TOL), divided by the normaliser Z; without a rejection there is no
    cancellation and the tolerance is purely relative."""
    z = np.maximum(ref_diag["last_residual_norm"], 2e-2)      # the screening keeps Z >= 2e-2
    return np.where(ref_diag["residual_passes"] > 0, RESIDUAL_ABS_TOL / z, 0.0)


MAX_SMALL_NORM_SHARE = 0.25   # at most this share of a workload's requests (one, in a tiny batch) may meet a
                              # small normaliser whatever is drawn and be compared only up to it


def assert_decisions_agree_in_both_precisions(w, ref, label):
    """The low-margin test is decided in fp32 on both sides (what the library computes in); the plain
    definition is the fp64 one.  A generated workload keeps its rows a guard band away from the threshold,
    so the two must agree on every row -- the mirrored decision can then hide no disagreement.  (Hand-made
    inputs that sit on a threshold on purpose carry no guard band and are exempt.)"""
    if "guard" in getattr(w, "meta", {}):
        assert np.array_equal(ref["stats"]["relax_ok"], ref["stats"]["relax_ok64"]), (
            f"{label}: the fp32 and the fp64 low-margin decisions differ on guarded data")


def assert_few_small_norm(clean, label):
    n = int((~clean).sum())
    allowed = max(1, int(np.ceil(MAX_SMALL_NORM_SHARE * clean.size)))
    say(f"[info] {label}: {n} of {clean.size} requests meet a small normaliser on every draw: compared up to it")
    assert n <= allowed, f"{label}: {n} of {clean.size} requests cannot be compared in full (at most {allowed})"


def assert_prefix_parity(w, ref, outs, b, label, k=None):
    """A request whose walk meets a residual normaliser below the floor on every likely path.  Up to that
    point -- ``small_norm_plen`` accepted drafts, the rejections at ``small_norm_node`` before it -- nothing the
    walk decided depends on the small normaliser, and the GPU must agree with the oracle on all of it; what
    comes after need only be a valid outcome (a root-to-node chain, mask and codes consistent with it, a
    token inside the vocabulary).  ``outs``: numpy outputs of the GPU for the whole batch (axis k first if given)."""
    sel = (lambda a: a[b]) if k is None else (lambda a: a[k][b])
    dg = sel(ref["diag"])
    L = int(dg["small_norm_plen"])
    assert L >= 0, f"{label}: request {b} is flagged but met no small normaliser"
    rpath, gpath = sel(ref["path_idx"]), sel(outs["path_idx"])
    glen = int(sel(outs["accept_len"]))
    gmask, gdec = sel(outs["accept_mask"]), sel(outs["decision"])
    assert glen >= L and np.array_equal(gpath[:L], rpath[:L]), f"{label}: request {b}: path prefix {gpath[:L]} vs {rpath[:L]}"
    for node in rpath[:L]:
        assert gdec[node] == sel(ref["decision"])[node], f"{label}: request {b}: code of node {node}"
    par = w.tree_parent[b]
    assert (gpath[:glen] > 0).all() and (gpath[glen:] == -1).all(), f"{label}: request {b}: path padding"
    prev = 0
    for node in gpath[:glen]:
        assert par[node] == prev, f"{label}: request {b}: node {node} does not hang under {prev}"
        prev = int(node)
    if L == glen:
        assert prev == int(dg["small_norm_node"]), f"{label}: request {b}: stopped at {prev}"
    want_mask = np.zeros(w.N, np.uint8)
    want_mask[0] = 1
    want_mask[gpath[:glen]] = 1
    assert np.array_equal(gmask, want_mask), f"{label}: request {b}: mask"
    assert ((gdec != 0) == (want_mask != 0))[1:].all() and gdec[0] == 0, f"{label}: request {b}: codes off the path"
    assert 0 <= int(sel(outs["bonus_token"])) < w.V and int(sel(outs["request_status"])) == 0


def compare(w, label=None, screened=True, cdf_guard=None, allow_small_norm=False, run=None):
    """Run both sides on workload ``w`` (uniforms are screened in place first) and assert parity.
    Returns a small summary dict.  With ``allow_small_norm`` a request that meets a residual normaliser
    below the screening floor whatever uniforms are drawn is compared up to that point
    (``assert_prefix_parity``) instead of in full; their share is bounded.  The row statistics, which do
    not depend on uniforms, are compared for every row.  ``run(w)`` replaces the plain mars_verify call (another
    entry point that produces the same outputs from ``w``'s inputs)."""
    label = label or w.name
    say(f"[case] {label}: B={w.B} N={w.N} V={w.V} dtype={w.dtype} T={w.temperature} "
        f"dense_q={w.draft_probs is not None}")
    ref = screen.screen_uniforms(w, cdf_guard=cdf_guard, allow_small_norm=allow_small_norm) if screened else mars_ref.verify(
        w.logits, w.draft_tokens, w.tree_parent, w.theta, w.temperature, w.uniforms, w.draft_probs)
    assert_decisions_agree_in_both_precisions(w, ref, label)
    clean = ref.get("clean", np.ones(w.B, bool))
    out = run(w) if run is not None else run_gpu(w)
    if not clean.all():
        assert_few_small_norm(clean, label)
        outs_np = {key: getattr(out, key).cpu().numpy() for key in
                   ("accept_len", "bonus_token", "request_status", "accept_mask", "path_idx", "decision")}
        for b in np.nonzero(~clean)[0]:
            assert_prefix_parity(w, ref, outs_np, int(b), label)
    sampling = w.temperature > 0
    for key in ("accept_len", "bonus_token", "request_status", "accept_mask", "path_idx", "decision"):
        g = getattr(out, key).cpu().numpy()
        bad = np.argwhere(g[clean] != ref[key][clean])
        assert bad.size == 0, f"{label}: {key} differs at (clean request, ...) {bad[:6].tolist()}"
    s_err = assert_stats_match(out.stats, ref["stats"], sampling, label)
    dg = {k: v.cpu().numpy() for k, v in M.unpack_diag(out.diag).items()}
    rd = ref["diag"]
    ok = (ref["request_status"] == 0) & clean
    assert np.array_equal(dg["last_node"][ok], rd["last_node"][ok]), f"{label}: last_node"
    d_err = 0.0
    if sampling:
        assert np.array_equal(dg["residual_passes"][ok], rd["residual_passes"][ok]), f"{label}: residual_passes"
        for key in ("bonus_prob", "last_residual_norm"):
            a, b = dg[key][ok].astype(np.float64), rd[key][ok]
            floor = RESIDUAL_ABS_TOL if key == "last_residual_norm" else bonus_prob_floor(rd[ok])
            rel = np.maximum(np.abs(a - b) - floor, 0.0) / np.maximum(np.abs(b), 1e-30)
            rel[(a == 0) & (b == 0)] = 0
            assert rel.max(initial=0) <= REL_TOL, f"{label}: {key} rel err {rel.max():.3e} at request {rel.argmax()}"
            d_err = max(d_err, float(rel.max(initial=0)))
    summary = dict(mean_tau=float(ref["accept_len"].mean() + 1), relaxed=int((ref["decision"] == 2).sum()),
                   sum_exp_rel=s_err, diag_rel=d_err)
    say(f"[ok]   {label}: {summary}")
    return summary


INDICATOR_CODE = {"logit_ratio": M.MARS_IND_LOGIT_RATIO, "prob_ratio": M.MARS_IND_PROB_RATIO,
                  "logit_gap": M.MARS_IND_LOGIT_GAP}


def compare_ex(w, label=None, indicator="logit_ratio", thetas=None, cdf_guard=None, commit=True,
               allow_small_norm=False):
    """mars_verify_ex against the oracle: chosen indicator, optional sweep thetas[K,B] (every output
    with a leading K axis), committed sequence and kept cache rows.  Same bar as ``compare``."""
    label = label or w.name
    code = INDICATOR_CODE[indicator]
    K = 1 if thetas is None else int(np.asarray(thetas).shape[0])
    say(f"[case] {label}: B={w.B} N={w.N} V={w.V} dtype={w.dtype} T={w.temperature} "
        f"dense_q={w.draft_probs is not None} indicator={indicator} K={K} commit={commit}")
    ref = screen.screen_uniforms(w, cdf_guard=cdf_guard, indicator=code, thetas=thetas,
                                 allow_small_norm=allow_small_norm)
    assert_decisions_agree_in_both_precisions(w, ref, label)
    clean = ref["clean"]                       # [B]: requests compared in full
    d = to_device(w)
    th = d["theta"] if thetas is None else torch.from_numpy(np.ascontiguousarray(thetas, dtype=np.float32)).to(
        d["logits"].device)
    out = M.mars_verify_ex(d["logits"], d["draft_tokens"], d["tree_parent"], th, w.temperature, d["uniforms"],
                           d["draft_probs"], indicator=code, n_theta=K, want_commit=commit)
    torch.cuda.synchronize()
    if not clean.all():
        assert_few_small_norm(clean, label)
        outs_np = {key: getattr(out, key).cpu().numpy() for key in
                   ("accept_len", "bonus_token", "request_status", "accept_mask", "path_idx", "decision")}
        for b in np.nonzero(~clean)[0]:
            for k in (range(K) if thetas is not None else [None]):
                if (ref["diag"][b] if k is None else ref["diag"][k][b])["small_norm_plen"] >= 0:
                    assert_prefix_parity(w, ref, outs_np, int(b), label, k)
    sampling = w.temperature > 0
    for key in ("accept_len", "bonus_token", "request_status", "accept_mask", "path_idx", "decision"):
        g = getattr(out, key).cpu().numpy()
        assert g.shape == ref[key].shape, (key, g.shape, ref[key].shape)
        sel = (slice(None), clean) if thetas is not None else (clean,)
        bad = np.argwhere(g[sel] != ref[key][sel])
        assert bad.size == 0, f"{label}: {key} differs at (clean request index, ...) {bad[:6].tolist()}"
    gs = out.stats.reshape(K, w.B * w.N, -1)
    rs = ref["stats"].reshape(K, w.B * w.N)
    for k in range(K):
        assert_stats_match(gs[k], rs[k], sampling, f"{label}[k={k}]")
    dg = {k: v.cpu().numpy().reshape(K, w.B) for k, v in M.unpack_diag(out.diag).items()}
    rd = ref["diag"].reshape(K, w.B)
    ok = (ref["request_status"].reshape(K, w.B) == 0) & clean[None, :]
    assert np.array_equal(dg["last_node"][ok], rd["last_node"][ok]), f"{label}: last_node"
    if sampling:
        assert np.array_equal(dg["residual_passes"][ok], rd["residual_passes"][ok]), f"{label}: residual_passes"
        a, b = dg["bonus_prob"][ok].astype(np.float64), rd["bonus_prob"][ok]
        bad = np.abs(a - b) > REL_TOL * np.abs(b) + bonus_prob_floor(rd[ok])
        assert not bad.any(), f"{label}: bonus_prob gpu {a[bad][:4]} ref {b[bad][:4]}"
    if commit:
        for k in range(K):
            sel = (lambda a: a[k]) if thetas is not None else (lambda a: a)
            want = mars_ref.commit(w.draft_tokens, sel(ref["accept_len"]), sel(ref["path_idx"]), sel(ref["bonus_token"]))
            for key in ("out_tokens", "out_len"):
                g = sel(getattr(out, key).cpu().numpy())
                bad = np.argwhere(g[clean] != want[key][clean])
                assert bad.size == 0, f"{label}[k={k}]: {key} differs at {bad[:6].tolist()}"
            if clean.all():   # the compacted list depends on every request
                for key in ("keep_rows", "keep_offsets"):
                    g = sel(getattr(out, key).cpu().numpy())
                    bad = np.argwhere(g != want[key])
                    assert bad.size == 0, f"{label}[k={k}]: {key} differs at {bad[:6].tolist()}"
    summary = dict(mean_tau=np.round(ref["accept_len"].reshape(K, -1).mean(axis=1) + 1, 3).tolist(),
                   relaxed=int((ref["decision"] == 2).sum()), low_margin_rows=int(ref["stats"]["relax_ok"].sum()))
    say(f"[ok]   {label}: {summary}")
    return summary


def compare_margin(w, ranges, bins, label=None, edge_tol=1e-4):
    """mars_margin_stats against the oracle.  Rows: z1, z2 and the fp32 ratio bit-exact, p2/p1 within
    rel 1e-5.  Histograms of z1 and of the ratio, and the summary, bit-exact.  The histogram of p2/p1 goes
    through an exponential evaluated differently on the two sides: rows whose p2/p1 lies within ``edge_tol``
    cells of a cell boundary (the oracle reports the distance) may fall on either side of it, every other
    row must be counted where the oracle counts it."""
    label = label or w.name
    say(f"[case] {label}: margin statistics B={w.B} N={w.N} V={w.V} dtype={w.dtype} T={w.temperature} bins={bins}")
    ref = mars_ref.margin_stats(w.logits, w.theta, w.temperature, ranges, bins)
    d = to_device(w)
    rows, counts = M.mars_margin_stats(d["logits"], d["theta"], w.temperature, np.asarray(ranges).reshape(6), bins)
    torch.cuda.synchronize()
    rows = rows.cpu().numpy()
    counts = counts.cpu().numpy().view(np.uint32)
    r = ref["rows"].reshape(-1)
    assert np.array_equal(rows[:, 0].astype(np.float64), r["z1"]) and np.array_equal(rows[:, 1].astype(np.float64), r["z2"])
    with np.errstate(divide="ignore", invalid="ignore"):
        want_ratio = r["z2"].astype(np.float32) / r["z1"].astype(np.float32)
    assert np.array_equal(rows[:, 2], want_ratio, equal_nan=True), f"{label}: ratio"
    pr = rows[:, 3].astype(np.float64)
    rel = np.abs(pr - r["prob_ratio"]) / np.maximum(r["prob_ratio"], 1e-300)
    rel[(pr == 0) & (r["prob_ratio"] < 1e-37)] = 0          # below the fp32 range: flushed to zero
    assert rel.max() <= REL_TOL, f"{label}: p2/p1 rel err {rel.max():.3e}"
    b0, b1, b2 = (int(b) + 2 for b in bins)
    h0, h1, h2, summary = counts[:b0], counts[b0:b0 + b1], counts[b0 + b1:b0 + b1 + b2], counts[b0 + b1 + b2:]
    assert h0.tolist() == ref["hist_z1"].tolist(), f"{label}: histogram of z1"
    assert h1.tolist() == ref["hist_ratio"].tolist(), f"{label}: histogram of z2/z1"
    assert summary.tolist() == ref["summary"].tolist(), f"{label}: summary {summary.tolist()} vs {ref['summary'].tolist()}"
    diff = h2.astype(np.int64) - ref["hist_prob"].astype(np.int64)
    near = int((ref["edge_dist"] < edge_tol).sum())
    assert diff.sum() == 0 and np.abs(diff).sum() <= 2 * near, (
        f"{label}: histogram of p2/p1 differs by {np.abs(diff).sum()} counts with {near} rows near a boundary")
    assert h2.sum() == w.B * w.N
    say(f"[ok]   {label}: p2/p1 rel {rel.max():.2e}, {near} boundary rows, moved {int(np.abs(diff).sum() // 2)}, "
        f"summary {summary.tolist()}")
    return dict(near=near, moved=int(np.abs(diff).sum() // 2), summary=summary.tolist())
