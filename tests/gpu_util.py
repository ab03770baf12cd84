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


def compare(w, label=None, screened=True, cdf_guard=None):
    """Run both sides on workload ``w`` (uniforms are screened in place first) and assert parity.
    Returns a small summary dict."""
    label = label or w.name
    say(f"[case] {label}: B={w.B} N={w.N} V={w.V} dtype={w.dtype} T={w.temperature} "
        f"dense_q={w.draft_probs is not None}")
    ref = screen.screen_uniforms(w, cdf_guard=cdf_guard) if screened else mars_ref.verify(
        w.logits, w.draft_tokens, w.tree_parent, w.theta, w.temperature, w.uniforms, w.draft_probs)
    out = run_gpu(w)
    sampling = w.temperature > 0
    for key in ("accept_len", "bonus_token", "request_status", "accept_mask", "path_idx", "decision"):
        g = getattr(out, key).cpu().numpy()
        bad = np.argwhere(g != ref[key])
        assert bad.size == 0, (f"{label}: {key} differs at {bad[:6].tolist()}: gpu "
                               f"{g[tuple(bad[0])]} ref {ref[key][tuple(bad[0])]}")
    s_err = assert_stats_match(out.stats, ref["stats"], sampling, label)
    dg = {k: v.cpu().numpy() for k, v in M.unpack_diag(out.diag).items()}
    rd = ref["diag"]
    ok = ref["request_status"] == 0
    assert np.array_equal(dg["last_node"][ok], rd["last_node"][ok]), f"{label}: last_node"
    d_err = 0.0
    if sampling:
        assert np.array_equal(dg["residual_passes"][ok], rd["residual_passes"][ok]), f"{label}: residual_passes"
        for key in ("bonus_prob", "last_residual_norm"):
            a, b = dg[key][ok].astype(np.float64), rd[key][ok]
            floor = RESIDUAL_ABS_TOL if key == "last_residual_norm" else 0.0
            rel = np.maximum(np.abs(a - b) - floor, 0.0) / np.maximum(np.abs(b), 1e-30)
            rel[(a == 0) & (b == 0)] = 0
            assert rel.max(initial=0) <= REL_TOL, f"{label}: {key} rel err {rel.max():.3e} at request {rel.argmax()}"
            d_err = max(d_err, float(rel.max(initial=0)))
    summary = dict(mean_tau=float(ref["accept_len"].mean() + 1), relaxed=int((ref["decision"] == 2).sum()),
                   sum_exp_rel=s_err, diag_rel=d_err)
    say(f"[ok]   {label}: {summary}")
    return summary
