"""Guard bands on the uniforms of a sampling-mode workload -- test infrastructure only.

The fp64 oracle and an fp32 implementation can only be asked for identical
decisions when no uniform sits within rounding distance of the probability it
is compared with.  ``screen_uniforms`` re-draws, per request and from a seed of
its own, the uniforms of every request whose smallest decision margin (as the
oracle reports it) is below ``guard``:

* acceptance tests (Eq. 1):  |u - f(x)/q(x)| >= guard;
* the final inverse-CDF draw: u * sum(f) at least ``cdf_guard`` * sum(f) away from
  the CDF steps on either side of the chosen token (``cdf_guard`` defaults to ``guard``;
  a flat distribution over a large vocabulary has no token wider than 2e-4 and needs a
  narrower band, which is sound as long as it stays well above the fp32 error of a
  normalised prefix sum, a few 1e-7);
* residual normalisers Z >= ``min_norm``: Z is a difference of probability masses of
  order 1, so an fp32 evaluation carries an absolute error of a few 1e-7 whatever its
  size, and the next acceptance probability inherits the relative error 1e-7/Z; below
  about 1e-2 that would come within reach of the guard band.

The path may change after a re-draw, so the oracle is run again until every
request is clean.  Returns the oracle's output for the final uniforms.
"""
import numpy as np

from . import mars_ref


def _sub(a, idx):
    return None if a is None else np.ascontiguousarray(a[idx])


def screen_uniforms(w, guard: float = 1e-4, min_norm: float = 2e-2, max_rounds: int = 200,
                    seed: int = 987654321, cdf_guard: float = None, indicator: int = 0, thetas=None,
                    drop_unscreenable: bool = False):
    """``w`` is a workload object with numpy fields (logits, draft_tokens, tree_parent, theta,
    temperature, uniforms, draft_probs); ``w.uniforms`` is updated in place.

    ``thetas`` [K,B] (optional) screens for a sweep: the same uniforms serve the K walks of a
    request, so a request is re-drawn until all K of them are clean; the outputs then carry a
    leading axis of length K.

    Some requests cannot be screened whatever is drawn (a peaked distribution whose residual mass stays
    below ``min_norm`` on every path that is at all likely).  With ``drop_unscreenable`` they are given
    up after ``max_rounds`` and flagged False in the returned ``"clean"`` mask [B] (their expected values
    are not well posed and a caller leaves them out of its comparison); otherwise that raises."""
    th = np.asarray(w.theta, np.float32)[None] if thetas is None else np.asarray(thetas, np.float32)
    K = th.shape[0]

    def run(idx=None):
        pick = (lambda a: a) if idx is None else (lambda a: _sub(a, idx))
        return [mars_ref.verify(pick(w.logits), pick(w.draft_tokens), pick(w.tree_parent),
                                th[k] if idx is None else th[k][idx], w.temperature, pick(w.uniforms),
                                pick(w.draft_probs), indicator) for k in range(K)]

    clean = np.ones(w.logits.shape[0], bool)

    def result(outs):
        r = outs[0] if thetas is None else {key: np.stack([o[key] for o in outs]) for key in outs[0]}
        r["clean"] = clean
        return r

    outs = run()
    if not w.temperature > 0:
        return result(outs)
    if cdf_guard is None:
        cdf_guard = guard
    rounds = 0
    while True:
        dirty = np.zeros(w.uniforms.shape[0], bool)
        for o in outs:
            d = o["diag"]
            dirty |= (d["min_accept_margin"] < guard) | (d["min_cdf_margin"] < cdf_guard) | (d["min_norm"] < min_norm)
        bad = np.nonzero(dirty & clean)[0]
        if bad.size == 0:
            return result(outs)
        rounds += 1
        if rounds > max_rounds:
            if not drop_unscreenable:
                raise RuntimeError(f"uniform guard band not reached for requests {bad.tolist()}")
            clean[bad] = False
            return result(outs)
        for b in bad:
            rng = np.random.default_rng(np.random.SeedSequence([seed, rounds, int(b)]))
            w.uniforms[b] = rng.random(w.uniforms.shape[1], dtype=np.float32)
        for o, sub in zip(outs, run(bad)):
            for k, v in sub.items():
                o[k][bad] = v
