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
request is clean.  Returns the oracle's output for the final uniforms.  A request
that meets a small normaliser whatever is drawn can be kept and flagged instead
(``allow_small_norm``): what its walk decided before that normaliser is still
well posed, and the oracle says where that was.
"""
import numpy as np

from . import mars_ref


def _sub(a, idx):
    return None if a is None else np.ascontiguousarray(a[idx])


def screen_uniforms(w, guard: float = 1e-4, min_norm: float = 2e-2, max_rounds: int = 200,
                    seed: int = 987654321, cdf_guard: float = None, indicator: int = 0, thetas=None,
                    allow_small_norm: bool = False, norm_rounds: int = 40):
    """``w`` is a workload object with numpy fields (logits, draft_tokens, tree_parent, theta,
    temperature, uniforms, draft_probs); ``w.uniforms`` is updated in place.

    ``thetas`` [K,B] (optional) screens for a sweep: the same uniforms serve the K walks of a
    request, so a request is re-drawn until all K of them are clean; the outputs then carry a
    leading axis of length K.

    A uniform too close to the probability it is compared with, or to a CDF step, is always cured by
    drawing again (``max_rounds`` is a safety net: exceeding it raises).  A small normaliser may not be:
    some requests meet one on every path that is at all likely (both distributions peaked on the same
    token).  Such a request is drawn again ``norm_rounds`` times; if a normaliser below ``min_norm`` is
    still met, then with ``allow_small_norm`` the request is kept with uniforms whose margins are clean
    and flagged False in the returned ``"clean"`` mask [B]: the oracle's diag then says where the first
    small normaliser was met (``small_norm_plen``, ``small_norm_node``), and a caller compares what the
    walk decided up to there, which does not depend on it.  Without ``allow_small_norm`` that raises."""
    th = np.asarray(w.theta, np.float32)[None] if thetas is None else np.asarray(thetas, np.float32)
    K = th.shape[0]
    mars_ref.set_norm_floor(min_norm)

    def run(idx=None):
        pick = (lambda a: a) if idx is None else (lambda a: _sub(a, idx))
        return [mars_ref.verify(pick(w.logits), pick(w.draft_tokens), pick(w.tree_parent),
                                th[k] if idx is None else th[k][idx], w.temperature, pick(w.uniforms),
                                pick(w.draft_probs), indicator) for k in range(K)]

    B = w.logits.shape[0]
    clean = np.ones(B, bool)
    norm_tries = np.zeros(B, np.int64)

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
        margin_dirty = np.zeros(B, bool)
        norm_dirty = np.zeros(B, bool)
        for o in outs:
            d = o["diag"]
            margin_dirty |= (d["min_accept_margin"] < guard) | (d["min_cdf_margin"] < cdf_guard)
            norm_dirty |= d["min_norm"] < min_norm
        gave_up = norm_dirty & ~margin_dirty & (norm_tries >= norm_rounds)
        if gave_up.any():
            if not allow_small_norm:
                raise RuntimeError(f"residual normaliser below {min_norm} on every draw for requests "
                                   f"{np.nonzero(gave_up)[0].tolist()}")
            clean[gave_up] = False
        clean[~norm_dirty] = True          # (a later draw may have found a path without a small normaliser)
        bad = np.nonzero(margin_dirty | (norm_dirty & clean))[0]
        if bad.size == 0:
            return result(outs)
        rounds += 1
        if rounds > max_rounds + norm_rounds:
            raise RuntimeError(f"uniform guard band not reached for requests {bad.tolist()}")
        norm_tries[bad] += norm_dirty[bad]
        for b in bad:
            rng = np.random.default_rng(np.random.SeedSequence([seed, rounds, int(b)]))
            w.uniforms[b] = rng.random(w.uniforms.shape[1], dtype=np.float32)
        for o, sub in zip(outs, run(bad)):
            for k, v in sub.items():
                o[k][bad] = v
