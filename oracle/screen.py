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
                    seed: int = 987654321, cdf_guard: float = None):
    """``w`` is a workload object with numpy fields (logits, draft_tokens, tree_parent, theta,
    temperature, uniforms, draft_probs); ``w.uniforms`` is updated in place."""
    out = mars_ref.verify(w.logits, w.draft_tokens, w.tree_parent, w.theta, w.temperature,
                          w.uniforms, w.draft_probs)
    if not w.temperature > 0:
        return out
    if cdf_guard is None:
        cdf_guard = guard
    rounds = 0
    while True:
        d = out["diag"]
        bad = np.nonzero((d["min_accept_margin"] < guard) | (d["min_cdf_margin"] < cdf_guard)
                         | (d["min_norm"] < min_norm))[0]
        if bad.size == 0:
            return out
        rounds += 1
        if rounds > max_rounds:
            raise RuntimeError(f"uniform guard band not reached for requests {bad.tolist()}")
        for b in bad:
            rng = np.random.default_rng(np.random.SeedSequence([seed, rounds, int(b)]))
            w.uniforms[b] = rng.random(w.uniforms.shape[1], dtype=np.float32)
        sub = mars_ref.verify(_sub(w.logits, bad), _sub(w.draft_tokens, bad), _sub(w.tree_parent, bad),
                              _sub(w.theta, bad), w.temperature, _sub(w.uniforms, bad),
                              _sub(w.draft_probs, bad))
        for k, v in sub.items():
            out[k][bad] = v
