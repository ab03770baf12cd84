"""CPU oracle for verification straight from the last hidden states -- test infrastructure only.

Eq. 2 of the paper: the logits of a row are z = W h.  With a bf16 model the logits leave the LM
head rounded to bf16; this module defines them as the exact product rounded once, to nearest even:

    z[r, v] = bf16( sum_k h[r, k] * W[v, k] )        (sum in fp64; products of bf16 values are exact)

and then runs the greedy pass of ``mars_ref`` on those logits.  An implementation that accumulates
in fp32 obtains the same bf16 value unless the exact sum lies within its accumulation error of a
rounding boundary; ``rounding_clearance`` reports that distance for the entries that can decide a
row (its largest ones), so that a test can keep its rows clear of the boundaries, the same way the
logits workloads keep their ratios clear of the threshold.
"""
import numpy as np

from . import mars_ref


def bf16_round(x):
    """Round doubles to bf16 (8 significant bits, nearest, ties to even) in one step.
    Returns (values as float64, bit patterns as uint16).  Normal range only."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0)                   # 8 significant bits; rint rounds ties to even
    v = np.ldexp(q, e - 8)
    bits = (v.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)  # exact: v fits bf16
    return v, bits


def bf16_widen(bits):
    """bf16 bit patterns (uint16) as float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def logits_exact(hidden_bits, weight_bits, chunk=4096):
    """Eq. 2 in fp64 for rows hidden_bits[R,H] against weight_bits[V,H]: [R,V] float64."""
    h = bf16_widen(hidden_bits)
    R = h.shape[0]
    V = weight_bits.shape[0]
    out = np.empty((R, V), dtype=np.float64)
    for v0 in range(0, V, chunk):
        v1 = min(V, v0 + chunk)
        out[:, v0:v1] = h @ bf16_widen(weight_bits[v0:v1]).T
    return out


def rounding_clearance(exact_row, window=2.0 ** -6):
    """Smallest relative distance to a bf16 rounding boundary among the entries of a row that can
    be one of its two largest after rounding: those within ``window`` (relative) of the second
    largest exact value.  A boundary is the midpoint of two neighbouring bf16 values."""
    x = np.asarray(exact_row, dtype=np.float64)
    second = np.partition(x, x.size - 2)[-2]
    cand = x[x >= second - window * abs(second)]
    cand = cand[cand != 0.0]
    if cand.size == 0:
        return np.inf
    m, _ = np.frexp(np.abs(cand))
    t = m * 256.0                            # in [128, 256): the bf16 grid is the integers here
    frac = t - np.floor(t)
    return float(np.min(np.abs(frac - 0.5) / t))


def lmhead_verify(hidden_bits, weight_bits, draft_tokens, tree_parent, theta, indicator=mars_ref.IND_LOGIT_RATIO,
                  exact=None):
    """Greedy verification (Alg. 1 on a chain or tree) from hidden states [B,N,H] and the LM-head
    weight [V,H], both bf16 bit patterns.  Returns the dict of ``mars_ref.verify`` plus
    ``logits_bits`` [B,N,V], ``exact`` [B*N,V] and ``clearance`` [B,N].  ``exact`` may be handed in
    (the caller updated a few rows or columns of an earlier result)."""
    B, N, H = hidden_bits.shape
    V = weight_bits.shape[0]
    if exact is None:
        exact = logits_exact(hidden_bits.reshape(B * N, H), weight_bits)
    _, bits = bf16_round(exact)
    bits = bits.reshape(B, N, V)
    out = mars_ref.verify(bits, draft_tokens, tree_parent, theta, 0.0, indicator=indicator)
    out["logits_bits"] = bits
    out["exact"] = exact
    out["clearance"] = np.array([rounding_clearance(exact[r]) for r in range(B * N)]).reshape(B, N)
    return out


def lmhead_verify_sampling(hidden_bits, weight_bits, draft_tokens, tree_parent, theta, temperature, uniforms,
                           draft_probs=None, indicator=mars_ref.IND_LOGIT_RATIO, exact=None):
    """Sampling-mode verification (Eq. 1 with the relaxed runner-up, residual resampling: ``mars_ref.verify`` at
    temperature > 0) on the logits of Eq. 2 as defined above: the exact product rounded once to bf16.  Eq. 3
    runs over the whole row, so every logit counts: an fp32-accumulating implementation agrees with this
    only where its sums are exact (lattice inputs) or where no entry sits on a rounding boundary.
    Returns the dict of ``mars_ref.verify`` plus ``logits_bits`` [B,N,V] and ``exact`` [B*N,V]."""
    B, N, H = hidden_bits.shape
    V = weight_bits.shape[0]
    if exact is None:
        exact = logits_exact(hidden_bits.reshape(B * N, H), weight_bits)
    _, bits = bf16_round(exact)
    bits = bits.reshape(B, N, V)
    out = mars_ref.verify(bits, draft_tokens, tree_parent, theta, temperature, uniforms, draft_probs, indicator)
    out["logits_bits"] = bits
    out["exact"] = exact
    return out


def screen_lmhead(w, clearance=4e-5, guard=1e-4, indicator=mars_ref.IND_LOGIT_RATIO, max_rounds=50, requests=None):
    """Redraw (``w.redraw_rows``) the rows of an LM-head workload whose deciding logits lie within
    ``clearance`` (relative) of a bf16 rounding boundary, or whose low-margin quantity lies within
    ``guard`` of the request's threshold, until none is left.  Returns ``lmhead_verify``'s result
    for the final inputs.  Only the redrawn rows and the two vocabulary columns each of them owns
    are recomputed between rounds.

    ``requests`` (a list of request indices) restricts the work to those requests: the result then
    describes the sub-batch they form, in the order given (a redrawn row still changes the weight
    rows it owns, which every request sees)."""
    B, N, H, V = w.B, w.N, w.H, w.V
    req = np.arange(B) if requests is None else np.asarray(requests, dtype=np.int64)
    flat = (req[:, None] * N + np.arange(N)[None, :]).reshape(-1)        # flat rows of the sub-batch
    theta = np.asarray(w.theta, np.float32)[req]
    exact = None
    for round_ in range(1, max_rounds + 1):
        hid = w.hidden.reshape(B * N, H)
        out = lmhead_verify(hid[flat].reshape(req.size, N, H), w.weight, w.draft_tokens[req], w.tree_parent[req],
                            theta, indicator, exact)
        exact = out["exact"]
        st = out["stats"]
        th = theta.astype(np.float64)[:, None]
        if indicator == mars_ref.IND_LOGIT_RATIO:
            near = (st["z1"] > 0) & (np.abs(st["ratio"] - th) < guard)
        elif indicator == mars_ref.IND_PROB_RATIO:
            near = np.abs(st["prob_ratio"] - th) < guard
        else:
            near = np.abs(st["gap"] - th) < guard
        dirty = np.nonzero(((out["clearance"] < clearance) | near).reshape(-1))[0]   # positions in the sub-batch
        if dirty.size == 0:
            return out
        w.redraw_rows(flat[dirty], round_)
        hid = w.hidden.reshape(B * N, H)
        exact[dirty] = logits_exact(hid[flat[dirty]], w.weight)
        cols = w.planted.reshape(B * N, 2)[flat[dirty]].reshape(-1)
        cols = cols[cols >= 0]
        if cols.size:
            exact[:, cols] = logits_exact(hid[flat], w.weight[cols])
    raise RuntimeError("rows still inside a guard band after the last round")
