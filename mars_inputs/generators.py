"""Seeded generators for logits, draft trees, draft tokens, uniforms and draft distributions.

Recipe (one request at a time, each with its own seed so the result does not
depend on how many threads generate):

* background logits: i.i.d. N(0, 3^2), or Gumbel(0, 2) for a long tail;
* in a stated fraction of rows two "planted" entries at random distinct ids:
  top ~ U(15, 30) and runner-up = r * top with r ~ U(r_lo, r_hi) -- the
  low-margin rows the paper's Sec. 3.1 / Fig. 5(b) describe;
* the row is rounded to its storage type (bf16: round-to-nearest-even) and is
  drawn again while the ratio of its two largest stored values lies within
  ``guard`` of the request's threshold (a guard band on the data, so that a test
  of "ratio > threshold" has the same answer in any precision);
* chains (parent(i) = i-1) or random trees with a depth and fan-out limit;
* the draft token of node i looks at the row of parent(i): the largest entry
  w.p. 0.6, the second largest w.p. 0.25, otherwise uniform over the vocabulary;
  siblings get distinct tokens;
* uniforms: fp32 in [0, 1), one per node plus one for the final draw;
* dense draft distribution (optional): softmax of the stored row plus N(0, 1)
  noise, kept in fp32.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

GUARD = 1e-4


# --------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- trees
def chain_parents(N: int) -> np.ndarray:
    p = np.arange(-1, N - 1, dtype=np.int32)
    return p


def random_tree(rng: np.random.Generator, N: int, depth: int, max_children: int) -> np.ndarray:
    """Parents of a random tree: node i hangs under a uniformly chosen earlier node that
    still has room; trees that do not reach exactly ``depth`` are drawn again."""
    if N == 1:
        return np.array([-1], dtype=np.int32)
    if depth * 1 > N - 1:
        raise ValueError("tree cannot reach the requested depth")
    capacity, level = 1, 1
    for _ in range(depth):
        level *= max_children
        capacity += level
        if capacity >= N:
            break
    if capacity < N:
        raise ValueError(f"a tree of depth {depth} with at most {max_children} children per node holds "
                         f"{capacity} nodes, not {N}")
    while True:
        parent = np.full(N, -1, dtype=np.int32)
        d = np.zeros(N, dtype=np.int32)
        nch = np.zeros(N, dtype=np.int32)
        ok = True
        for i in range(1, N):
            cands = np.nonzero((nch[:i] < max_children) & (d[:i] < depth))[0]
            if cands.size == 0:
                ok = False
                break
            p = int(cands[rng.integers(cands.size)])
            parent[i] = p
            d[i] = d[p] + 1
            nch[p] += 1
        if ok and int(d.max()) == depth:
            return parent


# --------------------------------------------------------------------------- workload container
@dataclass
class Workload:
    name: str
    B: int
    N: int
    V: int
    dtype: str                      # "f32" or "bf16": storage type of the logits
    temperature: float
    theta: np.ndarray               # [B] fp32
    logits: np.ndarray              # [B,N,V] float32, or uint16 bf16 bit patterns
    draft_tokens: np.ndarray        # [B,N] int32
    tree_parent: np.ndarray         # [B,N] int32
    uniforms: Optional[np.ndarray]  # [B,N+1] fp32 or None
    draft_probs: Optional[np.ndarray] = None  # [B,N,V] fp32 or None
    meta: dict = field(default_factory=dict)

    def logits_f32(self) -> np.ndarray:
        return bf16_bits_to_f32(self.logits) if self.dtype == "bf16" else self.logits

    @property
    def rows(self) -> int:
        return self.B * self.N

    @property
    def logits_bytes(self) -> int:
        return self.B * self.N * self.V * (2 if self.dtype == "bf16" else 4)


def _rng(seed: int, stream: int, b: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([int(seed), int(stream), int(b)]))


def _two_largest(row: np.ndarray):
    part = np.partition(row, row.size - 2)
    return float(part[-1]), float(part[-2])


def _margin_quantity(a: float, b2: float, indicator: str, temperature: float):
    """The quantity of the two largest stored values that a threshold is compared with (a property of the
    data, like the ratio): their ratio (None off the positive domain), exp(-(gap)/T'), or their gap."""
    if indicator == "logit_ratio":
        return b2 / a if a > 0.0 else None
    if indicator == "prob_ratio":
        return math.exp(-(a - b2) / (temperature if temperature > 0 else 1.0))
    if indicator == "logit_gap":
        return a - b2
    raise ValueError(indicator)


def _gen_row(rng, V, background, planted, r_range, thetas_b, dtype, guard, indicator="logit_ratio",
             temperature=0.0):
    while True:
        if background == "normal3":
            z = rng.standard_normal(V, dtype=np.float32) * np.float32(3.0)
        elif background == "gumbel2":
            z = rng.gumbel(0.0, 2.0, V).astype(np.float32)
        else:
            raise ValueError(background)
        if planted:
            ids = rng.choice(V, size=2, replace=False)
            top = rng.uniform(15.0, 30.0)
            r = rng.uniform(r_range[0], r_range[1])
            z[ids[0]] = np.float32(top)
            z[ids[1]] = np.float32(r * top)
        if dtype == "bf16":
            bits = f32_to_bf16_bits(z)
            stored = bf16_bits_to_f32(bits)
        else:
            bits = None
            stored = z
        a, b2 = _two_largest(stored)
        x = _margin_quantity(a, b2, indicator, temperature)
        if x is not None and any(abs(x - float(t)) < guard for t in thetas_b):
            continue  # inside the guard band of a threshold: draw the row again
        return stored, bits


def _top2_ids(row: np.ndarray):
    i1 = int(np.argmax(row))
    keep = row[i1]
    row[i1] = -np.inf
    i2 = int(np.argmax(row))
    row[i1] = keep
    return i1, i2


def _gen_request(b, *, seed, B, N, V, dtype, background, plant_frac, r_range, thetas_b,
                 tree, sampling, dense_q, guard, indicator, temperature):
    rl = _rng(seed, 1000, b)
    rt = _rng(seed, 2000, b)
    rk = _rng(seed, 3000, b)
    ru = _rng(seed, 4000, b)
    rq = _rng(seed, 5000, b)

    stored = np.empty((N, V), dtype=np.float32)
    bits = np.empty((N, V), dtype=np.uint16) if dtype == "bf16" else None
    for i in range(N):
        planted = bool(rl.random() < plant_frac)
        s, bt = _gen_row(rl, V, background, planted, r_range, thetas_b, dtype, guard, indicator, temperature)
        stored[i] = s
        if bits is not None:
            bits[i] = bt

    if tree["kind"] == "chain":
        parent = chain_parents(N)
    else:
        parent = random_tree(rt, N, tree["depth"], tree["max_children"])

    top = [_top2_ids(stored[i]) for i in range(N)]
    tokens = np.zeros(N, dtype=np.int32)
    tokens[0] = int(rk.integers(V))  # the committed root token; never read by the pass
    used = {}
    for i in range(1, N):
        p = int(parent[i])
        taken = used.setdefault(p, set())
        while True:
            c = rk.random()
            if c < 0.6:
                t = top[p][0]
            elif c < 0.85:
                t = top[p][1]
            else:
                t = int(rk.integers(V))
            if t not in taken:
                break
        taken.add(t)
        tokens[i] = t

    uniforms = ru.random(N + 1, dtype=np.float32) if sampling else None

    q = None
    if dense_q:
        q = np.empty((N, V), dtype=np.float32)
        for i in range(N):
            x = stored[i].astype(np.float64) + rq.standard_normal(V)
            x -= x.max()
            e = np.exp(x)
            q[i] = (e / e.sum()).astype(np.float32)
    return (bits if bits is not None else stored), parent, tokens, uniforms, q


def make_workload(name: str, *, B: int, N: int, V: int, dtype: str, temperature: float,
                  tree: dict, background: str = "normal3", plant_frac: float = 0.4,
                  r_range: Sequence[float] = (0.80, 1.00), theta_choices: Sequence[float] = (0.9,),
                  dense_q: bool = False, seed: int = 0, guard: float = GUARD,
                  threads: Optional[int] = None, indicator: str = "logit_ratio",
                  sweep_thetas: Sequence[float] = ()) -> Workload:
    """Generate one workload; every request has its own seeds (seed, stream, b).

    ``indicator`` names the quantity the thresholds are compared with (logit_ratio, prob_ratio, logit_gap):
    the guard band around theta is kept on that quantity.  ``sweep_thetas`` are further thresholds (of a
    sweep over theta) every row also keeps clear of."""
    assert dtype in ("f32", "bf16")
    if tree["kind"] != "chain" and tree["max_children"] > V:
        raise ValueError("siblings carry distinct draft tokens: max_children cannot exceed V")
    sampling = temperature > 0
    rth = _rng(seed, 6000, 0)
    theta = np.asarray(theta_choices, dtype=np.float32)[rth.integers(len(theta_choices), size=B)]
    if threads is None:
        threads = min(16, os.cpu_count() or 1, B)
    kw = dict(seed=seed, B=B, N=N, V=V, dtype=dtype, background=background, plant_frac=plant_frac,
              r_range=tuple(r_range), tree=tree, sampling=sampling, dense_q=dense_q, guard=guard,
              indicator=indicator, temperature=float(np.float32(temperature)))
    sweep = [float(np.float32(t)) for t in sweep_thetas]

    def job(b):
        return _gen_request(b, thetas_b=[float(theta[b])] + sweep, **kw)

    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            parts = list(ex.map(job, range(B)))
    else:
        parts = [job(b) for b in range(B)]

    ldt = np.uint16 if dtype == "bf16" else np.float32
    logits = np.empty((B, N, V), dtype=ldt)
    parents = np.empty((B, N), dtype=np.int32)
    tokens = np.empty((B, N), dtype=np.int32)
    uniforms = np.empty((B, N + 1), dtype=np.float32) if sampling else None
    dprobs = np.empty((B, N, V), dtype=np.float32) if dense_q else None
    for b, (lg, pa, tk, un, q) in enumerate(parts):
        logits[b] = lg
        parents[b] = pa
        tokens[b] = tk
        if sampling:
            uniforms[b] = un
        if dense_q:
            dprobs[b] = q
        parts[b] = None
    return Workload(name=name, B=B, N=N, V=V, dtype=dtype, temperature=float(temperature),
                    theta=theta, logits=logits, draft_tokens=tokens, tree_parent=parents,
                    uniforms=uniforms, draft_probs=dprobs,
                    meta=dict(seed=seed, tree=tree, background=background, plant_frac=plant_frac,
                              r_range=tuple(r_range), dense_q=dense_q, guard=guard, indicator=indicator,
                              sweep_thetas=tuple(sweep)))


# --------------------------------------------------------------------------- the five stated configurations
# N counts the root: a chain of 8 draft positions has 9 rows ("+1 bonus row").
CONFIGS = {
    0: dict(name="cfg0_greedy_chain8_V32000_f32", B=1, N=9, V=32000, dtype="f32", temperature=0.0,
            tree={"kind": "chain"}, background="normal3", plant_frac=0.4, r_range=(0.80, 1.00),
            theta_choices=(0.9,), dense_q=False),
    1: dict(name="cfg1_tree60_V151936_bf16", B=1, N=60, V=151936, dtype="bf16", temperature=1.0,
            tree={"kind": "tree", "depth": 6, "max_children": 4}, background="normal3",
            plant_frac=0.5, r_range=(0.80, 1.00), theta_choices=(0.9,), dense_q=False),
    2: dict(name="cfg2_B16_tree60_V151936_bf16_T0.7_denseq", B=16, N=60, V=151936, dtype="bf16",
            temperature=0.7, tree={"kind": "tree", "depth": 6, "max_children": 4},
            background="normal3", plant_frac=0.5, r_range=(0.80, 1.00), theta_choices=(0.9,),
            dense_q=True),
    3: dict(name="cfg3_B64_chain8_V128256_bf16_greedy", B=64, N=9, V=128256, dtype="bf16",
            temperature=0.0, tree={"kind": "chain"}, background="gumbel2", plant_frac=0.3,
            r_range=(0.80, 1.00), theta_choices=(0.85, 0.9, 0.95), dense_q=False),
    4: dict(name="cfg4_B256_tree26_V151936_f32_T1", B=256, N=26, V=151936, dtype="f32",
            temperature=1.0, tree={"kind": "tree", "depth": 5, "max_children": 4},
            background="normal3", plant_frac=0.6, r_range=(0.85, 1.00), theta_choices=(0.9,),
            dense_q=False),
    # Not one of the five stated configurations: the paper's "framework-decoupled" experiment runs the rule
    # inside standard speculative decoding with gamma = 6 drafts per step and a real draft distribution
    # (T = 1); the same shape at a serving batch size.
    5: dict(name="spd_B128_chain6_V151936_bf16_T1_dense_q", B=128, N=7, V=151936, dtype="bf16",
            temperature=1.0, tree={"kind": "chain"}, background="normal3", plant_frac=0.5,
            r_range=(0.80, 1.00), theta_choices=(0.9,), dense_q=True),
}


def make_config(cfg: int, *, temperature: Optional[float] = None, threads: Optional[int] = None,
                **override) -> Workload:
    """One of the five stated configurations (seed = cfg); keyword overrides (B=, N=, V=, ...)
    give reduced-size variants of the same recipe for quick parity cases."""
    spec = dict(CONFIGS[cfg])
    spec.update(override)
    if temperature is not None:
        spec["temperature"] = temperature
    name = spec.pop("name")
    seed = spec.pop("seed", cfg)
    if override or temperature is not None:
        name += "_variant"
    return make_workload(name, seed=seed, threads=threads, **spec)
