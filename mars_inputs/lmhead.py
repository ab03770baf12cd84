"""Seeded inputs for verification straight from the last hidden states (Eq. 2: z = W h).

Recipe:

* LM-head weight ``W[V,H]``: i.i.d. N(0, (3/sqrt(H))^2), rounded to bf16 -- with hidden states of
  unit variance the logits of a row are then N(0, 3^2) like the background of the logits workloads;
* hidden states ``h[B,N,H]``: i.i.d. N(0, 1), rounded to bf16, one seed per row;
* in a stated fraction of rows two "planted" vocabulary entries (ids taken from one seeded
  permutation of the vocabulary, so no two rows share one): their weight rows are replaced by
  ``(t / |h|^2) h`` and ``(r t / |h|^2) h`` with t ~ U(20, 30), r ~ U(r_lo, r_hi), which puts a logit
  of about t and one of about r t into that row (and only ~t/sqrt(H) into the other rows) -- the
  low-margin rows of Sec. 3.1, known by construction without forming any logit here;
* trees / chains and draft tokens as for the logits workloads: the token of node i is the planted
  top entry of its parent's row w.p. 0.6, the planted runner-up w.p. 0.25, otherwise uniform over
  the vocabulary (always uniform under an unplanted parent); siblings get distinct tokens.

With ``lattice=True`` every hidden state is a multiple of 2^-5 (below 8 in magnitude) and every weight a
multiple of 2^-10 (below 1/4): both are still bf16 values, every product is a multiple of 2^-15, and as long
as the sum of the products' magnitudes of a (row, vocabulary entry) pair stays below 512 -- it is about 125
for the background and at most 30 for a planted entry; a test checks it -- every partial sum, in any order
of addition, is a multiple of 2^-15 below 2^9 and therefore exact in fp32.  An fp32-accumulating LM head
then produces the exact product, and its bf16 rounding is that of the exact value: such workloads serve
paths in which every logit matters (sampling: Eq. 3 runs over the whole row), where keeping a few deciding
entries clear of the rounding boundaries is not enough.  Sampling-mode workloads also carry uniforms
[B,N+1] and, optionally, a dense fp32 draft distribution [B,N,V] (softmax of seeded N(0, 2^2) noise,
independent of the target: no logit is formed here).

``redraw_rows`` draws chosen rows again (hidden state and planted weight rows, same ids) from seeds
of their own; a test uses it to move rows whose exact logits sit too close to a rounding boundary
or to the threshold.  No logit is computed in this module.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Sequence

import numpy as np

from .generators import _rng, bf16_bits_to_f32, chain_parents, f32_to_bf16_bits, random_tree


@dataclass
class LmHeadWorkload:
    name: str
    B: int
    N: int
    H: int
    V: int
    theta: np.ndarray         # [B] fp32
    hidden: np.ndarray        # [B,N,H] uint16 (bf16 bit patterns)
    weight: np.ndarray        # [V,H] uint16 (bf16 bit patterns)
    draft_tokens: np.ndarray  # [B,N] int32
    tree_parent: np.ndarray   # [B,N] int32
    planted: np.ndarray       # [B,N,2] int32: planted (top, runner-up) ids of the row, -1 if none
    meta: dict = field(default_factory=dict)
    temperature: float = 0.0
    uniforms: np.ndarray = None     # [B,N+1] fp32 (sampling-mode workloads)
    draft_probs: np.ndarray = None  # [B,N,V] fp32 or None (one-hot draft distribution)

    @property
    def rows(self) -> int:
        return self.B * self.N

    def _draw_row(self, row: int, round_: int) -> None:
        rng = _rng(self.meta["seed"], 7100 + round_, row)
        h32 = rng.standard_normal(self.H, dtype=np.float32)
        if self.meta.get("lattice"):
            h32 = _to_lattice(h32, 5, 7.96875)
        hb = f32_to_bf16_bits(h32)
        self.hidden.reshape(self.rows, self.H)[row] = hb
        ids = self.planted.reshape(self.rows, 2)[row]
        if ids[0] < 0:
            return
        h = bf16_bits_to_f32(hb).astype(np.float64)
        t = rng.uniform(20.0, 30.0)
        r = rng.uniform(*self.meta["r_range"])
        unit = h / float(h @ h)
        top, second = (t * unit).astype(np.float32), (r * t * unit).astype(np.float32)
        if self.meta.get("lattice"):
            top, second = _to_lattice(top, 10, 0.2490234375), _to_lattice(second, 10, 0.2490234375)
        self.weight[ids[0]] = f32_to_bf16_bits(top)
        self.weight[ids[1]] = f32_to_bf16_bits(second)

    def redraw_rows(self, rows: Sequence[int], round_: int) -> None:
        """Draw the given flat rows (b*N + i) again; ``round_`` >= 1 selects the seed."""
        assert round_ >= 1
        for row in rows:
            self._draw_row(int(row), int(round_))


def _to_lattice(x: np.ndarray, bits: int, limit: float) -> np.ndarray:
    """Nearest multiple of 2^-bits, clipped to +-limit (itself such a multiple with at most 8 significant bits)."""
    s = np.float32(2.0 ** bits)
    return np.clip(np.rint(x * s) / s, -limit, limit).astype(np.float32)


def make_lmhead_workload(name: str, *, B: int, N: int, H: int, V: int, tree: dict, plant_frac: float = 0.6,
                         r_range: Sequence[float] = (0.80, 1.00), theta_choices: Sequence[float] = (0.9,),
                         seed: int = 0, lattice: bool = False, temperature: float = 0.0,
                         dense_q: bool = False) -> LmHeadWorkload:
    rows = B * N
    if V < 2 * rows + 2:
        raise ValueError("every row needs two vocabulary entries of its own: V >= 2*B*N + 2")
    if tree["kind"] != "chain" and tree["max_children"] > V:
        raise ValueError("siblings carry distinct draft tokens: max_children cannot exceed V")
    theta = np.asarray(theta_choices, dtype=np.float32)[_rng(seed, 6000, 0).integers(len(theta_choices), size=B)]

    weight = np.empty((V, H), dtype=np.uint16)
    scale = np.float32(3.0 / np.sqrt(H))
    step = max(1, (1 << 22) // H)
    for c, v0 in enumerate(range(0, V, step)):
        v1 = min(V, v0 + step)
        blk = _rng(seed, 7000, c).standard_normal((v1 - v0, H), dtype=np.float32) * scale
        weight[v0:v1] = f32_to_bf16_bits(_to_lattice(blk, 10, 0.2490234375) if lattice else blk)

    perm = _rng(seed, 7200, 0).permutation(V)[:2 * rows].astype(np.int32).reshape(rows, 2)
    is_planted = _rng(seed, 7201, 0).random(rows) < plant_frac
    planted = np.where(is_planted[:, None], perm, -1).astype(np.int32).reshape(B, N, 2)

    parents = np.empty((B, N), dtype=np.int32)
    tokens = np.empty((B, N), dtype=np.int32)
    for b in range(B):
        rt, rk = _rng(seed, 2000, b), _rng(seed, 3000, b)
        parent = chain_parents(N) if tree["kind"] == "chain" else random_tree(rt, N, tree["depth"], tree["max_children"])
        parents[b] = parent
        tokens[b, 0] = int(rk.integers(V))  # the committed root token; never read by the pass
        used = {}
        for i in range(1, N):
            p = int(parent[i])
            taken = used.setdefault(p, set())
            ids = planted[b, p]
            while True:
                c = rk.random()
                if ids[0] >= 0 and c < 0.6:
                    t = int(ids[0])
                elif ids[0] >= 0 and c < 0.85:
                    t = int(ids[1])
                else:
                    t = int(rk.integers(V))
                if t not in taken:
                    break
            taken.add(t)
            tokens[b, i] = t

    w = LmHeadWorkload(name=name, B=B, N=N, H=H, V=V, theta=theta,
                       hidden=np.empty((B, N, H), dtype=np.uint16), weight=weight, draft_tokens=tokens,
                       tree_parent=parents, planted=planted,
                       meta=dict(seed=seed, tree=tree, plant_frac=plant_frac, r_range=tuple(r_range), lattice=lattice),
                       temperature=float(temperature))
    for row in range(rows):
        w._draw_row(row, 0)
    if temperature > 0.0:
        w.uniforms = np.stack([_rng(seed, 4000, b).random(N + 1, dtype=np.float32) for b in range(B)])
        if dense_q:
            q = np.empty((B, N, V), dtype=np.float32)
            for b in range(B):
                x = _rng(seed, 5000, b).standard_normal((N, V), dtype=np.float32) * np.float32(2.0)
                x -= x.max(axis=1, keepdims=True)
                np.exp(x, out=x)
                q[b] = x / x.sum(axis=1, keepdims=True, dtype=np.float64).astype(np.float32)
            w.draft_probs = q
    return w


# Shapes of the LM heads of the paper's target models (Sec. 4.1): hidden size 4096 with the
# 151 936-entry (Qwen3-8B) and 128 256-entry (LLaMA-3.1-8B) vocabularies.
LMHEAD_CONFIGS = {
    "small": dict(name="lmhead_small", B=4, N=9, H=256, V=5000, tree={"kind": "chain"}, plant_frac=0.6),
    "headline": dict(name="lmhead_B16_tree60_H4096_V151936", B=16, N=60, H=4096, V=151936,
                     tree={"kind": "tree", "depth": 6, "max_children": 4}, plant_frac=0.6),
    "chains": dict(name="lmhead_B64_chain8_H4096_V128256", B=64, N=9, H=4096, V=128256,
                   tree={"kind": "chain"}, plant_frac=0.6, theta_choices=(0.85, 0.9, 0.95)),
}
