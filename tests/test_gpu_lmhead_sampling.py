"""GPU parity of sampling-mode verification from hidden states (LM head fused with the top-2 and the sum of
exponentials, logits written once) against the CPU oracle, through the C ABI.

Under sampling every logit of a row counts (Eq. 3 runs over all of them), so it is not enough to keep a few
deciding entries clear of the bf16 rounding boundaries: the workloads here are lattice workloads
(``mars_inputs/lmhead.py``), on which an fp32-accumulating LM head forms the exact product, whatever its
order of additions.  Bar: the stored logits bit for bit; everything behind them as for ``mars_verify`` in
sampling mode (decisions, paths, tokens bit-exact on screened uniforms; sum-exp, normalisers and the
probability of the drawn token within the tolerances of ``tests/gpu_util.py``).
"""
import numpy as np
import pytest
import torch

from mars_inputs.lmhead import LMHEAD_CONFIGS, make_lmhead_workload
from oracle import lmhead_ref
from paper_2601_15498_amd import binding as M

from tests.gpu_util import compare, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class LogitsView:
    """What ``compare`` needs of a workload: the oracle's logits of an LM-head workload (or of some of its
    requests) with the request inputs that go with them."""

    def __init__(self, w, bits, pick):
        self.name, self.N, self.V, self.dtype = w.name, w.N, w.V, "bf16"
        self.B = len(pick)
        self.temperature = w.temperature
        self.logits = bits
        self.draft_tokens, self.tree_parent = w.draft_tokens[pick], w.tree_parent[pick]
        self.theta = np.ascontiguousarray(w.theta[pick], np.float32)
        self.uniforms = np.ascontiguousarray(w.uniforms[pick])
        self.draft_probs = None if w.draft_probs is None else np.ascontiguousarray(w.draft_probs[pick])
        self.meta = {"guard": 1e-4}      # screen_lmhead has moved every row whose ratio was within 1e-4 of theta


def run_case(name, seed=0, temperature=1.0, dense_q=False, pick=None, spin_limit=0, **shape):
    say(f"[case] lmhead sampling {name}: {shape} T={temperature} dense_q={dense_q}")
    w = make_lmhead_workload(name, seed=seed, lattice=True, temperature=temperature, dense_q=dense_q, **shape)
    pick = list(range(w.B)) if pick is None else pick
    # rows whose ratio sits within 1e-4 of the threshold are drawn again; rounding boundaries need no clearance
    greedy = lmhead_ref.screen_lmhead(w, clearance=0.0, requests=None if len(pick) == w.B else pick)
    view = LogitsView(w, greedy["logits_bits"], pick)
    d = dict(h=torch.from_numpy(w.hidden).to(DEV), w=torch.from_numpy(w.weight).to(DEV),
             tok=torch.from_numpy(w.draft_tokens).to(DEV), par=torch.from_numpy(w.tree_parent).to(DEV),
             th=torch.from_numpy(np.ascontiguousarray(w.theta, np.float32)).to(DEV),
             q=None if w.draft_probs is None else torch.from_numpy(w.draft_probs).to(DEV))
    kept = {}

    def run(v):
        u = w.uniforms.copy()
        u[pick] = v.uniforms                      # the screened uniforms of the compared requests
        out, logits = M.mars_lmhead_verify_sampling(d["h"], d["w"], d["tok"], d["par"], d["th"], w.temperature,
                                                    torch.from_numpy(u).to(DEV), d["q"], spin_limit=spin_limit)
        torch.cuda.synchronize()
        kept["logits"] = logits
        if len(pick) == w.B:
            return out
        sel = torch.tensor(pick, device=DEV)
        rows = (sel[:, None] * w.N + torch.arange(w.N, device=DEV)[None, :]).reshape(-1)
        sub = M.VerifyOutputs(len(pick), w.N, DEV, want_diag=True)
        for key in ("accept_len", "bonus_token", "request_status", "accept_mask", "path_idx", "decision"):
            getattr(sub, key).copy_(getattr(out, key)[sel])
        sub.stats.view(-1, M.ROW_STAT_WORDS).copy_(out.stats.view(-1, M.ROW_STAT_WORDS)[rows])
        sub.diag.view(len(pick), -1).copy_(out.diag.view(w.B, -1)[sel])
        kept["all"] = out
        return sub

    summary = compare(view, label=name, run=run, allow_small_norm=True)
    got = kept["logits"].cpu().numpy()[pick]
    bad = np.argwhere(got != view.logits)
    assert bad.size == 0, f"{name}: stored logits differ from the rounded exact product at {bad[:6].tolist()} ({bad.shape[0]} in all)"
    return w, summary, kept


SHAPES = [
    dict(B=4, N=9, H=256, V=5000, tree={"kind": "chain"}),                                   # one slab of 64, ragged tile
    dict(B=3, N=24, H=512, V=20000, tree={"kind": "tree", "depth": 4, "max_children": 4}),   # several tiles per run
    dict(B=16, N=12, H=512, V=33000, tree={"kind": "chain"}),                                # 192 rows: one slab of 192
    dict(B=9, N=43, H=256, V=4096, tree={"kind": "tree", "depth": 5, "max_children": 4}),    # 387 rows: slabs of 128, ragged slab
    dict(B=1, N=1, H=128, V=104, tree={"kind": "chain"}),                                    # one row, one ragged tile
    dict(B=2, N=20, H=256, V=300008, tree={"kind": "chain"}),                                # 1172 tiles, the last one ragged
]


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_one_hot_draft_distribution(i):
    run_case(f"lm_sampling_onehot{i}", seed=300 + i, temperature=(1.0, 0.7)[i % 2], **SHAPES[i])


@pytest.mark.parametrize("i", [0, 1, 3])
def test_dense_draft_distribution(i):
    run_case(f"lm_sampling_dense{i}", seed=320 + i, temperature=(0.8, 1.0)[i % 2], dense_q=True, **SHAPES[i])


def test_work_groups_that_do_not_wait_for_their_partners():
    run_case("lm_sampling_nowait", seed=331, temperature=1.0, dense_q=True, spin_limit=1, **SHAPES[1])


def test_headline_shape_sampled_requests():
    """B = 16 trees of 60 nodes, H = 4096, V = 151 936 in the launch shape the benchmark times: three requests
    against the oracle in full, stored logits included; the others through what holds for any input."""
    spec = dict(LMHEAD_CONFIGS["headline"])
    name = spec.pop("name")
    w, _, kept = run_case(name + "_sampling", seed=11, temperature=0.7, dense_q=True, pick=[0, 7, 15], **spec)
    out = kept["all"]
    s = {k: v.cpu().numpy().reshape(w.B, w.N) for k, v in M.unpack_stats(out.stats).items()}
    alen, path = out.accept_len.cpu().numpy(), out.path_idx.cpu().numpy()
    assert (out.request_status.cpu().numpy() == 0).all()
    assert (s["z1"] >= s["z2"]).all() and (s["id1"] != s["id2"]).all() and (s["sum_exp"] > 0.999).all()
    for b in range(w.B):
        node = 0
        for dpt in range(alen[b]):
            k = path[b, dpt]
            assert w.tree_parent[b, k] == node
            node = k
