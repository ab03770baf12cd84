"""GPU parity of greedy verification from hidden states (LM head fused with the row reduction)
against the CPU oracle, through the C ABI.

Bar: bit-exact -- top-2 ids and (bf16) values of every row, low-margin flags, decisions, paths,
lengths and tokens.  The kernel accumulates the LM-head products in fp32, the oracle in fp64; the
workloads are screened (on the oracle's side) so that no deciding logit lies within 4e-5 (relative)
of a bf16 rounding boundary and no ratio within 1e-4 of its threshold.  The fp32 accumulation error
of a 4096-term product of this size is a few 1e-6 relative, ten times less than the band.
"""
import numpy as np
import pytest
import torch

from mars_inputs.lmhead import LMHEAD_CONFIGS, make_lmhead_workload
from oracle import lmhead_ref, mars_ref
from paper_2601_15498_amd import binding as M

from tests.gpu_util import say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_device(w):
    return dict(h=torch.from_numpy(w.hidden).to(DEV), w=torch.from_numpy(w.weight).to(DEV),
                tok=torch.from_numpy(w.draft_tokens).to(DEV), par=torch.from_numpy(w.tree_parent).to(DEV),
                th=torch.from_numpy(np.ascontiguousarray(w.theta, np.float32)).to(DEV))


def assert_rows_match(stats_gpu, ref_stats, label):
    s = {k: v.cpu().numpy() for k, v in M.unpack_stats(stats_gpu).items()}
    r = ref_stats.reshape(-1)
    for key in ("id1", "id2", "relax_ok"):
        bad = np.nonzero(s[key] != r[key])[0]
        assert bad.size == 0, f"{label}: {key} differs at rows {bad[:8]}: gpu {s[key][bad[:8]]} ref {r[key][bad[:8]]}"
    for key in ("z1", "z2"):
        bad = np.nonzero(s[key].astype(np.float64) != r[key])[0]
        assert bad.size == 0, f"{label}: {key} differs at rows {bad[:8]}: gpu {s[key][bad[:8]]} ref {r[key][bad[:8]]}"
    assert (s["sum_exp"] == 0).all()


def assert_requests_match(out, ref, label, pick=None):
    for key in ("accept_len", "bonus_token", "path_idx", "accept_mask", "decision", "request_status"):
        g = getattr(out, key).cpu().numpy()
        if pick is not None:
            g = g[pick]
        bad = np.nonzero(np.atleast_1d((g != ref[key]).reshape(g.shape[0], -1).any(axis=1)))[0]
        assert bad.size == 0, f"{label}: {key} differs for requests {bad[:8]}"


def run_case(name, indicator=mars_ref.IND_LOGIT_RATIO, theta_choices=(0.9,), seed=0, **shape):
    say(f"[case] lmhead {name}: {shape} indicator={indicator}")
    w = make_lmhead_workload(name, seed=seed, theta_choices=theta_choices, **shape)
    ref = lmhead_ref.screen_lmhead(w, indicator=indicator)
    d = to_device(w)
    out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"], indicator=indicator)
    torch.cuda.synchronize()
    assert_rows_match(out.stats, ref["stats"], name)
    assert_requests_match(out, ref, name)
    return w, ref, out


SHAPES = [
    dict(B=4, N=9, H=256, V=5000, tree={"kind": "chain"}),                                   # one slab of 64, ragged tile
    dict(B=2, N=18, H=128, V=100001, tree={"kind": "tree", "depth": 4, "max_children": 3}),  # several tiles per run
    dict(B=16, N=12, H=512, V=33000, tree={"kind": "chain"}),                                # 192 rows: one slab of 192
    dict(B=7, N=30, H=256, V=20011, tree={"kind": "tree", "depth": 5, "max_children": 4}),   # 210 rows: slabs of 64
    dict(B=5, N=60, H=384, V=9001, tree={"kind": "tree", "depth": 6, "max_children": 4}),    # 300 rows, H = 3 * 128
    dict(B=1, N=1, H=128, V=100, tree={"kind": "chain"}),                                    # one row, one ragged tile
    dict(B=3, N=40, H=1024, V=257, tree={"kind": "tree", "depth": 6, "max_children": 3}),    # tile of one entry
    dict(B=9, N=43, H=256, V=4096, tree={"kind": "tree", "depth": 5, "max_children": 4}),    # 387 rows: slabs of 128 + ragged slab
    dict(B=2, N=50, H=640, V=70001, tree={"kind": "chain"}),                                 # 100 rows: 137 runs, each from its own slab of the 10 along H
    dict(B=2, N=20, H=256, V=300007, tree={"kind": "chain"}),                                # a vocabulary of 1172 tiles, the last one ragged
]


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_shapes(i):
    _, ref, _ = run_case(f"shape{i}", seed=100 + i, **SHAPES[i])
    if SHAPES[i]["B"] * SHAPES[i]["N"] > 100:
        assert ref["accept_len"].max() >= 1


def test_seeded_sweep_of_shapes():
    """Sixteen shapes drawn from a seed: rows 1 .. 3000, H in {128 .. 2048}, odd and tile-aligned
    vocabularies, chains and trees, the three indicators, commit outputs included."""
    rng = np.random.default_rng(20260)
    for c in range(16):
        H = int(rng.choice([128, 256, 384, 512, 640, 1024, 2048]))
        B, N = int(rng.integers(1, 48)), int(rng.integers(1, 64))
        rows = B * N
        vmin = 2 * rows + 2
        V = int(rng.integers(vmin, max(vmin + 1, min(200000, int(2e10 / (rows * H)))) + 1))
        if rng.random() < 0.3:
            V = max(vmin, (V // 256) * 256 + int(rng.choice([0, 1, 255])))
        tree = {"kind": "chain"}
        if N >= 4 and rng.random() < 0.6:
            while True:
                dep, ch = int(rng.integers(2, min(6, N - 1) + 1)), int(rng.integers(2, 5))
                if sum(ch ** k for k in range(dep + 1)) >= 2 * N:
                    tree = {"kind": "tree", "depth": dep, "max_children": ch}
                    break
        ind = int(rng.choice([0, 0, 1, 2]))
        thetas = {0: (0.85, 0.9, 0.95), 1: (0.3,), 2: (1.5,)}[ind]
        say(f"[case] lmhead sweep {c}: B={B} N={N} H={H} V={V} {tree} indicator={ind}")
        w = make_lmhead_workload(f"sweep{c}", B=B, N=N, H=H, V=V, tree=tree, theta_choices=thetas, seed=500 + c)
        ref = lmhead_ref.screen_lmhead(w, indicator=ind)
        d = to_device(w)
        out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"], indicator=ind, want_commit=True)
        torch.cuda.synchronize()
        assert_rows_match(out.stats, ref["stats"], f"sweep {c}")
        assert_requests_match(out, ref, f"sweep {c}")
        want = mars_ref.commit(w.draft_tokens, ref["accept_len"], ref["path_idx"], ref["bonus_token"])
        for key in ("out_tokens", "out_len", "keep_rows", "keep_offsets"):
            assert np.array_equal(getattr(out, key).cpu().numpy(), want[key]), (c, key)


def test_per_request_thresholds_and_other_indicators():
    shape = dict(B=8, N=16, H=256, V=12000, tree={"kind": "tree", "depth": 4, "max_children": 3})
    run_case("thetas", theta_choices=(0.85, 0.9, 0.95), seed=21, **shape)
    _, ref, _ = run_case("prob_ratio", indicator=mars_ref.IND_PROB_RATIO, theta_choices=(0.3,), seed=22, **shape)
    assert 0 < ref["stats"]["relax_ok"].sum() < ref["stats"].size
    _, ref, _ = run_case("logit_gap", indicator=mars_ref.IND_LOGIT_GAP, theta_choices=(1.5,), seed=23, **shape)
    assert 0 < ref["stats"]["relax_ok"].sum() < ref["stats"].size


def test_committed_sequence_and_kept_rows():
    w = make_lmhead_workload("commit", B=6, N=20, H=256, V=8000, tree={"kind": "tree", "depth": 5, "max_children": 3}, seed=31)
    ref = lmhead_ref.screen_lmhead(w)
    want = mars_ref.commit(w.draft_tokens, ref["accept_len"], ref["path_idx"], ref["bonus_token"])
    d = to_device(w)
    out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"], want_commit=True)
    torch.cuda.synchronize()
    assert_requests_match(out, ref, "commit")
    for key in ("out_tokens", "out_len", "keep_rows", "keep_offsets"):
        assert np.array_equal(getattr(out, key).cpu().numpy(), want[key]), key


def test_threshold_sweep_from_one_pass():
    w = make_lmhead_workload("sweep", B=5, N=14, H=256, V=6000, tree={"kind": "chain"}, seed=41)
    thetas = np.float32([[0.82] * 5, [0.9] * 5, [0.97] * 5])
    for _ in range(20):                       # every row clear of all three thresholds
        before = w.hidden.copy()
        for k in range(3):
            w.theta = thetas[k]
            lmhead_ref.screen_lmhead(w)
        if np.array_equal(before, w.hidden):
            break
    else:
        raise AssertionError("screening did not settle")
    bits = lmhead_ref.lmhead_verify(w.hidden, w.weight, w.draft_tokens, w.tree_parent, thetas[0])["logits_bits"]
    ref = mars_ref.verify_sweep(bits, w.draft_tokens, w.tree_parent, thetas, 0.0)
    d = to_device(w)
    out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], torch.from_numpy(thetas).to(DEV), n_theta=3)
    torch.cuda.synchronize()
    for key in ("accept_len", "bonus_token", "path_idx", "accept_mask", "decision"):
        assert np.array_equal(getattr(out, key).cpu().numpy(), ref[key]), key
    assert ref["accept_len"][0].sum() >= ref["accept_len"][2].sum()      # a lower threshold accepts at least as much
    for k in range(3):
        assert_rows_match(out.stats[k], ref["stats"][k], f"sweep{k}")


def test_malformed_requests_are_flagged():
    w = make_lmhead_workload("bad", B=4, N=8, H=128, V=3000, tree={"kind": "chain"}, seed=51)
    ref0 = lmhead_ref.screen_lmhead(w)
    w.tree_parent[1, 3] = 5            # parent after child
    w.draft_tokens[2, 4] = w.V         # token out of range
    ref = lmhead_ref.lmhead_verify(w.hidden, w.weight, w.draft_tokens, w.tree_parent, w.theta)
    assert list(ref["request_status"]) == [0, 1, 2, 0]
    d = to_device(w)
    out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"])
    torch.cuda.synchronize()
    assert_requests_match(out, ref, "bad")
    assert np.array_equal(ref["accept_len"][[0, 3]], ref0["accept_len"][[0, 3]])


def test_batch_shape_does_not_change_the_result_on_screened_inputs():
    # The order in which a row's products are added depends on the launch plan (slab height, runs of tiles), so
    # on the batch shape; on inputs whose deciding logits keep clear of the bf16 rounding boundaries that must not
    # show.  The same requests verified in one batch (a tall slab, many rows) and one by one (a slab of 64 rows,
    # a different split of the vocabulary over the work-groups) give identical rows and identical outcomes.
    w = make_lmhead_workload("plan", B=7, N=30, H=512, V=20000, tree={"kind": "tree", "depth": 4, "max_children": 4},
                             seed=17)
    ref = lmhead_ref.screen_lmhead(w)
    d = to_device(w)
    whole = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"])
    torch.cuda.synchronize()
    assert_rows_match(whole.stats, ref["stats"], "plan: one batch")
    assert_requests_match(whole, ref, "plan: one batch")
    for b in range(w.B):
        one = M.mars_lmhead_verify(d["h"][b:b + 1].contiguous(), d["w"], d["tok"][b:b + 1].contiguous(),
                                   d["par"][b:b + 1].contiguous(), d["th"][b:b + 1].contiguous())
        torch.cuda.synchronize()
        for key in ("accept_len", "bonus_token", "path_idx", "accept_mask", "decision"):
            assert torch.equal(getattr(one, key)[0], getattr(whole, key)[b]), (b, key)
        assert torch.equal(one.stats.view(-1, M.ROW_STAT_WORDS), whole.stats.view(w.B, w.N, M.ROW_STAT_WORDS)[b]), b


def test_calls_on_two_streams_and_repeated_calls_agree():
    w = make_lmhead_workload("streams", B=6, N=16, H=256, V=30000, tree={"kind": "chain"}, seed=61)
    ref = lmhead_ref.screen_lmhead(w)
    d = to_device(w)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    torch.cuda.synchronize()
    for rep in range(3):
        for s in streams:
            with torch.cuda.stream(s):
                outs.append(M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"]))
    torch.cuda.synchronize()
    for i, out in enumerate(outs):
        assert_requests_match(out, ref, f"call {i}")
        assert_rows_match(out.stats, ref["stats"], f"call {i}")


def test_two_parts_of_a_call_and_graph_replays():
    """options.stages splits the call into the fused LM-head kernel and the per-request part; and the
    call only enqueues kernels, so a HIP graph may hold it: replays with the hidden states changed under
    the graph equal eager calls on the same inputs."""
    ws_host = [make_lmhead_workload("g0", B=5, N=20, H=256, V=20000, tree={"kind": "tree", "depth": 4, "max_children": 3}, seed=71),
               make_lmhead_workload("g1", B=5, N=20, H=256, V=20000, tree={"kind": "tree", "depth": 4, "max_children": 3}, seed=72)]
    refs = [lmhead_ref.screen_lmhead(w) for w in ws_host]
    devs = [to_device(w) for w in ws_host]
    B, N, H, V = ws_host[0].B, ws_host[0].N, ws_host[0].H, ws_host[0].V
    cur = {k: v.clone() for k, v in devs[0].items()}
    ws = torch.empty(M.mars_lmhead_workspace_bytes(B, N, V, H), dtype=torch.uint8, device=DEV)
    out_g = M.VerifyOutputs(B, N, DEV, want_diag=False, want_commit=True)
    out_s = M.VerifyOutputs(B, N, DEV, want_diag=False, want_commit=True)

    # the two parts one after the other
    M.mars_lmhead_verify(cur["h"], cur["w"], cur["tok"], cur["par"], cur["th"], out_s, ws, stages=M.MARS_STAGE_ROWS)
    M.mars_lmhead_verify(cur["h"], cur["w"], cur["tok"], cur["par"], cur["th"], out_s, ws, stages=M.MARS_STAGE_REQUESTS)
    torch.cuda.synchronize()
    assert_requests_match(out_s, refs[0], "two parts")
    assert_rows_match(out_s.stats, refs[0]["stats"], "two parts")

    def call(out):
        M.mars_lmhead_verify(cur["h"], cur["w"], cur["tok"], cur["par"], cur["th"], out, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(out_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(out_g)
    for rep in range(4):
        for k, v in cur.items():
            v.copy_(devs[rep % 2][k])
        for key in ("accept_len", "bonus_token", "path_idx", "out_tokens", "keep_rows"):
            getattr(out_g, key).fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_requests_match(out_g, refs[rep % 2], f"replay {rep}")
        assert_rows_match(out_g.stats, refs[rep % 2]["stats"], f"replay {rep}")
        want = mars_ref.commit(ws_host[rep % 2].draft_tokens, refs[rep % 2]["accept_len"], refs[rep % 2]["path_idx"],
                               refs[rep % 2]["bonus_token"])
        for key in ("out_tokens", "out_len", "keep_rows", "keep_offsets"):
            assert np.array_equal(getattr(out_g, key).cpu().numpy(), want[key]), (rep, key)
        torch.ones(1000, device=DEV).sum().item()        # eager work between the replays


def test_chain_batch_shape_sampled_requests():
    """B = 64 chains of 8 drafts, H = 4096, V = 128 256, per-request thresholds (three slabs of 192 rows):
    eight requests against the oracle, the others through what holds for any input."""
    spec = dict(LMHEAD_CONFIGS["chains"])
    name = spec.pop("name")
    say(f"[case] lmhead {name}: generating")
    w = make_lmhead_workload(name, seed=9, **spec)
    pick = [0, 5, 21, 22, 40, 41, 62, 63]
    say("[case] oracle on eight requests")
    ref = lmhead_ref.screen_lmhead(w, requests=pick)
    d = to_device(w)
    out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"], want_commit=True)
    torch.cuda.synchronize()
    rows = (np.asarray(pick)[:, None] * w.N + np.arange(w.N)[None, :]).reshape(-1)
    assert_rows_match(out.stats.view(-1, M.ROW_STAT_WORDS)[torch.from_numpy(rows).to(DEV)], ref["stats"], name)
    assert_requests_match(out, ref, name, pick=pick)
    s = {k: v.cpu().numpy().reshape(w.B, w.N) for k, v in M.unpack_stats(out.stats).items()}
    alen, bonus = out.accept_len.cpu().numpy(), out.bonus_token.cpu().numpy()
    out_tok, out_len = out.out_tokens.cpu().numpy(), out.out_len.cpu().numpy()
    assert (out.request_status.cpu().numpy() == 0).all()
    for b in range(w.B):          # a chain: accepted nodes are 1 .. alen, then the top-1 of the last node's row
        for k in range(1, alen[b] + 1):
            assert w.draft_tokens[b, k] in (s["id1"][b, k - 1], s["id2"][b, k - 1])
        if alen[b] + 1 < w.N:       # the next draft was rejected
            t, p = w.draft_tokens[b, alen[b] + 1], alen[b]
            assert t != s["id1"][b, p] and not (t == s["id2"][b, p] and s["relax_ok"][b, p])
        assert bonus[b] == s["id1"][b, alen[b]] and out_len[b] == alen[b] + 1
        assert list(out_tok[b, :alen[b]]) == list(w.draft_tokens[b, 1:alen[b] + 1]) and out_tok[b, alen[b]] == bonus[b]
    assert alen.max() >= 3


def test_headline_shape_sampled_requests():
    """B = 16 trees of 60 nodes, H = 4096, V = 151 936 in the launch shape the benchmark times: three
    requests are checked in full against the oracle (their rows screened), the others through what
    holds for any input."""
    spec = dict(LMHEAD_CONFIGS["headline"])
    name = spec.pop("name")
    say(f"[case] lmhead {name}: generating")
    w = make_lmhead_workload(name, seed=7, **spec)
    pick = [0, 7, 15]
    say("[case] oracle on three requests")
    ref = lmhead_ref.screen_lmhead(w, requests=pick)
    d = to_device(w)
    out = M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"])
    torch.cuda.synchronize()
    say("[case] compare")
    rows = (np.asarray(pick)[:, None] * w.N + np.arange(w.N)[None, :]).reshape(-1)
    assert_rows_match(out.stats.view(-1, M.ROW_STAT_WORDS)[torch.from_numpy(rows).to(DEV)], ref["stats"], name)
    assert_requests_match(out, ref, name, pick=pick)
    # every request: status ok, the path is a chain of parents, every accepted token is the top-1 or
    # the runner-up of its parent's row, the bonus token is the top-1 of the last node's row
    s = {k: v.cpu().numpy().reshape(w.B, w.N) for k, v in M.unpack_stats(out.stats).items()}
    alen, path, bonus = out.accept_len.cpu().numpy(), out.path_idx.cpu().numpy(), out.bonus_token.cpu().numpy()
    assert (out.request_status.cpu().numpy() == 0).all()
    assert (s["z1"] >= s["z2"]).all() and (s["id1"] != s["id2"]).all()
    planted = w.planted[..., 0] >= 0
    assert ((s["id1"] == w.planted[..., 0]) | ~planted).mean() > 0.99
    for b in range(w.B):
        node = 0
        for dpt in range(alen[b]):
            k = path[b, dpt]
            assert w.tree_parent[b, k] == node
            assert w.draft_tokens[b, k] in (s["id1"][b, node], s["id2"][b, node])
            node = k
        assert bonus[b] == s["id1"][b, node]
    assert alen.max() >= 2
