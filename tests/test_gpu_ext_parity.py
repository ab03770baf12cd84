"""GPU parity of the entry points beyond the core pass -- mars_verify_ex (other low-margin indicators,
threshold sweep, committed sequence with kept cache rows) and mars_margin_stats -- against the CPU
oracle on the same seeded inputs.  Every test here needs a real MI355X."""
import numpy as np
import pytest
import torch

from mars_inputs import f32_to_bf16_bits, make_config
from tests.gpu_util import compare_ex, compare_margin, say
from tests.test_gpu_parity import custom

pytestmark = pytest.mark.gpu

SWEEP = (0.84, 0.86, 0.88, 0.90, 0.92, 0.94, 0.96)   # the thresholds of the paper's ablation over theta


@pytest.fixture(scope="module", autouse=True)
def _gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2601_15498_amd import binding
    binding.lib()


def tiled(thetas, B):
    return np.tile(np.asarray(thetas, np.float32)[:, None], (1, B))


# ----------------------------------------------------------------------------- committed sequence + kept rows
def test_commit_cfg0_greedy_chain():
    compare_ex(make_config(0))


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_commit_cfg1_tree(T):
    compare_ex(make_config(1, temperature=T), label=f"commit_cfg1_T{T}")


def test_commit_cfg2_full_dense_q():
    compare_ex(make_config(2))


def test_commit_cfg3_full():
    compare_ex(make_config(3))


def test_commit_cfg4_reduced_many_requests():
    compare_ex(make_config(4, B=300, V=4096 + 24), label="commit_cfg4_B300_smallV")   # several scan rounds of 256


def test_commit_of_rejected_requests():
    rng = np.random.default_rng(3)
    B, N, V = 5, 6, 64
    z = rng.normal(0, 3, size=(B, N, V)).astype(np.float32)
    par = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    tok = z.argmax(-1).astype(np.int32)
    tok[:, 1:] = tok[:, :-1].copy()
    par[1, 3] = 4          # parent after child: malformed tree
    tok[3, 2] = V + 7      # token out of range
    u = rng.random((B, N + 1)).astype(np.float32)
    for T in (0.0, 1.0):
        compare_ex(custom(f"commit_malformed_T{T}", z, tok, par, 0.9, T, u if T > 0 else None))


# ----------------------------------------------------------------------------- other indicators (Sec. 3.3)
@pytest.mark.parametrize("indicator,theta", [("prob_ratio", 0.3), ("logit_gap", 1.0)])
def test_indicator_greedy_chain_f32(indicator, theta):
    s = compare_ex(make_config(0, B=8, indicator=indicator, theta_choices=(theta,)), indicator=indicator,
                   label=f"{indicator}_cfg0_B8")
    assert s["relaxed"] > 0


@pytest.mark.parametrize("indicator,theta", [("prob_ratio", 0.3), ("logit_gap", 1.0)])
@pytest.mark.parametrize("T", [0.0, 1.0])
def test_indicator_tree_bf16(indicator, theta, T):
    compare_ex(make_config(1, temperature=T, B=4, indicator=indicator, theta_choices=(theta,)), indicator=indicator,
               label=f"{indicator}_cfg1_B4_T{T}")


def test_indicator_prob_ratio_dense_q_uses_temperature():
    # T = 0.7: p2/p1 = exp(-gap / 0.7); per-request thresholds
    s = compare_ex(make_config(2, B=3, indicator="prob_ratio", theta_choices=(0.02, 0.2)), indicator="prob_ratio",
                   label="prob_ratio_cfg2_B3")
    assert 0 < s["low_margin_rows"] < 180


def test_indicator_gap_full_cfg3():
    compare_ex(make_config(3, indicator="logit_gap", theta_choices=(0.5, 1.0, 2.0)), indicator="logit_gap",
               label="logit_gap_cfg3")


def test_indicator_negative_top_logits():
    # every logit negative: the logit ratio never relaxes, the other two do
    rng = np.random.default_rng(4)
    B, N, V = 2, 8, 4096
    z = (rng.normal(0, 1, size=(B, N, V)) - 30.0).astype(np.float32)
    order = np.argsort(-z, axis=-1, kind="stable")
    par = np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1))
    tok = np.zeros((B, N), np.int32)
    tok[:, 1:] = order[:, :-1, 1]      # every draft is the runner-up
    assert compare_ex(custom("neg_ratio", z, tok, par, 0.5, 0.0), indicator="logit_ratio")["relaxed"] == 0
    assert compare_ex(custom("neg_gap", z, tok, par, 100.0, 0.0), indicator="logit_gap")["relaxed"] == B * (N - 1)
    assert compare_ex(custom("neg_prob", z, tok, par, 1e-30, 0.0), indicator="prob_ratio")["relaxed"] == B * (N - 1)


# ----------------------------------------------------------------------------- threshold sweep
@pytest.mark.parametrize("T", [0.0, 1.0])
def test_sweep_cfg1_seven_thresholds(T):
    w = make_config(1, temperature=T, sweep_thetas=SWEEP)
    s = compare_ex(w, thetas=tiled(SWEEP, w.B), label=f"sweep7_cfg1_T{T}")
    if T == 0.0:
        assert all(a >= b for a, b in zip(s["mean_tau"], s["mean_tau"][1:]))   # greedy: tau shrinks as theta rises


def test_sweep_cfg2_full_headline_shape():
    w = make_config(2, sweep_thetas=SWEEP)
    compare_ex(w, thetas=tiled(SWEEP, w.B), label="sweep7_cfg2_full")


def test_sweep_cfg3_per_request_thresholds():
    w = make_config(3, B=16, sweep_thetas=(0.8, 0.99))
    th = np.stack([w.theta, np.full(w.B, 0.8, np.float32), np.full(w.B, 0.99, np.float32)])
    compare_ex(w, thetas=th, label="sweep3_cfg3_B16")


def test_sweep_more_requests_than_compute_units():
    w = make_config(4, B=40, V=8192 + 8, sweep_thetas=SWEEP + (1.5,))
    compare_ex(w, thetas=tiled(SWEEP + (1.5,), w.B), label="sweep8_cfg4_B40")     # 320 walks, one work-group each


def test_sweep_with_other_indicator():
    ths = (0.1, 0.3, 0.6)
    w = make_config(1, temperature=1.0, B=3, indicator="prob_ratio", theta_choices=(0.3,), sweep_thetas=ths)
    compare_ex(w, thetas=tiled(ths, w.B), indicator="prob_ratio", label="sweep3_prob_ratio_cfg1_B3")


# ----------------------------------------------------------------------------- margin statistics
RANGES = ((-5.0, 35.0), (0.5, 1.0), (0.0, 1.0))
BINS = (40, 50, 50)


def test_margin_stats_cfg2_full():
    s = compare_margin(make_config(2), RANGES, BINS)
    assert s["summary"][0] == 960 and s["summary"][1] == 0      # no negative top-1 logit, as in the paper's figure


def test_margin_stats_cfg0_f32_greedy():
    compare_margin(make_config(0), RANGES, BINS)


def test_margin_stats_cfg3_full_gumbel():
    compare_margin(make_config(3), ((0.0, 40.0), (0.0, 1.0), (0.0, 1.0)), (64, 100, 1))


def test_margin_stats_cfg4_reduced():
    compare_margin(make_config(4, B=12), RANGES, (7, 13, 1000))


def test_margin_stats_negative_and_zero_top_logits_ragged_vocab():
    rng = np.random.default_rng(6)
    B, N, V = 3, 11, 1000 + 3
    z = rng.normal(0, 2, size=(B, N, V)).astype(np.float32)
    z[0] -= 20.0                                   # negative top-1
    z[1, :4] = np.minimum(z[1, :4], 0.0)           # top-1 exactly 0 (many ties)
    z[2, 0, :] = -np.inf
    z[2, 0, 5] = 3.0                               # a single unmasked token: z2 = -inf, ratio -inf, p2/p1 = 0
    s = compare_margin(custom("margin_edge_rows", z, np.zeros((B, N), np.int32),
                              np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1)), 0.9, 0.5),
                       ((-30.0, 10.0), (0.0, 1.0), (0.0, 1.0)), (8, 4, 4))
    assert s["summary"][1] == N and s["summary"][2] == N + 4
    zb = f32_to_bf16_bits(z)
    compare_margin(custom("margin_edge_rows_bf16", zb, np.zeros((B, N), np.int32),
                          np.tile(np.arange(-1, N - 1, dtype=np.int32), (B, 1)), 0.9, 0.0),
                   ((-30.0, 10.0), (0.0, 1.0), (0.0, 1.0)), (8, 4, 4))


# ----------------------------------------------------------------------------- SPD-shaped workload
def test_spd_chains_dense_q_reduced():
    compare_ex(make_config(5, B=6), label="spd_B6")


def test_spd_chains_dense_q_full():
    s = compare_ex(make_config(5), label="spd_B128")
    assert s["low_margin_rows"] > 0


# ----------------------------------------------------------------------------- failure handling, graphs
@pytest.mark.parametrize("case", ["resident_dense", "resident_onehot", "streamed_dense"])
def test_a_work_group_that_stops_waiting_for_its_partners_obtains_their_sums_itself(case):
    # Forced from the host: with a spin limit of one poll a work-group stops waiting for any partner that
    # is a moment late and works out that partner's slice sum itself (residual normalisers and the
    # totals of the final draw alike), with the partner's assignment of elements to threads and order
    # of additions.  The result must be the oracle's, bit for bit where the bar says so -- that is the
    # proof that the recomputed sums are the published ones -- and no request may carry a status.
    # Three shapes: slices resident in registers with a dense and with a one-hot draft distribution,
    # and slices streamed from memory (many requests, two work-groups each).
    from paper_2601_15498_amd import binding as M
    from oracle import screen
    from tests.gpu_util import to_device
    if case == "resident_dense":
        w = make_config(2, B=3)                 # 32 work-groups per request, several exchanges each
    elif case == "resident_onehot":
        w = make_config(1, temperature=1.0, B=2)
    else:
        w = make_config(5, B=96, N=8, tree={"kind": "tree", "depth": 3, "max_children": 3})   # dense q, 2 work-groups
                                                # per request, slices streamed; siblings, so Z is summed too
    ref = screen.screen_uniforms(w)
    d = to_device(w)
    ws = M.alloc_workspace(w.B, w.N, w.V, d["logits"].device)
    for limit in (1, 0):                        # never wait; then the default
        out = M.mars_verify_ex(d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], w.temperature,
                               d["uniforms"], d["draft_probs"], workspace=ws, spin_limit=limit)
        torch.cuda.synchronize()
        assert (out.request_status.cpu().numpy() == 0).all(), (case, limit)
        for key in ("accept_len", "bonus_token", "accept_mask", "path_idx", "decision"):
            assert np.array_equal(getattr(out, key).cpu().numpy(), ref[key]), (case, limit, key)
        dg = {k: v.cpu().numpy() for k, v in M.unpack_diag(out.diag).items()}
        assert np.array_equal(dg["residual_passes"], ref["diag"]["residual_passes"]), (case, limit)
        assert np.array_equal(dg["last_node"], ref["diag"]["last_node"]), (case, limit)
    say(f"[ok]   {case}: spin_limit 1 and default both exact; rejections per request "
        f"{ref['diag']['residual_passes'].tolist()[:8]}")


@pytest.mark.parametrize("T", [0.0, 0.7])
def test_graph_replays_equal_eager(T):
    # The calls only enqueue kernels (no allocation, no memset, no synchronisation), so a caller may
    # capture them in a HIP graph.  Every replay, with eager work and synchronisations in between and the
    # inputs changed under the graph, must equal the eager result on the same inputs.
    from paper_2601_15498_amd import binding as M
    from tests.gpu_util import to_device
    ws_list = [make_config(2, B=4, temperature=T), make_config(2, B=4, temperature=T, seed=77)]
    devs = [to_device(w) for w in ws_list]
    B, N, V = ws_list[0].B, ws_list[0].N, ws_list[0].V
    dev = devs[0]["logits"].device
    cur = {k: (None if v is None else v.clone()) for k, v in devs[0].items()}   # static inputs of the graph
    if T == 0.0:
        cur["uniforms"] = None
        cur["draft_probs"] = None
    ws = M.alloc_workspace(B, N, V, dev)
    out_g = M.VerifyOutputs(B, N, dev, want_commit=True)
    out_e = M.VerifyOutputs(B, N, dev, want_commit=True)

    def call(out):
        M.mars_verify_ex(cur["logits"], cur["draft_tokens"], cur["tree_parent"], cur["theta"], T, cur["uniforms"],
                         cur["draft_probs"], out=out, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(out_g)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(out_g)
    keys = ("accept_len", "bonus_token", "accept_mask", "path_idx", "decision", "request_status", "out_tokens",
            "out_len", "keep_rows", "keep_offsets", "stats")
    for rep in range(4):
        src = devs[rep % 2]
        for k, v in cur.items():
            if v is not None:
                v.copy_(src[k])
        torch.cuda.synchronize()
        call(out_e)
        torch.cuda.synchronize()
        want = {k: getattr(out_e, k).clone() for k in keys}
        for k in keys:
            getattr(out_g, k).fill_(-7 if getattr(out_g, k).dtype != torch.uint8 else 9)
        graph.replay()
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(getattr(out_g, k), want[k]), (rep, k)
    say(f"[ok]   graph T={T}: 4 replays equal eager")


# ----------------------------------------------------------------------------- edge sizes of the extended entry point
def test_ex_root_only_and_tiny_vocab_with_maximum_thresholds():
    # N = 1: nothing to verify, the committed sequence is the one token drawn from the root row; V = 2;
    # 64 thresholds per request (the maximum), both modes, every indicator.
    z = np.array([[[1.5, 1.25]], [[-2.0, 3.0]], [[0.5, 0.5]]], np.float32)
    tok = np.zeros((3, 1), np.int32)
    par = -np.ones((3, 1), np.int32)
    u = np.array([[0.3, 0.9], [0.2, 0.05], [0.7, 0.4999]], np.float32)
    ths = np.linspace(0.05, 1.3, 64).astype(np.float32)
    for T in (0.0, 0.9):
        for ind in ("logit_ratio", "prob_ratio", "logit_gap"):
            compare_ex(custom(f"root_only_T{T}_{ind}", z, tok, par, 0.9, T, u if T > 0 else None),
                       indicator=ind, thetas=tiled(ths, 3), label=f"root_only_K64_T{T}_{ind}")


@pytest.mark.parametrize("T", [0.0, 1.0])
def test_ex_maximum_nodes_with_commit_and_sweep(T):
    # N = 1024 (the maximum), a deep chain mixed with a bushy part, two thresholds
    rng = np.random.default_rng(21)
    B, N, V = 2, 1024, 512
    z = (rng.normal(0, 1, size=(B, N, V)) + 6.0).astype(np.float32)
    par = np.zeros((B, N), np.int32)
    par[:, 0] = -1
    for b in range(B):
        for i in range(1, N):
            par[b, i] = i - 1 if i < 700 else rng.integers(0, i)
    order = np.argsort(-z, axis=-1, kind="stable")
    tok = np.zeros((B, N), np.int32)
    for b in range(B):
        for i in range(1, N):
            tok[b, i] = order[b, par[b, i], 0 if rng.random() < 0.9 else 1]
    u = rng.random((B, N + 1)).astype(np.float32)
    w = custom(f"max_nodes_ex_T{T}", z, tok, par, 0.9, T, u if T > 0 else None)
    s = compare_ex(w, thetas=np.array([[0.5, 0.5], [2.0, 0.93]], np.float32), label=f"max_nodes_ex_T{T}")
    if T == 0.0:
        assert max(s["mean_tau"]) > 5      # long accepted chains: the path outputs are exercised in depth


def test_ex_tiny_vocab_every_indicator_sampling_dense():
    rng = np.random.default_rng(22)
    B, N = 6, 7
    for V in (2, 3, 9):
        z = rng.normal(0, 2, size=(B, N, V)).astype(np.float32)
        q = rng.dirichlet(np.ones(V), size=(B, N)).astype(np.float64)
        q = (q / q.sum(-1, keepdims=True)).astype(np.float32)
        par = np.tile(np.array([-1, 0, 0, 1, 1, 2, 3], np.int32), (B, 1))
        tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
        u = rng.random((B, N + 1)).astype(np.float32)
        for ind, th in (("prob_ratio", 0.4), ("logit_gap", 0.8)):
            compare_ex(custom(f"tiny_V{V}_{ind}", z, tok, par, th, 0.8, u, q), indicator=ind, cdf_guard=5e-6,
                       label=f"tiny_V{V}_{ind}")


# ----------------------------------------------------------------------------- seeded sweep over shapes and options
def sweep_case(rng, seed, case):
    """One randomly shaped, valid workload with its options."""
    from mars_inputs import make_workload
    B = int(rng.choice([1, 2, 3, 5, 9, 17, 40]))
    N = int(rng.choice([1, 2, 3, 8, 17, 33, 64]))
    V = int(rng.choice([2, 7, 8, 63, 64, 520, 1024, 4095, 4096, 8200, 16392, 40003]))
    dtype = str(rng.choice(["f32", "bf16"]))
    T = float(rng.choice([0.0, 0.0, 0.6, 1.0, 1.7]))
    dense = bool(rng.random() < 0.5) and T > 0
    ind, th = [("logit_ratio", 0.9), ("prob_ratio", 0.35), ("logit_gap", 1.25)][int(rng.integers(3))]
    K = int(rng.choice([1, 1, 2, 5]))
    ths = tuple(float(x) for x in np.round(np.linspace(0.6 * th, 1.3 * th, K), 4)) if K > 1 else ()
    tree = {"kind": "chain"}
    if rng.random() >= 0.4 and N >= 4:
        depth, fan = int(rng.integers(2, 7)), min(int(rng.integers(2, 5)), V)   # siblings carry distinct tokens
        depth = min(depth, N - 1)
        while sum(fan ** d for d in range(depth + 1)) < N:   # the tree must be able to hold N nodes
            depth += 1
        tree = {"kind": "tree", "depth": depth, "max_children": fan}
    w = make_workload(f"sweep_s{seed}_c{case}", B=B, N=N, V=V, dtype=dtype, temperature=T, tree=tree,
                      background=str(rng.choice(["normal3", "gumbel2"])), plant_frac=0.5 if V >= 64 else 0.0,
                      theta_choices=(th,), dense_q=dense, seed=5000 + 10 * seed + case, indicator=ind,
                      sweep_thetas=ths, threads=1)
    return w, ind, ths, tree


@pytest.mark.parametrize("seed", range(8))
def test_seeded_sweep_over_shapes_and_options(seed):
    # Valid inputs of many shapes: vocabulary sizes around the vector and tile boundaries, chains and trees,
    # both storage types, greedy and sampling with one-hot and dense q, every indicator, one to five thresholds.
    # A request that meets a residual normaliser below the conditioning floor whatever is drawn (a tiny or very
    # peaked vocabulary) is compared up to that point instead of in full; such requests are few (bounded).
    rng = np.random.default_rng(1000 + seed)
    ran = 0
    for case in range(6):
        w, ind, ths, tree = sweep_case(rng, seed, case)
        compare_ex(w, indicator=ind, thetas=tiled(ths, w.B) if ths else None,
                   cdf_guard=5e-6 if w.V > 20000 else None, allow_small_norm=True,
                   label=f"sweep_s{seed}_c{case}: ind={ind} K={max(1, len(ths))} tree={tree}")
        ran += 1
    assert ran == 6


@pytest.mark.timeout(7200)
def test_long_seeded_sweep_when_asked_for():
    # The same recipe over a range of seeds given in the environment (MARS_LONG_SWEEP=first:last, six cases per
    # seed; a thousand seeds take four minutes on the GPU).  Not part of a default run.  A case whose inputs the
    # screening cannot bring clear of the thresholds, or too many of whose requests meet a small normaliser
    # whatever is drawn, is counted and left out: these are properties of the inputs, and their share is bounded.
    import os
    span = os.environ.get("MARS_LONG_SWEEP")
    if not span:
        pytest.skip("set MARS_LONG_SWEEP=first:last to run it")
    first, last = (int(x) for x in span.split(":"))
    ran = left_out = 0
    for seed in range(first, last):
        rng = np.random.default_rng(1000 + seed)
        for case in range(6):
            w, ind, ths, tree = sweep_case(rng, seed, case)
            try:
                compare_ex(w, indicator=ind, thetas=tiled(ths, w.B) if ths else None,
                           cdf_guard=5e-6 if w.V > 20000 else None, allow_small_norm=True,
                           label=f"sweep_s{seed}_c{case}: ind={ind} K={max(1, len(ths))} tree={tree}")
                ran += 1
            except RuntimeError as e:
                if "guard band not reached" not in str(e):
                    raise
                left_out += 1
            except AssertionError as e:
                if "cannot be compared in full" not in str(e):
                    raise
                left_out += 1
    print(f"long sweep: {ran} cases compared, {left_out} left out")
    assert left_out * 100 <= max(ran, 100)


def test_margin_stats_many_cells_and_no_row_output():
    # half a million cells for the top-1 logit (the counters are cleared by the row reduction itself), and the
    # per-row table left out (rows_out = NULL)
    from oracle import mars_ref
    from paper_2601_15498_amd import binding as M
    from tests.gpu_util import to_device
    w = make_config(3, B=16)
    ranges, bins = ((0.0, 64.0), (0.0, 1.0), (0.0, 1.0)), (1 << 19, 3, 2)
    compare_margin(w, ranges, bins, label="margin_many_cells")
    d = to_device(w)
    rows, counts = M.mars_margin_stats(d["logits"], d["theta"], w.temperature, np.asarray(ranges).reshape(6), bins,
                                       want_rows=False)
    torch.cuda.synchronize()
    assert rows is None
    ref = mars_ref.margin_stats(w.logits, w.theta, w.temperature, ranges, bins)
    c = counts.cpu().numpy().view(np.uint32)
    assert np.array_equal(c[:bins[0] + 2], ref["hist_z1"]) and c[-4:].tolist() == ref["summary"].tolist()


def test_calls_on_two_streams_with_their_own_workspaces_overlap_and_stay_exact():
    # The library keeps no state: calls that do not share a workspace may run side by side.  Two different
    # headline-shaped batches alternate on two streams (the per-request kernel of one call beside the row
    # reduction of the next); after a burst of calls each stream's outputs equal the oracle's.
    from oracle import screen
    from paper_2601_15498_amd import binding as M
    from tests.gpu_util import to_device
    ws_list = [make_config(2, B=8), make_config(2, B=8, seed=92)]
    refs = [screen.screen_uniforms(w) for w in ws_list]
    devs = [to_device(w) for w in ws_list]
    dev = devs[0]["logits"].device
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [M.alloc_workspace(w.B, w.N, w.V, dev) for w in ws_list]
    outs = [M.VerifyOutputs(w.B, w.N, dev) for w in ws_list]
    torch.cuda.synchronize()
    for i in range(24):
        j = i % 2
        d = devs[j]
        with torch.cuda.stream(streams[j]):
            M.mars_verify(d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], ws_list[j].temperature,
                          d["uniforms"], d["draft_probs"], outs[j], wss[j])
    torch.cuda.synchronize()
    for j in range(2):
        assert (outs[j].request_status.cpu().numpy() == 0).all()
        for key in ("accept_len", "bonus_token", "accept_mask", "path_idx", "decision"):
            assert np.array_equal(getattr(outs[j], key).cpu().numpy(), refs[j][key]), (j, key)


def test_calls_on_four_streams_finish_and_stay_exact():
    # More calls side by side than the chip has room for: each call's per-request kernel wants one
    # work-group per compute unit, so with four streams many work-groups wait for a compute unit while their
    # partners already run.  Nobody waits for them for long (a partner's sum is worked out by whoever needs
    # it), so every call finishes, no request carries a status, and every output equals the oracle's.
    from oracle import screen
    from paper_2601_15498_amd import binding as M
    from tests.gpu_util import to_device
    ws_list = [make_config(2, B=8, seed=sd) for sd in (2, 92, 93, 94)]
    refs = [screen.screen_uniforms(w) for w in ws_list]
    devs = [to_device(w) for w in ws_list]
    dev = devs[0]["logits"].device
    streams = [torch.cuda.Stream() for _ in ws_list]
    wss = [M.alloc_workspace(w.B, w.N, w.V, dev) for w in ws_list]
    outs = [M.VerifyOutputs(w.B, w.N, dev) for w in ws_list]
    torch.cuda.synchronize()
    for i in range(32):
        j = i % 4
        d = devs[j]
        with torch.cuda.stream(streams[j]):
            M.mars_verify(d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], ws_list[j].temperature,
                          d["uniforms"], d["draft_probs"], outs[j], wss[j])
    torch.cuda.synchronize()
    for j in range(4):
        assert (outs[j].request_status.cpu().numpy() == 0).all(), j
        for key in ("accept_len", "bonus_token", "accept_mask", "path_idx", "decision"):
            assert np.array_equal(getattr(outs[j], key).cpu().numpy(), refs[j][key]), (j, key)


@pytest.mark.parametrize("T", [0.0, 0.7])
def test_pass_enqueued_in_two_parts_equals_the_whole(T):
    # stages: the row reduction and the per-request part as two calls with the same arguments, other work on
    # the stream in between; the result is that of the single call, bit for bit.
    from paper_2601_15498_amd import binding as M
    from tests.gpu_util import to_device
    w = make_config(2, B=5, temperature=T)
    d = to_device(w)
    dev = d["logits"].device
    ws = M.alloc_workspace(w.B, w.N, w.V, dev)
    args = (d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], T, d["uniforms"] if T > 0 else None,
            d["draft_probs"] if T > 0 else None)
    whole = M.mars_verify_ex(*args, workspace=ws, want_commit=True)
    torch.cuda.synchronize()
    parts = M.VerifyOutputs(w.B, w.N, dev, want_commit=True)
    M.mars_verify_ex(*args, out=parts, workspace=ws, stages=M.MARS_STAGE_ROWS)
    junk = torch.randn(1 << 20, device=dev).sum()          # unrelated work between the two parts
    M.mars_verify_ex(*args, out=parts, workspace=ws, stages=M.MARS_STAGE_REQUESTS)
    torch.cuda.synchronize()
    assert torch.isfinite(junk)
    for key in ("accept_len", "bonus_token", "accept_mask", "path_idx", "decision", "request_status", "stats", "diag",
                "out_tokens", "out_len", "keep_rows", "keep_offsets"):
        assert torch.equal(getattr(parts, key), getattr(whole, key)), key


def test_strict_sampling_on_the_gpu_reproduces_the_target_distribution():
    # Not through the oracle: with theta > 1 the pass is plain speculative sampling, which is lossless
    # (Sec. 2.3): whatever the draft distribution, the first committed token follows softmax(z / T).
    # 40 000 requests share one root row and one draft distribution; each draws its own draft token from
    # q and its own uniforms.  Chi-square against the closed form, and the same test must reject the
    # draft distribution itself.
    from scipy.stats import chi2
    from paper_2601_15498_amd import binding as M
    rng = np.random.default_rng(31)
    B, N, V, T = 40000, 2, 6, 0.8
    z0 = np.array([2.0, 1.2, 0.1, -0.5, 1.7, -2.0], np.float32)
    z1 = rng.normal(0, 1, V).astype(np.float32)
    q0 = np.array([0.05, 0.4, 0.2, 0.05, 0.1, 0.2], np.float32)
    p = np.exp(z0.astype(np.float64) / np.float64(np.float32(T)))
    p /= p.sum()
    z = np.tile(np.stack([z0, z1])[None], (B, 1, 1))
    q = np.tile(np.stack([q0, np.full(V, 1.0 / V, np.float32)])[None], (B, 1, 1)).astype(np.float32)
    tok = np.zeros((B, N), np.int32)
    qn = q0.astype(np.float64) / q0.astype(np.float64).sum()
    tok[:, 1] = rng.choice(V, size=B, p=qn)
    par = np.tile(np.array([-1, 0], np.int32), (B, 1))
    u = rng.random((B, N + 1), dtype=np.float32)
    dev = torch.device("cuda:0")
    out = M.mars_verify_ex(torch.from_numpy(z).to(dev), torch.from_numpy(tok).to(dev), torch.from_numpy(par).to(dev),
                           torch.full((B,), 2.0, dtype=torch.float32, device=dev), T, torch.from_numpy(u).to(dev),
                           torch.from_numpy(q).to(dev), want_commit=True)
    torch.cuda.synchronize()
    first = out.out_tokens[:, 0].cpu().numpy()
    counts = np.bincount(first, minlength=V).astype(np.float64)
    stat = ((counts - B * p) ** 2 / (B * p)).sum()
    limit = chi2.ppf(1 - 1e-4, V - 1)
    say(f"[info] first committed token: chi2 {stat:.2f} (limit {limit:.2f}), accepted {float(out.accept_len.float().mean()):.3f}")
    assert stat < limit
    assert ((counts - B * qn) ** 2 / (B * qn)).sum() > 10 * limit
