"""mars_verify_static -- the entry point for callers that cannot allocate: the pass runs on the
library's own static device array instead of a caller's workspace.  Its outputs are compared with
those of mars_verify_ex (caller's workspace) on the same inputs, through the C ABI: two calls in a
row on the one array, the second with a smaller input, in sampling mode with a dense draft
distribution (partial results, merged statistics and exchange words all live in the array), then
in greedy mode.  Integers, bytes and indices bit-exact; fp32 statistics within rel 1e-5 (the two
entry points share their kernels, so in practice every bit agrees)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

INT_KEYS = ("accept_mask", "accept_len", "path_idx", "bonus_token", "decision", "request_status",
            "out_tokens", "out_len", "keep_rows", "keep_offsets")


def _both(M, w, d, label):
    from tests.gpu_util import say
    say(f"[case] {label}: B={w.B} N={w.N} V={w.V} T={w.temperature} dense_q={w.draft_probs is not None}")
    a = M.mars_verify_ex(d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], w.temperature,
                         d["uniforms"], d["draft_probs"], want_commit=True)
    torch.cuda.synchronize()
    b = M.mars_verify_static(d["logits"], d["draft_tokens"], d["tree_parent"], d["theta"], w.temperature,
                             d["uniforms"], d["draft_probs"], want_commit=True)
    torch.cuda.synchronize()
    for key in INT_KEYS:
        x, y = getattr(a, key).cpu().numpy(), getattr(b, key).cpu().numpy()
        assert np.array_equal(x, y), f"{label}: {key} differs"
    sa = {k: v.cpu().numpy() for k, v in M.unpack_stats(a.stats).items()}
    sb = {k: v.cpu().numpy() for k, v in M.unpack_stats(b.stats).items()}
    for key in ("id1", "id2", "relax_ok", "z1", "z2"):
        assert np.array_equal(sa[key], sb[key]), f"{label}: stats.{key} differs"
    np.testing.assert_allclose(sb["sum_exp"], sa["sum_exp"], rtol=1e-5, atol=0)
    da = {k: v.cpu().numpy() for k, v in M.unpack_diag(a.diag).items()}
    db = {k: v.cpu().numpy() for k, v in M.unpack_diag(b.diag).items()}
    for key in ("residual_passes", "last_node"):
        assert np.array_equal(da[key], db[key]), f"{label}: diag.{key} differs"
    for key in ("bonus_prob", "last_residual_norm"):
        np.testing.assert_allclose(db[key], da[key], rtol=1e-5, atol=0)
    assert (a.request_status.cpu().numpy() == 0).all()
    say(f"[ok]   {label}: accept_len {a.accept_len.cpu().numpy().tolist()}")


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    from mars_inputs import make_config
    from paper_2601_15498_amd import binding as M
    from tests.gpu_util import to_device
    tree = {"kind": "tree", "depth": 4, "max_children": 4}
    big = make_config(2, B=6, N=30, V=40000, tree=tree)                 # sampling, dense q, bf16
    small = make_config(2, B=2, N=12, V=9001, tree={"kind": "tree", "depth": 3, "max_children": 4})
    dbig, dsmall = to_device(big), to_device(small)
    _both(M, big, dbig, "static_sampling_first")
    _both(M, small, dsmall, "static_sampling_second_smaller")
    g_big = make_config(3, B=5, N=9, V=50000)                           # greedy chains, per-request theta
    g_small = make_config(0, B=1, N=5, V=3000)
    _both(M, g_big, to_device(g_big), "static_greedy_first")
    _both(M, g_small, to_device(g_small), "static_greedy_second_smaller")


def test_static_scratch_entry_point_rejects_sizes_beyond_its_array():
    from paper_2601_15498_amd import binding as M
    import ctypes
    L = M.lib()
    # 1024 requests of 1024 nodes: the partial results alone need far more than the array holds
    assert M.mars_workspace_bytes(1024, 1024, 151936) > M.MARS_STATIC_SCRATCH_BYTES
    p = ctypes.c_void_p(0x1000)      # never dereferenced: the size check comes first
    null = ctypes.c_void_p(0)
    rc = L.mars_verify_static(p, 1, p, p, null, 0, p, ctypes.c_float(0.0), null, 1024, 1024, 151936,
                              p, p, p, p, null, null, null, null, null, None)
    assert rc == M.MARS_ERR_SCRATCH
    assert b"scratch" in L.mars_status_string(rc)
