"""The C-ABI library loads, exports every function include/mars.h declares, and rejects bad
arguments on the host before anything is enqueued.  No GPU needed: no call here reaches a kernel."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mars.h")
LIB = os.path.join(ROOT, "paper_2601_15498_amd", "libmars.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2601_15498_amd import build
        build.build()
    from paper_2601_15498_amd import binding
    return binding.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mars_[a-z_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert declared_functions() == ["mars_lmhead_verify", "mars_lmhead_verify_sampling", "mars_lmhead_workspace_bytes",
                                    "mars_margin_stats",
                                    "mars_row_reduce", "mars_row_stats", "mars_status_string",
                                    "mars_verify", "mars_verify_ex", "mars_verify_static", "mars_version",
                                    "mars_workspace_bytes",
                                    "mars_workspace_bytes_ex"]


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_struct_sizes_match_the_binding():
    from paper_2601_15498_amd import binding
    text = open(HEADER).read()
    row = re.search(r"typedef struct mars_row_stat \{(.*?)\}", text, re.S).group(1)
    diag = re.search(r"typedef struct mars_req_diag \{(.*?)\}", text, re.S).group(1)
    assert len(re.findall(r"\b(float|int32_t)\b", re.sub(r"/\*.*?\*/", "", row, flags=re.S))) == binding.ROW_STAT_WORDS
    assert len(re.findall(r"\b(float|int32_t)\b", re.sub(r"/\*.*?\*/", "", diag, flags=re.S))) == binding.REQ_DIAG_WORDS
    mrow = re.search(r"typedef struct mars_margin_row \{(.*?)\}", text, re.S).group(1)
    assert len(re.findall(r"\bfloat\b", mrow)) == binding.MARGIN_ROW_WORDS
    opt = re.sub(r"/\*.*?\*/", "", re.search(r"typedef struct mars_verify_options \{(.*?)\}", text, re.S).group(1), flags=re.S)
    fields = re.findall(r"(int32_t\s*\*?)\s*(\w+);", opt)
    assert [n for _, n in fields] == [n for n, _ in binding.VerifyOptionsStruct._fields_]
    assert ["*" in t for t, _ in fields] == [t is ctypes.c_void_p for _, t in binding.VerifyOptionsStruct._fields_]


def test_version_and_status_strings(lib):
    assert lib.mars_version() >= 100
    assert lib.mars_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert len(lib.mars_status_string(code)) > 0


def test_workspace_bytes(lib):
    assert lib.mars_workspace_bytes(16, 60, 151936) > 0
    assert lib.mars_workspace_bytes(16, 60, 151936) % 256 == 0
    assert lib.mars_workspace_bytes(1, 1, 2) > 0
    for B, N, V in ((0, 60, 100), (1, 0, 100), (1, 1025, 100), (1, 5, 1), (-3, 5, 100)):
        assert lib.mars_workspace_bytes(B, N, V) == 0


def test_host_side_argument_errors_enqueue_nothing(lib):
    p = ctypes.c_void_p(0x1000)  # never dereferenced: every case below fails validation first
    null = ctypes.c_void_p(0)
    ok = dict(logits=p, ldt=0, tok=p, par=p, dq=null, ddt=0, theta=p, T=0.0, u=null, B=2, N=4, V=100,
              mask=p, alen=p, path=p, bonus=p, dec=null, st=null, stats=null, diag=null, ws=p, wsb=1 << 20, stream=null)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.mars_verify(a["logits"], a["ldt"], a["tok"], a["par"], a["dq"], a["ddt"], a["theta"],
                               ctypes.c_float(a["T"]), a["u"], a["B"], a["N"], a["V"], a["mask"], a["alen"],
                               a["path"], a["bonus"], a["dec"], a["st"], a["stats"], a["diag"], a["ws"],
                               ctypes.c_size_t(a["wsb"]), a["stream"])

    assert call(logits=null) == -1 and call(tok=null) == -1 and call(par=null) == -1 and call(theta=null) == -1
    assert call(mask=null) == -1 and call(alen=null) == -1 and call(path=null) == -1 and call(bonus=null) == -1
    assert call(B=0) == -1 and call(N=0) == -1 and call(N=1025) == -1 and call(V=1) == -1
    assert call(T=-0.5) == -1 and call(T=float("nan")) == -1 and call(T=float("inf")) == -1
    assert call(T=1.0, u=null) == -1            # sampling needs uniforms
    assert call(ldt=7) == -2
    assert call(T=1.0, u=p, dq=p, ddt=5) == -2
    assert call(ws=null) == -3 and call(wsb=16) == -3 and call(ws=ctypes.c_void_p(0x1010)) == -3
    rr = lib.mars_row_reduce
    assert rr(null, 0, ctypes.c_float(0.0), 1, 1, 10, p, ctypes.c_size_t(1 << 20), null) == -1
    assert rr(p, 9, ctypes.c_float(0.0), 1, 1, 10, p, ctypes.c_size_t(1 << 20), null) == -2
    assert rr(p, 0, ctypes.c_float(-1.0), 1, 1, 10, p, ctypes.c_size_t(1 << 20), null) == -1
    assert rr(p, 0, ctypes.c_float(0.0), 1, 1, 10, null, ctypes.c_size_t(1 << 20), null) == -3
    assert lib.mars_workspace_bytes_ex(2, 4, 100, 1) == lib.mars_workspace_bytes(2, 4, 100)
    assert lib.mars_workspace_bytes_ex(2, 4, 100, 8) > lib.mars_workspace_bytes(2, 4, 100)
    assert lib.mars_workspace_bytes_ex(2, 4, 100, 0) == 0 and lib.mars_workspace_bytes_ex(2, 4, 100, 65) == 0

    from paper_2601_15498_amd.binding import VerifyOptionsStruct

    def call_ex(opt, **kw):
        a = dict(ok, **kw)
        return lib.mars_verify_ex(a["logits"], a["ldt"], a["tok"], a["par"], a["dq"], a["ddt"], a["theta"],
                                  ctypes.c_float(a["T"]), a["u"], a["B"], a["N"], a["V"], a["mask"], a["alen"],
                                  a["path"], a["bonus"], a["dec"], a["st"], a["stats"], a["diag"], a["ws"],
                                  ctypes.c_size_t(a["wsb"]), a["stream"], ctypes.byref(opt) if opt else None)

    assert call_ex(None, logits=null) == -1                                   # NULL options = mars_verify
    assert call_ex(VerifyOptionsStruct(3, 1, 0, 0, None, None, None, None)) == -1   # unknown indicator
    assert call_ex(VerifyOptionsStruct(-1, 1, 0, 0, None, None, None, None)) == -1
    assert call_ex(VerifyOptionsStruct(0, 65, 0, 0, None, None, None, None)) == -1  # too many thresholds
    assert call_ex(VerifyOptionsStruct(0, -2, 0, 0, None, None, None, None)) == -1
    assert call_ex(VerifyOptionsStruct(0, 1, 0, 0, 0x1000, None, None, None)) == -1  # commit outputs: all or none
    assert call_ex(VerifyOptionsStruct(0, 1, 0, 0, 0x1000, 0x1000, 0x1000, None)) == -1
    assert lib.mars_workspace_bytes(2, 4, 100) <= 2048 < lib.mars_workspace_bytes_ex(2, 4, 100, 8)
    assert call_ex(VerifyOptionsStruct(1, 8, 0, 0, None, None, None, None), wsb=2048) == -3  # the sweep needs more workspace
    assert call_ex(VerifyOptionsStruct(0, 1, -5, 0, None, None, None, None)) == -1  # negative spin limit
    assert call_ex(VerifyOptionsStruct(0, 1, 0, 7, None, None, None, None)) == -1   # unknown stages
    assert call_ex(VerifyOptionsStruct(0, 1, 0, -1, None, None, None, None)) == -1
    ms = lib.mars_margin_stats
    rg = (ctypes.c_float * 6)(0, 1, 0, 1, 0, 1)
    bn = (ctypes.c_int32 * 3)(4, 4, 4)

    def margin(logits=p, ldt=0, theta=p, T=0.0, B=1, N=1, V=10, rg=rg, bn=bn, counts=p, ws=p, wsb=1 << 20):
        return ms(logits, ldt, theta, ctypes.c_float(T), B, N, V, rg, bn, null, counts, ws, ctypes.c_size_t(wsb), null)

    assert margin(logits=null) == -1 and margin(theta=null) == -1 and margin(counts=null) == -1
    assert margin(rg=None) == -1 and margin(bn=None) == -1
    assert margin(ldt=4) == -2 and margin(T=-1.0) == -1 and margin(V=1) == -1
    assert margin(rg=(ctypes.c_float * 6)(0, 1, 1, 1, 0, 1)) == -1           # lo >= hi
    assert margin(bn=(ctypes.c_int32 * 3)(4, 0, 4)) == -1                    # no cells
    assert margin(bn=(ctypes.c_int32 * 3)(1 << 20, 1 << 20, 4)) == -1        # too many counters
    assert margin(ws=null) == -3 and margin(wsb=8) == -3
    rs = lib.mars_row_stats
    assert rs(null, 0, p, ctypes.c_float(0.0), 1, 1, 10, p, p, ctypes.c_size_t(1 << 20), null) == -1
    assert rs(p, 3, p, ctypes.c_float(0.0), 1, 1, 10, p, p, ctypes.c_size_t(1 << 20), null) == -2
    assert rs(p, 0, p, ctypes.c_float(0.0), 1, 1, 10, p, p, ctypes.c_size_t(8), null) == -3


def test_lmhead_argument_errors_enqueue_nothing(lib):
    from paper_2601_15498_amd.binding import VerifyOptionsStruct
    p = ctypes.c_void_p(0x1000)  # never dereferenced
    null = ctypes.c_void_p(0)
    wsb = lib.mars_lmhead_workspace_bytes
    assert wsb(16, 60, 151936, 4096, 1) > 0 and wsb(16, 60, 151936, 4096, 1) % 256 == 0
    assert wsb(16, 60, 151936, 4096, 0) == wsb(16, 60, 151936, 4096, 1) < wsb(16, 60, 151936, 4096, 7)
    for B, N, V, H, K in ((0, 4, 100, 128, 1), (1, 0, 100, 128, 1), (1, 1025, 100, 128, 1), (1, 4, 1, 128, 1),
                          (1, 4, 100, 0, 1), (1, 4, 100, 64, 1), (1, 4, 100, 200, 1), (1, 4, 100, 128, 65)):
        assert wsb(B, N, V, H, K) == 0, (B, N, V, H, K)
    ok = dict(h=p, w=p, H=256, tok=p, par=p, theta=p, B=2, N=4, V=100, mask=p, alen=p, path=p, bonus=p,
              ws=p, wsb=1 << 22, opt=None)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.mars_lmhead_verify(a["h"], a["w"], a["H"], a["tok"], a["par"], a["theta"], a["B"], a["N"], a["V"],
                                      a["mask"], a["alen"], a["path"], a["bonus"], null, null, null, a["ws"],
                                      ctypes.c_size_t(a["wsb"]), null, ctypes.byref(a["opt"]) if a["opt"] else None)

    for key in ("h", "w", "tok", "par", "theta", "mask", "alen", "path", "bonus"):
        assert call(**{key: null}) == -1, key
    assert call(h=ctypes.c_void_p(0x1008)) == -1 and call(w=ctypes.c_void_p(0x1004)) == -1   # 16-byte alignment
    assert call(H=0) == -1 and call(H=192) == -1 and call(H=-128) == -1                         # multiple of 128
    assert call(B=0) == -1 and call(N=1025) == -1 and call(V=1) == -1
    assert call(ws=null) == -3 and call(wsb=64) == -3 and call(ws=ctypes.c_void_p(0x1010)) == -3
    assert call(opt=VerifyOptionsStruct(5, 1, 0, 0, None, None, None, None)) == -1              # unknown indicator
    assert call(opt=VerifyOptionsStruct(0, 65, 0, 0, None, None, None, None)) == -1
    assert call(opt=VerifyOptionsStruct(0, 1, 0, 4, None, None, None, None)) == -1              # unknown stages
    assert call(opt=VerifyOptionsStruct(0, 1, 0, 0, 0x1000, None, None, None)) == -1            # commit outputs: all or none


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2601_15498_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(binding.MarsError):
        binding.lib()


def test_source_digest_ignores_comments_and_white_space():
    """bench.py ties a hardware-counter capture to the kernel's code: rewording a comment or
    re-indenting must not change the digest, changing a token must."""
    import bench
    a = 'int f(int x) { // add one\n  return x + 1;  /* really\n one */ }\nconst char* s = "// kept";\n'
    b = 'int f(int x) {\n    return x + 1; }\n\n\nconst char* s = "// kept";   // a note\n'
    c = a.replace("x + 1", "x + 2")
    assert bench._code_only(a) == bench._code_only(b)
    assert bench._code_only(a) != bench._code_only(c)
    assert '"// kept"' in bench._code_only(a)
    assert len(bench.kernel_source_digest()) == 16


def test_bench_refuses_more_than_one_gpu():
    """The pass is per request and this build measures one GPU: asked for more, bench.py says so and
    exits before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_capture_belongs_to_the_kernels_as_they_are():
    """The HBM-traffic figure of the benchmark line is a stored counter capture, valid for the kernel
    sources it names: committed together, the two must agree (otherwise the line says traffic_stale)."""
    import bench
    assert bench.measured_traffic() is not None
