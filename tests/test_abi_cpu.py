"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before any device
work."""
import ctypes
import os
import re

import pytest

from paper_2309_15531_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ctx():
    if not os.path.exists(B.LIB_PATH):
        from paper_2309_15531_amd.build import build
        build(verbose=False)
    c = B.Context(stream=0)
    yield c
    c.close()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "adadim.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adadim_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(ctx):
    lib = B.load_library()
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.adadim_version().decode().startswith("adadim-gfx950")


def test_no_torch_types_in_header():
    text = open(os.path.join(ROOT, "include", "adadim.h")).read()
    assert "torch" not in text.replace("torch.nn.Linear", "") and "at::" not in text
    assert 'extern "C"' in text


A16 = ctypes.c_void_p(0x1000)      # fake, aligned, never dereferenced: validation fails first
ODD = ctypes.c_void_p(0x1004)
F1 = ctypes.c_float(1.0)


def test_quantize_validation(ctx):
    q = lambda *a: ctx.raw("adadim_quantize", *a)
    tail = (A16, None, None, None, 0, None, None)
    assert q(None, 64, 64, 0, 3, 32, F1, *tail) == B.ENULL
    assert q(A16, 0, 64, 0, 3, 32, F1, *tail) == B.EINVAL
    assert q(A16, 64, 64, 2, 3, 32, F1, *tail) == B.EINVAL          # dim
    assert "dim" in ctx.last_error()
    assert q(A16, 64, 64, 0, 1, 32, F1, *tail) == B.EINVAL          # bits
    assert q(A16, 64, 64, 0, 9, 32, F1, *tail) == B.EINVAL
    assert q(A16, 64, 96, 0, 3, 64, F1, *tail) == B.EINVAL          # 96 % 64
    assert q(A16, 96, 64, 1, 3, 64, F1, *tail) == B.EINVAL          # per-IC groups run along out
    assert q(A16, 64, 64, 0, 3, -1, F1, *tail) == B.EINVAL
    assert q(A16, 64, 64, 0, 3, 32, ctypes.c_float(0.0), *tail) == B.EINVAL
    assert q(A16, 64, 64, 0, 3, 32, ctypes.c_float(1.5), *tail) == B.EINVAL
    assert q(A16, 64, 64, 0, 3, 32, ctypes.c_float(float("nan")), *tail) == B.EINVAL
    assert q(ODD, 64, 64, 0, 3, 32, F1, *tail) == B.EALIGN
    # scaled fp16 dW needs the column scales
    assert q(A16, 64, 64, 0, 3, 32, F1, None, None, None, A16, B.DW_F16_SCALED, None, None) == B.ENULL
    assert q(A16, 64, 64, 0, 3, 32, F1, None, None, None, A16, 7, None, None) == B.EINVAL


def test_hessian_validation(ctx):
    h = lambda *a: ctx.raw("adadim_hessian", *a)
    assert h(A16, 16, 64, 64, None, 0) == B.ENULL
    assert h(None, 16, 64, 64, A16, 0) == B.ENULL
    assert h(A16, -1, 64, 64, A16, 0) == B.EINVAL
    assert h(A16, 16, 64, 32, A16, 0) == B.EINVAL                   # ldx < in
    assert h(A16, 16, 64, 64, A16, 2) == B.EINVAL
    assert h(A16, 16, 60, 64, A16, 0) == B.EALIGN                   # in % 8
    assert h(ODD, 16, 64, 64, A16, 0) == B.EALIGN
    p = lambda *a: ctx.raw("adadim_hessian_prepare", *a)
    assert p(None, 64, A16, A16) == B.ENULL
    assert p(A16, 0, A16, A16) == B.EINVAL
    assert p(A16, 60, A16, A16) == B.EALIGN


def test_error_and_select_validation(ctx):
    e = lambda *a: ctx.raw("adadim_layer_error", *a)
    assert e(None, 0, 64, 64, A16, None, A16) == B.ENULL
    assert e(A16, 0, 64, 64, A16, None, None) == B.ENULL
    assert e(A16, 0, 0, 64, A16, None, A16) == B.EINVAL
    assert e(A16, B.DW_F16_SCALED, 64, 64, A16, None, A16) == B.EINVAL   # scaled dW needs the prepared form
    assert e(A16, 0, 64, 60, A16, None, A16) == B.EALIGN
    ep = lambda *a: ctx.raw("adadim_layer_error_prepared", *a)
    assert ep(A16, B.DW_F16_SCALED, 64, 64, A16, None, None, A16) == B.ENULL
    assert ep(A16, 5, 64, 64, A16, A16, None, A16) == B.EINVAL
    s = lambda *a: ctx.raw("adadim_select", *a)
    assert s(None, 2, A16, None) == B.ENULL
    assert s(A16, 0, A16, None) == B.EINVAL
    assert s(A16, 2, None, None) == B.ENULL
    assert "adadim_select" in ctx.last_error()


def test_gemv_validation(ctx):
    gv = lambda *a: ctx.raw("adadim_gemv_ic", *a)
    assert gv(None, A16, A16, A16, 64, 64, 4, 32, A16) == B.ENULL
    assert gv(A16, A16, A16, A16, 64, 64, 4, 32, None) == B.ENULL
    assert gv(A16, A16, A16, A16, 64, 64, 5, 32, A16) == B.EINVAL          # 2, 3 or 4 bits
    assert gv(A16, A16, A16, A16, 64, 64, 4, 48, A16) == B.EINVAL          # group not a multiple of 32
    assert gv(A16, A16, A16, A16, 96, 64, 4, 64, A16) == B.EINVAL          # group does not divide out
    assert gv(A16, A16, A16, A16, 64, 62, 4, 32, A16) == B.EINVAL          # in % 4
    assert gv(ctypes.c_void_p(A16.value + 4), A16, A16, A16, 64, 64, 4, 32, A16) == B.EALIGN
    assert "adadim_gemv_ic" in ctx.last_error()
    gm = lambda *a: ctx.raw("adadim_gemv_ic_meta16", *a)
    assert gm(A16, None, A16, 64, 64, 4, 32, A16) == B.ENULL
    assert gm(A16, A16, A16, 64, 64, 5, 32, A16) == B.EINVAL
    assert gm(A16, ctypes.c_void_p(A16.value + 4), A16, 64, 64, 4, 32, A16) == B.EALIGN
    assert "adadim_gemv_ic_meta16" in ctx.last_error()
    qm = lambda *a: ctx.raw("adadim_quantize_meta16", *a)
    assert qm(A16, 64, 64, 0, 5, 32, ctypes.c_float(1.0), None, A16, None, 0, None, None) == B.EINVAL   # 2, 3 or 4 bits
    assert qm(None, 64, 64, 0, 4, 32, ctypes.c_float(1.0), None, A16, None, 0, None, None) == B.ENULL
    assert qm(A16, 64, 64, 1, 4, 48, ctypes.c_float(1.0), None, A16, None, 0, None, None) == B.EINVAL
    assert ctx._lib.adadim_score_elems(300, 64) == 512 * 64 and ctx._lib.adadim_score_elems(300, 40) == 300 * 40


def test_gptq_validation(ctx):
    """GPTQ entry points: argument checks that run before any launch."""
    f1 = ctypes.c_float(0.01)
    pr = lambda *a: ctx.raw("adadim_gptq_prepare", *a)
    assert pr(None, 64, f1, 1, A16, A16, A16) == B.ENULL
    assert pr(A16, 0, f1, 1, A16, A16, A16) == B.EINVAL
    assert "adadim_gptq_prepare" in ctx.last_error()
    gq = lambda *a: ctx.raw("adadim_gptq_quantize", *a)
    assert gq(A16, 64, 64, 0, 4, 32, None, A16, A16, A16, A16, A16, None, None, None, None) == B.ENULL       # U
    assert gq(A16, 64, 64, 0, 4, 32, A16, A16, A16, None, None, A16, None, None, None, None) == B.ENULL     # static parameters
    assert gq(A16, 64, 64, 0, 4, 48, A16, A16, A16, A16, A16, A16, None, None, None, None) == B.EINVAL      # group does not divide in
    assert gq(A16, 128, 64, 1, 4, 32, A16, A16, A16, None, None, A16, A16, A16, None, None) == B.EINVAL     # per-IC group 64 or 128
    assert gq(A16, 128, 64, 1, 4, 64, A16, A16, A16, None, None, A16, None, None, None, None) == B.ENULL    # per-IC outputs
    assert gq(A16, 64, 64, 2, 4, 32, A16, A16, A16, A16, A16, A16, None, None, None, None) == B.EINVAL      # dim
    assert "adadim_gptq_quantize" in ctx.last_error()
    gm = lambda *a: ctx.raw("adadim_gptq_quantize_meta16", *a)
    assert gm(A16, 64, 64, 0, 5, 32, A16, A16, A16, A16, A16, None, None, None) == B.EINVAL                 # 2, 3 or 4 bits
    assert gm(A16, 64, 64, 0, 4, 32, A16, A16, A16, None, A16, None, None, None) == B.ENULL                 # static words
    assert gm(A16, 128, 64, 1, 4, 64, A16, A16, A16, None, A16, None, None, None) == B.ENULL                # word output
    assert gm(A16, 128, 64, 1, 4, 32, A16, A16, A16, None, A16, A16, None, None) == B.EINVAL
    assert "adadim_gptq_quantize_meta16" in ctx.last_error()


def test_capture_validation(ctx):
    """Graph recording: argument checks that need no device (the test context sits on the default stream)."""
    assert ctx._lib.adadim_capture_begin(None) == B.ENULL
    assert ctx.raw("adadim_capture_begin") == B.EINVAL                    # default stream cannot be recorded
    assert "default stream" in ctx.last_error()
    g = ctypes.c_void_p()
    assert ctx.raw("adadim_capture_end", ctypes.byref(g)) == B.EINVAL      # not recording
    assert ctx.raw("adadim_graph_launch", None) == B.ENULL
    ctx._lib.adadim_graph_destroy(None)


def test_profile_only_validation(ctx):
    assert ctx._lib.adadim_profile_only(None, b"gram_tiles") == B.ENULL
    assert ctx.raw("adadim_profile_only", b"gram_tiles") == B.OK
    assert ctx.raw("adadim_profile_only", b"x" * 32) == B.EINVAL          # at most 31 characters
    assert "adadim_profile_only" in ctx.last_error()
    assert ctx.raw("adadim_profile_only", None) == B.OK


def test_create_destroy():
    lib = B.load_library()
    assert lib.adadim_create(None, None) == B.ENULL
    assert b"NULL" in lib.adadim_last_error(None)
    lib.adadim_destroy(None)
    c = B.Context(stream=0)
    assert c.last_error() == "no error"
    c.close()
    c.close()


def test_code_field_plan_on_the_host(tmp_path):
    """csrc/code_fields.h (how the matrix-vector kernel reads 2-, 3- and 4-bit codes as fp16 patterns): the plan run
    on the CPU returns every code of random and extreme streams exactly, each once."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = tmp_path / "code_fields_check"
    src = os.path.join(ROOT, "tests", "host", "code_fields_check.cpp")
    subprocess.run(["g++", "-O2", "-std=c++17", src, "-o", str(exe)], check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout
    assert "2 bits: 0, 3 bits: 0, 4 bits: 0 mismatches" in res.stdout


def test_gram_launch_plans_cover_every_tile_once(tmp_path):
    """csrc/gram_plan.h (which workgroup of the Gram kernel runs which tile over which tokens, and where its partial
    tile goes): for the plans the library chooses over many shapes, and for hand-made ones at the corners of the
    arithmetic, every tile is taken whole once or covered by its pieces exactly once, no two pieces share a
    partial slot, and the reduction reads exactly the slots the pieces wrote.  The chosen plan for the 4096-wide
    layer at 65536 tokens must keep the 32 units of an XCD within 5 % of the even share."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = tmp_path / "gram_plan_check"
    src = os.path.join(ROOT, "tests", "host", "gram_plan_check.cpp")
    subprocess.run(["g++", "-O2", "-std=c++17", src, "-o", str(exe)], check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout
    assert " 0 mistakes" in res.stdout
    res = subprocess.run([str(exe), "65536", "4096"], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout
    share = [float(m) for m in re.findall(r"even share \d+ \(([0-9.]+)\)", res.stdout)]
    assert len(share) == 2 and min(share) >= 0.95, res.stdout


def test_bench_refuses_more_than_one_gpu():
    """One GPU per box: bench.py --gpus 2 says so and exits before anything touches a GPU."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "one GPU only" in res.stderr and res.stdout == ""


def test_product_does_not_import_oracle():
    """The product package must never reach into the oracle (and vice versa)."""
    pkg = os.path.join(ROOT, "paper_2309_15531_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "oracle/" not in src, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2309_15531_amd" not in src and "ctypes" not in src, f


def test_fast_division_matches_ieee(tmp_path):
    """The quantizer's three-operation quotient (csrc/fastdiv.h) must equal the IEEE
    division for every fp16-valued numerator; sampled here (2^12 scale significands per
    weight significand, four exponent pairs, both signs), exhaustive with argument 23."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = tmp_path / "fastdiv_check"
    src = os.path.join(ROOT, "tests", "host", "fastdiv_check.cpp")
    subprocess.run(["g++", "-O2", "-std=c++17", "-mfma", "-ffp-contract=off", "-pthread", src, "-o", str(exe)],
                   check=True)
    res = subprocess.run([str(exe), "12", "8"], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout
    assert " 0 mismatches" in res.stdout


def test_binding_refuses_tensors_the_library_would_misread():
    """The library sees addresses only; the binding must stop a transposed view, a wrong element type or a host
    tensor before its address goes in."""
    import torch
    from paper_2309_15531_amd.binding import _need

    class Dev:                                    # a device tensor's attributes without a device
        def __init__(self, t):
            self.t = t
        is_cuda, device = True, "cuda:0"
        dtype = property(lambda s: s.t.dtype)
        shape = property(lambda s: s.t.shape)
        def dim(self): return self.t.dim()
        def numel(self): return self.t.numel()
        def stride(self, *a): return self.t.stride(*a)
        def is_contiguous(self): return self.t.is_contiguous()

    w = torch.zeros((8, 16), dtype=torch.float16)
    _need(Dev(w), "W", "float16")
    _need(None, "W", "float16")
    _need(Dev(w[:, :8]), "X", "float16", pitched=True)           # a row pitch is fine where ldx carries it
    with pytest.raises(TypeError):
        _need(w, "W", "float16")                                  # host tensor
    with pytest.raises(TypeError):
        _need(Dev(w.float()), "W", "float16")                     # wrong element type
    with pytest.raises(ValueError):
        _need(Dev(w.t()), "W", "float16")                         # transposed view
    with pytest.raises(ValueError):
        _need(Dev(w[:, :8]), "W", "float16")                      # pitched where the ABI takes none


def test_host_checks_under_sanitizers(tmp_path):
    """The host builds of the device headers (fast division, code-field plan, Gram launch plan) compiled with the address and
    undefined-behaviour sanitizers: the constexpr plans and the bit manipulation the kernels share with these
    checks must be free of out-of-bounds indexing, signed overflow and shifts past the width."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1", "-std=c++17"]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env.pop("LD_PRELOAD", None)                   # the sanitizer runtime has to be first in the process
    for name, extra, argv, want in (("code_fields_check", [], [], "2 bits: 0, 3 bits: 0, 4 bits: 0 mismatches"),
                                    ("fastdiv_check", ["-mfma", "-ffp-contract=off", "-pthread"], ["10", "4"], " 0 mismatches"),
                                    ("gram_plan_check", [], [], " 0 mistakes")):
        exe = tmp_path / (name + "_san")
        build = subprocess.run(["g++", *san, *extra, os.path.join(ROOT, "tests", "host", name + ".cpp"), "-o", str(exe)],
                               capture_output=True, text=True)
        if build.returncode != 0 and "asan" in build.stderr.lower() and "cannot find" in build.stderr.lower():
            pytest.skip("the sanitizer runtime is not installed")
        assert build.returncode == 0, build.stderr
        res = subprocess.run([str(exe), *argv], capture_output=True, text=True, env=env)
        assert res.returncode == 0, res.stdout + res.stderr
        assert want in res.stdout and "runtime error" not in res.stderr
