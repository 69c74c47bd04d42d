"""Host-side sanitizer pass (CPU only): the oracle's C file and the library's host code (argument checking, shape and
size arithmetic) are rebuilt with AddressSanitizer + UndefinedBehaviorSanitizer and driven by small C / C++ programs
that call every entry point on exactly-sized heap buffers with ragged, degenerate and invalid arguments.  Device code
is not sanitized (not available for gfx950 here); the library driver only takes paths that return before any launch."""
import os
import shutil
import subprocess
import tempfile

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_00031_amd", "csrc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def test_oracle_c_file_under_asan_ubsan():
    tmp = tempfile.mkdtemp(prefix="zo_san_")
    try:
        exe = os.path.join(tmp, "oracle_san")
        subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-mfma", "-mavx2", "-fopenmp",
                               "-fsanitize=address,undefined,float-cast-overflow,float-divide-by-zero", "-fno-sanitize-recover=all",
                               os.path.join(ROOT, "oracle", "zo_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_main.c"),
                               "-lm", "-o", exe])
        r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
        assert r.returncode == 0 and "ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_reported_zero_point_saturates():
    """Found by the pass above: a constant group far from zero has a zero point beyond int32 (Background/Quantization:
    z = -round(min / step), not clamped; the step is at its floor).  The arithmetic keeps it as a float; the integer that
    is reported saturates (as the GPU's float -> int conversion does) instead of being undefined."""
    from oracle import zo_oracle as orc
    step, zp, codes, xhat = orc.quant_group(np.full(8, 1e30, np.float32), 4)
    assert step == np.float32(1e-5) and zp == -2 ** 31
    assert np.all(codes == 0) and np.all(np.isfinite(xhat))
    step, zp, codes, xhat = orc.quant_group(np.full(8, -1e30, np.float32), 4)
    assert zp == 2 ** 31 - 1


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_library_host_side_under_asan_ubsan():
    tmp = tempfile.mkdtemp(prefix="zo_san_")
    try:
        flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
                 "-packed-fp32-ops", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-option-ignored",
                 "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
        srcs = [f for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")] + ["sanitize_host_main.cpp"]
        procs = []
        for f in srcs:
            obj = os.path.join(tmp, f + ".o")
            procs.append((f, obj, subprocess.Popen(["hipcc", *flags, "-c", os.path.join(CSRC, f), "-o", obj],
                                                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        for f, obj, p in procs:
            out, _ = p.communicate()
            assert p.returncode == 0, "%s:\n%s" % (f, out[-3000:])
        exe = os.path.join(tmp, "host_san")
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-Wno-option-ignored",
                               *[o for _, o, _ in procs], "-o", exe], stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
        assert r.returncode == 0 and "ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
