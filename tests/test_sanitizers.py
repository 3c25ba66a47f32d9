"""CPU sanitizer leg: the oracle's C sources and the library's host-only helpers are rebuilt with
AddressSanitizer + UndefinedBehaviorSanitizer and exercised in a child process (the sanitizer runtime has to
be loaded first, so the instrumented code cannot run inside the pytest process).  No GPU is involved."""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = textwrap.dedent(r'''
    import ctypes as C, os, sys
    import numpy as np
    assert "libasan" in open("/proc/self/maps").read(), "the sanitizer runtime is not loaded"
    sys.path.insert(0, ROOT); sys.path.insert(0, os.path.join(ROOT, "tests"))
    from oracle import build_oracle
    build_oracle.LIB = ORACLE_SO                       # oracle_api loads the instrumented build
    build_oracle.build = lambda force=False: ORACLE_SO
    import oracle_api as O
    from paper_2507_19131_amd import synth
    # one small shifted, padded block with taps, both branches, three threads
    spec = synth.BlockSpec(2, 19, 24, 64, 2, shift=3)
    inp = synth.make_block_inputs(spec, 23, per_branch_bias=True)
    x = synth.make_feature_map(spec, 23, blobs=True)
    k = O.keep_count(spec.nW, 0.4)
    perm = O.select_windows(O.score_windows(inp, x), k)
    y, taps = O.block_forward(inp, x, perm, k, want_taps="all", threads=3)
    assert not np.isnan(y).any() and len(taps) == 14
    y2, _ = O.block_forward(inp, x, None, k, threads=1)
    assert np.array_equal(y, y2)
    y3, _ = O.block_forward(inp, x, O.select_windows(O.score_windows(inp, x), 3, k_low=4), 3, k_low=4)
    assert np.array_equal(O.uniform_block(inp, x, 0), O.block_forward(inp, x, None, spec.nW)[0])
    win, valid = O.gather_windows(spec, x, perm)
    assert np.array_equal(O.scatter_windows(spec, win, perm), x)
    # a layer between stages
    ds = synth.DownSpec(1, 1, 9, 11, 8, 32)
    out, codes, acc = O.downsample_forward(synth.make_downsample_inputs(ds, 5), np.random.default_rng(3).standard_normal((1, 9, 11, 8)).astype(np.float32), want_taps=True, threads=2)
    assert out.shape == (1, 5, 6, 32)
    # the library's host-only helpers: cost model and ratio sampler
    H = C.CDLL(HOST_SO)
    gm = (C.c_double * 6)(13.3, 13.56, 14.16, 14.16, 14.16, 14.02)
    r = (C.c_double * 6)(*[0.5] * 6)
    bits = C.c_double()
    assert H.mixaq_equivalent_act_bits(6, gm, C.c_double(3.0), r, None, C.c_double(4.0), C.byref(bits)) == 0
    assert abs(bits.value - 3.0347) < 1e-3
    rng = np.random.default_rng(1)
    for _ in range(50):
        u = np.ascontiguousarray(rng.uniform(1e-9, 1.0, 1 + 6 * 20000))
        ratios = (C.c_double * 6)()
        used = C.c_size_t()
        H.mixaq_sample_ratios.argtypes = [C.c_int32, C.c_double, C.c_double, C.c_double, C.c_void_p, C.c_size_t, C.POINTER(C.c_size_t), C.c_void_p]
        assert H.mixaq_sample_ratios(6, 0.6, 4.2, 0.8, u.ctypes.data, u.size, C.byref(used), ratios) == 0
        assert max(ratios) <= 0.8 + 1e-12 and (used.value - 1) % 6 == 0
    u = np.array([0.5, 0.1])
    assert H.mixaq_sample_ratios(6, 0.6, 4.2, 0.8, u.ctypes.data, u.size, None, ratios) == -4      # runs out: an error, no overrun
    k_out = C.c_int32()
    H.mixaq_keep_count.argtypes = [C.c_int32, C.c_double, C.POINTER(C.c_int32)]
    assert H.mixaq_keep_count(1369, 0.4, C.byref(k_out)) == 0 and k_out.value == 548
    print("SANITIZED RUN OK")
''')

HOST_SHIM = textwrap.dedent(r'''
    // host-only part of the library for the sanitizer build: the error channel and mixaq_keep_count as in api.hip
    #include <cmath>
    #include <cstdarg>
    #include <cstdio>
    #include "../include/mixaq.h"
    namespace mixaq {
    thread_local char g_err[512] = "";
    int fail(int code, const char* fmt, ...) { va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap); return code; }
    }
''')


def _find_runtime(name):
    out = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_oracle_and_host_helpers_under_asan_ubsan(tmp_path):
    asan = _find_runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    flags = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_so = str(tmp_path / "liboracle_san.so")
    srcs = [os.path.join(ROOT, "oracle", s) for s in ("mixaq_oracle.c", "uniform_block.c", "downsample.c")]
    subprocess.run(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared"] + flags + ["-o", oracle_so] + srcs + ["-lm"],
                   check=True)
    # keep_count is taken from api.hip's text so that the instrumented function is the product's own
    api = open(os.path.join(ROOT, "paper_2507_19131_amd", "csrc", "api.hip")).read()
    a = api.index("int mixaq_keep_count(")
    b = api.index("\n}\n", a) + 3
    shim = tmp_path / "host_shim.cpp"
    shim.write_text(HOST_SHIM.replace("../include/mixaq.h", os.path.join(ROOT, "include", "mixaq.h")) +
                    "using mixaq::fail;\nextern \"C\" {\n" + api[a:b] + "}\n")
    host_so = str(tmp_path / "libhost_san.so")
    subprocess.run(["g++", "-std=c++17", "-fPIC", "-shared"] + flags + ["-o", host_so, str(shim),
                    os.path.join(ROOT, "paper_2507_19131_amd", "csrc", "cost_sampler.cpp")], check=True)
    env = dict(os.environ, LD_PRELOAD=" ".join(filter(None, [asan, os.environ.get("LD_PRELOAD", "")])),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="3")
    code = "ROOT=%r\nORACLE_SO=%r\nHOST_SO=%r\n" % (ROOT, oracle_so, host_so) + DRIVER
    res = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0 and "SANITIZED RUN OK" in res.stdout, (res.stdout[-2000:], res.stderr[-4000:])
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
