"""The C-ABI library loads and exports every symbol include/mixaq.h declares (no GPU calls)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mixaq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mixaq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2507_19131_amd import binding, build
    if not os.path.exists(binding.lib_path()):
        build.build()
    lib = ctypes.CDLL(binding.lib_path())
    names = _declared()
    assert len(names) >= 11
    for n in names:
        assert hasattr(lib, n), n
    assert lib.mixaq_version() >= 100


def test_host_only_entry_points():
    from paper_2507_19131_amd import binding as M
    assert M.mixaq_keep_count(1369, 0.4) == 548 and M.mixaq_keep_count(361, 0.4) == 144
    assert M.mixaq_keep_count(1392, 0.5) == 696 and M.mixaq_keep_count(10, 0.0) == 0
    from paper_2507_19131_amd import synth
    d = M.make_desc(synth.BlockSpec(1, 200, 336, 96, 3))
    assert M.mixaq_num_windows(d) == 1392
    d = M.make_desc(synth.BlockSpec(4, 256, 256, 128, 4))
    assert M.mixaq_num_windows(d) == 1369
    try:
        M.mixaq_keep_count(10, 1.5)
        assert False
    except M.MixaqError as e:
        assert e.code == -2 and "keep_ratio" in str(e)


def test_benchmark_refuses_more_than_one_gpu():
    """The path has no collectives: `bench.py --gpus N` with N above 1 exits with a message and measures nothing."""
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
