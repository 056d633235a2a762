"""The C-ABI library loads and exports every symbol include/logoskg.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "logoskg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(logoskg_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2604_18913_amd as m
    path = m.library_path()
    if not os.path.exists(path):
        from paper_2604_18913_amd import build_ext
        build_ext.build(verbose=False)
    lib = ctypes.CDLL(path)
    syms = declared_symbols()
    assert {"logoskg_build", "logoskg_khop", "logoskg_paths"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), f"{s} is declared in logoskg.h but not exported"
    assert m.version().startswith("logoskg")


def test_struct_sizes_match_the_header():
    from paper_2604_18913_amd import binding as b
    # sizes follow from the field lists in logoskg.h under the x86-64 SysV ABI
    assert ctypes.sizeof(b._BuildOpts) == 64
    assert ctypes.sizeof(b._QueryBatch) == 56
    assert ctypes.sizeof(b._HopStats) == 56
    assert ctypes.sizeof(b._ResultInfo) == 48
    assert ctypes.sizeof(b._GraphInfo) == 120


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_18913_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f"{f} mentions the oracle"


def test_bench_refuses_more_than_one_gpu():
    # this build runs on exactly one GPU: bench.py says so and exits before it touches anything
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)


def test_bench_byte_model_of_the_list_writer():
    # the roofline of the dominant kernel prices 72 bytes per (entity, word) cell handed over by the
    # row walk plus 9 bytes per list entry (entity, hop, predecessor)
    import os
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    units = dict(rows=1000, edges=0, lines=0, items=50000, launches_per_step=1)
    got = bench.algorithmic_bytes("pred", units, 16, 3, False, 0.0, lists_fused=True)
    assert got == 72 * 1000 + 9 * 50000
