"""The C-ABI library loads and exports every symbol the header declares; pure host entry
points behave.  No compute call is made (no GPU here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1709_09393_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "slimdp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(slimdp_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = binding.load()
    names = header_functions()
    assert len(names) >= 16
    for name in names:
        assert hasattr(L, name), name
    assert sorted(binding.EXPORTS) == names


def test_header_constants_match_binding():
    src = open(os.path.join(ROOT, "include", "slimdp.h")).read()
    assert int(re.search(r"#define SLIMDP_TILE (\d+)u", src).group(1)) == binding.TILE
    assert int(re.search(r"#define SLIMDP_MAX_WORKERS (\d+)u", src).group(1)) == binding.MAX_WORKERS
    for name in ["OK", "ERR_INVALID_ARG", "ERR_OUT_OF_RANGE", "ERR_STALE_CORE", "ERR_WORKSPACE", "ERR_HIP",
                 "ERR_DEVICE_STATUS"]:
        m = re.search(r"SLIMDP_%s = (-?\d+)" % name, src)
        assert int(m.group(1)) == getattr(binding, name)


def test_num_tiles_and_workspace_are_pure_host_functions():
    assert binding.num_tiles(1) == 1
    assert binding.num_tiles(4096) == 1
    assert binding.num_tiles(4097) == 2
    assert binding.num_tiles(138_357_544) == (138_357_544 + 4095) // 4096
    # tiles never cross a segment
    assert binding.num_tiles(10000, [0, 1, 4097, 10000]) == 1 + 1 + 2
    # invalid shapes
    assert binding.num_tiles(0) == 0
    assert binding.num_tiles(10, [0, 5, 5, 10]) == 0        # empty segment
    assert binding.num_tiles(10, [0, 7, 5, 10]) == 0        # not increasing
    assert binding.num_tiles(10, [1, 10]) == 0
    assert binding.num_tiles(2 ** 31) == 2 ** 31 // 4096      # the largest model
    assert binding.num_tiles(2 ** 31 + 1) == 0
    assert binding.num_tiles(2 ** 32) == 0
    assert binding.workspace_bytes(10, 0) == 0
    assert binding.workspace_bytes(10, 33) == 0
    small = binding.workspace_bytes(1_000_000, 4)
    big = binding.workspace_bytes(138_357_544, 8)
    assert 0 < small < big < 2 * 2 ** 30           # 1.2 GiB at the VGG-16 size: bitmaps, counts, pair slots, lists
    assert 0 < binding.capture_bytes(138_357_544, 8) < 1.3 * 2 ** 30
    assert binding.capture_bytes(10, 0) == 0


def test_create_rejects_bad_arguments_before_touching_the_gpu():
    L = binding.load()
    h = C.c_void_p()
    so = (C.c_uint64 * 2)(0, 10)
    assert L.slimdp_create(None, 10, 1, 1, so, 0, None) == binding.ERR_INVALID_ARG
    assert L.slimdp_create(C.byref(h), 0, 1, 1, so, 0, None) == binding.ERR_INVALID_ARG
    assert L.slimdp_create(C.byref(h), 10, 0, 1, so, 0, None) == binding.ERR_INVALID_ARG
    assert L.slimdp_create(C.byref(h), 10, 64, 1, so, 0, None) == binding.ERR_INVALID_ARG
    bad = (C.c_uint64 * 3)(0, 12, 10)
    assert L.slimdp_create(C.byref(h), 10, 1, 2, bad, 0, None) == binding.ERR_INVALID_ARG
    assert b"seg_off" in L.slimdp_last_error(None)
    assert not h.value
    for fn in (L.slimdp_destroy, L.slimdp_synchronize):
        assert fn(None) == binding.ERR_INVALID_ARG


def test_workload_recipes():
    v = workloads.VGG16
    assert (v.n, v.W, v.k, v.m) == (138_357_544, 8, 13_835_754, 2_490_435)
    s = workloads.STRESS
    assert (s.W, s.k, s.m) == (16, 6_917_877, 1_314_396)
    t = workloads.TINY
    assert (t.n, t.W, t.k, t.m) == (1_000_000, 4, 100_000, 18_000)
    g = workloads.GOOGLENET
    off = g.segment_offsets()
    sizes = np.diff(off.astype(np.int64))
    assert off[0] == 0 and off[-1] == g.n == 6_998_552 and sizes.size == 57 and sizes.min() >= 1
    assert np.array_equal(g.k_seg(), (sizes * 10 // 100).astype(np.uint64))
    # seeded: same call, same bits; different worker or iteration, different draw
    a = workloads.TINY.scaled(1000)
    assert np.array_equal(a.gradient(0, 1), a.gradient(0, 1))
    assert not np.array_equal(a.gradient(0, 1), a.gradient(0, 2))
    assert not np.array_equal(a.gradient(0, 1), a.gradient(1, 1))
    st = workloads.STRESS.scaled(10000)
    wv = st.weights()
    assert np.array_equal(wv, wv.astype(np.float16).astype(np.float32))


def test_bench_refuses_more_than_one_gpu_and_models_the_stages():
    """bench.py runs on one GPU only and says so; its stream model of the headline workload is the 13.864 GB of the
    benchmark definition (no GPU needed for either)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert proc.returncode != 0 and "ONE GPU" in proc.stderr and proc.stdout.strip() == ""
    sys.path.insert(0, root)
    import bench
    wl = workloads.VGG16
    sb = bench.stage_bytes(wl.n, wl.W, wl.k, wl.m)
    assert abs(sum(sb.values()) - 13.864e9) < 1e6
    assert sb["score"] == 4 * wl.n * (wl.W + 2)


def test_product_path_and_oracle_do_not_know_each_other():
    """The library's package never imports, names or loads the oracle, and the oracle nothing of the package
    (the seeded input module is shared by the tests, not by the two sides); only tests, the smoke check and the
    bench's CPU leg may touch oracle/."""
    import subprocess
    import sys
    pkg = os.path.join(ROOT, "paper_1709_09393_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".c", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), os.path.join(dirpath, f)
                assert "slimdp_oracle" not in text and "oracle/" not in text, os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_1709_09393_amd" not in text and "slimdp.h" not in text and "libslimdp.so" not in text, f
    # importing the package and loading the library pulls in no oracle module
    code = ("import sys; from paper_1709_09393_amd import binding, workloads; binding.load(); "
            "assert not [m for m in sys.modules if m == 'oracle' or m.startswith('oracle.')]")
    subprocess.run([sys.executable, "-c", code], cwd=ROOT, check=True)
    # bench.py imports the oracle only inside its CPU leg
    bench_src = open(os.path.join(ROOT, "bench.py")).read()
    top_level = [l for l in bench_src.splitlines() if re.match(r"(import|from)\s+oracle\b", l)]
    assert not top_level


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    """No silent fallback: without the built library the binding raises and names the build step."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libslimdp.so"))
    with pytest.raises(FileNotFoundError) as e:
        binding.load()
    assert "build" in str(e.value)
    with pytest.raises(FileNotFoundError):
        binding.num_tiles(10)
