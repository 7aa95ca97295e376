"""CPU-only checks of the product's host side: the shared library loads and
exports what include/lasgd.h declares, argument validation happens before any
device call, and the workload generator gives the published architectures."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "lasgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lasgd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.load()
    names = _declared()
    assert len(names) >= 14
    for n in names:
        assert hasattr(L, n), f"{n} is declared in include/lasgd.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_library_is_built_from_the_current_sources():
    """The tests and the GPU runs load the in-tree library as it is; one left over from an
    experiment or an older source would be measured and tested instead of the code."""
    lib = os.path.getmtime(B.LIB_PATH)
    srcs = [os.path.join(ROOT, "paper_2203_13085_amd", "csrc", f) for f in os.listdir(os.path.join(ROOT, "paper_2203_13085_amd", "csrc"))]
    srcs.append(os.path.join(ROOT, "include", "lasgd.h"))
    stale = [os.path.relpath(f, ROOT) for f in srcs if os.path.getmtime(f) > lib]
    assert not stale, f"rebuild the library (python __graft_entry__.py): newer than it are {stale}"


def test_binding_struct_layouts_match_header():
    # field order and count of the two structs the binding mirrors
    text = open(os.path.join(ROOT, "include", "lasgd.h")).read()
    cfg = re.search(r"typedef struct \{([^{}]*)\} lasgd_config;", text, flags=re.S).group(1)
    cfg = re.sub(r"/\*.*?\*/", "", cfg, flags=re.S)
    fields = re.findall(r"(\w+)\s*;", cfg)
    assert fields == [f for f, _ in B.Config._fields_]
    tun = re.search(r"typedef struct \{([^{}]*)\} lasgd_tuning;", text, flags=re.S).group(1)
    tun = re.sub(r"/\*.*?\*/", "", tun, flags=re.S)
    assert re.findall(r"(\w+)\s*;", tun) == [f for f, _ in B.Tuning._fields_]
    assert ctypes.sizeof(B.Tuning) == 48


def _create(**kw):
    L = B.load()
    numel = kw.pop("numel", [16, 32])
    arr = (ctypes.c_int64 * len(numel))(*numel) if numel is not None else None
    wd = kw.pop("weight_decay", None)
    wda = (ctypes.c_float * len(wd))(*wd) if wd is not None else None
    cfg = B.Config(kw.pop("K", 2), kw.pop("n_tensors", len(numel) if numel else 0), arr,
                   kw.pop("storage", 0), kw.pop("momentum", 0.9), 1, wda, kw.pop("wd_scalar", 0.0), None, None)
    h = ctypes.c_void_p()
    st = L.lasgd_create(ctypes.byref(cfg), ctypes.byref(h))
    msg = L.lasgd_last_error(None).decode()
    if st == B.OK:
        L.lasgd_destroy(h)
    else:
        assert not h.value
    return st, msg


@pytest.mark.parametrize("kw", [dict(K=0), dict(K=65), dict(K=-3), dict(numel=[4, 0]), dict(numel=[-1]),
                                dict(storage=7), dict(momentum=float("nan")), dict(momentum=-0.1),
                                dict(wd_scalar=float("inf")), dict(weight_decay=[0.1, float("nan")]),
                                dict(numel=None)])
def test_create_rejects_bad_arguments_without_touching_the_device(kw):
    st, msg = _create(**kw)
    assert st == B.ERR_INVALID and msg


def test_create_rejects_oversized_replica():
    st, msg = _create(numel=[1 << 30, 1 << 30, 1 << 30])
    assert st == B.ERR_UNSUPPORTED and "elements" in msg


def test_null_arguments():
    L = B.load()
    assert L.lasgd_create(None, None) == B.ERR_INVALID
    for f in ("lasgd_local_step",):
        assert getattr(L, f)(None, 0.1) == B.ERR_INVALID
    for f in ("lasgd_snapshot", "lasgd_average", "lasgd_sync", "lasgd_init_master"):
        assert getattr(L, f)(None) == B.ERR_INVALID
    assert L.lasgd_merge(None, 1) == B.ERR_INVALID
    assert L.lasgd_step_merge(None, 0.1, 1) == B.ERR_INVALID
    L.lasgd_destroy(None)    # allowed


def test_static_global_update_validates_before_any_device_call():
    """No GPU here: every refusal below must come back as a status, not a HIP error."""
    buf = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    bad = (ctypes.c_void_p * 2)(0x1004, 0x2000)
    same = (ctypes.c_void_p * 2)(0x1000, 0x1010)          # 16 bytes apart, 32 bytes long: they overlap
    cross = (ctypes.c_void_p * 2)(0x2010, 0x3000)         # overlaps the second entry of buf
    L = B.load()
    assert L.lasgd_global_update_static(2, 8, None, buf, 1, None) == B.ERR_INVALID
    assert L.lasgd_global_update_static(0, 8, buf, buf, 1, None) == B.ERR_INVALID
    assert L.lasgd_global_update_static(65, 8, buf, buf, 1, None) == B.ERR_INVALID
    assert L.lasgd_global_update_static(2, 0, buf, buf, 1, None) == B.ERR_INVALID
    assert L.lasgd_global_update_static(2, 8, bad, buf, 1, None) == B.ERR_INVALID
    assert L.lasgd_global_update_static(2, 8, same, buf, 1, None) == B.ERR_INVALID
    assert L.lasgd_global_update_static(2, 8, buf, cross, 1, None) == B.ERR_INVALID
    assert b"overlaps" in L.lasgd_last_error(None)
    assert L.lasgd_global_update_static(2, B.STATIC_MAX_N + 1, buf, same, 1, None) == B.ERR_UNSUPPORTED
    assert b"LASGD_STATIC_MAX_N" in L.lasgd_last_error(None)
    text = open(os.path.join(ROOT, "include", "lasgd.h")).read()
    m = re.search(r"#define LASGD_STATIC_MAX_N \((\d+)ll << (\d+)\)", text)
    assert int(m.group(1)) << int(m.group(2)) == B.STATIC_MAX_N


def test_shape_lists_match_published_architectures():
    # tensor and parameter counts of the torchvision-style models these rules describe
    for shapes, nt, npar in ((W.resnet_shapes(18), 62, 11689512), (W.resnet_shapes(50), 161, 25557032),
                             (W.mobilenet_v2_shapes(), 158, 3504872)):
        assert len(shapes) == nt
        assert sum(W.numel(s) for _, s in shapes) == npar
        assert all(W.numel(s) % 4 == 0 for _, s in shapes)
    r50 = [W.numel(s) for _, s in W.resnet_shapes(50)]
    assert min(r50) == 64 and max(r50) == 2359296
    mb = [W.numel(s) for _, s in W.mobilenet_v2_shapes()]
    assert min(mb) == 16 and max(mb) == 1280000


def test_inputs_are_pure_functions_of_their_key():
    w = W.config(1)
    a = W.gradient_tensor(w, 3, 2, 5)
    b = W.gradient_tensor(w, 3, 2, 5)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, W.gradient_tensor(w, 3, 1, 5))
    assert not np.array_equal(a, W.gradient_tensor(w, 4, 2, 5))
    assert abs(float(a.std()) - 1e-3) < 2e-4
    x0 = W.initial_tensor(w, 0)                     # 64x3x7x7 conv: He-normal, fan_in 147
    assert abs(float(x0.std()) - (2 / 147) ** 0.5) < 0.01
    assert np.all(W.initial_tensor(w, 1) == 1.0) and np.all(W.initial_tensor(w, 2) == 0.0)
    bits = W.to_bf16_bits(a)
    assert np.all(np.abs(W.bf16_bits_to_f32(bits) - a) <= np.abs(a) * 2.0 ** -8)


def test_product_path_never_touches_the_oracle():
    """The HIP path and the oracle share no code: nothing in the package imports,
    loads or names the oracle, and bench.py reaches it only inside cpu_baseline()."""
    import ast
    pkg = os.path.join(ROOT, "paper_2203_13085_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"(import\s+oracle|from\s+oracle|liblasgd_oracle|lasgd_oracle|lasgd_ref64)", text), \
                    f"{f} reaches for the oracle"
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for node in ast.walk(tree):
        if isinstance(node, ast.FunctionDef):
            uses = any(isinstance(n, (ast.Import, ast.ImportFrom)) and "oracle" in ast.dump(n) for n in ast.walk(node))
            if uses:
                assert node.name == "cpu_baseline", f"bench.py imports the oracle in {node.name}()"
    top = [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom))]
    assert not any("oracle" in ast.dump(n) for n in top)
    # and the oracle does not import the package or load its library
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert not re.search(r"(import\s+paper_2203_13085_amd|from\s+paper_2203_13085_amd|liblasgd_hip|hip_runtime|#include\s+\"lasgd)", text), f


def test_algorithmic_bytes_match_the_per_unit_figures():
    """The roofline's numerator: 20 B per replica-parameter for a local step (either storage), 28 B + 4 B/K for
    the fused step + global update, 4 (K + 1) B per parameter for the mean, 28 B + 8 B/K with the mean inside."""
    import bench
    for cfg, (step, sm, av) in {0: (83_886_080, 121_634_816, 20_971_520),
                                2: (4_089_125_120, 5_827_003_296, 920_053_152),
                                3: (1_121_559_040, 1_584_202_144, 238_331_296),
                                4: (16_356_500_480, 23_001_328_800, 3_373_528_224)}.items():
        w = W.config(cfg)
        a = bench.algorithmic_bytes(w.K, w.N, w.storage == "bf16")
        assert (a["local_step"], a["step_merge"], a["average"]) == (step, sm, av)
        assert a["local_step"] == 20 * w.K * w.N
        assert a["step_merge"] == 28 * w.K * w.N + 4 * w.N
        assert a["average"] == 4 * (w.K + 1) * w.N
        assert a["step_merge_average"] == 28 * w.K * w.N + 8 * w.N
    # one cycle of the default workload (m = 4): 19.01 GB
    w = W.config(2)
    a = bench.algorithmic_bytes(w.K, w.N, False)
    assert round(((w.m - 1) * a["local_step"] + a["step_merge"] + a["average"]) / 1e9, 2) == 19.01


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and not r.stdout.strip()


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "paper_2203_13085_amd", "no_such_library.so"))
    with pytest.raises(FileNotFoundError):
        B.load()
