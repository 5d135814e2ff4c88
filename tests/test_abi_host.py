"""Host-only checks of the C-ABI library: it loads, exports every function the public
header declares, and its pure host helpers (validation, workspace sizing, status strings)
behave.  No GPU compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    from paper_2605_08632_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_08632_amd import build
        build.build(verbose=False)
    return binding


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(pard2_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol(b):
    L = b.lib()
    declared = _declared_functions()
    assert {"pard2_cat_fwd", "pard2_cat_bwd", "pard2_cat_weights"} <= declared
    for name in declared:
        assert hasattr(L, name), f"{name} declared in include/ but not exported"
    assert set(b.EXPORTS) == declared
    assert L.pard2_cat_abi_version() == 1


def test_descriptor_layout_matches_header(b):
    # 12 four-byte fields then two int64: 64 bytes, strides at offsets 48 and 56
    assert ctypes.sizeof(b.pard2_cat_desc) == 64
    assert b.pard2_cat_desc.ldH.offset == 48 and b.pard2_cat_desc.ldW.offset == 56


def test_validate_and_workspace(b):
    ok = b.make_desc(8192, 2048, 128256, 1024, 8, b.PARD2_BF16)
    assert b.pard2_cat_validate(ok) == 0
    n = b.pard2_cat_workspace_bytes(ok)
    assert 0 < n < 8 << 30
    # never the T x V logits: far below T*V*2 bytes
    assert n < 8192 * 128256 * 2
    bad = [
        (dict(T=8191), -2),                      # T != B*K
        (dict(d=2044, ldH=2044, ldW=2044), -2),  # bf16 needs d % 8 == 0
        (dict(ldH=2040), -2),                    # stride below d
        (dict(dtype=7), -3),
        (dict(weight_mode=3), -3),
        (dict(reduction=2), -3),
        (dict(flags=2), -3),                     # unknown descriptor flag
        (dict(beta=float("nan")), -6),
        (dict(weight_mode=b.PARD2_W_DECAY, gamma=0.0), -6),
        (dict(weight_mode=b.PARD2_W_DECAY, gamma=1.5), -6),
        (dict(ignore_index=5), -6),              # ignore_index must not be a real id
        (dict(V=0), -2),
    ]
    for change, code in bad:
        d = b.make_desc(8192, 2048, 128256, 1024, 8, b.PARD2_BF16)
        for k, v in change.items():
            setattr(d, k, v)
        assert b.pard2_cat_validate(d) == code, change
        assert b.pard2_cat_workspace_bytes(d) == 0
    assert b.lib().pard2_cat_validate(None) == -1
    f32 = b.make_desc(64, 250, 4099, 8, 8, b.PARD2_FP32)          # fp32 has no multiple-of-8 rule
    assert b.pard2_cat_validate(f32) == 0 and b.pard2_cat_workspace_bytes(f32) > 0


def test_status_strings(b):
    seen = {b.pard2_status_string(c) for c in range(0, -8, -1)}
    assert len(seen) == 8 and "ok" in seen
    assert "unknown" in b.pard2_status_string(-99)


def test_null_arguments_rejected_before_any_launch(b):
    L = b.lib()
    d = b.make_desc(64, 256, 4096, 8, 8, b.PARD2_FP32)
    args = [ctypes.byref(d)] + [None] * 13 + [None, 0, None]
    assert L.pard2_cat_fwd(*args) == -1
    args = [ctypes.byref(d)] + [None] * 9 + [0, None, 0, None]
    assert L.pard2_cat_bwd(*args) == -1
    assert L.pard2_cat_weights(ctypes.byref(d), None, None, None, None, None, None) == -1
    # non-null data pointers but no workspace -> workspace error (still no launch)
    one = ctypes.c_void_p(256)
    args = [ctypes.byref(d)] + [one] * 3 + [None, None, one, one, one, one, None, None, None, None] + [None, 0, None]
    assert L.pard2_cat_fwd(*args) == -4


def test_kd_entry_points_validate_on_the_host(b):
    L = b.lib()
    desc = b.make_desc(64, 64, 512, 8, 8, b.PARD2_BF16)
    assert b.pard2_cat_kd_workspace_bytes(desc, 128) > 0
    assert b.pard2_cat_kd_workspace_bytes(desc, 100) == 0            # teacher width not a multiple of 8
    assert b.pard2_cat_kd_workspace_bytes(b.make_desc(64, 60, 513, 8, 8, b.PARD2_FP32), 100) > 0   # fp32: no multiple-of-8 rule
    assert b.pard2_cat_kd_workspace_bytes(b.make_desc(64, 64, 512, 8, 8, b.PARD2_BF16, beta=-0.1), 128) == 0
    assert ctypes.sizeof(b.pard2_kd_teacher) == 40
    one = 256
    te = b.pard2_kd_teacher(one, one, 128, 128, 128, 0)
    # null teacher / null data pointers / fp32 storage / missing workspace: all rejected before any launch
    assert L.pard2_cat_kd_fwd(ctypes.byref(desc), one, one, None, *([None] * 13), None, 0, None) == -1
    assert L.pard2_cat_kd_fwd(ctypes.byref(desc), None, one, ctypes.byref(te), *([None] * 13), None, 0, None) == -1
    neg = b.make_desc(64, 64, 512, 8, 8, b.PARD2_BF16, beta=-1.0)
    assert L.pard2_cat_kd_fwd(ctypes.byref(neg), one, one, ctypes.byref(te), *([None] * 13), None, 0, None) == -6
    args = [one, None, None, None, one, one, one] + [None] * 6        # y .. dev_status
    assert L.pard2_cat_kd_fwd(ctypes.byref(desc), one, one, ctypes.byref(te), *args, None, 0, None) == -4
    bad = b.pard2_kd_teacher(one, one, 64, 128, 128, 0)              # stride below the teacher's width
    assert L.pard2_cat_kd_fwd(ctypes.byref(desc), one, one, ctypes.byref(bad), *args, None, 0, None) == -2
    assert L.pard2_cat_kd_bwd(ctypes.byref(desc), one, one, ctypes.byref(te), *([None] * 8), 0, None, None, None,
                              None, 0, None) == -1


def test_inject_entry_points_validate_on_the_host(b):
    L = b.lib()
    one = 256
    feats = (ctypes.c_void_p * 3)(one, one, one)
    # only calls that are rejected before any launch: the pointers here are not device memory
    assert L.pard2_inject_fwd(64, 60, 32, 3, one, feats, 32, one, one, one, None) == -2     # d % 8
    assert L.pard2_inject_fwd(64, 64, 32, 9, one, feats, 32, one, one, one, None) == -2     # F > 8
    assert L.pard2_inject_fwd(64, 64, 32, 3, one, feats, 24, one, one, one, None) == -2     # stride < dt
    assert L.pard2_inject_fwd(64, 64, 32, 3, None, feats, 32, one, one, one, None) == -1
    assert L.pard2_inject_fwd(64, 64, 32, 3, one, None, 32, one, one, one, None) == -1
    hole = (ctypes.c_void_p * 3)(one, None, one)
    assert L.pard2_inject_bwd(64, 64, 32, 3, one, hole, 32, one, one, one, 0, None) == -1
    assert L.pard2_inject_bwd(64, 64, 32, 3, one, feats, 32, one, None, one, 0, None) == -1


def test_binding_raises_without_library(b, monkeypatch, tmp_path):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(b.Pard2Error):
        b.lib()


def test_header_is_plain_c_and_links(b, tmp_path):
    """gcc -std=c99 -pedantic compiles a C program against include/pard2_cat.h, links the library and runs
    its host-only calls (layout of the two structs, validation, refusal of null pointers)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("gcc not found")
    b.lib()                                              # the library must exist
    exe = str(tmp_path / "abi_host_check")
    libdir = os.path.dirname(b.LIB_PATH)
    src = os.path.join(ROOT, "tests", "c", "abi_host_check.c")
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), src,
           "-o", exe, "-L", libdir, "-lpard2cat", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib",
           "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "abi_host_check ok" in r.stdout, r.stdout + r.stderr


def test_product_path_is_independent_of_the_oracle():
    """Nothing under the package (Python or HIP sources) imports, includes or names a file of oracle/,
    and the oracle imports nothing from the package; bench.py touches the oracle in its CPU-baseline
    leg only."""
    pkg = os.path.join(ROOT, "paper_2605_08632_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath or "__pycache__" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "cat_oracle" not in text and "inject_oracle" not in text and "oracle/" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2605_08632_amd" not in open(os.path.join(ROOT, "oracle", f), encoding="utf-8").read(), f
    bench = open(os.path.join(ROOT, "bench.py"), encoding="utf-8").read()
    uses = [m.start() for m in re.finditer(r"from oracle import", bench)]
    start = bench.index("def cpu_baseline")
    end = bench.index("\ndef ", start + 1)
    assert len(uses) == 1 and start < uses[0] < end
