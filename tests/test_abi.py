"""The C-ABI library loads without a GPU and exports every symbol include/ss.h declares (CPU only)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ss.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    import paper_2509_11076_amd.binding as B
    names = declared_functions()
    assert "ss_swap_out" in names and "ss_timeline_scan" in names and len(names) >= 20
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "libss.so does not export %s" % n
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert callable(getattr(B, n)), "binding lacks %s" % n


def test_hook_library_exports_what_its_header_declares():
    import paper_2509_11076_amd.torch_hook as H
    text = open(os.path.join(ROOT, "include", "ss_torch_hook.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(ss_hook_[a-z_0-9]+)\s*\(", text)))
    assert len(names) == 10 and names == sorted(H.EXPORTS)
    lib = ctypes.CDLL(H.LIB_PATH)
    for n in names:
        assert hasattr(lib, n) and callable(getattr(H, n))
    assert H.ss_hook_get_stats()["ops"] == 0          # nothing is hooked until ss_hook_install
    with pytest.raises(H.B.SsError):
        H.ss_hook_set_mode(7)


def test_record_layouts_match_the_header_sizes():
    import paper_2509_11076_amd.binding as B
    import workloads as W
    text = open(os.path.join(ROOT, "include", "ss.h")).read()
    for name, dt in (("ss_op_t", B.OP_DT), ("ss_event_t", B.EVENT_DT), ("ss_tensor_t", B.TENSOR_DT),
                     ("ss_anchor_t", B.ANCHOR_DT), ("ss_policy_item_t", B.POLICY_DT),
                     ("ss_desc_t", B.DESC_DT), ("ss_action_t", B.ACTION_DT)):
        m = re.search(r"\}\s*%s;\s*/\*\s*(\d+) B" % name, text)
        assert m and int(m.group(1)) == dt.itemsize, name
    for a, b in ((B.OP_DT, W.OP_DT), (B.EVENT_DT, W.EVENT_DT), (B.TENSOR_DT, W.TENSOR_DT),
                 (B.POLICY_DT, W.POLICY_DT), (B.DESC_DT, W.DESC_DT), (B.ACTION_DT, W.ACTION_DT)):
        assert a == b


def test_configuration_record_has_the_librarys_size():
    """ss_config_default clears the whole record before it sets the defaults: on a buffer of 0xFF bytes it
    rewrites exactly as many bytes as the binding's record is long"""
    import paper_2509_11076_amd.binding as B
    n = ctypes.sizeof(B.ss_config_t)
    buf = (ctypes.c_ubyte * (n + 64))(*([0xFF] * (n + 64)))
    lib = ctypes.CDLL(B.LIB_PATH)
    lib.ss_config_default.argtypes = [ctypes.c_void_p]
    assert lib.ss_config_default(ctypes.addressof(buf)) == 0
    raw = bytes(buf)
    assert raw[n:] == b"\xff" * 64 and raw[n - 8:n] == b"\x00" * 8      # flag_wait_ms and the reserved word: 0
    header = open(os.path.join(ROOT, "include", "ss.h")).read()
    body = re.search(r"typedef struct \{([^}]*)\} ss_config_t;", re.sub(r"/\*.*?\*/", "", header, flags=re.S)).group(1)
    names = re.findall(r"\b(?:uint64_t|uint32_t)\s+([a-z_0-9, ]+);", body)
    fields = [x.strip() for grp in names for x in grp.split(",")]
    assert fields == [f for f, _ in B.ss_config_t._fields_]


def test_host_only_calls_work_without_a_gpu():
    import paper_2509_11076_amd.binding as B
    cfg = B.ss_config_default()
    assert (cfg.align, cfg.stage_m, cfg.stage_n, cfg.guard_bytes) == (256, 2, 5, 0)
    assert B.ss_strerror(B.SS_E_INFEASIBLE).startswith("no candidate")
    assert B.ss_strerror(0) == "ok"
    cfg.align = 24                      # not a power of two: refused before anything touches the GPU
    with pytest.raises(B.SsError) as e:
        B.ss_create(cfg)
    assert e.value.code == B.SS_E_INVAL


def test_product_does_not_import_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2509_11076_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", src, flags=re.M), f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith(".py"):
                src = open(os.path.join(dirpath, f)).read()
                assert "paper_2509_11076_amd" not in src, f


def test_bench_refuses_more_than_one_gpu():
    """the build is for one GPU: asking the benchmark for more ends with a message, before any GPU work"""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
