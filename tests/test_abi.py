"""The C-ABI library builds, loads without a GPU and exports every function include/nrt.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nrt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nrt_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_declared_symbols():
    from paper_2603_20622_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_20622_amd import build
        build.build()
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = declared_functions()
    assert "nrt_graph_create" in names and "nrt_cache_init" in names and "nrt_apply_batch" in names
    for name in names:
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(names)
    lib.nrt_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.nrt_version()


def test_argument_errors_without_gpu():
    """Pure host-side argument checks: no device call is reached."""
    from paper_2603_20622_amd import binding as nb
    L = nb.lib()
    out = ctypes.c_size_t()
    assert L.nrt_graph_workspace_bytes(0, 10, 0, ctypes.byref(out)) == nb.NRT_ERR_INVALID_ARG
    assert L.nrt_graph_workspace_bytes(10, -1, 0, ctypes.byref(out)) == nb.NRT_ERR_INVALID_ARG
    assert L.nrt_graph_workspace_bytes(1000, 5000, 1, ctypes.byref(out)) == nb.NRT_OK
    assert out.value > 2 * 5000 * 8
    h = ctypes.c_void_p()
    st = L.nrt_graph_create(10, 5, 4, 0, None, None, None, None, None, None, None, 0, None, ctypes.byref(h))
    assert st == nb.NRT_ERR_INVALID_ARG and b"e_capacity" in L.nrt_last_error()
    assert L.nrt_get_stats(None, None) == nb.NRT_ERR_INVALID_ARG


def test_struct_sizes_match_header():
    from paper_2603_20622_amd import binding as nb
    # int32*2 + int32*5 + int32*2 + float*2 = 44 bytes, padded to 48, then 8+8+4+4 pointers, then 4 floats, an int32 (padded to 8),
    # 4+4 more pointers and three int32 (padded to 16)
    assert ctypes.sizeof(nb.nrt_model_desc) == 48 + 8 * (8 + 8 + 4 + 4) + 4 * 4 + 8 + 8 * (4 + 4) + 16
    assert ctypes.sizeof(nb.nrt_batch) == 10 * 8
    assert ctypes.sizeof(nb.nrt_layer_stats) == 5 * 8 + 6 * 4


def test_mode_and_profiling_reject_null_handles():
    from paper_2603_20622_amd import binding as nb
    L = nb.lib()
    assert L.nrt_set_mode(None, nb.NRT_MODE_RECOMPUTE) == nb.NRT_ERR_INVALID_ARG
    assert L.nrt_set_profiling(None, 1) == nb.NRT_ERR_INVALID_ARG
    assert (nb.NRT_MODE_INCREMENTAL, nb.NRT_MODE_RECOMPUTE, nb.NRT_MODE_FULL, nb.NRT_MODE_AUTO) == (0, 1, 2, 3)
    text = open(os.path.join(ROOT, "include", "nrt.h")).read()
    assert re.search(r"NRT_MODE_INCREMENTAL\s*=\s*0,\s*NRT_MODE_RECOMPUTE\s*=\s*1,\s*NRT_MODE_FULL\s*=\s*2,\s*NRT_MODE_AUTO\s*=\s*3", text)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_model_kinds_agree_between_header_generators_and_oracle():
    """One numbering of the model kinds everywhere: the C header, the workload generators and the oracle."""
    from paper_2603_20622_amd import workloads as wl
    from oracle import rtec_oracle as orc
    text = open(os.path.join(ROOT, "include", "nrt.h")).read()
    enum = re.search(r"typedef enum \{([^}]*)\} nrt_model_kind;", text).group(1)
    header = {k: int(v) for k, v in re.findall(r"(NRT_[A-Z_]+)\s*=\s*(\d+)", enum)}
    names = {"NRT_GCN": "GCN", "NRT_SAGE_MEAN": "SAGE_MEAN", "NRT_GIN": "GIN", "NRT_GAT": "GAT", "NRT_COMMNET": "COMMNET",
             "NRT_PINSAGE": "PINSAGE", "NRT_AGNN": "AGNN", "NRT_MONET": "MONET", "NRT_GGCN": "GGCN", "NRT_RGCN": "RGCN", "NRT_RGAT": "RGAT"}
    assert set(header) == set(names)
    for c_name, py_name in names.items():
        assert header[c_name] == getattr(wl, py_name) == getattr(orc, py_name), c_name
    assert sorted(header.values()) == list(range(1, len(names) + 1))
