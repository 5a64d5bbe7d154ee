"""CPU-side checks of the boundary: the shared library loads and exports exactly the entry
points that include/gelo.h declares, and the Python binding mirrors them."""
import ctypes
import os
import re

from paper_2603_05035_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gelo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gelo_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_five_protocol_calls():
    names = _declared()
    for required in ("gelo_sample_mixing", "gelo_mix", "gelo_project", "gelo_unmix", "gelo_qkv_forward"):
        assert required in names


def test_library_exports_every_declared_symbol():
    assert os.path.exists(binding.LIB_PATH), "build the library first: python -m paper_2603_05035_amd.build"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name


def test_binding_mirrors_the_header():
    assert sorted(binding.SIGNATURES) == _declared()
    for name in _declared():
        if name not in ("gelo_last_error", "gelo_status_string"):
            assert callable(getattr(binding, name)), name


def test_status_strings_without_a_gpu():
    lib = binding.load_library()
    assert lib.gelo_status_string(0) == b"ok"
    assert b"reused" in lib.gelo_status_string(8)
    assert len(binding.STATUS_NAMES) == 11


def test_product_sources_do_not_reach_for_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_05035_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")) and f != "workloads.py":   # the shared input generator may mention it
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"(import|from)\s+oracle|gelo_oracle", text), f


def test_enumerators_agree_between_header_binding_and_workloads():
    """the numbers behind gelo_kind / gelo_dtype / gelo_norm_stat as the header spells them"""
    from paper_2603_05035_amd import workloads as wl
    text = open(os.path.join(ROOT, "include", "gelo.h")).read()
    values = {name: int(v) for name, v in re.findall(r"\b(GELO_[A-Z0-9_]+)\s*=\s*(\d+)", text)}
    for name in ("GELO_ORTHOGONAL", "GELO_GAUSSIAN", "GELO_CONDITIONED", "GELO_STRUCTURED", "GELO_BLOCK_ORTHOGONAL", "GELO_REFLECTOR_PRODUCT", "GELO_F32", "GELO_BF16",
                 "GELO_NORM_MEDIAN", "GELO_NORM_MEAN", "GELO_OK"):
        assert getattr(binding, name) == values[name], name
    assert (wl.KIND_ORTHOGONAL, wl.KIND_GAUSSIAN, wl.KIND_CONDITIONED, wl.KIND_STRUCTURED, wl.KIND_BLOCK_ORTHOGONAL,
            wl.KIND_REFLECTOR_PRODUCT) == (
        values["GELO_ORTHOGONAL"], values["GELO_GAUSSIAN"], values["GELO_CONDITIONED"], values["GELO_STRUCTURED"],
        values["GELO_BLOCK_ORTHOGONAL"], values["GELO_REFLECTOR_PRODUCT"])
    assert binding.STATUS_NAMES[values["GELO_ESHAPE"]] == "GELO_ESHAPE" and binding.STATUS_NAMES[values["GELO_EHIP"]] == "GELO_EHIP"
    assert int(re.search(r"#define GELO_MAX_N (\d+)", text).group(1)) == binding.GELO_MAX_N


def test_bench_refuses_more_than_one_gpu():
    """the measurement is a one-GPU figure: asking for more must end with a message, before anything touches a GPU"""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
