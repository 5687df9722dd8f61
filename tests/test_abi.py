"""The C-ABI library loads and exports every function include/rapidgnn.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rapidgnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(rg_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_three_entry_points():
    names = declared_functions()
    for must in ("rg_build_schedule", "rg_build_cache", "rg_gather_batch"):
        assert must in names


def test_library_exports_every_declared_function():
    from paper_2509_05207_amd import binding, build
    build.build(force=False)
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2509_05207_amd", "librapidgnn_hip.so"))
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared but not exported"
    assert set(binding.EXPORTS) == set(declared_functions())


def test_binding_has_the_same_names():
    from paper_2509_05207_amd import binding
    for name in declared_functions():
        if name in ("rg_schedule_destroy", "rg_cache_destroy", "rg_last_error", "rg_schedule_info",
                    "rg_cache_pair_destroy", "rg_prefetcher_destroy"):
            continue        # folded into the handle classes / error type
        assert hasattr(binding, name), name


def test_no_product_module_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_05207_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in src and "from oracle" not in src and "rapidgnn_oracle" not in src, fn
