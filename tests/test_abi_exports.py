"""The C-ABI library loads without a GPU and exports every function the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe_offload.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|size_t|const char \*)\s*\*?\s*(\w+)\s*\(", text)
    return sorted(set(n for n in names if n.startswith(("moe_", "expert_cache_", "predictor_"))))


def test_header_functions_are_exported():
    from paper_2509_07379_amd import binding
    assert os.path.exists(binding.LIB_PATH), "build first: python -m paper_2509_07379_amd.build"
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = declared_functions()
    assert {"moe_prefill_layer", "moe_decode_layer", "expert_cache_prefetch", "predictor_score"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_argument_errors_without_gpu():
    from paper_2509_07379_amd import binding
    lib = binding.load()
    cfg = binding.MoeConfig(256, 128, 8, 9, 1, 8, 0, 1)  # k > E: rejected before any HIP call
    h = ctypes.c_void_p()
    assert lib.moe_create(ctypes.byref(cfg), ctypes.byref(h)) == -1
    assert b"exceeds" in lib.moe_last_error()
    assert lib.moe_workspace_bytes(ctypes.byref(cfg), 4) == 0
    ok = binding.MoeConfig(4096, 14336, 8, 2, 1, 2, 0, 1)
    assert lib.moe_workspace_bytes(ctypes.byref(ok), 2048) > 2048 * 2 * 14336 * 2
