"""The C-ABI shared library loads and exports every entry point that include/cats.h
declares; host-side validation paths that never touch a GPU are exercised too."""
import ctypes
import re
from pathlib import Path

import paper_2605_11186_amd as cats

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "cats.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cats_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert declared_functions() == cats.exported_symbols()


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(str(cats.library_path()))
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_status_strings_and_kernel_name():
    assert cats.cats_strerror(cats.CATS_OK) == "ok"
    assert "max_ctx" in cats.cats_strerror(cats.CATS_ECAPACITY)
    assert "tree" in cats.cats_strerror(cats.CATS_ESTATE)
    assert cats.cats_gemm_kernel_name() == "cats_gemm_skinny_bf16"


def test_struct_layouts_match_header_sizes():
    # 8 int32 + 2 float + 1 int32; 9 pointers; 2 pointers; 1 + 17 + 17 + 1 + 1 int32
    assert ctypes.sizeof(cats.ModelDesc) == 44
    assert ctypes.sizeof(cats.LayerWeights) == 72
    assert ctypes.sizeof(cats.KVLayer) == 16
    assert ctypes.sizeof(cats.AcceptResult) == 4 * (1 + 17 + 17 + 1 + 1)


def test_null_arguments_are_rejected_before_any_device_work():
    lib = cats.library()
    assert lib.cats_create(None, None) == cats.CATS_EINVAL
    assert lib.cats_destroy(None) == cats.CATS_EINVAL
    assert lib.cats_set_tree(None, None, None) == cats.CATS_EINVAL
    assert lib.cats_verify_layer(None, None, None, None, 0, None) == cats.CATS_EINVAL
    assert lib.cats_tree_attention(None, None, None, 0, None, None) == cats.CATS_EINVAL
    bad = cats.ModelDesc(2, 250, 4, 64, 688, 1024, 320, 128, 1e-6, 10000.0, 0)   # hidden % 64 != 0
    handle = ctypes.c_void_p()
    assert lib.cats_create(ctypes.byref(bad), ctypes.byref(handle)) == cats.CATS_EINVAL
