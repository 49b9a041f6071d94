"""Host-side checks of the boundary: the shared library loads, exports every symbol the
header declares, and refuses to compute without a GPU (no CPU fallback)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    inc = os.path.join(ROOT, "include")        # every header under include/: the boundary and the test hooks
    src = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kge_[a-z_0-9]+)\s*\(", src)))


@pytest.fixture(scope="module")
def kb():
    from paper_2201_02791_amd import build, binding
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    binding.load()
    return binding


def test_header_declares_the_five_calls():
    syms = declared_symbols()
    for name in ("kge_build_partition", "kge_rgcn_forward", "kge_rgcn_backward", "kge_sample_negatives",
                 "kge_distmult_score_loss"):
        assert name in syms


def test_library_exports_every_declared_symbol(kb):
    lib = kb.load()
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(kb.EXPORTED) == declared_symbols()


def test_struct_layouts_match_the_header(kb):
    # five int32, padding, three pointers, the dropout rate, padding, its seed and step
    assert C.sizeof(kb._Layer) == 5 * 4 + 4 + 3 * 8 + 4 + 4 + 2 * 8
    assert C.sizeof(kb._LayerGrad) == 3 * 8
    assert C.sizeof(kb._PartInfo) == 6 * 8 + 8 * 4


def test_argument_errors_need_no_gpu(kb):
    lib = kb.load()
    out = C.c_void_p()
    rc = lib.kge_build_partition(None, None, None, C.c_int64(3), C.c_int32(4), C.c_int32(1), C.c_int32(1),
                                 C.c_int32(0), C.c_int32(2), C.c_int32(0), C.byref(out))
    assert rc == -1 and b"NULL" in lib.kge_last_error()
    rc = lib.kge_build_partition(None, None, None, C.c_int64(0), C.c_int32(4), C.c_int32(1), C.c_int32(2),
                                 C.c_int32(5), C.c_int32(2), C.c_int32(0), C.byref(out))
    assert rc == -1
    assert lib.kge_partition_info(None, None) == -1
    assert lib.kge_workspace_bytes(None, None, C.c_int32(1), C.c_int32(0)) == 0


def test_product_path_fails_loudly_without_a_gpu(kb):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(kb.KgeError) as e:
        kb.build_partition(np.array([0], np.int32), np.array([0], np.int32), np.array([1], np.int32), 2, 1)
    assert e.value.status == -3


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2201_02791_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|liborc|kge_oracle|orc_[a-z]", text, flags=re.M), \
                    os.path.join(dirpath, f)
