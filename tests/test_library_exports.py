"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol that include/kge.h declares,
and fails loudly (no fallback) when there is no device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kge.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kge_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2004_08532_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = _declared_functions()
    assert "kge_create" in names and "kge_train_step" in names and "kge_score" in names and "kge_destroy" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_binding_struct_matches_header_layout():
    from paper_2004_08532_amd import binding
    # int32 x2, int64 x2, int32 x7 (5 + gemm_input + adagrad_mode), float x2, int32
    assert ctypes.sizeof(binding.kge_config) == 8 + 16 + 7 * 4 + 8 + 4 + 0 or ctypes.sizeof(binding.kge_config) % 8 == 0
    fields = [f[0] for f in binding.kge_config._fields_]
    header = open(HEADER).read()
    body = header[header.index("typedef struct {"):header.index("} kge_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    declared = re.findall(r"\b(?:int32_t|int64_t|float)\s+(\w+)\s*;", body)
    assert fields == declared


def test_no_device_means_an_error_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import paper_2004_08532_amd as kge
    with pytest.raises(kge.KgeError) as e:
        kge.KgeContext("transe_l2", 100, 10, 64)
    assert e.value.code == kge.KGE_ERR_DEVICE


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2004_08532_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "kge_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2004_08532_amd" not in text and "libkge.so" not in text, f
