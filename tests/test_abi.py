"""The C-ABI library loads without a GPU and exports everything include/rsr.h declares."""
import os
import re

import paper_2603_27462_amd as rsr

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "rsr.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rsr_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared_functions() == sorted(rsr.exported_symbols)


def test_library_exports_every_declared_symbol():
    lib = rsr.load_library()
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_error_strings_without_gpu():
    assert rsr.rsr_error_string(0) == "ok"
    for code in range(1, 8):
        assert rsr.rsr_error_string(code) not in ("ok", "unknown error")
    assert rsr.rsr_error_string(99) == "unknown error"


def test_deserialize_rejects_what_it_did_not_write():
    # header checks run on the host, before any device call
    import numpy as np
    import pytest
    for blob in (np.zeros(16, np.uint8), np.zeros(4096, np.uint8),
                 np.frombuffer(b"RSRS" + bytes(200), dtype=np.uint8)):
        with pytest.raises(rsr.RsrError) as e:
            rsr.rsr_deserialize(blob)
        assert e.value.code == 1


def test_no_oracle_in_product():
    # the product never imports the oracle
    pkg = os.path.dirname(rsr.__file__)
    for root, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(root, f)).read()
                assert "import oracle" not in src and "rsr_oracle" not in src, f
