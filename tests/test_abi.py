"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_2412_18910_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.LIB):
        build.build()
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "adaeagle.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ae_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"ae_init", "ae_ldlp", "ae_draft", "ae_verify", "ae_accept", "ae_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in adaeagle.h but not exported"
    assert set(binding.EXPORTS) == set(names)


def test_struct_layouts_match_header():
    # field order and count of the POD structs, checked against the header text
    text = open(os.path.join(ROOT, "include", "adaeagle.h")).read()
    cfg = re.search(r"typedef struct \{(.*?)\} ae_config;", text, re.S).group(1)
    cfg = re.sub(r"/\*.*?\*/", "", cfg, flags=re.S)
    names = [n.strip() for decl in cfg.split(";") for n in re.sub(r"^\s*\w+\s", "", decl.strip()).split(",") if n.strip()]
    assert names == [n for n, _ in binding.AeConfig._fields_]
    assert C.sizeof(binding.AeConfig) == 19 * 4
    assert C.sizeof(binding.AeLayerW) == 9 * 8


def test_init_rejects_bad_arguments_without_a_gpu(lib):
    h = C.c_void_p()
    assert lib.ae_init(None, None, None, C.byref(h)) == binding.AE_EINVAL
    assert b"NULL" in lib.ae_last_error(None)
    cfg = binding.AeConfig()
    w = binding.AeWeights()
    assert lib.ae_init(C.byref(cfg), C.byref(w), None, C.byref(h)) == binding.AE_EINVAL
    assert h.value is None
    assert lib.ae_version().startswith(b"adaeagle")


def test_engine_fails_loudly_when_library_is_missing(tmp_path):
    saved = binding._lib
    binding._lib = None
    try:
        with pytest.raises(RuntimeError, match="no fallback"):
            binding.load_library(str(tmp_path / "libadaeagle.so"))
    finally:
        binding._lib = saved
