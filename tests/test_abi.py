"""CPU-side checks of the C ABI: the built library loads and exports every function include/freqcache.h declares,
host-side argument validation works without a GPU, and the product path never falls back to the CPU."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "freqcache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^(?:int|float\s*\*|const\s+char\s*\*)\s*(\w+)\s*\(", text, flags=re.M)
    return names


@pytest.fixture(scope="module")
def lib():
    from paper_2208_05321_amd.binding import load_library, LIB_PATH
    if not os.path.exists(LIB_PATH):
        from paper_2208_05321_amd.build import build
        build()
    return load_library()


def test_every_declared_symbol_is_exported(lib):
    from paper_2208_05321_amd.binding import EXPORTS
    names = declared_functions()
    assert len(names) >= 18 and "cache_prepare" in names and "embedding_bag_bwd_sgd" in names
    assert sorted(names) == sorted(EXPORTS)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in freqcache.h but not exported"


def test_strerror_and_profile_names(lib):
    assert lib.cache_strerror(0) == b"ok"
    assert b"cache" in lib.cache_strerror(-4)
    names = [lib.cache_profile_name(k).decode() for k in range(lib.cache_profile_count())]
    assert "miss_fill" in names and "bag_fwd" in names and "bwd_reduce" in names and all(names)


def test_host_side_validation_needs_no_gpu(lib):
    h = ctypes.c_void_p()
    fr = np.arange(10, dtype=np.int32)
    assert lib.cache_create(10, 4, 0, fr.ctypes.data, None, 0, 0, None, ctypes.byref(h)) == -1      # cache_rows = 0
    assert lib.cache_create(10, 4, 11, fr.ctypes.data, None, 0, 0, None, ctypes.byref(h)) == -1     # > num_rows
    assert lib.cache_create(10, 4, 3, None, None, 0, 0, None, ctypes.byref(h)) == -1
    assert lib.cache_create(10, 4, 3, fr.ctypes.data, None, 0, 1024, None, ctypes.byref(h)) == -1   # unknown flag
    bad = fr.copy()
    bad[0] = 1
    assert lib.cache_create(10, 4, 3, bad.ctypes.data, None, 0, 0, None, ctypes.byref(h)) == -5
    assert lib.cache_prepare(None, None, 0, None, 0, None) == -1
    assert lib.cache_flush(None) == -1 and lib.cache_destroy(None) == -1


def test_no_cpu_fallback_without_gpu():
    """Without a GPU the product must fail loudly, not compute on the CPU."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2208_05321_amd import FreqCache, FreqCacheError
    with pytest.raises(FreqCacheError) as e:
        FreqCache(10, 4, 3, np.arange(10, dtype=np.int32))
    assert e.value.name == "HIP"
    lib = __import__("paper_2208_05321_amd").load_library()
    h = ctypes.c_void_p()
    fr = np.arange(10, dtype=np.int32)
    assert lib.cache_create(10, 4, 3, fr.ctypes.data, None, 0, 0, None, ctypes.byref(h)) == -8


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2208_05321_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp", ".c")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2208_05321_amd" not in text and "freqcache" not in text
