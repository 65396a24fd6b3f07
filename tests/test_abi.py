"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the public header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2604_16402_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_16402_amd import build
        build.build(verbose=False)
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "grab.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(grab_[a-z0-9_]+)\s*\(", header))
    assert {"grab_build_buckets", "grab_load_graph", "grab_search_range", "grab_append_batch"} <= declared
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in grab.h but not exported"
    from paper_2604_16402_amd import binding
    assert declared == set(binding.EXPORTS)


def test_create_validates_arguments(lib):
    h = ctypes.c_void_p()
    assert lib.grab_create(ctypes.byref(h), 100, 0, None) == 1      # dim not a multiple of 32
    assert lib.grab_create(ctypes.byref(h), 4096, 0, None) == 1     # dim too large
    supported = [32, 64, 96, 128, 160, 192, 256, 384, 512, 640, 768, 960, 1024, 1536, 2048]
    for dim in range(32, 2049, 32):                                  # a length without kernels is refused up front
        rc = lib.grab_create(ctypes.byref(h), dim, 0, None)
        assert rc == (0 if dim in supported else 1), dim
        if rc == 0:
            lib.grab_destroy(h)
    assert lib.grab_create(ctypes.byref(h), 128, 7, None) == 1      # unknown metric
    assert lib.grab_create(None, 128, 0, None) == 1
    assert lib.grab_create(ctypes.byref(h), 128, 0, None) == 0 and h.value
    lib.grab_destroy(h)
    lib.grab_destroy(None)


def test_calls_out_of_order_and_bad_parameters():
    from paper_2604_16402_amd import binding as B
    ix = B.Index(128)
    q = np.zeros((2, 128), np.float32)
    lo = np.zeros(2, np.int32)
    with pytest.raises(B.GrabError) as e:
        ix.search_range(q, lo, lo, 10, 64)
    assert e.value.status == B.ESTATE and "graph" in str(e.value)
    with pytest.raises(B.GrabError) as e:
        ix.get_layout()
    assert e.value.status == B.ESTATE
    with pytest.raises(B.GrabError) as e:
        ix.load_graph(np.zeros((0, 4), np.uint32), np.zeros((0, 1), np.uint32))
    assert e.value.status == B.ESTATE
    for name, bad in [("search_width", 0), ("search_width", 9), ("visited_cap", 0), ("visited_cap", 1e6),
                      ("alpha", 0.0), ("alpha", 1.5), ("append_beam", 0), ("max_iter", -1), ("n_seeds", -3),
                      ("profile", 2), ("remote_mode", 2), ("n_proximal", 65), ("remote_window", 1.5)]:
        with pytest.raises(B.GrabError) as e:
            ix.set_param(name, bad)
        assert e.value.status == B.EINVAL
    ix.set_param("search_width", 4)
    ix.set_param("alpha", 1.0)
    x = np.zeros((10, 128), np.float32)
    a = np.zeros(10, np.int32)
    for n_buckets, n_cap in [(0, 10), (11, 10), (2, 9), (2000, 10)]:
        with pytest.raises(B.GrabError) as e:
            ix.build_buckets(x, a, n_buckets, n_cap)
        assert e.value.status == B.EINVAL
    with pytest.raises(ValueError):
        ix.build_buckets(np.zeros((10, 64), np.float32), a, 2)
    assert ix.sizes()["n"] == 0 and ix.sizes()["has_graph"] == 0
    ix.close()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_attribute_image_is_the_oracle_order_key(lib):
    # the two host functions need no device: compare them with the oracle's key on special values
    # and random bit patterns, and check the round trip
    from oracle import oracle as O
    from paper_2604_16402_amd import binding as B
    rng = np.random.default_rng(3)
    v = np.concatenate([np.array([0.0, -0.0, 1e-45, -1e-45, 1.0, -1.0, 0.5, np.inf, -np.inf, 3.4028235e38, -3.4028235e38],
                                 np.float32), rng.integers(-2**31, 2**31, 500).astype(np.int32).view(np.float32)])
    v = v[~np.isnan(v)]
    want = O.float_order_key(v)
    for x, k in zip(v.tolist(), want.tolist()):
        assert B.attr_image(x) == k, x
        back = B.attr_value(k)
        assert back == x and (x != 0.0 or np.signbit(np.float32(back)) == False)
