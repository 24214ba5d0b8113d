"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, validates arguments before touching a GPU, and its host-only
query encoder agrees with the oracle's encoder bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_1802_06466_amd as rbe
from paper_1802_06466_amd import _build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(_build.LIB) or _build.is_stale():
        _build.build(force=True)
    return rbe.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rbe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rbe_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"rbe_load_corpus", "rbe_encode_query", "rbe_search"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in rbe.h but not exported"
    assert set(names) == set(rbe.PROTOTYPES), "binding prototypes and header disagree"


def test_binding_has_same_names():
    for n in declared_functions():
        if n in ("rbe_last_error", "rbe_n_items", "rbe_dim", "rbe_n_planes"):
            continue
        assert callable(getattr(rbe, n)), f"python binding lacks {n}"


def test_no_torch_types_in_header():
    text = open(os.path.join(ROOT, "include", "rbe.h")).read()
    assert "torch" not in re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert "at::" not in text and "#include <hip" not in text


def test_constants_match_header():
    text = open(os.path.join(ROOT, "include", "rbe.h")).read()
    for name in ("RBE_MAX_PLANES", "RBE_MAX_QUERIES", "RBE_MAX_K", "RBE_MAX_ITEMS", "RBE_MAX_LEVELS"):
        m = re.search(r"#define\s+%s\s+(\d+)" % name, text)
        assert m and int(m.group(1)) == getattr(rbe, name), name
    for name in ("RBE_COSINE", "RBE_DYADIC"):
        m = re.search(r"%s\s*=\s*1u\s*<<\s*(\d+)" % name, text)
        assert m and (1 << int(m.group(1))) == getattr(rbe, name), name
    assert ctypes.sizeof(rbe.rbe_search_stats) == 16 + 8 * 8 * 2 + 4 * 8 * 2 + 8


def test_argument_validation_needs_no_gpu(lib):
    out = ctypes.c_void_p(None)
    for args in [(0, 64, 3, 0), (10, 65, 3, 0), (10, 64, 0, 0), (10, 64, 5, 0), (10, 64, 3, 1), (2**32, 64, 3, 0)]:
        assert lib.rbe_index_create(ctypes.byref(out), *args) == rbe.RBE_EINVAL
        assert out.value is None
        assert lib.rbe_last_error()
    assert lib.rbe_search(None, None, None, 1, 1, 1, 0, 0, None, None, None) == rbe.RBE_EINVAL
    assert lib.rbe_strerror(rbe.RBE_EINVAL) == b"invalid argument"
    assert lib.rbe_strerror(0) == b"ok"
    lib.rbe_free(None)


@pytest.mark.parametrize("d,P", [(64, 1), (64, 3), (128, 4), (256, 2)])
def test_encode_query_matches_oracle_bit_for_bit(lib, d, P):
    rng = np.random.default_rng(d + P)
    for t in range(50):
        x = rng.standard_normal(d).astype(np.float32)
        if t == 0:
            x[5] = 0.0
        planes, scales = rbe.rbe_encode_query(x, P)
        o_planes, o_scales = oracle.encode(x, P)
        np.testing.assert_array_equal(planes, o_planes[:, 0])
        np.testing.assert_array_equal(scales.view(np.uint32), o_scales[:, 0].view(np.uint32))


def test_encode_query_rejects_bad_input(lib):
    with pytest.raises(rbe.RbeError):
        rbe.rbe_encode_query(np.zeros(65, np.float32), 2)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_encode_query(np.zeros(64, np.float32), 5)
    x = np.zeros(64, np.float32); x[3] = np.nan
    with pytest.raises(rbe.RbeError):
        rbe.rbe_encode_query(x, 2)


@pytest.mark.parametrize("n_tiles,ratio", [(1, 64), (2, 2), (31, 2), (64, 64), (65, 64), (977, 8), (4097, 64),
                                           (5000, 3), (300000, 64)])
def test_tile_order_is_a_bijection_with_nested_sample_prefixes(lib, n_tiles, ratio):
    to_phys = lambda t: rbe.rbe_debug_tile_to_phys(n_tiles, ratio, t)
    to_tile = lambda p: rbe.rbe_debug_phys_to_tile(n_tiles, ratio, p)
    step = max(1, n_tiles // 5000)
    tiles = sorted(set(range(0, n_tiles, step)) | {n_tiles - 1})
    phys = [to_phys(t) for t in tiles]
    assert all(0 <= p < n_tiles for p in phys) and len(set(phys)) == len(tiles)
    assert [to_tile(p) for p in phys] == tiles
    assert to_phys(0) == 0
    if n_tiles <= 5000:
        assert sorted(phys) == list(range(n_tiles))
    # number of sample levels: split while the coarsest sample still has more than 32 tiles
    top, n_ge = 0, n_tiles
    while n_ge > 32 and ratio ** (top + 1) < n_tiles and top + 1 < 8:
        top += 1
        n_ge = -(-n_tiles // ratio ** top)
    for c in range(1, top + 1):
        # the stride-r^c sample of tiles is exactly the first ceil(T / r^c) physical tiles
        size = -(-n_tiles // ratio ** c)
        probe = range(size) if size <= 3000 else list(range(0, size, size // 1000)) + [size - 1]
        assert all(to_tile(p) % ratio ** c == 0 for p in probe)
        if size < n_tiles:
            assert to_tile(size) % ratio ** c != 0
        # and within a class tiles ascend
        ts = [to_tile(p) for p in (probe if size <= 3000 else range(min(size, 200)))]
        lo = -(-n_tiles // ratio ** (c + 1)) if c < top else 0
        seg = ts[lo:] if size <= 3000 else ts[lo:200]
        assert seg == sorted(seg)


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_1802_06466_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_1802_06466_amd" not in open(os.path.join(ROOT, "oracle", f)).read()
