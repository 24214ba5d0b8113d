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


HEADERS = ("rbe.h", "rbe_debug.h")


def declared_functions(headers=HEADERS):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(rbe_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"rbe_load_corpus", "rbe_encode_query", "rbe_search", "rbe_workspace_bytes", "rbe_set_workspace",
            "rbe_index_create_in", "rbe_search_static"} <= set(declared_functions(("rbe.h",)))
    assert not [n for n in declared_functions(("rbe.h",)) if n.startswith("rbe_debug_")], "test hooks belong in rbe_debug.h"
    for n in names:
        assert hasattr(lib, n), f"{n} declared in a header but not exported"
    assert set(names) == set(rbe.PROTOTYPES), "binding prototypes and header disagree"


def test_binding_has_same_names():
    for n in declared_functions():
        if n in ("rbe_last_error", "rbe_n_items", "rbe_dim", "rbe_n_planes"):
            continue
        assert callable(getattr(rbe, n)), f"python binding lacks {n}"


def test_no_torch_types_in_header():
    for h in HEADERS:
        text = open(os.path.join(ROOT, "include", h)).read()
        assert "torch" not in re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        assert "at::" not in text and "#include <hip" not in text


def test_constants_match_header():
    text = open(os.path.join(ROOT, "include", "rbe.h")).read()
    for name in ("RBE_MAX_PLANES", "RBE_MAX_QUERIES", "RBE_MAX_K", "RBE_MAX_ITEMS", "RBE_MAX_LEVELS"):
        m = re.search(r"#define\s+%s\s+(\d+)" % name, text)
        assert m and int(m.group(1)) == getattr(rbe, name), name
    m = re.search(r"#define\s+RBE_STATIC_SCRATCH_BYTES\s+(\d+)u", text)
    assert m and int(m.group(1)) == rbe.RBE_STATIC_SCRATCH_BYTES
    for name in ("RBE_BORROW", "RBE_COSINE", "RBE_DYADIC"):
        m = re.search(r"%s\s*=\s*1u\s*<<\s*(\d+)" % name, text)
        assert m and (1 << int(m.group(1))) == getattr(rbe, name), name
    assert ctypes.sizeof(rbe.rbe_search_stats) == 16 + 8 * 8 * 2 + 4 * 8 * 2 + 8 + 4 * 8 + 4 + 4 * 8 + 4
    for code, name in rbe.KERNEL_NAMES.items():
        assert re.search(r"RBE_KERNEL_[A-Z0-9_]+\s*=\s*%d\b" % code, text), name


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


def test_caller_owned_memory_entry_points_validate_without_a_gpu(lib):
    """rbe_index_bytes is a pure host function; the other calls reject bad arguments before any GPU work."""
    def expect(N, d, P, flags):
        tiles = -(-N // 1024)
        W = d // 64
        dyadic, cosine = bool(flags & rbe.RBE_DYADIC), bool(flags & rbe.RBE_COSINE)
        S = (1 if cosine else 0) if dyadic else P
        up = lambda b: -(-b // 256) * 256
        total = up(tiles * 1024 * (8 * W * P + 4 * S))
        total += up(2 * tiles * 4 * 4 if S else 0)                      # two floats per row of 256 items
        nw = 0 if (dyadic or P < 2) else (4 if P - 1 == 3 else P - 1)   # one-byte scale copies, a word per 4 items and array
        nw += 1 if (nw and P >= 3) else 0                               # ... and of the last array, for the two-stage scan
        total += up(tiles * 256 * nw * 4)
        return total + 256
    for N, d, P, flags in [(1, 64, 1, 0), (1_000_000_000, 64, 3, 0), (100_000_000, 128, 4, 0), (1025, 256, 2, 0),
                           (1_212_153_856, 64, 2, rbe.RBE_DYADIC | rbe.RBE_COSINE), (5000, 128, 3, rbe.RBE_DYADIC),
                           (5000, 64, 3, rbe.RBE_COSINE | rbe.RBE_BORROW)]:
        assert rbe.rbe_index_bytes(N, d, P, flags) == expect(N, d, P, flags), (N, d, P, flags)
    assert rbe.rbe_index_bytes(0, 64, 3) == 0 and rbe.rbe_index_bytes(10, 65, 3) == 0 and rbe.rbe_index_bytes(10, 64, 5) == 0
    assert rbe.rbe_index_bytes(10, 256, 2, rbe.RBE_DYADIC) == 0
    assert rbe.rbe_index_bytes(10, 64, 3, 0, 1) == 0 and rbe.rbe_index_bytes(10, 64, 3, 0, 8) == rbe.rbe_index_bytes(10, 64, 3)
    out = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)
    assert lib.rbe_index_create_in(ctypes.byref(out), 10, 64, 3, 0, 0, fake, 1 << 20) == rbe.RBE_EINVAL      # RBE_BORROW missing
    assert lib.rbe_index_create_in(ctypes.byref(out), 10, 64, 3, rbe.RBE_BORROW, 0, None, 1 << 20) == rbe.RBE_EINVAL
    assert lib.rbe_index_create_in(ctypes.byref(out), 10, 65, 3, rbe.RBE_BORROW, 0, fake, 1 << 20) == rbe.RBE_EINVAL
    assert out.value is None
    assert lib.rbe_workspace_bytes(None, 1, 10, 0) == 0
    assert lib.rbe_set_workspace(None, None, 0) == rbe.RBE_EINVAL
    assert lib.rbe_search_static(None, None, None, 1, 1, 1, 0, 0, None, None, None) == rbe.RBE_EINVAL
    assert lib.rbe_debug_index_info(None, None) == rbe.RBE_EINVAL


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


# ------------------------------------------------------------------ host logic: refinement plan of the exact mode
@pytest.mark.parametrize("n_items,ratio,cap,k", [
    (1_000_000_000, 64, 131072, 1000), (1_000_000_000, 64, 131072, 4000), (10_000_000, 64, 131072, 1000),
    (1_000_000, 64, 131072, 100), (100_000_000, 8, 6144, 100), (5000, 64, 131072, 100), (1, 64, 131072, 1),
    (4_294_966_272, 64, 131072, 4096), (1_212_153_856, 64, 131072, 1000), (3_000_000, 2, 8192, 50)])
def test_exact_plan_partitions_the_corpus(lib, n_items, ratio, cap, k):
    """Levels are contiguous physical ranges, each starting where the previous one ended, together
    covering every tile exactly once; the first (threshold-free) level fits the candidate list;
    each level is a nested strided sample: its end is ceil(T / ratio^c) for decreasing c."""
    T = -(-n_items // 1024)
    plan = rbe.rbe_debug_exact_plan(n_items, ratio, cap, k)
    if not plan:                       # nothing fits: the library uses its bounded-segment path
        assert T * 1024 > cap
        return
    assert plan[0][0] == 0 and plan[-1][1] == T
    for (b0, e0), (b1, e1) in zip(plan, plan[1:]):
        assert e0 == b1 and b1 < e1
    assert plan[0][1] * 1024 <= cap
    c = len(plan) - 1
    for i, (_, e) in enumerate(plan):
        assert e == -(-T // ratio ** (c - i))
    # the start level holds at least 4k items whenever a coarser choice would not
    if len(plan) > 1:
        assert plan[0][1] * 1024 >= min(4 * k, cap // 2) or plan[0][1] * ratio * 1024 > cap


def test_exact_plan_levels_are_strided_samples(lib):
    """Physical prefix [0, end) of level i is exactly the set of logical tiles that are multiples of
    ratio^(c-i): checked through the tile-order functions on a corpus of 70,001 tiles."""
    T, ratio = 70_001, 8
    plan = rbe.rbe_debug_exact_plan(T * 1024, ratio, 32768, 100)
    assert len(plan) >= 3
    c = len(plan) - 1
    for i, (b, e) in enumerate(plan[:-1]):
        step = ratio ** (c - i)
        got = sorted(rbe.rbe_debug_phys_to_tile(T, ratio, p) for p in range(0, e))
        assert got == list(range(0, T, step))


# ------------------------------------------------------------------ host logic: query operands of the matrix-core scan
def _halves_to_float(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _emulated_contraction(A, start, q, bits, parts, copy=0):
    """What the kernel's MFMAs add up for query q against one plane of item bits: lane group g takes bits
    10 + t and 26 + t of each 32-bit part rotated left by 4g, as halves worth 0 or val_t."""
    val = np.array([2.0 ** -14, 2.0 ** -13, 2.0 ** -11, 2.0 ** -7])
    got = 0.0
    for part in range(parts):
        b32 = bits[32 * part: 32 * part + 32]
        for g in range(4):
            for e in range(8):
                t, h = e >> 1, e & 1
                got += A[q // 16, copy, part, 16 * g + q % 16, e] * (b32[(10 + 16 * h + t - 4 * g) % 32] * val[t])
    return got


@pytest.mark.parametrize("dim,P,Pq,Q,dyadic", [(64, 3, 3, 16, False), (64, 2, 3, 5, True), (128, 4, 4, 33, False),
                                                (128, 3, 4, 20, True), (64, 1, 1, 1, False)])
def test_matrix_core_operands_reproduce_the_score(lib, dim, P, Pq, Q, dyadic):
    """Emulates the kernel's side of the contract on the CPU: the sum over lanes, parts and plane copies
    plus the start value must equal qhat . rho (times the item-plane weights in the dyadic case) --
    exactly for dyadic queries, within the reported filter margin for general scales."""
    rng = np.random.default_rng(dim + P + Q)
    W = dim // 64
    qp = rng.integers(0, 2**64, size=(Q, Pq, W), dtype=np.uint64)
    qs = None if dyadic else rng.uniform(0.05, 1.0, size=(Q, Pq)).astype(np.float32)
    halves, unscale, start, margin = rbe.rbe_debug_batch_operands(qp, qs, dim, P, dyadic)
    tiles, copies, parts = halves.shape[:3]
    assert (tiles, copies, parts) == ((Q + 15) // 16, P if dyadic else 1, 2 * W)
    assert (margin == 0.0) if dyadic else (margin > 0.0)
    A = _halves_to_float(halves)                                  # [tile][copy][part][lane][8]
    coef = np.array([2.0 ** -i for i in range(Pq)]) if dyadic else None
    n_items = 7
    item_planes = rng.integers(0, 2**64, size=(P, n_items, W), dtype=np.uint64)
    for q in range(Q):
        c = coef if dyadic else qs[q].astype(np.float64)
        qbits = ((qp[q][:, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64)   # [Pq][W][64]
        qhat = (c[:, None, None] * (2 * qbits - 1)).sum(axis=0).reshape(dim)
        for z in range(n_items):
            want_all, got_all = 0.0, float(start[q])
            for j in range(P):
                word_bits = ((item_planes[j, z][:, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.int64).reshape(dim)
                want = float(qhat @ (2 * word_bits - 1))
                if dyadic:
                    want_all += 2.0 ** -j * want
                    got_all += _emulated_contraction(A, start, q, word_bits, parts, copy=j)
                else:
                    got = (float(start[q]) + _emulated_contraction(A, start, q, word_bits, parts)) * float(unscale[q])
                    assert abs(got - want) <= margin * float(unscale[q]), (q, z, j, got, want)
            if dyadic:
                assert got_all * float(unscale[q]) == want_all, (q, z, got_all, want_all)


def test_matrix_core_operands_stay_in_half_range(lib):
    """2 v / val_t is below 2^15 and the scaled query's largest component is at least 0.5: no
    overflow to infinity, the halves are normal numbers or zero (never subnormal: the margin must not
    depend on how the matrix cores treat those)."""
    rng = np.random.default_rng(5)
    qp = rng.integers(0, 2**64, size=(64, 4, 2), dtype=np.uint64)
    qs = rng.uniform(1e-3, 50.0, size=(64, 4)).astype(np.float32)
    halves, unscale, start, _ = rbe.rbe_debug_batch_operands(qp, qs, 128, 4, False)
    A = _halves_to_float(halves)
    assert np.isfinite(A).all() and np.abs(A).max() < 2.0 ** 15
    assert (np.abs(A).reshape(4, -1).max(axis=1) >= 2.0 ** 7).all()
    assert ((A == 0) | (np.abs(A) >= 2.0 ** -14)).all()
    assert np.isfinite(start).all() and (unscale > 0).all()
    lg = np.log2(unscale.astype(np.float64))
    assert np.array_equal(lg, np.round(lg))       # powers of two


# ------------------------------------------------------------------ compiled code: wave-wide steps stay wave-wide
def test_scan_kernels_have_no_lane_peeling_loops():
    """Compiles the scan units to gfx950 assembly (no GPU needed) and checks that no kernel with
    wave-wide survivor staging contains a loop that removes lanes from the execution mask: such a
    loop once made the two halves of a wave run their ballots and flushes separately and lose
    entries.  Kernels whose per-lane loops are intended are listed in the checker."""
    import check_isa
    assert check_isa.main() == 0


@pytest.mark.parametrize("kind", ["binary", "fp32", "fp32_wide_range"])
def test_matrix_core_filter_operands_stay_within_their_margin(lib, kind):
    """General scales: the emulated contraction may differ from q . rho by at most the margin the host
    reports (per unit of item scale), and the margin is a small fraction of the query's mass -- otherwise
    the filter would pass far more than the survivors.  fp32 queries (hybrid scoring) included, also with
    components so small that their halves would be subnormal (those are dropped and counted as lost)."""
    rng = np.random.default_rng(321)
    dim, P, Pq, Q = 128, 3, 4, 19
    W = dim // 64
    if kind == "binary":
        qp = rng.integers(0, 2**64, size=(Q, Pq, W), dtype=np.uint64)
        qs = rng.uniform(0.01, 3.0, size=(Q, Pq)).astype(np.float32)
        halves, unscale, start, margin = rbe.rbe_debug_batch_operands(qp, qs, dim, P, False)
        qbits = ((qp[:, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64)
        qhat = (qs.astype(np.float64)[:, :, None, None] * (2 * qbits - 1)).sum(axis=1).reshape(Q, dim)
    else:
        qf = rng.standard_normal((Q, dim)).astype(np.float32)
        if kind == "fp32_wide_range":
            qf *= (2.0 ** rng.integers(-40, 1, size=(Q, dim))).astype(np.float32)
        halves, unscale, start, margin = rbe.rbe_debug_batch_operands(None, None, dim, P, False, q_float=qf)
        qhat = qf.astype(np.float64)
    assert halves.shape[:3] == ((Q + 15) // 16, 1, 2 * W) and margin > 0
    A = _halves_to_float(halves)
    assert ((A == 0) | (np.abs(A) >= 2.0 ** -14)).all()
    worst = 0.0
    for q in range(Q):
        v = qhat[q] / float(unscale[q])                  # the scaled query the operands describe
        assert 0.5 <= np.abs(v).max() < 1.0
        assert margin <= 2.0 ** -9 * np.abs(v).sum() + 2.0 ** -9       # a few 1e-4 of the query's mass
        for _ in range(40):
            bits = rng.integers(0, 2, size=dim)
            got = float(start[q]) + _emulated_contraction(A, start, q, bits, 2 * W)
            worst = max(worst, abs(got - float(v @ (2 * bits - 1))))
    assert worst <= margin, (worst, margin)
    assert worst > 0                                     # the halves really are roundings


@pytest.mark.parametrize("kind", ["binary", "fp32"])
def test_matrix_core_filter_at_the_margin_never_drops_a_survivor(lib, kind):
    """Adversarial case for the matrix-core filter (general scales).  The contraction is linear in the item bits,
    so per dimension its coefficient can be read off, and the item plane that makes (contraction - true value) as
    negative as possible can be written down: the filter then under-estimates by nearly the whole margin.  Such
    planes in positions 0 .. P-2, the plane that attains the query's mass in the last position, the row's largest
    last scale on that item, and a threshold EQUAL to the item's own score: the first look (last plane left out,
    row-wide threshold in fp32 as the kernel forms it) and the second look must both let the pair through."""
    rng = np.random.default_rng(77)
    dim, P, Pq, Q = 64, 3, 3, 16
    W = dim // 64
    if kind == "binary":
        qp = rng.integers(0, 2**64, size=(Q, Pq, W), dtype=np.uint64)
        qs = rng.uniform(0.01, 3.0, size=(Q, Pq)).astype(np.float32)
        halves, unscale, start, margin = rbe.rbe_debug_batch_operands(qp, qs, dim, P, False)
        qbits = ((qp[:, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64)
        qhat = (qs.astype(np.float64)[:, :, None, None] * (2 * qbits - 1)).sum(axis=1).reshape(Q, dim)
    else:
        qf = rng.standard_normal((Q, dim)).astype(np.float32)
        halves, unscale, start, margin = rbe.rbe_debug_batch_operands(None, None, dim, P, False, q_float=qf)
        qhat = qf.astype(np.float64)
    A = _halves_to_float(halves)
    f32 = np.float32
    tight = []
    for q in range(Q):
        v = qhat[q] / float(unscale[q])
        zero = float(start[q]) + _emulated_contraction(A, start, q, np.zeros(dim, dtype=np.int64), 2 * W)
        coef = np.array([float(start[q]) + _emulated_contraction(A, start, q, np.eye(dim, dtype=np.int64)[i], 2 * W) - zero
                         for i in range(dim)])
        # contraction(b) - true(b) = (zero + sum v) + sum_d (coef_d - 2 v_d) b_d : most negative with b_d = [coef_d < 2 v_d]
        low = (coef < 2 * v).astype(np.int64)
        worst_under = (zero + v.sum()) + ((coef - 2 * v) * low).sum()
        assert -margin <= worst_under <= 0
        tight.append(-worst_under / margin)
        best_last = (v > 0).astype(np.int64)                      # attains sum_d |v_d|
        mass = np.abs(v).sum()
        qmass = f32(mass * (1 + 2.0 ** -20)); qmass = np.nextafter(qmass, f32(np.inf)) if float(qmass) < mass * (1 + 2.0 ** -20) else qmass
        a = np.array([0.11, 0.052, 0.027], dtype=f32)            # decaying scales, the last one the row's largest
        amax, smax = a[P - 1], f32(float(a.astype(np.float64).sum()) * (1 + 1e-6))
        D = [f32(zero + (coef * low).sum())] * (P - 1)            # what the MFMAs deliver for the adversarial planes
        DL = f32(zero + (coef * best_last).sum())
        true = sum(float(a[j]) * float(v @ (2 * low - 1)) for j in range(P - 1)) + float(a[P - 1]) * mass
        taus = f32(true)                                          # threshold = the pair's own score (scaled domain)
        row_tau = f32(taus - f32(1.000001) * f32(np.float64(amax) * np.float64(qmass) + np.float64(f32(margin)) * np.float64(smax)))
        first = f32(0.0)
        for j in range(P - 1):
            first = f32(np.float64(a[j]) * np.float64(D[j]) + np.float64(first))      # one rounding per fused multiply-add
        assert first >= row_tau, (q, float(first), float(row_tau))
        asum = f32(f32(a[P - 1] + a[0]) + a[1])
        second = f32(f32(np.float64(a[P - 1]) * np.float64(DL) + np.float64(first)) + f32(f32(margin) * asum))
        assert second >= taus, (q, float(second), float(taus))
        # and it is a near miss: without the slack the first look would have dropped the pair
        assert first < f32(taus - f32(np.float64(amax) * np.float64(qmass)) * f32(0.999)) or -worst_under < 0.02 * margin
    assert max(tight) > 0.3, tight          # the adversarial plane comes within a factor of the margin: the bound is not slack by orders


# ------------------------------------------------------------------ host logic: eight-bit integer operands of the batch scan
K_ACC = 12582912.0          # 1.5 * 2^23: the float whose bit pattern the integer accumulators start from


def _i8_operand_view(ops, q, dim):
    """(T [dim], stored [dim], odd [dim]) of query q from the operand bytes, through the documented placement:
    byte 4t + m of lane (g, q % 16) is dimension 64 part + 32 (t // 2) + 8 m + 2 g + (t % 2)."""
    T = np.zeros(dim, dtype=np.int64); stored = np.zeros(dim, dtype=np.int64); odd = np.zeros(dim, dtype=bool)
    for part in range(dim // 64):
        for g in range(4):
            for t in range(4):
                for m in range(4):
                    d = 64 * part + 32 * (t // 2) + 8 * m + 2 * g + (t % 2)
                    v = int(ops[q // 16, part, 16 * g + q % 16, 4 * t + m])
                    stored[d] = v; odd[d] = bool(t % 2); T[d] = -2 * v if t % 2 else v
    return T, stored, odd


def _i8_accumulator(start_q, stored, odd, bits):
    """The accumulator of v_mfma_i32_16x16x64_i8 read as a float: it starts at the bit pattern of start_q and adds
    stored_d times the item byte (64 where an even-slot bit is set, -128 where an odd-slot bit is set)."""
    acc = int(np.float32(start_q).view(np.int32)) + int((stored * np.where(odd, -128, 64) * bits).sum())
    return np.array([acc], dtype=np.int32).view(np.float32)[0]


@pytest.mark.parametrize("dim,Pq,Q", [(64, 3, 16), (128, 4, 33), (64, 1, 3), (64, 0, 5), (128, 0, 17)])
def test_integer_operands_contract_to_the_rounded_query(lib, dim, Pq, Q):
    """The integer contraction, emulated from the operand bytes alone, equals 1.5 2^23 + 32 sum_d T_d rho_d for
    every plane tried; T is qhat rounded to integers times a power of two, |T| <= 126 (odd slots even); and the
    value is within the margin of qhat . rho in the filter's units."""
    rng = np.random.default_rng(dim + Pq)
    W = dim // 64
    if Pq == 0:         # fp32 queries (hybrid scoring): the query itself takes the place of qhat
        qf = rng.standard_normal((Q, dim)).astype(np.float32)
        qf[0] *= np.float32(2.0 ** -40); qf[1] *= np.float32(2.0 ** 30)
        ops, unscale, start, mass, margin = rbe.rbe_debug_batch_operands_i8(None, None, dim, q_float=qf)
        qhat = qf.astype(np.float64)
    else:
        qp = rng.integers(0, 2**64, size=(Q, Pq, W), dtype=np.uint64)
        qs = rng.uniform(0.01, 3.0, size=(Q, Pq)).astype(np.float32)
        qs[0] *= np.float32(2.0 ** -40); qs[1 % Q] *= np.float32(2.0 ** 30)       # the unit follows the query's size
        ops, unscale, start, mass, margin = rbe.rbe_debug_batch_operands_i8(qp, qs, dim)
        qbits = ((qp[:, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64)
        qhat = (qs.astype(np.float64)[:, :, None, None] * (2 * qbits - 1)).sum(axis=1).reshape(Q, dim)
    lg = np.log2(unscale.astype(np.float64))
    assert np.array_equal(lg, np.round(lg))
    for q in range(Q):
        T, stored, odd = _i8_operand_view(ops, q, dim)
        unit = float(unscale[q])
        assert np.abs(stored).max() <= 126 and np.abs(T).max() <= 126 and np.abs(T).max() >= 32
        assert np.abs(qhat[q] / (32 * unit) - T).max() <= 1.0 and np.abs(qhat[q] / (32 * unit) - T)[~odd].max() <= 0.5
        assert float(start[q]) == K_ACC - 32 * T.sum()
        assert np.abs(qhat[q]).sum() / unit <= float(mass[q]) <= np.abs(qhat[q]).sum() / unit * (1 + 2.0 ** -18)
        lost = np.abs(qhat[q] / unit - 32 * T).sum()
        assert lost + 4 <= margin
        for trial in range(6):
            bits = rng.integers(0, 2, size=dim) if trial else (T * 32 < qhat[q] / unit).astype(np.int64)
            rho = 2 * bits - 1
            f = 0.0
            for part in range(W):        # one instruction per 64-dimension part, chained through the accumulator
                sl = slice(64 * part, 64 * part + 64)
                f = _i8_accumulator(start[q] if part == 0 else f, stored[sl], odd[sl], bits[sl])
            assert float(f) == K_ACC + 32 * int((T * rho).sum())
            assert abs((float(f) - K_ACC) - float(qhat[q] @ rho) / unit) <= lost * (1 + 1e-12)


@pytest.mark.parametrize("exact_query", [False, True])
def test_integer_filter_at_the_margin_never_drops_a_survivor(lib, exact_query):
    """Adversarial case for the integer filter.  The item plane that makes (contraction - true value) as negative
    as possible is rho_d = -sign(32 T_d - qhat_d / unit); with such planes in positions 0 .. P-2, the plane that
    attains the query's mass last, and a threshold EQUAL to the pair's own score, the first look (row-wide
    threshold, fp32 steps as the kernel takes them: the start constant leaves through a multiply-add with the
    scale sum) and the second look must both let the pair through.  exact_query: coefficients the integers hold
    exactly, so that the margin is the arithmetic allowance alone and the multiply-adds' rounding is what is tested,
    over scale triples of very different sizes."""
    rng = np.random.default_rng(99 if exact_query else 98)
    dim, P, Pq, Q = 64, 3, 3, 16
    f32, f64 = np.float32, np.float64
    qp = rng.integers(0, 2**64, size=(Q, Pq, 1), dtype=np.uint64)
    if exact_query:
        qs = np.tile(np.array([64, 32, 16], dtype=np.float32) * np.float32(2.0 ** -9), (Q, 1))    # qhat / 2^-9 in {+-16 .. +-112}, even
    else:
        qs = rng.uniform(0.01, 3.0, size=(Q, Pq)).astype(np.float32)
    ops, unscale, start, mass, margin = rbe.rbe_debug_batch_operands_i8(qp, qs, dim)
    qbits = ((qp[:, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64)
    qhat = (qs.astype(np.float64)[:, :, None, None] * (2 * qbits - 1)).sum(axis=1).reshape(Q, dim)
    worst_seen = 0.0
    for q in range(Q):
        T, stored, odd = _i8_operand_view(ops, q, dim)
        unit = float(unscale[q])
        v = qhat[q] / unit
        if exact_query:
            assert np.array_equal(32 * T, v)
        low = np.where(32 * T - v > 0, 0, 1)                                          # rho = -sign(32 T - v); ties: +1
        under = float(((32 * T - v) * (2 * low - 1)).sum())
        assert -margin <= under <= 0
        best_last = (v > 0).astype(np.int64)
        fa = _i8_accumulator(start[q], stored, odd, low)
        fl = _i8_accumulator(start[q], stored, odd, best_last)
        for trial in range(40):
            a = (rng.uniform(0.02, 1.0, size=P) * 10.0 ** rng.uniform(-6, 6) * np.array([1.0, 10.0 ** rng.uniform(-4, 1), 10.0 ** rng.uniform(-6, 1)])).astype(f32)
            amax = a[P - 1]
            smax = f32(float(a.astype(f64).sum()) * (1 + 1e-6))
            true = sum(float(a[j]) * float(v @ (2 * low - 1)) for j in range(P - 1)) + float(a[P - 1]) * float(v @ (2 * best_last - 1))
            taus = f32(true)
            row_tau = f32(taus - f32(1.000001) * f32(f64(amax) * f64(mass[q]) + f64(f32(margin)) * f64(smax)))
            asum_f = f32(a[0] + a[1])
            first = f32(f64(-K_ACC) * f64(asum_f))                                   # fma(-K, asum, 0)
            for j in range(P - 1):
                first = f32(f64(a[j]) * f64(fa) + f64(first))
            assert first >= row_tau, (q, trial, float(first), float(row_tau))
            # the constant is gone, up to the allowance of 4 units per unit of scale sum
            ideal = sum(float(a[j]) * (float(fa) - K_ACC) for j in range(P - 1))
            worst_seen = max(worst_seen, abs(float(first) - ideal) / float(a.astype(f64).sum()))
            asum = f32(f32(a[P - 1] + a[0]) + a[1])
            sofar = f32(f64(-K_ACC) * f64(a[P - 1]) + f64(first))
            second = f32(f32(f64(a[P - 1]) * f64(fl) + f64(sofar)) + f32(f32(margin) * asum))
            assert second >= taus, (q, trial, float(second), float(taus))
            ideal2 = ideal + float(a[P - 1]) * (float(fl) - K_ACC)
            worst_seen = max(worst_seen, abs(float(f32(f64(a[P - 1]) * f64(fl) + f64(sofar))) - ideal2) / float(a.astype(f64).sum()))
    assert worst_seen <= 3.0, worst_seen        # what the multiply-adds lose stays inside the allowance of 4
    if exact_query:
        assert margin < 4.5                      # nothing but the arithmetic allowances (multiply-adds, XOR/popcount score)


@pytest.mark.parametrize("dim,P,Pq,Q", [(64, 2, 3, 16), (128, 3, 4, 19), (64, 4, 3, 5), (128, 2, 1, 33), (64, 3, 3, 1)])
def test_integer_operands_of_the_dyadic_modes_contract_to_the_exact_score(lib, dim, P, Pq, Q):
    """Dyadic index: the integer contraction over ALL item planes, emulated from the operand bytes alone (one copy of
    the query operand per item plane, every plane adding into one accumulator that starts at `start`), read as a
    float and freed of 1.5 2^23, times unscale, IS the oracle's score with the weights 2^-i, 2^-j -- exactly; `mass`
    is the most the last plane can add to an accumulator that holds the start value; every byte fits."""
    rng = np.random.default_rng(10 * dim + 3 * P + Pq)
    W = dim // 64
    N = 40
    qp = rng.integers(0, 2**64, size=(Q, Pq, W), dtype=np.uint64)
    planes = rng.integers(0, 2**64, size=(P, N, W), dtype=np.uint64)
    ops, unscale, start, mass = rbe.rbe_debug_batch_operands_i8_dyadic(qp, dim, P)
    assert np.abs(ops.astype(np.int64)).max() <= 127
    qs = np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32)
    scales = np.tile(np.array([2.0 ** -j for j in range(P)], dtype=np.float32)[:, None], (1, N))
    item_bits = ((planes[:, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.int64).reshape(P, N, dim)
    for q in range(Q):
        want = oracle.scores(planes, scales, qp[q], qs)
        views = [_i8_operand_view(ops[:, j], q, dim) for j in range(P)]
        assert np.all(unscale[q] == np.float32(2.0 ** -(P + Pq + 4)))
        sum_all = sum(int(v[0].sum()) for v in views)
        assert float(start[q]) == K_ACC - 32 * sum_all
        for z in range(N):
            acc = int(np.float32(start[q]).view(np.int32))
            for j in range(P):
                T, stored, odd = views[j]
                acc += int((stored * np.where(odd, -128, 64) * item_bits[j, z]).sum())
            got = (float(np.array([acc], dtype=np.int32).view(np.float32)[0]) - K_ACC) * float(unscale[q])
            assert got == float(want[z]), (q, z, got, float(want[z]))
        # the last plane's copy: with the start value in place it adds 64 sum over its set bits, at most mass
        T_last = views[P - 1][0]
        assert float(mass[q]) == 32 * (int(np.abs(T_last).sum()) + int(T_last.sum()))
        assert np.all(T_last % 2 == 0) and np.all(np.abs(T_last) < 2 ** (Pq + 1))


def test_integer_operands_of_the_dyadic_modes_are_refused_when_they_do_not_fit(lib):
    qp = np.zeros((3, 4, 1), dtype=np.uint64)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_debug_batch_operands_i8_dyadic(qp, 64, 4)          # 2 * 15 * 8 = 240


def test_lean_first_look_with_scale_copies_never_drops_a_survivor(lib):
    """The matrix-core scan's lean stream forms its first look with the one-byte copies h_j of the scales of planes
    0 .. P-2 and lowers the row's threshold by the most the copies can be off:
        hs = 1.016 smax + floor,  off = 0.015875 hs + floor,
        row_tau = tau - 1.000001 (amax mass + margin hs + off (mass + margin)),
    floor the sum of the arrays' smallest codes.  With the planes that make the integer contraction fall short of
    the true value most, the last plane attaining the query's mass, scales spread over many binades (zeros and values
    far below the smallest code included) and a threshold equal to the pair's own score, the first look -- fp32
    steps as the kernel takes them -- lets every pair through."""
    rng = np.random.default_rng(321)
    dim, P, Pq, Q, N = 64, 3, 3, 16, 600
    f32, f64 = np.float32, np.float64
    qp = rng.integers(0, 2**64, size=(Q, Pq, 1), dtype=np.uint64)
    qs = rng.uniform(0.01, 3.0, size=(Q, Pq)).astype(np.float32)
    ops, unscale, start, mass, margin = rbe.rbe_debug_batch_operands_i8(qp, qs, dim)
    qbits = ((qp[:, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64)
    qhat = (qs.astype(np.float64)[:, :, None, None] * (2 * qbits - 1)).sum(axis=1).reshape(Q, dim)
    scales = (rng.uniform(0.02, 1.0, size=(P, N)) * 10.0 ** rng.uniform(-9, 0, size=(P, N))).astype(f32)
    scales[:, :20] = 0.0
    scales[0, 20:60] = f32(0.97)
    scales[1, 40:80] = f32(0.5)
    # items whose copies read as low as copies can (scales just under the midpoint of two codes) and whose last scale
    # is the row's largest: with planes that agree with the query, nothing but the allowance for the copies lets them pass
    under = np.arange(N) % 5 == 0
    for j in range(P - 1):
        m = 1.0 + (rng.integers(0, 32, size=N) + 0.49) / 32.0
        scales[j, under] = (m * 2.0 ** rng.integers(-3, 0, size=N)).astype(f32)[under]
    scales[P - 1, under] = f32(0.25)
    scales[P - 1, ~under] = np.minimum(scales[P - 1, ~under], f32(0.25))
    h = np.zeros((P - 1, N)); floor = 0.0
    for j in range(P - 1):
        h[j], base = _scale_copy_codec(scales[j])
        floor += 2.0 ** (base - 127)
    h = h.astype(f32)
    floor = f32(f32(floor) * f32(1.0001))
    closest = np.inf
    for rows in np.array_split(np.arange(N), 12):            # a row of the corpus: its largest last scale and scale sum
        a = scales[:, rows]
        amax = a[P - 1].max()
        smax = f32(float(a.astype(f64).sum(axis=0).max()) * (1 + 1e-6))
        hs = f32(f64(f32(1.016)) * f64(smax) + f64(floor))
        off = f32(f64(f32(0.015875)) * f64(hs) + f64(floor))
        for q in range(Q):
            T, stored, odd = _i8_operand_view(ops, q, dim)
            v = qhat[q] / float(unscale[q])
            low = np.where(32 * T - v > 0, 0, 1)
            best_last = (v > 0).astype(np.int64)
            fa_low = _i8_accumulator(start[q], stored, odd, low)
            fa_best = _i8_accumulator(start[q], stored, odd, best_last)
            slack = f32(f32(f64(amax) * f64(mass[q]) + f64(f32(f32(margin) * hs))) + f32(off * f32(mass[q] + f32(margin))))
            for z in range(a.shape[1]):
                first_planes = best_last if under[rows[z]] else low
                fa = fa_best if under[rows[z]] else fa_low
                true = sum(float(a[j, z]) * float(v @ (2 * first_planes - 1)) for j in range(P - 1)) + float(a[P - 1, z]) * float(v @ (2 * best_last - 1))
                taus = f32(true)
                if float(taus) < true:
                    taus = np.nextafter(taus, f32(np.inf))
                row_tau = f32(taus - f32(f32(1.000001) * slack))
                hz = h[:, rows[z]]
                first = f32(f64(-K_ACC) * f64(f32(hz[0] + hz[1])))
                for j in range(P - 1):
                    first = f32(f64(hz[j]) * f64(fa) + f64(first))
                assert first >= row_tau, (q, int(rows[z]), float(first), float(row_tau))
                closest = min(closest, (float(first) - float(row_tau)) / max(float(slack), 1e-30))
    assert closest < 1.0           # (the cases do come within the allowance: it is not idle)


# ------------------------------------------------------------------ host logic: query mass of the progressive scan
@pytest.mark.parametrize("dim,Pq", [(64, 1), (64, 3), (128, 4), (256, 2)])
def test_query_mass_bounds_every_plane(lib, dim, Pq):
    """M = sum_d |qhat_d| is reached by the plane whose signs are those of qhat and by no other; the
    reported mass is at least M, and above it only by a rounding allowance.  Checked against the
    oracle's score of single-plane items with unit scale (the inner sum itself)."""
    rng = np.random.default_rng(dim + Pq)
    W = dim // 64
    for trial in range(20):
        qp = rng.integers(0, 2**64, size=(Pq, W), dtype=np.uint64)
        qs = rng.uniform(0.01, 2.0, size=Pq).astype(np.float32)
        if trial == 0 and Pq >= 2:
            qp[1] = ~qp[0]; qs[1] = qs[0] * np.float32(1 - 2.0 ** -10)     # cancelling planes: M far below dim * sum|c|
        x, y = rbe.rbe_debug_query_mass(qp, qs, dim)
        qbits = ((qp[:, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64).reshape(Pq, dim)
        qhat = (qs.astype(np.float64)[:, None] * (2 * qbits - 1)).sum(axis=0)
        M = np.abs(qhat).sum()
        B = dim * np.abs(qs.astype(np.float64)).sum()
        assert M + 2.0 ** -21 * B <= x <= (M + 2.0 ** -19 * B) * (1 + 2.0 ** -18)
        assert y == np.float32(x) * np.float32(2.0 ** -19)
        # the best plane and random planes, through the oracle's scoring (one item plane, scale 1)
        best = np.zeros((1, 1, W), dtype=np.uint64)
        for d_ in range(dim):
            if qhat[d_] > 0:
                best[0, 0, d_ // 64] |= np.uint64(1) << np.uint64(d_ % 64)
        planes = np.concatenate([best, rng.integers(0, 2**64, size=(1, 200, W), dtype=np.uint64)], axis=1)
        s = oracle.scores(planes, np.ones((1, 201), dtype=np.float32), qp, qs)
        assert abs(s[0] - M) <= 1e-9 * B and np.all(np.abs(s) <= M + 1e-9 * B)


def test_last_plane_bound_holds_for_scales_at_least_zero_and_fails_below(lib):
    """Host-side evaluation of the pruning scans' bound, written out in float64:
        bound(z) = sum_{j < P-1} a_j[z] t_j(z) + max(0, largest last scale of the row) * M,
    t_j = sum_i c_i (b_q^i . b_z^j), M = the library's query mass.  For scales >= 0 it is never below the
    oracle's score.  With a negative last scale it can be: the last plane then adds up to |a| M while the
    bound allows for nothing.  That is why an index holding a negative scale gets no pruning scan
    (rbe_finalize marks it; the GPU tests check that the plain scans find such items)."""
    rng = np.random.default_rng(91)
    d, P, Pq, N = 64, 3, 3, 2000
    planes = rng.integers(0, 2**64, size=(P, N, 1), dtype=np.uint64)
    scales = rng.uniform(0.0, 1.0, size=(P, N)).astype(np.float32)
    qp = rng.integers(0, 2**64, size=(Pq, 1), dtype=np.uint64)
    qs = rng.uniform(0.05, 1.0, size=Pq).astype(np.float32)
    M, _ = rbe.rbe_debug_query_mass(qp, qs, d)

    def bound(planes, scales):
        part = oracle.scores(planes[:P - 1], scales[:P - 1], qp, qs)           # planes 0 .. P-2, exactly
        return part + max(0.0, float(scales[P - 1].max())) * M                  # one row: the whole corpus here

    true = oracle.scores(planes, scales, qp, qs)
    assert np.all(bound(planes, scales) >= true)
    # item 0: last plane = complement of the sign pattern of qhat, last scale -0.9 -> contributes +0.9 M
    qbits = ((qp[:, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64).reshape(Pq, d)
    qhat = (qs.astype(np.float64)[:, None] * (2 * qbits - 1)).sum(axis=0)
    word = np.uint64(0)
    for i in range(d):
        if qhat[i] <= 0:
            word |= np.uint64(1) << np.uint64(i)
    planes[P - 1, 0, 0] = word
    scales[:, 0] = 0.0
    scales[P - 1, 0] = -0.9
    scales[P - 1, 1:] = np.minimum(scales[P - 1, 1:], np.float32(0.1))          # the row's largest last scale is small
    true = oracle.scores(planes, scales, qp, qs)
    assert true[0] == pytest.approx(0.9 * np.abs(qhat).sum(), rel=1e-6)
    assert bound(planes, scales)[0] < true[0] - 0.5 * M, "the bound no longer covers the last plane"


def _scale_copy_codec(a):
    """One-byte copies of a scale array as rbe_finalize makes them (written out from their description: a 3-bit
    exponent above a per-array base -- the array's largest value gets exponent field 7 -- and the top 5 mantissa
    bits, rounded to nearest; smaller values, zeros included, get the smallest code).  Returns (decoded copies, base)."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.int64)
    base = max(1, int((bits.max() + (1 << 17)) >> 23) - 7)
    code = np.clip(((bits + (1 << 17)) >> 18) - (base << 5), 0, 255)
    return ((code + (base << 5)) << 18).astype(np.uint32).view(np.float32).astype(np.float64), base


@pytest.mark.parametrize("P,A", [(3, 1), (4, 2)])
def test_first_stage_bound_of_the_two_stage_scan_is_an_upper_bound(lib, P, A):
    """Host-side evaluation, in float64, of the bound the two-stage one-query scan forms from the planes of its
    stream (plane 0 with three planes, planes 0 and 1 with four) and the one-byte scale copies:
        bound(z) = sum_{j<A} [h_j t_j + (e h_j + 2^(base_j - 127)) |t_j|] + (1 + e) M sum_{j>=A} h_j,   e = 0.015875,
    h_j the decoded copies, t_j = qhat . rho_j, M the library's query mass.  It is never below the oracle's score:
    on random items with scales spread over many binades (zeros and values far below the smallest code included),
    and on the items that attain it -- every plane outside the stream the sign pattern of qhat.  And it is not
    slack by more than the copies' precision on those."""
    rng = np.random.default_rng(123 + P)
    d, Pq, N = 64, 3, 4000
    planes = rng.integers(0, 2**64, size=(P, N, 1), dtype=np.uint64)
    scales = (rng.uniform(0.0, 1.0, size=(P, N)) * 10.0 ** rng.uniform(-12, 0, size=(P, N))).astype(np.float32)
    scales[:, :50] = 0.0
    scales[0, 50:100] = np.float32(0.93)
    qp = rng.integers(0, 2**64, size=(Pq, 1), dtype=np.uint64)
    qs = rng.uniform(0.05, 1.0, size=Pq).astype(np.float32)
    M, _ = rbe.rbe_debug_query_mass(qp, qs, d)
    qbits = ((qp[:, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64).reshape(Pq, d)
    qhat = (qs.astype(np.float64)[:, None] * (2 * qbits - 1)).sum(axis=0)
    best = np.uint64(0)
    for i in range(d):
        if qhat[i] > 0:
            best |= np.uint64(1) << np.uint64(i)
    planes[A:, 100:600, 0] = best                      # planes outside the stream that attain +M each
    scales[:, 100:600] = rng.uniform(0.05, 1.0, size=(P, 500)).astype(np.float32)

    def bound(planes, scales):
        e = 0.015875
        copies = [_scale_copy_codec(scales[j]) for j in range(P)]
        h = [c[0] for c in copies]
        out = (1 + e) * M * sum(h[A:])
        for j in range(A):
            bits = ((planes[j, :, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.float64).reshape(-1, d)
            t = (2 * bits - 1) @ qhat
            floor_j = 2.0 ** (copies[j][1] - 127)     # a scale of array j below its smallest copy is above it by less than this
            out = out + h[j] * t + (e * h[j] + floor_j) * np.abs(t)
        return out, h, [c[1] for c in copies]

    true = oracle.scores(planes, scales, qp, qs)
    b, h, bases = bound(planes, scales)
    assert np.all(b >= true), float((true - b).max())
    # the copies are what their description says: within 2^-6 of every scale that is at least the smallest code
    for j in range(P):
        a = scales[j].astype(np.float64)
        big = a >= 2.0 ** (bases[j] - 127)
        assert np.all(np.abs(h[j][big] - a[big]) <= 2.0 ** -6 * 1.016 * h[j][big])
        assert np.all(h[j][~big] >= a[~big])
    # attained up to the copies' precision where the residual planes are the best ones and the scales are not tiny
    sel = np.arange(100, 600)
    sel = sel[(scales[:, sel] > 1e-3).all(axis=0)]
    assert sel.size > 20
    assert np.all(b[sel] - true[sel] <= 0.035 * scales[:, sel].astype(np.float64).sum(axis=0) * M + sum(2.0 ** (bases[j] - 127) for j in range(A)) * M)


@pytest.mark.parametrize("dim,Pq", [(64, 1), (64, 3), (128, 4)])
def test_query_mass_dyadic_is_the_least_mismatch_count(lib, dim, Pq):
    """Dyadic index: h_min = min over planes K of sum_i 2^(Pq-1-i) popcount(Q_i XOR K).  The minimum
    separates over dimensions, so brute force over the two choices per dimension gives it."""
    rng = np.random.default_rng(7 * dim + Pq)
    W = dim // 64
    for _ in range(20):
        qp = rng.integers(0, 2**64, size=(Pq, W), dtype=np.uint64)
        h_min, y = rbe.rbe_debug_query_mass(qp, None, dim, dyadic=True)
        qbits = ((qp[:, :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(np.int64).reshape(Pq, dim)
        wts = 2 ** np.arange(Pq - 1, -1, -1, dtype=np.int64)
        cost1 = (wts[:, None] * (1 - qbits)).sum(axis=0)      # item bit 1: mismatches where the query bit is 0
        cost0 = (wts[:, None] * qbits).sum(axis=0)
        assert h_min == int(np.minimum(cost0, cost1).sum()) and y == 0.0
