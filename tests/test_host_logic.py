"""CPU tests of the library's host logic and of the integer/float building blocks its kernels use.

No GPU and no compute calls: the C-ABI library is loaded only to check its exports and its host-only
fcv2_get_layout; the building blocks (csrc/fcv2_bits.h) are compiled for the host and held to the oracle.
"""
import ctypes as C
import importlib.util
import os
import re

import numpy as np
import pytest

import oracle as O
from paper_2508_03760_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _hostcheck_build():
    spec = importlib.util.spec_from_file_location("fcv2_hostcheck_build", os.path.join(ROOT, "tests", "hostcheck", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.fixture(scope="module")
def hc():
    so = _hostcheck_build().build(sanitize=os.environ.get("FCV2_ORACLE_SANITIZE") == "1")
    L = C.CDLL(so)
    L.hc_div_mismatches.restype = C.c_uint64
    L.hc_div_mismatches.argtypes = [C.c_int, C.c_uint32, C.c_uint32]
    for f in ("hc_key_of_bf16", "hc_bf16_of_key", "hc_bf16_rne_bits", "hc_bf16_round_up_bits"):
        getattr(L, f).restype = C.c_uint32
        getattr(L, f).argtypes = [C.c_uint32]
    L.hc_scale_int_of.restype = None
    L.hc_scale_int_of.argtypes = [C.c_uint32, C.c_uint32, C.POINTER(C.c_int8), C.POINTER(C.c_uint32)]
    L.hc_scale_int_from_tables.restype = None
    L.hc_scale_int_from_tables.argtypes = L.hc_scale_int_of.argtypes
    L.hc_scale_tables_mismatches.restype = C.c_int
    L.hc_scale_tables_mismatches.argtypes = []
    L.hc_scale_int_estimate.restype = C.c_int
    L.hc_scale_int_estimate.argtypes = [C.c_float]
    L.hc_scale_of_int.restype = C.c_float
    L.hc_scale_of_int.argtypes = [C.c_int]
    L.hc_rows_plan.restype = None
    L.hc_rows_plan.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_int, C.c_uint32, C.POINTER(C.c_uint64)]
    return L


@pytest.fixture(scope="module")
def lib():
    path = B.lib_path()
    if not os.path.exists(path):
        B.build()
    return C.CDLL(path)


def test_library_exports_every_declared_symbol(lib):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fcv2_[a-z_0-9]+)\s*\(", header))
    assert names >= {"fcv2_get_layout", "fcv2_quantize_pack", "fcv2_unpack_dequant", "fcv2_reduce_requant",
                     "fcv2_dispatch_workspace_bytes", "fcv2_dispatch_quant", "fcv2_status_string", "fcv2_version",
                     "fcv2_quantize_pack_slices", "fcv2_unpack_dequant_slices", "fcv2_stream_copy"}
    for n in names:
        assert hasattr(lib, n), n
    lib.fcv2_status_string.restype = C.c_char_p
    assert lib.fcv2_status_string(0) == b"ok" and lib.fcv2_version() >= 100


def test_get_layout_matches_oracle_and_rejects_bad_input(lib):
    from paper_2508_03760_amd import fcv2
    for bits in range(2, 9):
        for group in (32, 64, 128, 256):
            for flags in (0, 1, 2, 3, 4, 5, 9, 11, 13):
                for align in (16, 256):
                    for n in (group, 4096, 7168 * 4):
                        if n % group:
                            continue
                        a = fcv2.get_layout(n, bits, group, flags, align)
                        b = O.get_layout(n, bits, group, flags, align)
                        assert a.__dict__ == b.__dict__
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4096, 9, 128, 1)
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4096, 4, 48, 1)
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4100, 4, 128, 1)
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(0, 4, 128, 1)
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4096, 4, 128, 16)  # unknown flag
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4096, 4, 128, 8)  # BF16 spike positions without spikes
    with pytest.raises(ValueError):
        O.get_layout(4096, 4, 128, 8)
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4096, 4, 128, 1, 48)
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.get_layout(4096, 4, 128, 2 | 4)  # fp32 and integer metadata exclude each other
    assert fcv2.dispatch_workspace_bytes(8192, 8, 256) > 8192 * 8 * 4


def test_null_and_misaligned_arguments_are_refused_on_the_host(lib):
    from paper_2508_03760_amd.fcv2 import _Fmt
    fmt = _Fmt(4, 128, 1)
    vp = C.c_void_p
    lib.fcv2_quantize_pack.argtypes = [vp, C.c_uint64, C.POINTER(_Fmt), vp, vp]
    assert lib.fcv2_quantize_pack(None, 4096, C.byref(fmt), vp(256), None) == -1
    assert lib.fcv2_quantize_pack(vp(256), 4096, C.byref(fmt), vp(264), None) == -3  # not 16-byte aligned
    assert lib.fcv2_quantize_pack(vp(256), 4000, C.byref(fmt), vp(512), None) == -1
    assert lib.fcv2_quantize_pack(vp(256), (1 << 31) + 4096, C.byref(fmt), vp(512), None) == -2  # above the largest tensor
    lib.fcv2_unpack_dequant.argtypes = [vp, C.c_uint64, C.POINTER(_Fmt), vp, C.c_int, vp]
    assert lib.fcv2_unpack_dequant(vp(256), (1 << 31) + 4096, C.byref(fmt), vp(512), 0, None) == -2
    assert lib.fcv2_unpack_dequant(vp(256), 4096, C.byref(fmt), vp(512), 7, None) == -1  # unknown output type
    lib.fcv2_reduce_requant.argtypes = [C.POINTER(vp), C.c_int, C.c_uint64, C.POINTER(_Fmt), C.POINTER(_Fmt), vp, vp, vp]
    peers = (vp * 2)(256, 512)
    assert lib.fcv2_reduce_requant(peers, 0, 4096, C.byref(fmt), C.byref(fmt), vp(1024), None, None) == -1
    assert lib.fcv2_reduce_requant(peers, 17, 4096, C.byref(fmt), C.byref(fmt), vp(1024), None, None) == -1
    other = _Fmt(4, 64, 1)  # another group size
    assert lib.fcv2_reduce_requant(peers, 2, 4096, C.byref(fmt), C.byref(other), vp(1024), None, None) == -2
    other = _Fmt(4, 128, 0)  # spike reserving on one side only
    assert lib.fcv2_reduce_requant(peers, 2, 4096, C.byref(fmt), C.byref(other), vp(1024), None, None) == -2
    lib.fcv2_dispatch_quant.argtypes = [vp, vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(_Fmt), vp, vp,
                                        vp, vp, C.c_size_t, vp]
    assert lib.fcv2_dispatch_quant(vp(256), vp(256), 64, 512, 4, 16, C.byref(fmt), vp(256), vp(256), vp(256), vp(256), 16,
                                   None) == -4  # workspace too small


@pytest.mark.parametrize("bits", range(2, 9))
def test_plane_packing_sequences_match_oracle(hc, bits):
    rng = np.random.default_rng(bits)
    cases = [rng.integers(0, 2 ** bits, 8).astype(np.uint8) for _ in range(300)]
    cases += [np.full(8, 2 ** bits - 1, np.uint8), np.zeros(8, np.uint8)]
    cases += [np.eye(8, dtype=np.uint8)[i] * (2 ** bits - 1) for i in range(8)]
    for codes in cases:
        out = (C.c_uint32 * 5)()
        assert hc.hc_planes_of_codes(bits, codes.ctypes.data_as(C.POINTER(C.c_uint8)), out) == 0
        L = O.get_layout(8, bits, 8, 0, align=1)
        packed = O.split_pack(codes, bits, 8, 0, align=1)
        want = {}
        for w, nbytes in ((8, 8), (4, 4), (2, 2), (1, 1)):
            off = getattr(L, f"off_plane{w}")
            want[w] = None if off == O.ABSENT else int.from_bytes(packed[off:off + nbytes].tobytes(), "little")
        if want[8] is not None:
            assert out[0] | (out[1] << 32) == want[8]
        for w, got in ((4, out[2]), (2, out[3]), (1, out[4])):
            if want[w] is not None:
                assert got == want[w], (bits, w, codes)
        if bits < 8:  # and back
            back = np.zeros(8, np.uint8)
            assert hc.hc_codes_of_planes(bits, out[2], out[3], out[4], back.ctypes.data_as(C.POINTER(C.c_uint8))) == 0
            assert np.array_equal(back, codes)
        back = np.zeros(8, np.uint8)  # the "pair" decoding used with mixed-precision FMAs
        assert hc.hc_pairs_of_planes(bits, out[0], out[1], out[2], out[3], out[4],
                                     back.ctypes.data_as(C.POINTER(C.c_uint8))) == 0
        assert np.array_equal(back, codes), (bits, codes, back)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_sixteen_element_pair_decoding(hc, bits):
    """The reduce kernel's decoder for 16 elements per lane: planes packed by the oracle come back as the same codes,
    every 16-bit half holds code << pos and nothing else."""
    rng = np.random.default_rng(40 + bits)
    cases = [rng.integers(0, 2 ** bits, 16).astype(np.uint8) for _ in range(400)]
    cases += [np.full(16, 2 ** bits - 1, np.uint8), np.zeros(16, np.uint8)]
    cases += [np.eye(16, dtype=np.uint8)[i] * (2 ** bits - 1) for i in range(16)]
    cases += [np.eye(16, dtype=np.uint8)[i] for i in range(16)]
    for codes in cases:
        L = O.get_layout(16, bits, 16, 0, align=1)
        packed = O.split_pack(codes, bits, 16, 0, align=1)
        plane = {}
        for w, nbytes in ((4, 8), (2, 4), (1, 2)):
            off = getattr(L, f"off_plane{w}")
            plane[w] = 0 if off == O.ABSENT else int.from_bytes(packed[off:off + nbytes].tobytes(), "little")
        back = np.zeros(16, np.uint8)
        rc = hc.hc_pairs16_of_planes(bits, plane[4] & 0xFFFFFFFF, plane[4] >> 32, plane[2], plane[1],
                                     back.ctypes.data_as(C.POINTER(C.c_uint8)))
        assert rc == 0, (bits, codes)
        assert np.array_equal(back, codes), (bits, codes, back)


def test_bf16_helpers_match_oracle(hc):
    for u in range(0, 65536, 7):
        assert hc.hc_key_of_bf16(u) == O.key(u)
        assert hc.hc_bf16_of_key(hc.hc_key_of_bf16(u)) == u
    rng = np.random.default_rng(0)
    vals = rng.standard_normal(3000).astype(np.float32) * np.float32(10.0) ** rng.integers(-8, 8, 3000).astype(np.float32)
    for v in np.concatenate([vals, np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.00390625, 1.01171875], np.float32)]):
        u = int(np.float32(v).view(np.uint32))
        assert hc.hc_bf16_rne_bits(u) == O.bf16_rne(v)
    for u in (0x3F800000, 0x3F800001, 0x3F80FFFF, 0x3F810000, 0x00810000):
        r = hc.hc_bf16_round_up_bits(u)
        assert r >= u and r & 0xFFFF == 0 and r - u < 0x10000


@pytest.mark.parametrize("qmax", [3, 7, 15, 31, 63, 127, 255])
def test_short_division_is_ieee_division(hc, qmax):
    # every significand of one binade (scaling by powers of two is exact), plus the ranges where the exponent
    # matters: around the 2^-64 threshold of the codec, the largest finite values, denormal quotients, inf
    assert hc.hc_div_mismatches(qmax, 0x3F800000, 1 << 23) == 0
    assert hc.hc_div_mismatches(qmax, 0x1F000000, 1 << 21) == 0
    assert hc.hc_div_mismatches(qmax, 0x7F000000, 0x00800001) == 0  # up to and including +inf
    assert hc.hc_div_mismatches(qmax, 0x00000000, 1 << 20) == 0
    assert hc.hc_div_mismatches(qmax, 0x00800000, 1 << 22) == 0


# ---- integer scale (Eq. 1) as the kernels compute it: table thresholds instead of a logarithm -------------------------

def _scale_int_block(hc, first_bits, count, tables=False):
    k = np.zeros(count, np.int8)
    sb = np.zeros(count, np.uint32)
    fn = hc.hc_scale_int_from_tables if tables else hc.hc_scale_int_of
    fn(first_bits, count, k.ctypes.data_as(C.POINTER(C.c_int8)), sb.ctypes.data_as(C.POINTER(C.c_uint32)))
    return k, sb.view(np.float32)


@pytest.mark.parametrize("exponent", [-14, -13, -7, -1, 0, 1, 5, 12, 13])
def test_scale_int_every_significand(hc, exponent):
    """Eq. 1 for every fp32 significand of a binade against float64 log2; the decoded scale is 2^(k/10)."""
    first = (127 + exponent) << 23
    k, s = _scale_int_block(hc, first, 1 << 23)
    x = (np.arange(1 << 23, dtype=np.uint32) + np.uint32(first)).view(np.float32).astype(np.float64)
    t = np.log2(x) * 10.0
    want = np.clip(np.rint(t), -128, 127)
    far = np.abs(t - np.floor(t) - 0.5) > 1e-9  # float64 log2 decides everything that is not within 1e-9 of a tie
    assert far.sum() >= (1 << 23) - 40
    assert np.array_equal(k[far].astype(np.float64), want[far])
    assert np.all(np.abs(k.astype(np.float64) - want) <= 1)
    assert np.array_equal(s, np.exp2(k.astype(np.float64) / 10.0).astype(np.float32))
    k2, s2 = _scale_int_block(hc, first, 1 << 23, tables=True)  # the table form the kernels keep in LDS
    assert np.array_equal(k, k2) and np.array_equal(s, s2)


def test_compile_time_scale_tables_are_the_table_functions(hc):
    """The 515 floats the kernels copy into LDS are written out at compile time (a table entry times an exact power of
    two); each must be bit for bit what the table functions compute with ldexpf."""
    assert hc.hc_scale_tables_mismatches() == 0


def test_scale_int_estimate_is_within_one(hc):
    rng = np.random.default_rng(5)
    for x in np.exp2(rng.uniform(-20, 20, 20000)).astype(np.float32):
        exact = int(np.clip(np.rint(np.log2(np.float64(x)) * 10), -128, 127))
        assert abs(hc.hc_scale_int_estimate(float(x)) - exact) <= 1


def test_scale_int_ends_and_specials(hc):
    for bits, want in ((0x00000000, -128), (0x00000001, -128), (0x007FFFFF, -128), (0x80000000, -128), (0xBF800000, -128),
                       (0x7FC00000, -128), (0x7F800000, 127), (0x7F7FFFFF, 127), (0x3F800000, 0), (0x40000000, 10)):
        for tables in (False, True):
            k, s = _scale_int_block(hc, bits, 1, tables)
            assert int(k[0]) == want, hex(bits)
            assert s[0] == np.float32(2.0 ** (want / 10.0))
    for kk in range(-128, 128):
        assert np.float32(hc.hc_scale_of_int(kk)) == np.float32(np.exp2(np.float64(kk) / 10.0))


def test_bench_byte_formula_is_the_unpadded_record():
    """The algorithmic bytes the benchmark divides by are the record's sections without alignment padding."""
    import bench
    for bits in range(2, 9):
        for group in (32, 128, 256):
            for spike in (False, True):
                for int_meta in (False, True):
                    flags = (O.F_SPIKE if spike else 0) | (O.F_META_INT if int_meta else 0)
                    assert bench.packed_bytes(1 << 16, bits, group, spike, int_meta) == O.get_layout(1 << 16, bits, group, flags, align=1).total_bytes


def test_dispatch_launch_plan(hc):
    """The row-staged dispatch kernel's launch shape: whole tokens per block, whole waves, at most 512 threads and
    64 KiB of LDS, the fewest idle lanes; shapes that do not fit get no plan (the direct kernel takes them)."""
    def plan(lpr, K, row_bytes, int_meta=0, E=256):
        out = (C.c_uint64 * 3)()
        hc.hc_rows_plan(lpr, K, row_bytes, int_meta, E, out)
        return tuple(int(v) for v in out)

    starts = (256 + 8) * 4  # the block's copy of the expert starts, and the words its scan needs

    # the DeepSeek-V3-shaped workload: H = 7168 = 224 lanes, 2-bit rows of 2,352 bytes, 8 copies: two tokens would fill 7
    # waves exactly, but one token in four waves (an eighth of the lanes idle) is the smaller block, and it is taken
    assert plan(224, 8, 2352) == (1, 256, 4 * 4096 + 2352 + 8 * 4 + starts)
    assert plan(256, 8, 2688) == (1, 256, 4 * 4096 + 2688 + 32 + starts)  # H = 8192: one token is four whole waves
    assert plan(128, 8, 1344)[:2] == (1, 128)                         # H = 4096: the first count without idle lanes
    assert plan(160, 8, 1680)[:2] == (2, 320)                         # H = 5120: one token would leave a sixth of three waves idle
    assert plan(1, 2, 32)[:2] == (64, 64)                             # H = 32: 64 tokens share a wave
    assert plan(513, 8, 5000) == (0, 0, 0)                            # more than 512 lanes per token
    assert plan(512, 8, 8 * 4096 + 30000) == (0, 0, 0)                # record too large for the LDS
    assert plan(224, 8, 2256, 1) == (1, 256, 4 * 4096 + 2256 + 32 + starts + (258 + 257) * 4)
    assert plan(224, 8, 2352, 0, 2048)[2] == 4 * 4096 + 2352 + 32 + (2048 + 8) * 4   # the most experts a call takes
    for lpr in list(range(1, 70)) + [96, 160, 224, 300, 448, 512]:
        for K in (1, 8, 33):
            for row_bytes in (16 * lpr, 40 * lpr + 48):
                rows, threads, lds = plan(lpr, K, row_bytes)
                assert rows >= 1 and threads % 64 == 0 and 64 <= threads <= 512
                assert rows * lpr <= threads < rows * lpr + 64 and lds <= 65536
                # the rule, stated once more: fewest idle lanes (smallest such count), unless that block is larger than four
                # waves and a smaller count fills at least four waves with at most an eighth of the lanes idle
                cands = []
                for r in range(1, 65):
                    if r * lpr > 512:
                        break
                    w = -(-r * lpr // 64)
                    if w * 4096 + r * row_bytes + r * K * 4 + starts > 65536:
                        break
                    cands.append((r, w, (w * 64 - r * lpr) * 1024 // (w * 64)))
                best = min(cands, key=lambda c: (c[2], c[0]))
                small = next((c for c in cands if c[1] >= 4 and c[2] <= 128), None)
                want = small if (best[1] > 4 and small and small[0] < best[0]) else best
                assert (rows, threads) == (want[0], want[1] * 64)


def test_bench_reads_its_counters_from_the_committed_profile():
    """bench.py takes `traffic` and the VALU counts of its roofline objects from the rocprofv3 summary under profiles/;
    the machine-readable line it parses must say what the summary's counter table says."""
    import bench
    pc = bench.profile_counters()
    assert pc and {"quantize_pack", "reduce_requant", "unpack_dequant"} <= set(pc)
    text = open(bench.PROFILE).read()
    text = text[text.index("## Counters, averages per launch"):]
    text = text[:text.index("\n## ", 4)]
    rows = {}
    for line in text.splitlines():
        m = re.match(r"\| fcv2::k_(quantize_pack|reduce_requant|unpack_dequant)\S*.*?\|(.*)\|\s*$", line)
        cells = [c.strip().replace(",", "") for c in (m.group(2).split("|") if m else [])]
        if m and len(cells) >= 4 and m.group(1) not in rows and re.fullmatch(r"[0-9.]+", cells[0]) and re.fullmatch(r"[0-9.]+", cells[3]):
            try:
                rows[m.group(1)] = (float(cells[0]), float(cells[1]), float(cells[3]))  # FETCH_SIZE, WRITE_SIZE, SQ_INSTS_VALU
            except ValueError:
                pass
    assert set(rows) == {"quantize_pack", "reduce_requant", "unpack_dequant"}, rows
    n = 4096 * 4096
    for k, (fetch, write, valu) in rows.items():
        assert abs(pc[k]["hbm_bytes_per_launch"] - (2.0 * fetch + write) * 1024) <= 2048, k
        assert abs(pc[k]["valu_per_element"] - valu * 64 / n) <= 0.06, k
