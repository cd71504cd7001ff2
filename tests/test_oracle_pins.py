"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU, no HIP library).

Each test names the passage or the fact it holds the oracle to.  A plausible mistake in the oracle (a
dropped term, a wrong index, a swapped plane, a wrong tie rule) fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle as O
from paper_2508_03760_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SR = O.F_SPIKE
F32 = O.F_META_FP32
INT = O.F_META_INT


def bf(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def f32(b):
    return W.bf16_bits_to_f32(np.asarray(b, np.uint16))


def bfs(v) -> int:
    """bf16 bits of one value, as a Python int"""
    return int(bf([v])[0])


def f32s(b) -> float:
    return float(f32([b])[0])


def rand_group(rng, G, kind):
    if kind == "normal":
        v = rng.standard_normal(G)
    elif kind == "outlier":
        v = rng.standard_normal(G)
        v[rng.integers(G)] *= 60
    elif kind == "coarse":  # many ties
        v = rng.integers(-3, 4, G).astype(np.float64) * 0.5
    elif kind == "positive":
        v = np.abs(rng.standard_normal(G)) + 1.0
    else:
        v = np.full(G, 1.25)
    return bf(v)


# ---- Table 4 ------------------------------------------------------------------------------------------------

def test_table4_footprint():
    rows = {}
    for line in open(os.path.join(GOLD, "table4_footprint.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = list(map(int, v))
    data, quant, sz, spikes, meta, total = rows["scale"]
    L = O.get_layout(4096, 2, 32, SR, align=1)
    assert 4096 * 2 == data
    assert L.off_plane2 == 0 and L.off_scale == quant  # payload section
    assert L.off_spike_val - L.off_scale == sz  # bf16 scale + bf16 zero
    assert L.off_spike_idx - L.off_spike_val == 512  # bf16 spike values
    byte_idx = L.total_bytes - L.off_spike_idx
    assert (L.off_spike_idx - L.off_spike_val) + byte_idx == rows["scale_int"][3]  # 768: byte indices
    assert (L.off_spike_idx - L.off_spike_val) + 2 * byte_idx == spikes  # 1024 with 2-byte indices
    assert quant + sz + spikes == total and sz + spikes == meta
    assert L.total_bytes == quant + sz + rows["scale_int"][3]  # the default format: bf16 scale/zero, byte indices
    # the table's first row as a layout of its own: spike positions as BF16 numbers, two bytes each
    L1 = O.get_layout(4096, 2, 32, SR | O.F_IDX_BF16, align=1)
    assert L1.total_bytes == total == 2560
    assert (L1.off_plane2, L1.off_scale, L1.off_zero, L1.off_spike_val, L1.off_spike_idx) == (0, 1024, 1280, 1536, 2048)
    assert L1.total_bytes - L1.off_spike_val == spikes and L1.total_bytes - L1.off_scale == meta


def test_spike_positions_as_bf16_numbers():
    """Table 4, first row: the positions written as BF16 numbers.  Nothing else in the record changes, the numbers are
    exactly the byte positions, and decoding gives the same values as with byte positions."""
    rng = np.random.default_rng(8)
    for bits, G in ((2, 32), (3, 64), (4, 128), (8, 256)):
        n = G * 40
        x = bf(rng.standard_normal(n) * np.exp(rng.standard_normal(n)))
        a = O.quantize_pack(x, bits, G, SR)
        b = O.quantize_pack(x, bits, G, SR | O.F_IDX_BF16)
        La, Lb = O.get_layout(n, bits, G, SR), O.get_layout(n, bits, G, SR | O.F_IDX_BF16)
        assert Lb.off_spike_idx == La.off_spike_idx and Lb.total_bytes >= La.total_bytes
        assert np.array_equal(a[:La.off_spike_idx], b[:Lb.off_spike_idx])  # planes, scale, zero, spike values
        pos_bytes = a[La.off_spike_idx:La.off_spike_idx + 2 * La.n_groups]
        pos_bf16 = f32(b[Lb.off_spike_idx:Lb.off_spike_idx + 4 * Lb.n_groups].view(np.uint16))
        assert np.array_equal(pos_bf16, pos_bytes.astype(np.float32))
        va = O.unpack_dequant(a, n, bits, G, SR)
        vb = O.unpack_dequant(b, n, bits, G, SR | O.F_IDX_BF16)
        assert np.array_equal(va.view(np.uint32), vb.view(np.uint32))
        # the reduce step reads either kind and writes either kind
        r1 = O.reduce_requant([b, b], n, (bits, G, SR | O.F_IDX_BF16), (bits, G, SR))
        r2 = O.reduce_requant([a, a], n, (bits, G, SR))
        assert np.array_equal(r1, r2)


@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_layout_sections(bits, group):
    n = 4096
    for flags in (0, SR, F32, SR | F32):
        for align in (1, 16, 256):
            L = O.get_layout(n, bits, group, flags, align)
            widths = {2: [2], 3: [2, 1], 4: [4], 5: [4, 1], 6: [4, 2], 7: [4, 2, 1], 8: [8]}[bits]
            assert sum(widths) == bits
            secs = []
            for w in (8, 4, 2, 1):
                off = getattr(L, f"off_plane{w}")
                if w in widths:
                    secs.append((off, n * w // 8))
                else:
                    assert off == O.ABSENT
            m = 4 if flags & F32 else 2
            secs += [(L.off_scale, m * n // group), (L.off_zero, m * n // group)]
            if flags & SR:
                secs += [(L.off_spike_val, 4 * n // group), (L.off_spike_idx, 2 * n // group)]
            else:
                assert L.off_spike_val == O.ABSENT and L.off_spike_idx == O.ABSENT
            end = 0
            for off, size in secs:  # in order, aligned, not overlapping, padding < align
                assert off % align == 0 and end <= off < end + align
                end = off + size
            assert L.total_bytes == -(-end // align) * align


# ---- order key ----------------------------------------------------------------------------------------------

def test_key_is_numeric_order_on_all_finite_bf16():
    u = np.arange(65536, dtype=np.uint32)
    finite = (u & 0x7F80) != 0x7F80
    u = u[finite].astype(np.uint16)
    keys = np.array([O.key(v) for v in u])
    vals = f32(u).astype(np.float64)
    order = np.argsort(keys, kind="stable")
    assert np.all(np.diff(vals[order]) >= 0)  # sorted by key == sorted numerically
    assert len(set(keys.tolist())) == len(keys)  # injective
    assert O.key(0x8000) < O.key(0x0000)  # -0 below +0


# ---- bf16 rounding against an independent library conversion -------------------------------------------------

def test_bf16_rne_matches_torch():
    rng = np.random.default_rng(1)
    v = np.concatenate([rng.standard_normal(4000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 4000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], np.float32)])
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([O.bf16_rne(x) for x in v], np.uint16)
    assert np.array_equal(got, want)


# ---- spike selection (Section 3.3) ---------------------------------------------------------------------------

def sorted_closed_form(x):
    """min/max spikes are the extremes; the shrunk range is [2nd smallest, 2nd largest] of the multiset."""
    keys = sorted(O.key(v) for v in x)
    return keys[0], keys[-1], keys[1], keys[-2]


@pytest.mark.parametrize("kind", ["normal", "outlier", "coarse", "positive", "const"])
@pytest.mark.parametrize("G", [32, 64, 128, 256])
def test_spike_select_closed_form(kind, G):
    rng = np.random.default_rng(G * 7 + len(kind))
    for _ in range(40):
        x = rand_group(rng, G, kind)
        codes, s, z, sv, si = O.quantize_group(x, 8, SR | F32)
        kmin, kmax, klo, khi = sorted_closed_form(x)
        assert O.key(sv[0]) == kmin and O.key(sv[1]) == kmax
        assert x[si[0]] == sv[0] and x[si[1]] == sv[1] and si[0] != si[1]
        # lowest index on ties; the max is looked for among the other positions
        assert si[0] == min(i for i in range(G) if O.key(x[i]) == kmin)
        assert si[1] == min(i for i in range(G) if O.key(x[i]) == kmax and i != si[0])
        assert O.key(bfs(z)) == klo  # zero = new minimum
        rest = [i for i in range(G) if i not in (si[0], si[1])]
        hi = max(f32(x[rest]))
        lo = min(f32(x[rest]))
        assert z == lo
        want_s = np.float32(np.float32(hi - lo) / np.float32(255))
        assert s == (want_s if want_s >= 2.0 ** -64 else np.float32(1))
        assert O.key(bfs(hi)) == khi


def test_spike_select_brute_force_tiny_groups():
    alphabet = bf([-1.5, -0.0, 0.0, 2.0])
    for G in (4, 5, 6):
        for tup in itertools.product(range(4), repeat=G):
            x = alphabet[list(tup)]
            codes, s, z, sv, si = O.quantize_group(x, 2, SR | F32)
            keys = [O.key(v) for v in x]
            # every way of taking out one minimal and one maximal element leaves the same multiset
            kmin, kmax = min(keys), max(keys)
            imin = keys.index(kmin)
            imax = [i for i in range(G) if keys[i] == kmax and i != imin][0]
            assert (si[0], si[1]) == (imin, imax)
            rest = [keys[i] for i in range(G) if i not in (imin, imax)]
            assert O.key(bfs(z)) == min(rest)
            assert codes[imin] == 0 and codes[imax] == 0
            # codes of the rest: nearest level of the 4-level grid over [min(rest), max(rest)]
            lo = f32s(x[keys.index(min(rest))])
            hi = f32s(x[keys.index(max(rest))])
            for i in range(G):
                if i in (imin, imax):
                    continue
                xi = f32s(x[i])
                if hi == lo:
                    assert codes[i] == 0
                else:
                    levels = [lo + q * (hi - lo) / 3 for q in range(4)]
                    best = min(abs(xi - l) for l in levels)
                    assert abs(xi - levels[codes[i]]) <= best + 1e-6


# ---- quantizer invariants (Sections 3.1, 3.3) ----------------------------------------------------------------

@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("flags", [0, SR, F32, SR | F32])
def test_quantizer_invariants(bits, flags):
    rng = np.random.default_rng(bits * 11 + flags)
    qmax = 2 ** bits - 1
    for G in (32, 128, 256):
        for kind in ("normal", "outlier", "coarse", "positive", "const"):
            x = rand_group(rng, G, kind)
            codes, s, z, sv, si = O.quantize_group(x, bits, flags)
            xf = f32(x).astype(np.float64)
            rest = np.ones(G, bool)
            if flags & SR:
                rest[[si[0], si[1]]] = False
                assert codes[si[0]] == 0 and codes[si[1]] == 0
            assert codes.max() <= qmax
            lo, hi = xf[rest].min(), xf[rest].max()
            assert float(z) == lo
            # the stored scale covers the range and is the smallest representable one that does
            if hi - lo >= qmax * 2.0 ** -64:
                assert qmax * float(s) >= (hi - lo) * (1 - 2 ** -23)
                if not flags & F32:
                    assert bfs(s) << 16 == int(np.float32(s).view(np.uint32))  # exactly a bf16
                    assert qmax * f32s(bfs(s) - 1) < (hi - lo) * (1 + 2 ** -22)
            recon = codes.astype(np.float64) * float(s) + lo
            err = np.abs(recon - xf)[rest]
            assert np.all(err <= float(s) * (0.5 + 2.0 ** -10))  # half a step
            assert codes[rest][np.argmin(xf[rest])] == 0  # new minimum sits on level 0
            order = np.argsort(xf[rest], kind="stable")
            assert np.all(np.diff(codes[rest][order].astype(int)) >= 0)  # monotone


def test_round_half_to_even_and_clamp():
    # no spikes, fp32 metadata, 2 bits: lo=0, hi=3 -> scale exactly 1, so x is its own quantizer argument
    x = bf([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 0.25] + [0.75] * 24)
    codes, s, z, _, _ = O.quantize_group(x, 2, F32)
    assert s == 1.0 and z == 0.0
    assert codes[:8].tolist() == [0, 3, 0, 2, 2, 1, 2, 0]  # .5 -> 0, 1.5 -> 2, 2.5 -> 2


@pytest.mark.parametrize("bits", range(2, 9))
def test_reduces_to_textbook_rtn_without_spikes(bits):
    """Spike reserving off and fp32 metadata: plain per-group asymmetric min-max round-to-nearest,
    here recomputed in float64."""
    rng = np.random.default_rng(bits)
    qmax = 2 ** bits - 1
    for _ in range(30):
        x = rand_group(rng, 128, "outlier")
        codes, s, z, _, _ = O.quantize_group(x, bits, F32)
        xf = f32(x).astype(np.float64)
        lo, hi = xf.min(), xf.max()
        t = (xf - lo) / ((hi - lo) / qmax)
        want = np.clip(np.rint(t), 0, qmax)
        near_half = np.abs(t - np.floor(t) - 0.5) < 1e-4
        assert np.array_equal(codes[~near_half], want[~near_half].astype(np.uint8))
        assert np.all(np.abs(codes.astype(float) - t) <= 0.5 + 1e-4)
        assert abs(float(s) - (hi - lo) / qmax) <= 2 ** -23 * float(s) and float(z) == lo


# ---- bit splitting (Section 3.2, Fig. 3) ---------------------------------------------------------------------

@pytest.mark.parametrize("bits", range(2, 9))
def test_planes_reassemble_every_code(bits):
    n = 2 ** bits * 8
    codes = np.repeat(np.arange(2 ** bits, dtype=np.uint8), 8)
    rng = np.random.default_rng(bits)
    for c in (codes, rng.permutation(codes)):
        packed = O.split_pack(c, bits, 8, 0, align=1)
        L = O.get_layout(n, bits, 8, 0, align=1)
        assert L.off_scale == n * bits // 8  # planes hold exactly n*b/8 bytes
        assert np.array_equal(O.unpack_codes(packed, n, bits, 8, 0, align=1), c)


def test_int5_is_four_bits_plus_one_bit():
    # Fig. 3: a 5-bit value is stored as its first four bits, all together, and one extra bit, all together
    codes = np.array([0b10111, 0b00001, 0b11110, 0b01010, 0, 0, 0, 0b10000], np.uint8)
    packed = O.split_pack(codes, 5, 8, 0, align=1)
    L = O.get_layout(8, 5, 8, 0, align=1)
    p4 = packed[L.off_plane4:L.off_plane4 + 4]
    p1 = packed[L.off_plane1]
    assert p4.tolist() == [0b1011 | (0b0000 << 4), 0b1111 | (0b0101 << 4), 0, 0 | (0b1000 << 4)]
    assert p1 == 0b00000011  # extra bits of elements 0 and 1
    assert L.off_plane1 == 4 and L.off_scale == 5


def test_plane_membership_for_every_width():
    # 3 = 2+1, 6 = 4+2, 7 = 4+2+1: the wider plane holds the more significant bits
    for bits, parts in {3: [(2, 1), (1, 0)], 6: [(4, 2), (2, 0)], 7: [(4, 3), (2, 1), (1, 0)], 2: [(2, 0)],
                        4: [(4, 0)], 8: [(8, 0)], 5: [(4, 1), (1, 0)]}.items():
        codes = (np.arange(64) * 37 % (2 ** bits)).astype(np.uint8)
        packed = O.split_pack(codes, bits, 8, 0, align=1)
        L = O.get_layout(64, bits, 8, 0, align=1)
        for w, shift in parts:
            off = getattr(L, f"off_plane{w}")
            per = 8 // w
            for e in range(64):
                got = (packed[off + e // per] >> ((e % per) * w)) & (2 ** w - 1)
                assert got == (codes[e] >> shift) & (2 ** w - 1)


# ---- whole records: encode -> decode (Section 3.3: spikes go back to their place) ----------------------------

@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_roundtrip_record(bits, group):
    n = 4096
    x = W.tensor(1, 0, rows=1, cols=n).reshape(-1)
    xf = f32(x)
    for flags in (SR, 0, SR | F32):
        packed = O.quantize_pack(x, bits, group, flags)
        L = O.get_layout(n, bits, group, flags)
        v = O.unpack_dequant(packed, n, bits, group, flags, O.DT_FP32)
        vb = O.unpack_dequant(packed, n, bits, group, flags, O.DT_BF16)
        m = 4 if flags & F32 else 2
        sc = packed[L.off_scale:L.off_scale + m * L.n_groups].view(np.float32 if flags & F32 else np.uint16)
        sc = sc if flags & F32 else f32(sc)
        step = np.repeat(sc, group)
        spike = np.zeros(n, bool)
        if flags & SR:
            idx = packed[L.off_spike_idx:L.off_spike_idx + 2 * L.n_groups].reshape(-1, 2).astype(np.int64)
            pos = (np.arange(L.n_groups)[:, None] * group + idx).reshape(-1)
            spike[pos] = True
            assert np.array_equal(vb[spike], x[spike])  # restored bit for bit
            assert np.array_equal(v[spike], xf[spike])
            val = packed[L.off_spike_val:L.off_spike_val + 4 * L.n_groups].view(np.uint16)
            assert np.array_equal(val, x[pos])
        assert np.all(np.abs(v - xf)[~spike] <= step[~spike] * (0.5 + 2.0 ** -7))
        assert np.array_equal(vb[~spike], W.f32_to_bf16_bits(v[~spike]))
        # codes are what the per-group quantizer said
        codes = O.unpack_codes(packed, n, bits, group, flags)
        g0 = O.quantize_group(x[:group], bits, flags)[0]
        assert np.array_equal(codes[:group], g0)


def test_spike_reserving_beats_plain_rtn_on_outlier_data():
    # direction of Tables 3, 7 and 8: at low bit widths keeping the spikes in float lowers the error
    n = 1 << 16
    x = W.tensor(2, 0, rows=16, cols=4096).reshape(-1)
    xf = f32(x).astype(np.float64)
    for bits in (2, 3, 4):
        mse = {}
        for flags in (0, SR):
            v = O.unpack_dequant(O.quantize_pack(x, bits, 128, flags), n, bits, 128, flags)
            mse[flags] = np.mean((v - xf) ** 2)
        assert mse[SR] < mse[0]


# ---- local reduce step (Sections 3.1, 3.4) -------------------------------------------------------------------

@pytest.mark.parametrize("bits,group", [(2, 32), (3, 128), (4, 128), (5, 64), (6, 256), (7, 128), (8, 128)])
def test_reduce_requant(bits, group):
    n, N = 8192, 5
    fmt = (bits, group, SR)
    xs = [W.tensor(2, p, rows=2, cols=4096).reshape(-1) for p in range(N)]
    peers = [O.quantize_pack(x, *fmt) for x in xs]
    out, s = O.reduce_requant(peers, n, fmt, want_sum=True)
    vs = [O.unpack_dequant(p, n, *fmt).astype(np.float64) for p in peers]
    exact = np.sum(vs, axis=0)
    bound = N * 2.0 ** -23 * np.sum(np.abs(vs), axis=0) + 1e-30
    assert np.all(np.abs(s - exact) <= bound)
    # the packed result is the quantized bf16 sum
    assert np.array_equal(out, O.quantize_pack(W.f32_to_bf16_bits(s), *fmt))
    # one peer: decode to bf16, encode again
    one = O.reduce_requant(peers[:1], n, fmt)
    assert np.array_equal(one, O.quantize_pack(O.unpack_dequant(peers[0], n, *fmt, O.DT_BF16), *fmt))
    # identical peers, power-of-two count: the sum is exact
    _, s4 = O.reduce_requant([peers[0]] * 4, n, fmt, want_sum=True)
    assert np.array_equal(s4, (4 * vs[0]).astype(np.float32))
    # peer order matters only through rounding: any order stays inside the bound
    _, s_rev = O.reduce_requant(peers[::-1], n, fmt, want_sum=True)
    assert np.all(np.abs(s_rev - exact) <= bound)


def test_reduce_requant_different_output_format():
    n = 4096
    xs = [W.tensor(4, p, rows=1, cols=n).reshape(-1) for p in range(3)]
    fin, fout = (6, 64, SR), (3, 128, SR | F32)
    peers = [O.quantize_pack(x, *fin) for x in xs]
    out, s = O.reduce_requant(peers, n, fin, fout, want_sum=True)
    assert np.array_equal(out, O.quantize_pack(W.f32_to_bf16_bits(s), *fout))


def _spike_group(G, first, second):
    """A group whose elements 0 and 1 are its two spikes (restored exactly on decode), the rest zeros."""
    x = np.zeros(G, np.float32)
    x[0], x[1] = first, second
    return bf(x)


def test_reduce_peer_order_is_sequential_from_peer_zero():
    """Sections 3.1, 3.4: the local step adds the peers' chunks one after the other.  fp32 addition is not
    associative, so the order is part of the result: with the decoded values 2^24, 1, -2^24 at one position
    (spikes, hence exact) the chain ((2^24 + 1) + -2^24) loses the 1 to a tie-to-even rounding and gives 0,
    every other order gives 1, and a sum carried in higher precision gives 1 as well."""
    G, fmt = 32, (4, 32, SR)
    big = float(2 ** 24)
    A, B, C_ = _spike_group(G, big, -5.0), _spike_group(G, 1.0, -1.0), _spike_group(G, -big, 5.0)
    pa, pb, pc = (O.quantize_pack(x, *fmt) for x in (A, B, C_))
    for rec, x in ((pa, A), (pb, B), (pc, C_)):
        assert np.array_equal(O.unpack_dequant(rec, G, *fmt)[:2], f32(x[:2]))  # the spikes decode exactly
    s = lambda peers: O.reduce_requant(peers, G, fmt, want_sum=True)[1][0]
    assert s([pa, pb, pc]) == 0.0
    assert s([pc, pb, pa]) == 1.0 and s([pb, pc, pa]) == 1.0 and s([pa, pc, pb]) == 1.0
    # four peers: sequential ((A + 1) + 1) + -A = 0; a pairwise tree (A + 1) + (1 + -A) would give 1, and a sum
    # rounded only once would give 2
    assert s([pa, pb, pb, pc]) == 0.0
    # position 1 holds -5, -1, 5 (exact in every order): the neighbour is untouched
    assert O.reduce_requant([pa, pb, pc], G, fmt, want_sum=True)[1][1] == -1.0


def _round_fraction_to_f32(fr):
    """Correctly rounded (nearest, ties to even) float32 of an exact rational, by integer arithmetic only."""
    from fractions import Fraction
    if fr == 0:
        return np.float32(0.0)
    sign, a = (-1, -fr) if fr < 0 else (1, fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1  # 2^e <= a < 2^(e+1)
    e = max(e, -126)  # below the normal range the spacing stays 2^-149
    q = a / Fraction(2) ** (e - 23)  # a in units of the last place
    n, r = divmod(q.numerator, q.denominator)
    twice = 2 * r
    if twice > q.denominator or (twice == q.denominator and (n & 1)):
        n += 1
    return np.float32(sign * float(Fraction(n) * Fraction(2) ** (e - 23)))  # exact in float64, then exact in float32


def test_decode_is_one_fused_multiply_add():
    """Section 3.1 / 3.3: a value is reconstructed as code * scale + zero.  The oracle rounds that expression once
    (a fused multiply-add): every decoded non-spike value equals the exact rational code * scale + zero rounded
    to fp32 a single time.  Rounding the product first is a different function, and the data below tells them apart."""
    from fractions import Fraction
    rng = np.random.default_rng(31)
    G, n = 32, 32 * 64
    differs = 0
    for bits in (4, 8):
        for flags in (F32, SR | F32, SR):
            x = bf(rng.standard_normal(n) * np.exp(rng.standard_normal(n)))
            rec = O.quantize_pack(x, bits, G, flags)
            L = O.get_layout(n, bits, G, flags)
            codes = O.unpack_codes(rec, n, bits, G, flags)
            v = O.unpack_dequant(rec, n, bits, G, flags)
            m = 4 if flags & F32 else 2
            raw_s = rec[L.off_scale:L.off_scale + m * L.n_groups]
            raw_z = rec[L.off_zero:L.off_zero + m * L.n_groups]
            sc = raw_s.view(np.float32) if flags & F32 else f32(raw_s.view(np.uint16))
            zr = raw_z.view(np.float32) if flags & F32 else f32(raw_z.view(np.uint16))
            spikes = set()
            if flags & SR:
                si = rec[L.off_spike_idx:L.off_spike_idx + 2 * L.n_groups]
                spikes = {g * G + int(si[2 * g + k]) for g in range(L.n_groups) for k in (0, 1)}
            for e in range(n):
                if e in spikes:
                    continue
                g = e // G
                q, s_, z_ = int(codes[e]), float(sc[g]), float(zr[g])
                want = _round_fraction_to_f32(Fraction(q) * Fraction(s_) + Fraction(z_))
                assert v[e] == want, (bits, flags, e, q, s_, z_)
                two_step = np.float32(np.float32(np.float32(q) * np.float32(s_)) + np.float32(z_))
                differs += int(two_step != want)
    assert differs > 0  # the inputs do separate one rounding from two


# ---- integer metadata (Section 3.3, Eq. 1, second row of Table 4) ---------------------------------------------

def test_table4_footprint_with_integer_scales():
    """Second row of Table 4: one-byte scale and zero (256 B for 128 groups), bf16 spike values + byte indices
    (768 B), 1024 B of metadata, 2048 B in all."""
    rows = {}
    for line in open(os.path.join(GOLD, "table4_footprint.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = list(map(int, v))
    data, quant, sz, spikes, meta, total = rows["scale_int"]
    L = O.get_layout(4096, 2, 32, SR | INT, align=1)
    assert L.off_scale == quant
    assert L.off_zero - L.off_scale == sz // 2 and L.off_spike_val - L.off_scale == sz
    assert L.total_bytes - L.off_spike_val == spikes
    assert L.total_bytes - L.off_scale == meta
    assert L.total_bytes == total
    assert total == rows["scale"][5] * 4 // 5  # "reduce the memory footprint by 20 %"
    with pytest.raises(ValueError):
        O.get_layout(4096, 2, 32, SR | INT | F32)  # one precision of the metadata at a time


def _exact_pow2_tenths(k):
    """2^(k/10) to 60 digits."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    return (Decimal(k) / 10 * Decimal(2).ln()).exp()


def test_scale_int_is_eq1():
    """Eq. 1 with theta = 10 on closed forms: powers of two, the tenth-octave points themselves, the clamps of a
    signed byte, monotonicity, and the decision points 2^((k + 1/2)/10) located with 60-digit arithmetic."""
    from decimal import Decimal
    for m in range(-12, 13):
        assert O.scale_int(2.0 ** m) == 10 * m
    assert O.scale_int(0.0) == -128 and O.scale_int(1e-30) == -128 and O.scale_int(float("nan")) == -128
    assert O.scale_int(1e30) == 127 and O.scale_int(float("inf")) == 127
    assert O.scale_int(3.0) == 16 and O.scale_int(0.1) == -33 and O.scale_int(1000.0) == 100  # 15.85, -33.2, 99.66
    for k in range(-128, 128):
        assert O.scale_int(float(np.float32(float(_exact_pow2_tenths(k))))) == k
    xs = np.exp2(np.linspace(-14, 14, 5001)).astype(np.float32)
    ks = [O.scale_int(float(x)) for x in xs]
    assert all(a <= b for a, b in zip(ks, ks[1:]))
    for k in range(-127, 127, 7):
        from decimal import getcontext
        getcontext().prec = 60
        thr = ((Decimal(2 * k + 1) / 20) * Decimal(2).ln()).exp()  # 2^((k + 1/2)/10): above it the code is k + 1
        up = np.float32(float(thr))
        if Decimal(float(up)) < thr:
            up = np.nextafter(up, np.float32(np.inf))
        dn = np.nextafter(up, np.float32(-np.inf))
        assert Decimal(float(dn)) < thr < Decimal(float(up))
        assert O.scale_int(float(up)) == k + 1 and O.scale_int(float(dn)) == k


def test_scale_of_int_is_the_rounded_power():
    """The receiver's scale is 2^(scale_int/10) correctly rounded to fp32 (checked with 60-digit arithmetic);
    it inverts Eq. 1 and stays within 2^(1/20) of any scale that maps to the same byte."""
    from decimal import Decimal
    for k in range(-128, 128):
        got = O.scale_of_int(k)
        exact = _exact_pow2_tenths(k)
        err = abs(Decimal(float(got)) - exact)
        for other in (np.nextafter(got, np.float32(np.inf)), np.nextafter(got, np.float32(-np.inf))):
            assert err < abs(Decimal(float(other)) - exact)
        assert O.scale_int(float(got)) == k
        if k % 10 == 0:
            assert float(got) == 2.0 ** (k // 10)
    rng = np.random.default_rng(3)
    for s in np.exp2(rng.uniform(-12.7, 12.6, 2000)).astype(np.float32):
        r = float(O.scale_of_int(O.scale_int(float(s)))) / float(s)
        assert 2 ** -0.0501 <= r <= 2 ** 0.0501


def test_meta_int_worked_examples():
    """Hand-computed groups.  [-1.8, 1.9] at 2 bits: scale 3.7/3 = 1.2333, log2 = 0.3025 -> scale_int 3, decoded
    2^0.3 = 1.2311; zero = round(1.8/1.2311 = 1.46) = 1.  [0.5, 2] at 2 bits: the range is widened to [0, 2]:
    2/3 -> log2 = -0.585 -> -6, zero 0.  [-4, -1] at 4 bits: widened to [-4, 0]: 4/15 -> log2 = -1.907 -> -19,
    decoded 2^-1.9 = 0.26794, zero = round(4/0.26794 = 14.93) = 15.  A group of zeros: lowest scale, zero 0."""
    k, z, sd, zf = O.meta_int(-1.8, 1.9, 2)
    assert (k, z) == (3, 1) and abs(float(sd) - 2 ** 0.3) < 1e-6 and abs(float(zf) + 2 ** 0.3) < 1e-6
    k, z, sd, zf = O.meta_int(0.5, 2.0, 2)
    assert (k, z) == (-6, 0) and float(zf) == 0.0
    k, z, sd, zf = O.meta_int(-4.0, -1.0, 4)
    assert (k, z) == (-19, 15) and abs(float(zf) + 15 * 2 ** -1.9) < 1e-5
    k, z, sd, zf = O.meta_int(0.0, 0.0, 3)
    assert (k, z) == (-128, 0) and float(zf) == 0.0
    # the zero always fits its byte: it is at most about qmax * 2^(1/20) + 1/2
    rng = np.random.default_rng(9)
    for _ in range(2000):
        lo, hi = np.sort(rng.standard_normal(2) * 10.0 ** rng.uniform(-3, 3))
        bits = int(rng.integers(2, 9))
        k, z, sd, zf = O.meta_int(float(np.float32(lo)), float(np.float32(hi)), bits)
        qmax = 2 ** bits - 1
        assert 0 <= z <= min(255, int(qmax * 2 ** 0.05 + 1))
        assert float(zf) == -float(np.float32(z) * sd)
        if z < 255 and -128 < k < 127:
            assert abs(float(zf) - min(float(np.float32(lo)), 0.0)) <= float(sd) * 0.5001


@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("flags", [INT, SR | INT])
def test_integer_metadata_is_textbook_zero_point_quantization(bits, flags):
    """With integer metadata the codes are the usual affine quantization with an integer zero-point,
    q = clamp(round(x / s) + z, 0, qmax), recomputed here in float64 from the stored bytes; decoding is
    (q - z) * s.  Codes may differ only where x / s is within 1e-4 of a tie."""
    rng = np.random.default_rng(bits * 5 + flags)
    qmax = 2 ** bits - 1
    for kind in ("normal", "outlier", "coarse", "positive", "const"):
        for G in (32, 128):
            x = rand_group(rng, G, kind)
            codes, s, zf, sv, si = O.quantize_group(x, bits, flags)
            xf = f32(x).astype(np.float64)
            rest = np.ones(G, bool)
            if flags & SR:
                rest[[int(si[0]), int(si[1])]] = False
                assert codes[int(si[0])] == 0 and codes[int(si[1])] == 0
            lo, hi = xf[rest].min(), xf[rest].max()
            k, z, sd, zf2 = O.meta_int(lo, hi, bits)
            assert (s, zf) == (sd, zf2)
            # Eq. 1 on the widened range, in float64
            s64 = (max(hi, 0.0) - min(lo, 0.0)) / qmax
            if s64 > 0:
                t = np.log2(s64) * 10
                if abs(t - np.floor(t) - 0.5) > 1e-4:
                    assert k == int(np.clip(np.rint(t), -128, 127))
            t = xf / float(sd)
            want = np.clip(np.rint(t) + z, 0, qmax)
            near_tie = np.abs(t - np.floor(t) - 0.5) < 1e-4
            ok = (codes == want) | near_tie | ~rest
            assert ok.all()
            assert codes.max() <= qmax
            # error: half a step inside the covered range; the top may clamp by the 2^(1/20) slack of Eq. 1
            v = (codes.astype(np.float64) - z) * float(sd)
            err = np.abs(v - xf)[rest]
            assert np.all(err <= float(sd) * (1.0 + 0.036 * qmax))
            inside = ((t + z) <= qmax + 0.5)[rest]
            assert np.all(err[inside] <= float(sd) * (0.5 + 1e-3))


@pytest.mark.parametrize("bits,group", [(2, 32), (3, 32), (4, 32), (2, 128), (5, 64), (8, 256)])
def test_roundtrip_record_with_integer_metadata(bits, group):
    n = 4096
    x = W.tensor(1, 0, rows=1, cols=n).reshape(-1)
    xf = f32(x)
    flags = SR | INT
    packed = O.quantize_pack(x, bits, group, flags)
    L = O.get_layout(n, bits, group, flags)
    v = O.unpack_dequant(packed, n, bits, group, flags, O.DT_FP32)
    vb = O.unpack_dequant(packed, n, bits, group, flags, O.DT_BF16)
    kb = packed[L.off_scale:L.off_scale + L.n_groups].view(np.int8)
    zb = packed[L.off_zero:L.off_zero + L.n_groups]
    idx = packed[L.off_spike_idx:L.off_spike_idx + 2 * L.n_groups].reshape(-1, 2).astype(np.int64)
    pos = (np.arange(L.n_groups)[:, None] * group + idx).reshape(-1)
    spike = np.zeros(n, bool)
    spike[pos] = True
    assert np.array_equal(vb[spike], x[spike]) and np.array_equal(v[spike], xf[spike])  # Section 3.3: restored exactly
    codes = O.unpack_codes(packed, n, bits, group, flags)
    sd = np.exp2(kb.astype(np.float64) / 10)
    want = (codes.astype(np.float64) - np.repeat(zb, group)) * np.repeat(sd, group)  # (q - z) * 2^(k/10)
    # two fp32 roundings: the offset z * s, then the fused multiply-add
    tol = 2.0 ** -22 * (codes + np.repeat(zb, group).astype(np.float64)) * np.repeat(sd, group) + 1e-30
    assert np.all(np.abs(v - want)[~spike] <= tol[~spike])
    assert np.array_equal(vb[~spike], W.f32_to_bf16_bits(v[~spike]))
    for g in (0, 5, L.n_groups - 1):
        cg, s, zf, sv, si = O.quantize_group(x[g * group:(g + 1) * group], bits, flags)
        assert np.array_equal(codes[g * group:(g + 1) * group], cg)
        assert float(s) == float(O.scale_of_int(int(kb[g]))) and float(zf) == -float(np.float32(zb[g]) * s)
    # at the low widths Eq. 1 is meant for, the bytes cost little accuracy against bf16 metadata (within 1 dB on
    # this data); at 7 and 8 bits the 2^(1/20) slack of the scale clamps the top codes and costs several dB
    if bits <= 5:
        v16 = O.unpack_dequant(O.quantize_pack(x, bits, group, SR), n, bits, group, SR)
        e_int, e_16 = np.mean((v - xf) ** 2), np.mean((v16 - xf) ** 2)
        assert e_int <= e_16 * 10 ** 0.1


def test_reduce_requant_with_integer_metadata():
    n, N = 4096, 4
    fmt = (2, 32, SR | INT)
    xs = [W.tensor(2, p, rows=1, cols=n).reshape(-1) for p in range(N)]
    peers = [O.quantize_pack(x, *fmt) for x in xs]
    out, s = O.reduce_requant(peers, n, fmt, want_sum=True)
    vs = [O.unpack_dequant(p, n, *fmt).astype(np.float64) for p in peers]
    exact = np.sum(vs, axis=0)
    assert np.all(np.abs(s - exact) <= N * 2.0 ** -23 * np.sum(np.abs(vs), axis=0) + 1e-30)
    assert np.array_equal(out, O.quantize_pack(W.f32_to_bf16_bits(s), *fmt))
    out2 = O.reduce_requant(peers, n, fmt, (4, 32, SR))  # integer metadata in, bf16 metadata out
    assert np.array_equal(out2, O.quantize_pack(W.f32_to_bf16_bits(s), 4, 32, SR))


# ---- dispatch (Sections 3.1, 4.4) ----------------------------------------------------------------------------

def test_dispatch_quant():
    T, H, K, E = 64, 512, 4, 16
    x = W.tensor(3, 0, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3), T, E, K)
    ids[5, 2] = -1
    ids[9, :] = -1
    send, offs, src = O.dispatch_quant(x, ids, E, 2, 128, SR)
    flat = ids.reshape(-1)
    R = int((flat != -1).sum())
    assert offs[0] == 0 and offs[E] == R and len(src) == R
    assert np.array_equal(np.diff(offs), np.bincount(flat[flat >= 0], minlength=E))
    assert sorted(src.tolist()) == np.nonzero(flat != -1)[0].tolist()  # a permutation of the routed copies
    for e in range(E):
        seg = src[offs[e]:offs[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)  # grouped by expert, stable inside
    L = O.get_layout(H, 2, 128, SR, 16)
    assert send.shape == (R, L.total_bytes)
    for r in range(R):
        assert np.array_equal(send[r], O.quantize_pack(x[src[r] // K], 2, 128, SR, align=16))
