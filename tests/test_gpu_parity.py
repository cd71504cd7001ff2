"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on the same
seeded inputs.  Packed planes, metadata, spike values/indices, offsets and row maps must be bit-identical;
fp32 outputs must agree within 1e-3 absolute + 1e-3 relative (they are expected to be identical too).
"""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2508_03760_amd import fcv2
from paper_2508_03760_amd import workloads as W

pytestmark = pytest.mark.gpu

SR, F32, INT, IDX16 = fcv2.F_SPIKE, fcv2.F_META_FP32, fcv2.F_META_INT, fcv2.F_IDX_BF16
DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    fcv2.lib()  # fails loudly if the HIP library is missing
    yield
    torch.cuda.synchronize()


def to_dev_bf16(bits_u16):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).to(DEV).view(torch.bfloat16)


def sections(L, flags):
    m = 4 if flags & F32 else 1 if flags & INT else 2
    out = []
    for w in (8, 4, 2, 1):
        off = getattr(L, f"off_plane{w}")
        if off != O.ABSENT:
            out.append((f"plane{w}", off, L.n * w // 8))
    out += [("scale", L.off_scale, m * L.n_groups), ("zero", L.off_zero, m * L.n_groups)]
    if flags & SR:
        out += [("spike_val", L.off_spike_val, 4 * L.n_groups), ("spike_idx", L.off_spike_idx, (4 if flags & IDX16 else 2) * L.n_groups)]
    return out


def assert_packed_equal(got, want, L, flags, what=""):
    got = np.asarray(got).reshape(-1)
    want = np.asarray(want).reshape(-1)
    for name, off, size in sections(L, flags):
        a, b = got[off:off + size], want[off:off + size]
        if not np.array_equal(a, b):
            bad = np.nonzero(a != b)[0]
            raise AssertionError(f"{what}: section {name} differs at {bad.size} of {size} bytes, first at {bad[0]}: "
                                 f"gpu {a[bad[0]]} oracle {b[bad[0]]}")


def assert_close(got, want, what=""):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    bad = np.abs(got - want) > 1e-3 + 1e-3 * np.abs(want)
    assert not bad.any(), f"{what}: {bad.sum()} values outside 1e-3 abs + 1e-3 rel, first at {np.nonzero(bad)[0][0]}"


def check_codec(x_u16, bits, group, flags, what):
    """quantize_pack + both unpack_dequant outputs against the oracle; returns the GPU packed record."""
    x_u16 = np.ascontiguousarray(x_u16).reshape(-1)
    n = x_u16.size
    L = O.get_layout(n, bits, group, flags)
    want = O.quantize_pack(x_u16, bits, group, flags)
    got = fcv2.quantize_pack(to_dev_bf16(x_u16), bits, group, flags)
    assert got.numel() == L.total_bytes
    assert_packed_equal(got.cpu().numpy(), want, L, flags, f"quantize_pack {what}")
    v = fcv2.unpack_dequant(got, n, bits, group, flags, torch.float32).cpu().numpy()
    vo = O.unpack_dequant(want, n, bits, group, flags, O.DT_FP32)
    assert_close(v, vo, f"unpack_dequant fp32 {what}")
    assert np.array_equal(v.view(np.uint32), vo.view(np.uint32)), f"unpack_dequant fp32 {what}: not bit-identical"
    vb = fcv2.unpack_dequant(got, n, bits, group, flags, torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(vb, O.unpack_dequant(want, n, bits, group, flags, O.DT_BF16)), f"unpack_dequant bf16 {what}"
    return got


# ---- small shapes: several tiles and a ragged tail, every format -----------------------------------------------

@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_codec_all_formats(bits, group):
    n = 2048 * 3 + 3 * 256  # three full 256-lane blocks plus a partial one
    x = W.tensor(2, 0, rows=1, cols=n).reshape(-1)
    for flags in (SR, 0, SR | F32, F32, SR | INT, INT, SR | IDX16, SR | INT | IDX16):
        check_codec(x, bits, group, flags, f"b{bits} g{group} f{flags}")


@pytest.mark.parametrize("bits", [2, 3, 5, 8])
def test_codec_single_group_and_tiny_inputs(bits):
    for group in (32, 64, 128, 256):
        for ngroups in (1, 2, 7):
            x = W.tensor(4, 1, rows=1, cols=group * ngroups).reshape(-1)
            check_codec(x, bits, group, SR, f"tiny b{bits} g{group} x{ngroups}")


def test_table4_rows_are_layouts_of_the_library():
    assert fcv2.get_layout(4096, 2, 32, SR | IDX16, 1).total_bytes == 2560  # Table 4, first row
    assert fcv2.get_layout(4096, 2, 32, SR | INT, 1).total_bytes == 2048    # second row


def _edge_groups(group):
    rng = np.random.default_rng(group)
    rows = []
    rows.append(np.full(group, 1.25))                                   # constant group
    rows.append(np.zeros(group))                                        # all +0
    r = np.zeros(group); r[::2] = -0.0; rows.append(r)                  # -0 / +0 mix (ties in value, not in key)
    rows.append(rng.integers(-2, 3, group) * 0.5)                       # many ties
    r = np.full(group, 3.0); r[5] = -7.0; rows.append(r)                # everything but the minimum equal
    r = np.full(group, -3.0); r[group - 1] = 9.0; rows.append(r)        # everything but the maximum equal
    r = np.full(group, 2.0); r[3] = 2.0; r[9] = 100.0; r[17] = -100.0; rows.append(r)
    r = rng.standard_normal(group); r[0] = 1e30; r[1] = -1e30; rows.append(r)       # spikes far outside
    rows.append(rng.standard_normal(group) * 1e-30)                     # tiny magnitudes
    rows.append(rng.standard_normal(group) * 1e-42)                     # range below the 2^-64 threshold
    rows.append(rng.standard_normal(group) * 3e37)                      # near the top of the range
    rows.append(np.linspace(-1, 1, group))                              # exact halves appear at some widths
    rows.append(np.arange(group, dtype=np.float64))                     # integers: ties to even at .5
    r = np.abs(rng.standard_normal(group)) + 4; rows.append(r)          # all positive
    r = -np.abs(rng.standard_normal(group)) - 4; rows.append(r)         # all negative
    for pos in (0, 7, 8, group - 1):                                    # spikes on lane borders
        r = rng.standard_normal(group); r[pos] = 50.0; r[(pos + 8) % group] = -50.0; rows.append(r)
    return W.f32_to_bf16_bits(np.concatenate(rows).astype(np.float32))


@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_codec_edge_cases(bits, group):
    x = _edge_groups(group)
    for flags in (SR, 0, SR | F32, SR | INT, INT, SR | IDX16):
        check_codec(x, bits, group, flags, f"edge b{bits} g{group} f{flags}")


def test_range_overflow_is_deterministic():
    """hi - lo = +inf (inputs beyond 2^127 apart): outside the contract of finite ranges, but the packed record
    still matches the oracle (infinite scale, all codes 0) and decoding yields NaN at the same positions."""
    rng = np.random.default_rng(3)
    x = W.f32_to_bf16_bits(np.clip(rng.standard_normal(1024) * 3e38, -3.3e38, 3.3e38).astype(np.float32))
    for bits in (2, 5, 8):
        L = O.get_layout(x.size, bits, 128, SR)
        want = O.quantize_pack(x, bits, 128, SR)
        got = fcv2.quantize_pack(to_dev_bf16(x), bits, 128, SR)
        assert_packed_equal(got.cpu().numpy(), want, L, SR, f"overflow b{bits}")
        v = fcv2.unpack_dequant(got, x.size, bits, 128, SR).cpu().numpy()
        vo = O.unpack_dequant(want, x.size, bits, 128, SR)
        assert np.array_equal(np.isnan(v), np.isnan(vo))
        assert np.array_equal(v[~np.isnan(v)], vo[~np.isnan(vo)])


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_every_scale_value(bits):
    """Groups [0, hi, hi/2, ...] for every positive finite bf16 hi: sweeps every scale significand and exponent
    the encoder's reciprocal can meet."""
    hi = np.arange(0x0080, 0x7F80, dtype=np.uint16)  # all positive normal bf16 values
    hf = W.bf16_bits_to_f32(hi).astype(np.float64)
    frac = np.concatenate([[0.0, 1.0], np.linspace(0.02, 0.98, 30)])
    x = W.f32_to_bf16_bits((hf[:, None] * frac[None, :]).astype(np.float32)).reshape(-1)
    check_codec(x, bits, 32, 0, f"scales b{bits}")
    check_codec(x, bits, 32, SR, f"scales sr b{bits}")
    # the same sweep passes every decision point of the integer scale (Eq. 1)
    check_codec(x, bits, 32, INT, f"scales int b{bits}")
    check_codec(x, bits, 32, SR | INT, f"scales sr int b{bits}")


def test_random_shapes_and_formats():
    """Forty seeded draws of (length, bits, group, flags): lengths are any whole number of groups (multiples of 8
    elements), so tiles end anywhere; codec, reduce over a random number of peers, and the sliced calls where the
    length allows them."""
    rng = np.random.default_rng(2508)
    for case in range(40):
        bits = int(rng.integers(2, 9))
        group = int(rng.choice([32, 64, 128, 256]))
        flags = int(rng.choice([0, SR, SR | F32, SR | INT, INT, F32]))
        n = group * int(rng.integers(1, 200))
        kind = int(rng.integers(1, 6))
        x = W.tensor(kind, case % 8, rows=1, cols=n).reshape(-1)
        check_codec(x, bits, group, flags, f"random case {case}: n={n} b{bits} g{group} f{flags}")
        n_peers = int(rng.integers(1, 7))
        xs = [W.tensor(kind, (case + p) % 8, rows=1, cols=n).reshape(-1) for p in range(n_peers)]
        check_reduce(xs, bits, group, flags, f"random case {case}: reduce N={n_peers} n={n} b{bits} g{group} f{flags}")


@pytest.mark.parametrize("bits", [2, 8])
def test_maximum_tensor_size(bits):
    """2^31 elements, the largest tensor a call takes (4 GiB of bf16): the 16M-element payload repeated 128 times on the
    GPU.  Groups are independent, so every 16M-element block of the packed record must equal the oracle's record of
    the payload, section by section; the same for the decoded tensor.  Exercises the 32-bit offsets at their limit: at
    8 bits the byte plane alone is 2 GiB, so the metadata sections lie beyond offset 2^31."""
    group, flags = 128, SR
    base = W.tensor(2, 0).reshape(-1)
    reps = (1 << 31) // base.size
    n = base.size * reps
    Lb = O.get_layout(base.size, bits, group, flags)
    want = O.quantize_pack(base, bits, group, flags)
    x = to_dev_bf16(base).repeat(reps)
    assert x.numel() == 1 << 31
    got = fcv2.quantize_pack(x, bits, group, flags)
    L = fcv2.get_layout(n, bits, group, flags)
    assert L.total_bytes < 1 << 32 and (bits != 8 or L.off_scale >= 1 << 31)
    want_d = torch.from_numpy(want).to(DEV)
    for name, off, size in sections(L, flags):
        per = size // reps
        boff = getattr(Lb, "off_" + name)
        blocks = got[off:off + size].view(reps, per)
        assert torch.equal(blocks, want_d[boff:boff + per].expand(reps, per)), f"max size: section {name}"
    out = fcv2.unpack_dequant(got, n, bits, group, flags, torch.bfloat16)
    want_out = torch.from_numpy(O.unpack_dequant(want, base.size, bits, group, flags, O.DT_BF16).view(np.int16)).to(DEV)
    assert torch.equal(out.view(torch.int16).view(reps, base.size), want_out.expand(reps, base.size)), "max size: unpack_dequant"
    del x, out
    # the local reduce step at the same size: two peers, the second one the first record again
    red = fcv2.reduce_requant([got, got], n, (bits, group, flags))
    want_red = torch.from_numpy(O.reduce_requant([want, want], base.size, (bits, group, flags))).to(DEV)
    for name, off, size in sections(L, flags):
        per = size // reps
        boff = getattr(Lb, "off_" + name)
        assert torch.equal(red[off:off + size].view(reps, per), want_red[boff:boff + per].expand(reps, per)), f"max size reduce: {name}"
    del got, red
    torch.cuda.empty_cache()


# ---- reduce_requant -----------------------------------------------------------------------------------------------

def check_reduce(xs, bits, group, flags, what, flags_out=None, bits_out=None):
    n = xs[0].size
    fin = (bits, group, flags)
    fout = (bits if bits_out is None else bits_out, group, flags if flags_out is None else flags_out)
    peers_o = [O.quantize_pack(x, *fin) for x in xs]
    peers_g = [torch.from_numpy(p).to(DEV) for p in peers_o]
    want, s_want = O.reduce_requant(peers_o, n, fin, fout, want_sum=True)
    got, s_got = fcv2.reduce_requant(peers_g, n, fin, fout, want_sum=True)
    assert_close(s_got.cpu().numpy(), s_want, f"reduce sum {what}")
    assert np.array_equal(s_got.cpu().numpy().view(np.uint32), s_want.view(np.uint32)), f"reduce sum {what}: bits differ"
    Lout = O.get_layout(n, *fout)
    assert_packed_equal(got.cpu().numpy(), want, Lout, fout[2], f"reduce_requant {what}")
    got2 = fcv2.reduce_requant(peers_g, n, fin, fout)  # without the optional sum output
    assert_packed_equal(got2.cpu().numpy(), want, Lout, fout[2], f"reduce_requant (no sum) {what}")


@pytest.mark.parametrize("bits", range(2, 9))
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_reduce_requant_all_formats(bits, group):
    n = 2048 * 2 + 512
    xs = [W.tensor(2, p, rows=1, cols=n).reshape(-1) for p in range(8)]
    check_reduce(xs, bits, group, SR, f"b{bits} g{group} N8")
    check_reduce(xs[:3], bits, group, 0, f"b{bits} g{group} N3 no-sr")
    check_reduce(xs[:5], bits, group, SR | INT, f"b{bits} g{group} N5 integer metadata")
    check_reduce(xs[:4], bits, group, SR | IDX16, f"b{bits} g{group} N4 BF16 positions")
    check_reduce(xs[:2], bits, group, SR | IDX16, f"b{bits} g{group} N2 BF16 positions in, bytes out", flags_out=SR)


@pytest.mark.parametrize("flags_in", [0, SR, SR | F32])
def test_reduce_requant_of_sums_that_are_not_numbers(flags_in):
    """A peer whose values span more than the fp32 range is packed with an infinite scale and decodes to NaN (the
    documented behaviour of the sender); sums with it are NaN, sums of the largest finite values are infinite.  The
    requantized record still matches the oracle in every output format: a NaN takes code 0."""
    group, n = 128, 2048 + 256
    rng = np.random.default_rng(17)
    v = np.clip(rng.standard_normal(n) * 3e38, -3.3e38, 3.3e38).astype(np.float32)
    v[n // 2:] = rng.standard_normal(n - n // 2)  # only the first half of this peer decodes to NaN
    huge = W.f32_to_bf16_bits(v)
    big = W.f32_to_bf16_bits(np.where(np.arange(n) % 256 < 128, 3.0e38, 1.0).astype(np.float32))  # finite ranges, infinite sums
    xs = [W.tensor(2, 0, rows=1, cols=n).reshape(-1), huge, big, big, W.tensor(2, 1, rows=1, cols=n).reshape(-1)]
    for bits_in, bits_out, flags_out in ((4, 2, INT), (4, 3, SR | INT), (3, 5, SR | INT), (8, 8, INT), (5, 4, SR), (2, 6, F32)):
        fin, fout = (bits_in, group, flags_in), (bits_out, group, (flags_out & ~SR) | (flags_in & SR))
        peers_o = [O.quantize_pack(x, *fin) for x in xs]
        want, s_want = O.reduce_requant(peers_o, n, fin, fout, want_sum=True)
        assert np.isnan(s_want).any() and np.isinf(s_want).any()
        got, s_got = fcv2.reduce_requant([torch.from_numpy(p).to(DEV) for p in peers_o], n, fin, fout, want_sum=True)
        sg = s_got.cpu().numpy()
        assert np.array_equal(np.isnan(sg), np.isnan(s_want)), f"{fin} -> {fout}: NaN positions"
        ok = ~np.isnan(s_want)
        assert np.array_equal(sg[ok].view(np.uint32), s_want[ok].view(np.uint32)), f"{fin} -> {fout}: sums"
        assert_packed_equal(got.cpu().numpy(), want, O.get_layout(n, *fout), fout[2], f"reduce of NaN sums {fin} -> {fout}")


@pytest.mark.parametrize("n_peers", [1, 2, 5, 16])
def test_reduce_requant_peer_counts(n_peers):
    n = 4096 + 256
    xs = [W.tensor(4, p, rows=1, cols=n).reshape(-1) for p in range(n_peers)]
    check_reduce(xs, 3, 128, SR, f"N{n_peers}")
    check_reduce(xs, 6, 64, SR | F32, f"N{n_peers} fp32 meta", flags_out=SR)
    check_reduce(xs, 2, 32, SR | INT, f"N{n_peers} integer meta in, bf16 out", flags_out=SR)
    check_reduce(xs, 4, 32, SR, f"N{n_peers} bf16 meta in, integer out", flags_out=SR | INT)


@pytest.mark.parametrize("bits_in,bits_out", [(2, 8), (3, 5), (4, 3), (5, 2), (6, 7), (7, 4), (8, 6)])
def test_reduce_requant_other_output_width(bits_in, bits_out):
    n = 2048 * 2 + 512
    for group in (32, 128):
        xs = [W.tensor(2, p, rows=1, cols=n).reshape(-1) for p in range(5)]
        check_reduce(xs, bits_in, group, SR, f"in b{bits_in} out b{bits_out} g{group}", bits_out=bits_out)
    check_reduce(xs[:2], bits_in, 64, 0, f"in b{bits_in} out b{bits_out} no-sr", bits_out=bits_out, flags_out=F32)
    check_reduce(xs[:3], bits_in, 32, SR | INT, f"in b{bits_in} out b{bits_out} integer meta", bits_out=bits_out)


def test_reduce_requant_edge_cases():
    for group in (32, 128, 256):
        base = _edge_groups(group)
        xs = [base, base[::-1].copy(), np.roll(base, group)]
        check_reduce(xs, 4, group, SR, f"edge g{group}")
        check_reduce(xs, 2, group, SR, f"edge g{group} b2")
        check_reduce(xs, 3, group, SR | INT, f"edge g{group} b3 integer meta")


# ---- slices and the whole two-step AllReduce on one GPU (Sections 3.1, 3.4) ----------------------------------

@pytest.mark.parametrize("bits,group", [(2, 32), (3, 128), (5, 64), (8, 256)])
def test_slices_match_per_slice_records(bits, group):
    R, n = 4, 4 * 2048 * 3
    x = W.tensor(2, 0, rows=1, cols=n).reshape(-1)
    L = O.get_layout(n // R, bits, group, SR)
    got = fcv2.quantize_pack_slices(to_dev_bf16(x), R, bits, group, SR)
    assert got.shape == (R, L.total_bytes)
    recs_o = [O.quantize_pack(x[j * n // R:(j + 1) * n // R], bits, group, SR) for j in range(R)]
    for j in range(R):
        assert_packed_equal(got[j].cpu().numpy(), recs_o[j], L, SR, f"slice {j} b{bits} g{group}")
    want = np.concatenate([O.unpack_dequant(r, n // R, bits, group, SR) for r in recs_o])
    for dt, view in ((torch.float32, np.uint32), (torch.bfloat16, np.uint16)):
        out = fcv2.unpack_dequant_slices([torch.from_numpy(r).to(DEV) for r in recs_o], n, bits, group, SR, dt)
        if dt == torch.float32:
            assert np.array_equal(out.cpu().numpy().view(view), want.view(view))
        else:
            wb = np.concatenate([O.unpack_dequant(r, n // R, bits, group, SR, O.DT_BF16) for r in recs_o])
            assert np.array_equal(out.view(torch.int16).cpu().numpy().view(view), wb)


def test_slice_arguments_are_checked():
    x = to_dev_bf16(W.tensor(2, 0, rows=1, cols=8192).reshape(-1))
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.quantize_pack_slices(x, 3, 4, 128, SR)  # 8192 not a multiple of 3
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.quantize_pack_slices(x, 8, 4, 128, SR)  # slices of 1024 elements: not whole wave tiles
    with pytest.raises(fcv2.Fcv2Error):
        fcv2.quantize_pack_slices(x, 32, 4, 128, SR)  # more than 16 slices


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_two_step_allreduce_on_one_gpu(bits):
    """R simulated ranks: every rank packs its payload as R slices, rank j reduces the R copies of slice j, every
    rank unpacks the R reduced slices.  The GPU pipeline equals the oracle's bit for bit, and the result stays within
    the quantization error bound of the exact sum."""
    R, n, group = 8, 8 * 2048 * 2, 128
    fmt = (bits, group, SR)
    xs = [W.tensor(2, r, rows=1, cols=n).reshape(-1) for r in range(R)]
    m = n // R
    L = O.get_layout(m, *fmt)
    # oracle pipeline
    send_o = [[O.quantize_pack(x[j * m:(j + 1) * m], *fmt) for j in range(R)] for x in xs]
    red_o = [O.reduce_requant([send_o[r][j] for r in range(R)], m, fmt) for j in range(R)]
    out_o = np.concatenate([O.unpack_dequant(red_o[j], m, *fmt, O.DT_BF16) for j in range(R)])
    # GPU pipeline, through the C ABI
    send_g = [fcv2.quantize_pack_slices(to_dev_bf16(x), R, *fmt) for x in xs]
    red_g = [fcv2.reduce_requant([send_g[r][j] for r in range(R)], m, fmt) for j in range(R)]
    out_g = fcv2.unpack_dequant_slices(red_g, n, *fmt, torch.bfloat16)
    for j in range(R):
        assert_packed_equal(red_g[j].cpu().numpy(), red_o[j], L, SR, f"reduced slice {j}")
    assert np.array_equal(out_g.view(torch.int16).cpu().numpy().view(np.uint16), out_o)
    # against the exact sum: every term is off by at most half a step of its group (spikes are exact), the sum is
    # rounded to bf16, and the second quantization adds half a step of the output group
    exact = np.sum([W.bf16_bits_to_f32(x).astype(np.float64) for x in xs], axis=0)
    got = W.bf16_bits_to_f32(out_o).astype(np.float64)

    def steps(rec, layout):
        sc = W.bf16_bits_to_f32(rec[layout.off_scale:layout.off_scale + 2 * layout.n_groups].view(np.uint16))
        return np.repeat(sc.astype(np.float64), group)

    bound = np.zeros(n)
    for j in range(R):
        b = sum(steps(send_o[r][j], L) for r in range(R)) * (0.5 + 2.0 ** -7)
        s_exact = np.abs(exact[j * m:(j + 1) * m]) + b
        b = b + s_exact * 2.0 ** -8 + steps(red_o[j], L) * (0.5 + 2.0 ** -7) + s_exact * 2.0 ** -8
        bound[j * m:(j + 1) * m] = b
    assert np.all(np.abs(got - exact) <= bound)


def test_micro_chunks_on_two_streams_match_the_whole_payload():
    """Section 3.4 cuts the payload into micro-chunks and overlaps their stages.  On one GPU: the chunks' quantize ->
    reduce -> unpack chains alternate between two streams.  Groups never straddle a chunk, so the pipelined result
    is bit-identical to processing the whole payload at once, and to the oracle's."""
    N, C, group, bits = 4, 4, 128, 3
    fmt = (bits, group, SR)
    n = C * 2048 * 3
    m = n // C
    xs = [W.tensor(2, p, rows=1, cols=n).reshape(-1) for p in range(N)]
    xd = to_dev_bf16(xs[0])
    others = [[fcv2.quantize_pack(to_dev_bf16(x[c * m:(c + 1) * m]), *fmt) for c in range(C)] for x in xs[1:]]
    L = fcv2.get_layout(m, *fmt)
    q = [torch.zeros(L.total_bytes, dtype=torch.uint8, device=DEV) for _ in range(C)]
    r = [torch.zeros(L.total_bytes, dtype=torch.uint8, device=DEV) for _ in range(C)]
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]  # default priority
    start = torch.cuda.Event()
    start.record()
    for c in range(C):
        st = streams[c % 2]
        st.wait_event(start)
        with torch.cuda.stream(st):
            fcv2.quantize_pack(xd[c * m:(c + 1) * m], *fmt, out=q[c])
            fcv2.reduce_requant([q[c]] + [o[c] for o in others], m, fmt, out=r[c])
            fcv2.unpack_dequant(r[c], m, *fmt, torch.bfloat16, out=out[c * m:(c + 1) * m])
    for st in streams:
        torch.cuda.current_stream().wait_stream(st)
    torch.cuda.synchronize()
    # the whole payload at once
    whole = fcv2.unpack_dequant(fcv2.reduce_requant([fcv2.quantize_pack(to_dev_bf16(x), *fmt) for x in xs], n, fmt), n, *fmt,
                                torch.bfloat16)
    assert torch.equal(out.view(torch.int16), whole.view(torch.int16))
    want = O.unpack_dequant(O.reduce_requant([O.quantize_pack(x, *fmt) for x in xs], n, fmt), n, *fmt, O.DT_BF16)
    assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), want)


# ---- dispatch_quant -------------------------------------------------------------------------------------------------

def check_dispatch(x, ids, E, bits, group, flags, what):
    T, H = x.shape
    send_o, offs_o, src_o = O.dispatch_quant(x, ids, E, bits, group, flags)
    send, offs, src = fcv2.dispatch_quant(to_dev_bf16(x).view(T, H), torch.from_numpy(ids).to(DEV), E, bits, group, flags)
    R = int(offs_o[E])
    assert np.array_equal(offs.cpu().numpy(), offs_o), f"{what}: expert_offsets"
    assert np.array_equal(src.cpu().numpy()[:R], src_o), f"{what}: row_src"
    L = O.get_layout(H, bits, group, flags, 16)
    got = send.cpu().numpy()[:R]
    for name, off, size in sections(L, flags):
        assert np.array_equal(got[:, off:off + size], send_o[:, off:off + size]), f"{what}: rows differ in {name}"


@pytest.mark.parametrize("bits,group,flags", [(2, 128, SR), (3, 32, SR), (4, 64, 0), (5, 128, SR | F32), (7, 256, SR), (8, 128, SR),
                                              (2, 32, SR | INT), (4, 128, INT), (2, 32, SR | IDX16), (6, 256, SR | INT | IDX16)])
def test_dispatch_quant_small(bits, group, flags):
    T, H, K, E = 300, 768, 4, 40  # slots not a multiple of the planning chunk, rows not a multiple of a block
    x = W.tensor(3, 0, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3), T, E, K)
    ids[5, 2] = -1
    ids[9, :] = -1
    ids[T - 1, 0] = -1
    check_dispatch(x, ids, E, bits, group, flags, f"dispatch b{bits} g{group}")


@pytest.mark.parametrize("bits,group,flags", [(2, 128, SR), (3, 32, SR), (4, 64, 0), (5, 128, SR | F32), (6, 32, SR | INT), (7, 64, SR | INT),
                                              (8, 128, SR), (2, 256, SR), (4, 128, SR | INT), (3, 256, F32), (8, 32, 0)])
def test_dispatch_quant_rows_of_whole_kilo_blocks(bits, group, flags):
    """Rows of whole 1024-element blocks (so wave tiles straddle tokens half-way), more formats, and a tensor that
    ends in the middle of a wave."""
    T, H, K, E = 37, 3072, 3, 11
    x = W.tensor(3, 2, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3) + 1, T, E, K)
    ids[4, 1] = -1
    ids[T - 1, :] = -1
    check_dispatch(x, ids, E, bits, group, flags, f"dispatch wide rows b{bits} g{group} f{flags}")


def test_dispatch_quant_nine_copies_per_token():
    T, H, K, E = 20, 1024, 9, 16  # more copies than one batch of destination loads
    x = W.tensor(3, 3, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3) + 2, T, E, K)
    check_dispatch(x, ids, E, 2, 128, SR, "dispatch K=9")
    check_dispatch(x, ids, E, 5, 64, SR, "dispatch K=9 b5")


@pytest.mark.parametrize("bits,group,flags", [(2, 128, SR), (8, 32, SR), (4, 64, SR | INT), (5, 256, F32)])
def test_dispatch_quant_rows_beyond_one_block(bits, group, flags):
    """Rows too long for a block to hold a whole record (32,768 elements = 1,024 lanes), and one length that just fits
    (16,384): two code paths, one result."""
    for T, H in ((5, 32768), (7, 16384)):
        K, E = 3, 7
        x = W.tensor(3, 5, rows=T, cols=H)
        ids = W.topk_routing(W.seed_for(3) + 4, T, E, K)
        ids[1, 1] = -1
        check_dispatch(x, ids, E, bits, group, flags, f"dispatch long rows H{H} b{bits} g{group} f{flags}")


@pytest.mark.parametrize("H,group", [(32, 32), (64, 32), (96, 32), (256, 128), (2560, 256)])
def test_dispatch_quant_short_and_odd_rows(H, group):
    """Rows of one to a few lanes (many tokens per block, the last block short) and a row length that leaves idle lanes."""
    T, K, E = 203, 2, 9
    x = W.tensor(3, 7, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3) + 6, T, E, K)
    ids[0, 0] = -1
    check_dispatch(x, ids, E, 4, group, SR, f"dispatch H{H} g{group}")
    check_dispatch(x, ids, E, 2, group, INT, f"dispatch H{H} g{group} int")


def test_dispatch_quant_send_buffer_off_the_line_grid():
    """The copies are cut on 128-byte lines of the send buffer: every 16-byte phase of the buffer's address gives the
    same bytes."""
    T, H, K, E = 50, 1024, 2, 5
    bits, group, flags = 3, 128, SR
    x = W.tensor(3, 6, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3) + 5, T, E, K)
    want, _, _ = O.dispatch_quant(x, ids, E, bits, group, flags)
    L = fcv2.get_layout(H, bits, group, flags, fcv2.ROW_ALIGN)
    xd, idd = to_dev_bf16(x).view(T, H), torch.from_numpy(ids).to(DEV)
    for phase in range(8):
        back = torch.zeros(T * K * L.total_bytes + 256, dtype=torch.uint8, device=DEV)
        base = (-back.data_ptr()) % 128 + 16 * phase
        send = back[base:base + T * K * L.total_bytes].view(T * K, L.total_bytes)
        fcv2.dispatch_quant(xd, idd, E, bits, group, flags, send_buf=send)
        got = send.cpu().numpy()[:want.shape[0]]
        assert np.array_equal(got, want), f"phase {phase}"
        assert int(back[:base].max() if base else 0) == 0 and int(back[base + T * K * L.total_bytes:].max()) == 0, f"phase {phase}: wrote outside"


def test_dispatch_quant_ids_outside_the_expert_range_are_dropped():
    """An id outside [-1, E) cannot be reported by an asynchronous call without a device-to-host round trip; the
    library documents that it treats such a slot as dropped.  So the result must be the reference result of the same
    routing with those ids replaced by -1 (the reference itself refuses such ids and stays as it is)."""
    T, H, K, E = 257, 512, 4, 24
    x = W.tensor(3, 8, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3) + 9, T, E, K)
    bad = ids.copy()
    rng = np.random.default_rng(5)
    for v in (E, E + 1, 2047, 2048, 1 << 20, 2**31 - 1, -2, -7, -(2**31)):
        t, k = int(rng.integers(T)), int(rng.integers(K))
        bad[t, k] = v
    clean = np.where((bad < 0) | (bad >= E), -1, bad).astype(np.int32)
    assert (clean != ids).sum() >= 5
    with pytest.raises(ValueError):
        O.dispatch_quant(x, bad, E, 2, 128, SR)  # the reference refuses them
    send_o, offs_o, src_o = O.dispatch_quant(x, clean, E, 2, 128, SR)
    send, offs, src = fcv2.dispatch_quant(to_dev_bf16(x).view(T, H), torch.from_numpy(bad).to(DEV), E, 2, 128, SR)
    R = int(offs_o[E])
    assert np.array_equal(offs.cpu().numpy(), offs_o)
    assert np.array_equal(src.cpu().numpy()[:R], src_o)
    assert np.array_equal(send.cpu().numpy()[:R], send_o)


@pytest.mark.parametrize("E", [257, 1024, 1025, 2048])
def test_dispatch_quant_many_experts(E):
    """More experts than one lane-mask table or one four-word share per lane holds: the planning kernels switch to their
    general paths (ballot rounds for the in-chunk ranks, looped reads of the expert totals)."""
    T, H, K = 700, 256, 6
    x = W.tensor(3, 9, rows=T, cols=H)
    rng = np.random.default_rng(E)
    ids = rng.integers(0, E, (T, K)).astype(np.int32)
    ids[rng.integers(0, T, 40), rng.integers(0, K, 40)] = -1
    ids[:50, 0] = E - 1  # a run of one expert across wave and chunk borders
    check_dispatch(x, ids, E, 3, 128, SR, f"dispatch E={E}")


def test_dispatch_quant_degenerate_routing():
    T, H, K, E = 130, 512, 8, 256
    x = W.tensor(3, 1, rows=T, cols=H)
    one = np.full((T, K), 7, np.int32)  # every copy to one expert: longest possible stable run
    check_dispatch(x, one, E, 2, 128, SR, "all to one expert")
    none = np.full((T, K), -1, np.int32)  # nothing routed
    send, offs, src = fcv2.dispatch_quant(to_dev_bf16(x).view(T, H), torch.from_numpy(none).to(DEV), E, 2, 128, SR)
    assert int(offs.cpu().numpy().max()) == 0


def test_dispatch_maximum_input_size():
    """T x H = 2^31 elements (262,144 tokens of 8,192, one copy each): 1,024 seeded tokens repeated on the GPU.  The
    routing is checked against its definition (stable sort by expert), every row against the oracle's record of its
    token."""
    bits, group, flags = 2, 128, SR
    base_T, H, E, K = 1024, 8192, 64, 1
    reps = (1 << 31) // (base_T * H)
    T = base_T * reps
    base = W.tensor(3, 4, rows=base_T, cols=H)
    x = to_dev_bf16(base).view(base_T, H).repeat(reps, 1)
    rng = np.random.default_rng(77)
    ids = rng.integers(0, E, (T, K)).astype(np.int32)
    ids[rng.integers(0, T, 1000), 0] = -1
    send, offs, src = fcv2.dispatch_quant(x, torch.from_numpy(ids).to(DEV), E, bits, group, flags)
    flat = ids.reshape(-1)
    routed = np.nonzero(flat >= 0)[0]
    order = routed[np.argsort(flat[routed], kind="stable")]
    R = order.size
    want_offs = np.concatenate([[0], np.cumsum(np.bincount(flat[routed], minlength=E))]).astype(np.int32)
    assert np.array_equal(offs.cpu().numpy(), want_offs)
    assert np.array_equal(src.cpu().numpy()[:R], order.astype(np.int32))
    L = O.get_layout(H, bits, group, flags, 16)
    rows_o = np.stack([O.quantize_pack(base[t], bits, group, flags, align=16) for t in range(base_T)])
    rows_d = torch.from_numpy(rows_o).to(DEV)
    tok = torch.from_numpy((order // K) % base_T).to(DEV)
    for name, off, size in sections(L, flags):
        assert torch.equal(send[:R, off:off + size], rows_d[tok][:, off:off + size]), f"max dispatch: section {name}"


# ---- the five workloads at full size, in the launch configuration the benchmark times ----------------------------------

def test_workload1_full():
    x = W.tensor(1, 0).reshape(-1)
    check_codec(x, 4, 128, SR, "workload 1")
    xs = [W.tensor(1, p).reshape(-1) for p in range(4)]
    check_reduce(xs, 4, 128, SR, "workload 1 N4")


@pytest.mark.parametrize("bits", [3, 2, 4, 5, 6, 7, 8])
def test_workload2_full(bits):
    xs = [W.tensor(2, p).reshape(-1) for p in range(8)]
    check_codec(xs[0], bits, 128, SR, f"workload 2 b{bits}")
    check_reduce(xs, bits, 128, SR, f"workload 2 b{bits} N8")


def test_workload2_paper_default_low_bit_shape():
    """Section 4.1's default for INT2: groups of 32, spike reserving, integer scale and zero (Eq. 1, Table 4); and the
    table's first row (bf16 scale and zero, spike positions as BF16 numbers) on the sender and the receiver."""
    xs = [W.tensor(2, p).reshape(-1) for p in range(8)]
    check_codec(xs[0], 2, 32, SR | INT, "workload 2 b2 g32 integer meta")
    check_reduce(xs, 2, 32, SR | INT, "workload 2 b2 g32 integer meta N8")
    check_codec(xs[0], 2, 32, SR | IDX16, "workload 2 b2 g32 BF16 positions")


def test_workload3_full():
    w = W.WORKLOADS[3]
    x = W.tensor(3, 0)
    ids = W.topk_routing(W.seed_for(3), w["rows"], w["experts"], w["topk"])
    check_dispatch(x, ids, w["experts"], 2, 128, SR, "workload 3")


@pytest.mark.parametrize("bits,group", [(5, 64), (5, 256), (6, 64), (6, 256)])
def test_workload4_full(bits, group):
    xs = [W.tensor(4, p).reshape(-1) for p in range(8)]
    check_codec(xs[0], bits, group, SR, f"workload 4 b{bits} g{group}")
    check_reduce(xs, bits, group, SR, f"workload 4 b{bits} g{group} N8")


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_workload5_full(bits):
    xs = [W.tensor(5, p).reshape(-1) for p in range(8)]
    g = check_codec(xs[0], bits, 128, SR, f"workload 5 b{bits}")
    # back-to-back calls on one stream give the same record every time
    xd = to_dev_bf16(xs[0])
    outs = [fcv2.quantize_pack(xd, bits, 128, SR) for _ in range(50)]
    torch.cuda.synchronize()
    assert all(torch.equal(o, g) for o in outs)
    check_reduce(xs, bits, 128, SR, f"workload 5 b{bits} N8")
