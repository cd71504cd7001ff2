"""GPU parity on seeded random cases: formats, sizes, peer counts, routing and value patterns drawn at random
(normal values at three magnitudes, injected outliers, constant tensors, integers with many ties, all-zero groups,
bf16 denormals, values near the largest finite bf16, signed zeros), every output compared with the CPU oracle bit
for bit.  The sizes are small, so that the oracle is quick; the cases are many."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2508_03760_amd import fcv2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FLAGS = [0, 1, 2, 3, 4, 5]  # spike reserving x (bf16 | fp32 | integer) metadata


def bf16_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def dev16(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)


def values(rng, n, group):
    kind = int(rng.integers(0, 8))
    x = rng.standard_normal(n) * rng.choice([1e-4, 1.0, 300.0])
    if kind == 1:
        x[rng.random(n) < 0.01] *= 50
    elif kind == 2:
        x[:] = x[0]
    elif kind == 3:
        x = np.round(x)
    elif kind == 4:
        g = int(rng.integers(0, n // group))
        x[g * group:(g + 1) * group] = 0.0
    elif kind == 5:
        x = x * 1e-38
    elif kind == 6:
        x = np.clip(x * 1e36, -3.3e38, 3.3e38)  # the range of a group overflows fp32: infinite scale, NaN on decode
    elif kind == 7:
        x = np.where(rng.random(n) < 0.5, 0.0, -0.0) + (rng.random(n) < 0.05) * x
    return bf16_bits(x)


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_random_tensors_all_calls(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(150):
        group = int(rng.choice([32, 64, 128, 256]))
        bits = int(rng.integers(2, 9))
        flags = int(rng.choice(FLAGS))
        n = group * int(rng.integers(1, max(2, 1 << int(rng.integers(3, 13)))))
        n -= n % 8
        if n < group or n % group:
            n = group * 8
        what = f"seed {seed} case {case}: n {n} b{bits} g{group} f{flags}"
        xb = values(rng, n, group)
        want = O.quantize_pack(xb, bits, group, flags)
        got = fcv2.quantize_pack(dev16(xb), bits, group, flags)
        assert np.array_equal(got.cpu().numpy(), want), f"quantize_pack {what}"
        d32 = fcv2.unpack_dequant(got, n, bits, group, flags, torch.float32).cpu().numpy()
        assert np.array_equal(d32.view(np.uint32), O.unpack_dequant(want, n, bits, group, flags, O.DT_FP32).view(np.uint32)), f"unpack fp32 {what}"
        d16 = fcv2.unpack_dequant(got, n, bits, group, flags, torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(d16, O.unpack_dequant(want, n, bits, group, flags, O.DT_BF16)), f"unpack bf16 {what}"
        n_peers = int(rng.integers(1, 17))
        fout = (int(rng.integers(2, 9)) if rng.random() < 0.5 else bits, group, (flags & 1) | int(rng.choice([0, 2, 4])))
        peers = [O.quantize_pack(values(rng, n, group), bits, group, flags) for _ in range(n_peers)]
        w_r, w_s = O.reduce_requant(peers, n, (bits, group, flags), fout, want_sum=True)
        g_r, g_s = fcv2.reduce_requant([torch.from_numpy(p).to(DEV) for p in peers], n, (bits, group, flags), fout, want_sum=True)
        assert np.array_equal(g_s.cpu().numpy().view(np.uint32), w_s.view(np.uint32)), f"reduce sums {what} -> {fout} N{n_peers}"
        assert np.array_equal(g_r.cpu().numpy(), w_r), f"reduce_requant {what} -> {fout} N{n_peers}"


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_dispatch(seed):
    rng = np.random.default_rng(2000 + seed)
    for case in range(200):
        group = int(rng.choice([32, 64, 128, 256]))
        bits = int(rng.integers(2, 9))
        flags = int(rng.choice(FLAGS))
        kind = int(rng.integers(0, 4))
        if kind == 0:
            H = group * int(rng.integers(1, 9))
        elif kind == 1:
            H = group * int(rng.integers(1, 80))
        elif kind == 2:
            H = int(rng.choice([4096, 5120, 7168, 8192, 16384, 16384 + group, 32768]))  # the last two: the direct kernel
        else:
            H = 256 * int(rng.integers(1, 40))
        H = max(group, H - H % group)
        T = int(rng.integers(1, max(1, min(400, (3 << 20) // H)) + 1))
        K, E = int(rng.integers(1, 13)), int(rng.integers(1, 300))
        what = f"seed {seed} case {case}: T{T} H{H} K{K} E{E} b{bits} g{group} f{flags}"
        x = (rng.standard_normal((T, H)) * rng.choice([1e-3, 1.0, 50.0])).astype(np.float32)
        if rng.random() < 0.3:
            x[int(rng.integers(0, T))] = x[0, 0]  # a constant token
        if rng.random() < 0.2:
            x = np.round(x)
        xb = bf16_bits(x)
        ids = rng.integers(-1 if rng.random() < 0.5 else 0, E, size=(T, K)).astype(np.int32)
        want, offs_o, src_o = O.dispatch_quant(xb, ids, E, bits, group, flags)
        send, offs, src = fcv2.dispatch_quant(dev16(xb).view(T, H), torch.from_numpy(ids).to(DEV), E, bits, group, flags)
        R = int(offs_o[E])
        assert np.array_equal(offs.cpu().numpy(), offs_o), f"expert_offsets {what}"
        assert np.array_equal(src.cpu().numpy()[:R], src_o), f"row_src {what}"
        assert np.array_equal(send.cpu().numpy()[:R], want), f"rows {what}"
