"""Seeded synthetic inputs for the five benchmark/parity workloads.

Data only: nothing here quantizes, packs or reduces.  Both the HIP library's tests and the CPU oracle's
tests draw their inputs from this module, so the two sides always see the same bits.  The generator is a
counter-based splitmix64 (value i of stream k depends only on (seed, i, k)), so results do not depend on
chunking, threading or the numpy version.  Activations of real models are not available offline; these
distributions stand in for them (heavy-tailed, per-channel scaled, with injected outliers).

bf16 tensors are returned as numpy uint16 bit patterns.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 21
_STREAMS = 4  # uniforms available per element


def seed_for(cfg: int, peer: int = 0) -> int:
    return 0xFC520000 + 0x100 * cfg + peer


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def uniform(seed: int, start: int, count: int, stream: int) -> np.ndarray:
    """float64 uniforms in (0, 1] for elements start..start+count of one stream."""
    with np.errstate(over="ignore"):
        i = np.arange(start, start + count, dtype=np.uint64)
        ctr = i * np.uint64(_STREAMS) + np.uint64(stream) + np.uint64(1)
        z = _mix(_mix(np.uint64(seed)) + ctr * _GOLD)
    return ((z >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def _normal_pair(seed, start, count):
    u1 = uniform(seed, start, count, 0)
    u2 = uniform(seed, start, count, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    a = (2.0 * np.pi) * u2
    return r * np.cos(a), r * np.sin(a), u1


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of finite float32 values to bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _chunked(n, fn, threads=8):
    out = np.empty(n, np.uint16)
    spans = [(s, min(_CHUNK, n - s)) for s in range(0, n, _CHUNK)]

    def work(span):
        s, c = span
        out[s:s + c] = fn(s, c)

    if len(spans) == 1:
        work(spans[0])
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, spans))
    return out


def _outliers(v, seed, start, count, prob=0.001, factor=50.0):
    u = uniform(seed, start, count, 2)
    hit = u <= prob
    sign = np.where(u <= prob / 2, -1.0, 1.0)
    return np.where(hit, v * factor * sign, v)


def column_scales(seed: int, n_blocks: int, sigma: float = 0.5) -> np.ndarray:
    z, _, _ = _normal_pair(seed ^ 0x5CA1E5, 0, n_blocks)
    return np.exp(sigma * z)


def activations(seed: int, rows: int, cols: int, col_block: int = 128, channel_scale: bool = True) -> np.ndarray:
    """N(0,1) times a lognormal(0, 0.5) scale per block of `col_block` columns (shared by all rows);
    0.1 % of the elements multiplied by +-50.  Shape [rows, cols], bf16 bits.  (Workloads 1, 2, 3.)"""
    n = rows * cols
    c = column_scales(seed, -(-cols // col_block)) if channel_scale else None  # a last, shorter block gets a scale too

    def fn(s, cnt):
        z, _, _ = _normal_pair(seed, s, cnt)
        if c is not None:
            col = (np.arange(s, s + cnt, dtype=np.int64) % cols) // col_block
            z = z * c[col]
        z = _outliers(z, seed, s, cnt)
        return f32_to_bf16_bits(z.astype(np.float32))

    return _chunked(n, fn).reshape(rows, cols)


def student_t3(seed: int, rows: int, cols: int, scale: float = 0.02) -> np.ndarray:
    """scale * Student-t with 3 degrees of freedom: Z0 / sqrt((Z1^2 + E) / 3) where E = -2 ln U is the sum
    of two squared standard normals (chi-square with 2 degrees of freedom).  (Workload 4.)"""
    n = rows * cols

    def fn(s, cnt):
        z0, z1, _ = _normal_pair(seed, s, cnt)
        e = -2.0 * np.log(uniform(seed, s, cnt, 2))
        t = z0 / np.sqrt((z1 * z1 + e) / 3.0)
        return f32_to_bf16_bits((scale * t).astype(np.float32))

    return _chunked(n, fn).reshape(rows, cols)


def decode_spiky(seed: int, rows: int, cols: int, group: int = 128, spike: float = 100.0) -> np.ndarray:
    """N(0,1) with exactly one element per group of `group` set to +-spike at a seeded position.  (Workload 5.)"""
    n = rows * cols
    z, _, _ = _normal_pair(seed, 0, n)
    ng = n // group
    u = uniform(seed ^ 0x51DE, 0, ng, 0)
    v = uniform(seed ^ 0x51DE, 0, ng, 1)
    pos = np.minimum((u * group).astype(np.int64), group - 1)
    z[np.arange(ng) * group + pos] = np.where(v <= 0.5, -spike, spike)  # elements past the last whole group stay plain
    return f32_to_bf16_bits(z.astype(np.float32)).reshape(rows, cols)


def topk_routing(seed: int, tokens: int, experts: int, k: int, zipf_a: float = 1.1) -> np.ndarray:
    """k distinct experts per token, drawn without replacement with weights (e+1)^-a (exponential race).
    Returns int32 [tokens, k], in order of selection."""
    w = (np.arange(1, experts + 1, dtype=np.float64)) ** (-zipf_a)
    u = uniform(seed ^ 0x70C4, 0, tokens * experts, 0).reshape(tokens, experts)
    race = -np.log(u) / w
    return np.argsort(race, axis=1, kind="stable")[:, :k].astype(np.int32)


# ---- the five workloads -----------------------------------------------------------------------------------

WORKLOADS = {
    1: dict(name="cfg1_1M_b4_g128", rows=256, cols=4096, bits=(4,), groups=(128,), peers=4),
    2: dict(name="cfg2_llama8b_allreduce_4096x4096", rows=4096, cols=4096, bits=(3, 2, 4, 5, 6, 7, 8),
            groups=(128,), peers=8),
    3: dict(name="cfg3_dsv3_dispatch_8192x7168", rows=8192, cols=7168, bits=(2,), groups=(128,), experts=256, topk=8),
    4: dict(name="cfg4_large_allreduce_8192x8192", rows=8192, cols=8192, bits=(5, 6), groups=(64, 256), peers=8),
    5: dict(name="cfg5_decode_64x7168", rows=64, cols=7168, bits=(2, 3, 4), groups=(128,), peers=8),
}


def tensor(cfg: int, peer: int = 0, rows: int = None, cols: int = None) -> np.ndarray:
    """bf16 bits of workload `cfg`, peer chunk `peer` (optionally at a reduced shape for quick tests)."""
    w = WORKLOADS[cfg]
    rows = rows or w["rows"]
    cols = cols or w["cols"]
    seed = seed_for(cfg, peer)
    if cfg in (1, 2):
        return activations(seed, rows, cols)
    if cfg == 3:
        return activations(seed, rows, cols, channel_scale=False)
    if cfg == 4:
        return student_t3(seed, rows, cols)
    if cfg == 5:
        return decode_spiky(seed, rows, cols)
    raise KeyError(cfg)
