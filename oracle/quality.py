"""Quality proxy for Section 3.3 / Table 3: signal-to-quantization-noise of the four methods the table compares --
plain round-to-nearest (RTN), RTN after a Hadamard rotation, LogFMT, and spike reserving -- on synthetic activations.

TEST INFRASTRUCTURE ONLY (numpy, float64), like the rest of oracle/.  The table's own figures are C4 perplexities
of trained models, which cannot be reproduced offline; this checks the DIRECTION only.  RTN and spike reserving go
through the oracle's codec.  The two comparison methods are minimal forms of the published ideas, written here
from their descriptions:
  * Hadamard: every block of `block` consecutive values is multiplied by the orthonormal Walsh-Hadamard matrix
    (which spreads an outlier over the block), quantized with plain group RTN, and rotated back.
  * LogFMT-n: one sign bit and n-1 bits of magnitude per value; magnitudes are quantized uniformly in the log domain
    between the group's smallest and largest log|x| (the smallest clamped to 32 octaves below the largest), code 0
    stands for zero.  With n = 2 a group has a single magnitude level.
"""
import numpy as np

import oracle as O
from paper_2508_03760_amd import workloads as W


def sqnr_db(x, v):
    x, v = np.asarray(x, np.float64), np.asarray(v, np.float64)
    return float(10.0 * np.log10(np.sum(x * x) / np.sum((v - x) ** 2)))


def codec(x_bits, bits, group, flags):
    """Decoded fp32 values of the oracle's quantize_pack -> unpack_dequant round trip."""
    n = x_bits.size
    return O.unpack_dequant(O.quantize_pack(x_bits, bits, group, flags), n, bits, group, flags)


def hadamard(n):
    h = np.array([[1.0]])
    while h.shape[0] < n:
        h = np.block([[h, h], [h, -h]])
    assert h.shape[0] == n, "block size must be a power of two"
    return h / np.sqrt(n)


def hadamard_rtn(x, bits, group, block=128):
    """Rotate blocks of `block` values, asymmetric min-max RTN per group in float64, rotate back."""
    x = np.asarray(x, np.float64)
    H = hadamard(block)
    r = (x.reshape(-1, block) @ H).reshape(-1, group)
    lo, hi = r.min(axis=1, keepdims=True), r.max(axis=1, keepdims=True)
    qmax = 2 ** bits - 1
    s = np.where(hi > lo, (hi - lo) / qmax, 1.0)
    q = np.clip(np.rint((r - lo) / s), 0, qmax)
    back = (q * s + lo).reshape(-1, block) @ H.T
    return back.reshape(-1)


def logfmt(x, bits, group):
    x = np.asarray(x, np.float64).reshape(-1, group)
    mag = np.abs(x)
    nz = mag > 0
    with np.errstate(divide="ignore"):
        L = np.where(nz, np.log(np.where(nz, mag, 1.0)), -np.inf)
    Lmax = L.max(axis=1, keepdims=True)
    Lmin = np.maximum(np.where(nz, L, np.inf).min(axis=1, keepdims=True), Lmax - 32.0 * np.log(2.0))
    levels = 2 ** (bits - 1) - 1  # codes 1..levels carry magnitudes, code 0 is zero
    step = np.where(levels > 1, (Lmax - Lmin) / max(levels - 1, 1), 0.0)
    with np.errstate(invalid="ignore", divide="ignore"):
        k = np.where(step > 0, np.rint((np.maximum(L, Lmin) - Lmin) / np.where(step > 0, step, 1.0)), levels - 1.0)
    k = np.clip(k, 0, levels - 1)
    # a single level (n = 2) sits at the top of the range: the largest value is what the format keeps
    dec = np.exp(np.where(levels > 1, Lmin + k * step, Lmax + 0.0 * k))
    out = np.where(nz & np.isfinite(Lmax), np.sign(x) * dec, 0.0)
    return out.reshape(-1)


def table(x_bits, group=32, widths=(4, 3, 2)):
    """{bits: {method: SQNR in dB}} for the four methods of Table 3 at one group size."""
    xf = W.bf16_bits_to_f32(x_bits).astype(np.float64)
    out = {}
    for b in widths:
        out[b] = {
            "rtn": sqnr_db(xf, codec(x_bits, b, group, 0)),
            "hadamard": sqnr_db(xf, hadamard_rtn(xf, b, group)),
            "logfmt": sqnr_db(xf, logfmt(xf, b, group)),
            "spike_reserving": sqnr_db(xf, codec(x_bits, b, group, O.F_SPIKE)),
        }
    return out
