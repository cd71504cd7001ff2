"""Direction of Table 3 (Section 3.3) on synthetic activations, CPU only: at 32 values per group spike reserving has
the best signal-to-noise ratio of the four methods at INT4, INT3 and INT2; the gap to plain RTN grows as the width
shrinks; and at INT2 the two comparison methods fall behind (LogFMT keeps one magnitude per group; the rotation spreads
every outlier over its whole block before a 4-level quantizer).  The paper's numbers are perplexities of trained
models and are not reproduced here; the comparison methods are minimal numpy forms (oracle/quality.py)."""
import numpy as np

import oracle.quality as Q
from paper_2508_03760_amd import workloads as W


def test_hadamard_is_orthonormal_and_logfmt_is_exact_where_it_can_be():
    H = Q.hadamard(128)
    assert np.allclose(H @ H.T, np.eye(128), atol=1e-12)
    # eight bits are plenty for a group of equal magnitudes and mixed signs, zeros included
    x = np.array([0.5, -0.5, 0.0, 0.5] * 8)
    assert np.allclose(Q.logfmt(x, 8, 32), x)
    # two bits: sign and one magnitude per group
    y = Q.logfmt(np.array([1.0, -4.0, 2.0, 0.0] * 8), 2, 32)
    assert set(np.unique(np.abs(y))) <= {0.0, 4.0}


def test_direction_of_table3_on_synthetic_activations():
    x = W.tensor(2, 0, rows=64, cols=4096).reshape(-1)  # outlier-injected, per-channel scaled
    t = Q.table(x, group=32)
    for b in (4, 3, 2):
        best = max(t[b], key=t[b].get)
        assert best == "spike_reserving", (b, t[b])
    gain = {b: t[b]["spike_reserving"] - t[b]["rtn"] for b in (4, 3, 2)}
    assert min(gain.values()) > 1.0, gain  # reserving the spikes is worth decibels at every width
    # Table 3's other direction: the comparison methods hold up at INT4 and fall furthest behind spike reserving at INT2
    assert t[2]["logfmt"] < t[2]["rtn"] and t[2]["logfmt"] < t[2]["spike_reserving"] - 6.0
    assert t[2]["hadamard"] < t[2]["spike_reserving"]
    assert t[4]["logfmt"] > t[2]["logfmt"] + 6.0 and t[4]["hadamard"] > t[2]["hadamard"] + 6.0
