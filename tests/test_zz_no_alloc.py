"""The dispatch entry point that allocates nothing (fcv2_dispatch_quant_noalloc: planning scratch in a static device
array) against fcv2_dispatch_quant, through the C ABI: two calls in a row on one stream, the second with a smaller
input, every output byte for byte; then the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2508_03760_amd import fcv2
from paper_2508_03760_amd import workloads as W

pytestmark = pytest.mark.gpu

SR = fcv2.F_SPIKE
DEV = "cuda:0"


def _inputs(T, H, K, E, seed):
    x = W.tensor(3, seed, rows=T, cols=H)
    ids = W.topk_routing(W.seed_for(3) + seed, T, E, K)
    ids[T // 3, 0] = -1
    xd = torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16).view(T, H)
    return xd, torch.from_numpy(ids).to(DEV)


def _outputs(T, K, E, row_bytes, fill):
    return (torch.full((T * K, row_bytes), fill, dtype=torch.uint8, device=DEV),
            torch.full((E + 1,), -7, dtype=torch.int32, device=DEV),
            torch.full((T * K,), -7, dtype=torch.int32, device=DEV))


def test_noalloc_dispatch_equals_the_workspace_call_twice_in_a_row():
    assert torch.cuda.is_available()
    fcv2.lib()
    bits, group = 2, 128
    cases = [(2048, 1024, 8, 64, 11), (300, 768, 4, 40, 12)]  # the second call is smaller: stale scratch must not matter
    results = []
    # the very first launch from a code object makes the runtime load it (that takes device memory once per process):
    # get that out of the way with a tiny call before watching the free memory
    xd, idd = _inputs(16, 128, 2, 4, 10)
    fcv2.dispatch_quant_noalloc(xd, idd, 4, bits, group, SR, *_outputs(16, 2, 4, fcv2.get_layout(128, bits, group, SR, fcv2.ROW_ALIGN).total_bytes, 0))
    torch.cuda.synchronize()
    for T, H, K, E, seed in cases:
        xd, idd = _inputs(T, H, K, E, seed)
        L = fcv2.get_layout(H, bits, group, SR, fcv2.ROW_ALIGN)
        assert fcv2.dispatch_workspace_bytes(T, K, E) <= fcv2.STATIC_SCRATCH_BYTES
        got = _outputs(T, K, E, L.total_bytes, 0)
        free_before = torch.cuda.mem_get_info()[0]
        fcv2.dispatch_quant_noalloc(xd, idd, E, bits, group, SR, *got)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before  # the call took no device memory
        results.append((xd, idd, E, L, got))
    for xd, idd, E, L, got in results:
        T, K = idd.shape
        want = _outputs(T, K, E, L.total_bytes, 0)
        fcv2.dispatch_quant(xd, idd, E, bits, group, SR, send_buf=want[0], expert_offsets=want[1], row_src=want[2])
        torch.cuda.synchronize()
        R = int(want[1][E])
        assert R > 0 and torch.equal(got[1], want[1]), "expert_offsets"
        assert torch.equal(got[2][:R], want[2][:R]), "row_src"
        assert torch.equal(got[0][:R], want[0][:R]), "send buffer rows"
        assert torch.equal(got[2][R:], want[2][R:]) and torch.equal(got[0][R:], want[0][R:]), "rows past the routed ones untouched"


def test_noalloc_dispatch_other_format_after_the_first():
    """A third and fourth call with another format and integer metadata, larger then smaller again, on a side stream."""
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for (T, H, K, E, seed), (bits, group, flags) in (((1024, 2048, 8, 256, 13), (4, 32, SR | fcv2.F_META_INT)),
                                                           ((64, 512, 2, 8, 14), (8, 64, 0))):
            xd, idd = _inputs(T, H, K, E, seed)
            L = fcv2.get_layout(H, bits, group, flags, fcv2.ROW_ALIGN)
            got = _outputs(T, K, E, L.total_bytes, 0)
            want = _outputs(T, K, E, L.total_bytes, 0)
            fcv2.dispatch_quant_noalloc(xd, idd, E, bits, group, flags, *got)
            fcv2.dispatch_quant(xd, idd, E, bits, group, flags, send_buf=want[0], expert_offsets=want[1], row_src=want[2])
            st.synchronize()
            for g, w in zip(got, want):
                assert torch.equal(g, w)


def test_noalloc_dispatch_refuses_shapes_beyond_the_static_scratch():
    T, H, K, E = 8192, 128, 8, 2048  # 256 chunks x 2048 experts x 4 bytes = 2 MiB of histograms alone
    assert fcv2.dispatch_workspace_bytes(T, K, E) > fcv2.STATIC_SCRATCH_BYTES
    xd = torch.zeros((T, H), dtype=torch.bfloat16, device=DEV)
    idd = torch.zeros((T, K), dtype=torch.int32, device=DEV)
    L = fcv2.get_layout(H, 2, 128, SR, fcv2.ROW_ALIGN)
    out = _outputs(T, K, E, L.total_bytes, 0)
    with pytest.raises(fcv2.Fcv2Error, match="static scratch"):
        fcv2.dispatch_quant_noalloc(xd, idd, E, 2, 128, SR, *out)
    rc = fcv2.lib().fcv2_dispatch_quant_noalloc(None, None, 16, 128, 2, 4, None, None, None, None, None)
    assert rc == -1  # null arguments: invalid argument, nothing launched
