"""The hot path under HIP graph capture: the library only launches kernels on the caller's stream (no allocation,
no memset, no synchronisation), so a caller may record the three calls once and replay them.  Every replay is
checked against eager calls on the same inputs, with eager work and synchronisation between the replays, and the
first one against the CPU oracle as well."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2508_03760_amd import fcv2
from paper_2508_03760_amd import workloads as W

pytestmark = pytest.mark.gpu
SR = fcv2.F_SPIKE
DEV = "cuda:0"


def to_dev_bf16(bits_u16):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).to(DEV).view(torch.bfloat16)


@pytest.mark.parametrize("bits,group,flags", [(3, 128, SR), (2, 32, SR | fcv2.F_META_INT)])
def test_step_replays_under_graph_capture(bits, group, flags):
    assert torch.cuda.is_available()
    fmt = (bits, group, flags)
    hosts = [W.tensor(5, p).reshape(-1) for p in range(8)]  # the decode-sized payload: launch-bound, the case for graphs
    n = hosts[0].size
    L = fcv2.get_layout(n, *fmt)
    x = to_dev_bf16(hosts[0]).clone()
    others = [fcv2.quantize_pack(to_dev_bf16(h), *fmt) for h in hosts[1:]]
    q = torch.zeros(L.total_bytes, dtype=torch.uint8, device=DEV)
    r = torch.zeros(L.total_bytes, dtype=torch.uint8, device=DEV)
    o = torch.empty(n, dtype=torch.bfloat16, device=DEV)

    def step(q, r, o):
        fcv2.quantize_pack(x, *fmt, out=q)
        fcv2.reduce_requant([q] + others, n, fmt, out=r)
        fcv2.unpack_dequant(r, n, *fmt, torch.bfloat16, out=o)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(q, r, o)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(q, r, o)
    torch.cuda.synchronize()

    for trial, src in enumerate((0, 3, 6, 0)):
        x.copy_(to_dev_bf16(hosts[src]))
        q.fill_(0xAB)
        r.fill_(0xCD)
        o.fill_(7.0)  # stale contents must not survive a replay
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        q2, r2, o2 = torch.zeros_like(q), torch.zeros_like(r), torch.empty_like(o)
        step(q2, r2, o2)  # eager, between the replays
        torch.cuda.synchronize()
        # padding bytes between sections are never written: compare the sections only
        lay = O.get_layout(n, *fmt)
        m = 1 if flags & fcv2.F_META_INT else 2
        secs = [(getattr(lay, f"off_plane{w}"), n * w // 8) for w in (8, 4, 2, 1) if getattr(lay, f"off_plane{w}") != O.ABSENT]
        secs += [(lay.off_scale, m * lay.n_groups), (lay.off_zero, m * lay.n_groups),
                 (lay.off_spike_val, 4 * lay.n_groups), (lay.off_spike_idx, 2 * lay.n_groups)]
        for off, size in secs:
            assert torch.equal(q[off:off + size], q2[off:off + size]), f"replay {trial}: quantize_pack differs"
            assert torch.equal(r[off:off + size], r2[off:off + size]), f"replay {trial}: reduce_requant differs"
        assert torch.equal(o.view(torch.int16), o2.view(torch.int16)), f"replay {trial}: unpack_dequant differs"
        if trial == 0:
            peers_o = [O.quantize_pack(h, *fmt) for h in hosts]
            want = O.unpack_dequant(O.reduce_requant(peers_o, n, fmt), n, *fmt, O.DT_BF16)
            assert np.array_equal(o.view(torch.int16).cpu().numpy().view(np.uint16), want)


def test_dispatch_replays_under_graph_capture():
    """fcv2_dispatch_quant is four launches on the caller's stream and nothing else: recorded once, replayed with new
    tokens and new routing in the same buffers, every replay equals the eager call and the oracle."""
    T, H, K, E = 96, 2048, 4, 12
    bits, group, flags = 2, 128, SR
    L = fcv2.get_layout(H, bits, group, flags, fcv2.ROW_ALIGN)
    x = torch.zeros((T, H), dtype=torch.bfloat16, device=DEV)
    ids = torch.zeros((T, K), dtype=torch.int32, device=DEV)

    def bufs():
        return dict(send_buf=torch.zeros((T * K, L.total_bytes), dtype=torch.uint8, device=DEV),
                    expert_offsets=torch.zeros(E + 1, dtype=torch.int32, device=DEV),
                    row_src=torch.zeros(T * K, dtype=torch.int32, device=DEV),
                    workspace=torch.empty(fcv2.dispatch_workspace_bytes(T, K, E), dtype=torch.uint8, device=DEV))

    b = bufs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fcv2.dispatch_quant(x, ids, E, bits, group, flags, **b)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fcv2.dispatch_quant(x, ids, E, bits, group, flags, **b)
    torch.cuda.synchronize()
    for trial in range(3):
        xh = W.tensor(3, 8 + trial, rows=T, cols=H)
        idh = W.topk_routing(W.seed_for(3) + 10 + trial, T, E, K)
        idh[trial, 0] = -1
        x.copy_(to_dev_bf16(xh).view(T, H))
        ids.copy_(torch.from_numpy(idh))
        b["send_buf"].fill_(0xEE)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        e = bufs()
        fcv2.dispatch_quant(x, ids, E, bits, group, flags, **e)  # eager, between the replays
        torch.cuda.synchronize()
        want, offs, src = O.dispatch_quant(xh, idh, E, bits, group, flags)
        R = int(offs[E])
        assert np.array_equal(b["expert_offsets"].cpu().numpy(), offs), f"replay {trial}: offsets"
        assert np.array_equal(b["row_src"].cpu().numpy()[:R], src), f"replay {trial}: row_src"
        assert np.array_equal(b["send_buf"].cpu().numpy()[:R], want), f"replay {trial}: rows differ from the oracle"
        assert torch.equal(b["send_buf"][:R], e["send_buf"][:R]), f"replay {trial}: rows differ from the eager call"
