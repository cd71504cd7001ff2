"""Benchmark of libfcv2 on one MI355X.

One "step" is the pair of calls the metric names, on the Llama-3-8B-shaped AllReduce payload (bf16 [4096 x 4096],
3-bit = 2+1 split, group 128, spike reserving, 8 simulated peer chunks):
    fcv2_quantize_pack(x)  ->  fcv2_reduce_requant(8 packed peer chunks)
`value` = algorithmic bytes of the two calls / time of a step (effective HBM GB/s).  The step with the third local call
of a two-step quantized AllReduce added (fcv2_unpack_dequant of the result) is reported beside it as
`three_call_step`.  All inputs are resident in HBM before the timed region.  Buffer sets are rotated so that every step
reads lines that are not in the 256 MB last-level cache (the working set of one step is smaller than that cache).
Before the warm-up the same step runs untimed for about 30 ms, so that the GPU is at its sustained clocks when the W
warm-up steps and the K timed steps run; the figure is sustained throughput, not the first milliseconds after idling.

Prints ONE JSON line.  `roofline` is the dominant kernel (reduce_requant) against HBM: algorithmic bytes per launch
divided by its launch duration, measured here with HIP events on the launch stream, over the 8 TB/s peak; `traffic` and
the instruction counts of `alu_roofline` are read from the committed rocprofv3 summary under profiles/ (counters cannot
be read inside this process).  Extra keys: per-kernel figures, a sweep over bit widths 2..8, the dispatch workload and
the CPU oracle timed beside it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
LLC_BYTES = 256 << 20
ALU_PEAK_TLOPS = 256 * 4 * 16 * 2.4e9 / 1e12  # 39.3 T lane-operations/s: VALU issue without packed fp32
PROFILE = os.path.join(ROOT, "profiles", "headline_step_b3_g128_n8.md")


def profile_counters(path=PROFILE):
    """Per-kernel counter figures of the headline shape from the committed rocprofv3 summary: the line that starts with
    `counters-json:` holds {kernel: {"hbm_bytes_per_launch": ..., "valu_per_element": ...}}.  None if the file or the
    line is missing (the bench line then carries null for what it cannot know)."""
    try:
        for line in open(path):
            if line.startswith("counters-json:"):
                return json.loads(line[len("counters-json:"):])
    except (OSError, ValueError):
        pass
    return None


def packed_bytes(n, bits, group, spike=True, int_meta=False):
    """Algorithmic size of a packed record: planes + per-group metadata (no alignment padding).  Per group:
    scale + zero (2 x 2 bytes, 2 x 1 with the integer metadata of Eq. 1) and, with spike reserving, 2 x (2 + 1)."""
    return n * bits // 8 + ((2 if int_meta else 4) + (6 if spike else 0)) * (n // group)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-sweep", action="store_true", help="skip the bit-width sweep and the dispatch workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--attribution", action="store_true",
                    help="only launch reduce_requant over peer counts, with and without spike reserving, float and integer "
                         "metadata, each case on a tensor size of its own (so a profiler's per-kernel, per-grid counters "
                         "can be told apart), print the cases and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2508_03760_amd import fcv2
    from paper_2508_03760_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    fcv2.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    SR = fcv2.F_SPIKE
    w = W.WORKLOADS[2]
    rows, cols, n_peers, group = w["rows"], w["cols"], w["peers"], 128
    n = rows * cols

    def bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    xs_host = [W.tensor(2, p).reshape(-1) for p in range(n_peers)]
    xs = [bf16(x) for x in xs_host]

    if args.attribution:
        # For rocprofv3 --pmc SQ_INSTS_VALU: the slope over the peer count is the cost of a peer, the intercept the
        # requantization.  Case i runs on n - i * 262,144 elements, so every case has a grid size of its own.
        import ctypes as C
        lib = fcv2.lib()
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        cases, i = [], 0
        for label, bits, grp, flags in (("b3_g128_sr", 3, 128, SR), ("b3_g128_plain", 3, 128, 0), ("b3_g32_sr", 3, 32, SR),
                                        ("b3_g32_sr_int_meta", 3, 32, SR | fcv2.F_META_INT), ("b2_g128_sr", 2, 128, SR),
                                        ("b5_g128_sr", 5, 128, SR), ("b8_g128_sr", 8, 128, SR)):
            for N in (1, 2, 4, 8, 16):
                n_i = n - i * 262144
                i += 1
                peers = [fcv2.quantize_pack(xs[p % n_peers][:n_i], bits, grp, flags) for p in range(N)]
                out = torch.zeros(fcv2.get_layout(n_i, bits, grp, flags).total_bytes, dtype=torch.uint8, device=dev)
                fmt = fcv2._Fmt(bits, grp, flags)
                arr = (C.c_void_p * N)(*[p.data_ptr() for p in peers])
                for _ in range(3):
                    rc = lib.fcv2_reduce_requant(arr, N, n_i, C.byref(fmt), C.byref(fmt), C.c_void_p(out.data_ptr()), None, stream)
                    assert rc == 0, rc
                torch.cuda.synchronize()
                cases.append(dict(case=label, bits=bits, group=grp, peers=N, elements=n_i, lanes=n_i // 16))
        print(json.dumps({"attribution_cases": cases}))
        return

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def make_sets(bits, n_sets, group=group, flags=SR):
        """n_sets independent copies of (x, 8 packed peers, outputs) at different addresses."""
        L = fcv2.get_layout(n, bits, group, flags)
        sets = []
        for _ in range(n_sets):
            peers = [fcv2.quantize_pack(x, bits, group, flags) for x in xs]
            sets.append(dict(x=xs[0].clone(), peers=peers, group=group, flags=flags,
                             q=torch.zeros(L.total_bytes, dtype=torch.uint8, device=dev),
                             r=torch.zeros(L.total_bytes, dtype=torch.uint8, device=dev),
                             o=torch.empty(n, dtype=torch.bfloat16, device=dev)))
        torch.cuda.synchronize()
        return sets

    def algo_bytes(bits, group=group, int_meta=False):
        P = packed_bytes(n, bits, group, True, int_meta)
        return dict(quantize_pack=2 * n + P, reduce_requant=(n_peers + 1) * P, unpack_dequant=P + 2 * n)

    def n_sets_for(bits):
        """Buffer sets to rotate: enough that even the kernel with the smallest footprint per set, timed alone, cycles
        through three times the last-level cache before it sees a set again."""
        smallest = min(algo_bytes(bits).values())
        return max(8, -(-3 * LLC_BYTES // smallest))

    def bind_calls(sets, bits):
        """Arguments marshalled once per buffer set: a timed loop is C-ABI calls and nothing else."""
        import ctypes as C
        lib = fcv2.lib()
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        for s in sets:
            if s.get("bits") != bits:
                fmt = fcv2._Fmt(bits, s["group"], s["flags"])
                arr = (C.c_void_p * n_peers)(*[p.data_ptr() for p in s["peers"]])
                s["bits"] = bits
                s["keep"] = (arr, fmt)
                s["calls"] = dict(
                    quantize_pack=(lib.fcv2_quantize_pack, (C.c_void_p(s["x"].data_ptr()), n, C.byref(fmt), C.c_void_p(s["q"].data_ptr()), stream)),
                    reduce_requant=(lib.fcv2_reduce_requant, (arr, n_peers, n, C.byref(fmt), C.byref(fmt), C.c_void_p(s["r"].data_ptr()), None, stream)),
                    unpack_dequant=(lib.fcv2_unpack_dequant, (C.c_void_p(s["r"].data_ptr()), n, C.byref(fmt), C.c_void_p(s["o"].data_ptr()), fcv2.DT_BF16, stream)),
                )

    KERNELS = ("quantize_pack", "reduce_requant", "unpack_dequant")
    STEP = ("quantize_pack", "reduce_requant")  # the calls the metric names

    def timed(fn, count, warmup):
        """HIP events on the launch stream around `count` back-to-back calls; returns ms per call."""
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        t0, t1 = ev(), ev()
        t0.record()
        for i in range(count):
            fn(i)
        t1.record()
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) / count

    def call(s, name):
        fn, a = s["calls"][name]
        rc = fn(*a)
        if rc != 0:
            raise RuntimeError(f"libfcv2 {name} failed: {rc}")

    def run_steps(sets, bits, steps, warmup, names=STEP):
        """ms per step: one step = the calls `names` one after the other, on rotating buffer sets."""
        bind_calls(sets, bits)

        def step(i):
            s = sets[i % len(sets)]
            for name in names:
                call(s, name)

        return timed(step, steps, warmup)

    def run_kernels(sets, bits, steps, warmup):
        """ms per launch of each kernel, each timed over its own run of `steps` back-to-back launches."""
        bind_calls(sets, bits)
        out = {}
        for name in KERNELS:  # median of 5 repeats of `steps` launches each
            reps = sorted(timed(lambda i, name=name: call(sets[i % len(sets)], name), steps, warmup) for _ in range(5))
            out[name] = reps[2]
        return out

    # ---- headline: 3-bit ------------------------------------------------------------------------------------
    bits = 3
    sets = make_sets(bits, n_sets_for(bits))
    # Bring the GPU to its sustained clocks first: after idling it needs some tens of milliseconds of work to get there
    # (measured: the first 100 steps after set-up run 8 % slower than steps 300 onwards).  Untimed, like the warm-up.
    run_steps(sets, bits, 600, 0, KERNELS)
    ms_step = run_steps(sets, bits, args.steps, args.warmup)  # the timed region proper: quantize_pack + reduce_requant
    ms_step3 = run_steps(sets, bits, args.steps, args.warmup, KERNELS)  # with unpack_dequant: one rank's three local calls
    kern_ms = run_kernels(sets, bits, args.steps, 3)           # the same launches, one kernel at a time
    ab = algo_bytes(bits)
    total_bytes = sum(ab[k] for k in STEP)
    total_bytes3 = sum(ab.values())
    value = total_bytes / (ms_step * 1e-3) / 1e9
    kernels = {k: dict(us=round(kern_ms[k] * 1e3, 2), algorithmic_bytes=ab[k],
                       gbs=round(ab[k] / (kern_ms[k] * 1e-3) / 1e9, 1),
                       frac_of_hbm_peak=round(ab[k] / (kern_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)) for k in ab}
    dom = "reduce_requant"
    kname = f"k_reduce_requant ({dom}, 3 bits, G=128, N={n_peers})"
    prof = profile_counters() or {}
    pk = prof.get(dom, {})
    traffic = pk.get("hbm_bytes_per_launch")
    traffic_source = ("profiles/headline_step_b3_g128_n8.md (rocprofv3 FETCH_SIZE and WRITE_SIZE, each scaled by the same counter "
                      "on a copy of known size)") if traffic is not None else None
    # The dominant kernel against HBM, the bound the metric is stated in: algorithmic bytes per launch ((N + 1) x the
    # packed record) / the launch duration measured above with HIP events / 8 TB/s.
    roofline = dict(bound="hbm", kernel=kname, achieved=kernels[dom]["gbs"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(kernels[dom]["gbs"] / HBM_PEAK_GBS, 4), traffic=traffic, traffic_source=traffic_source,
                    algorithmic_bytes=ab[dom], us_per_launch=kernels[dom]["us"])
    # What limits it in practice is VALU time; the executed instruction rate of the same launch, for context (not a
    # roofline: the nominal rate of 256 CU x 4 SIMD x 16 lanes x 2.4 GHz assumes 4 cycles per wave-wide instruction, and the
    # two-operand forms this kernel mostly uses occupy a SIMD for 2.4, so the executed rate can exceed it).  executed = VALU
    # instructions per output element from the same rocprofv3 summary (SQ_INSTS_VALU).
    alu_roofline = None
    if pk.get("valu_per_element") is not None:
        ops_s = pk["valu_per_element"] * n / (kern_ms[dom] * 1e-3) / 1e12
        alu_roofline = dict(kernel=kname, executed_ops_per_element=pk["valu_per_element"], executed_rate=round(ops_s, 2),
                            nominal_rate_at_4_cycles_per_instruction=round(ALU_PEAK_TLOPS, 2), unit="T lane-op/s",
                            source="profiles/headline_step_b3_g128_n8.md (SQ_INSTS_VALU x 64 lanes / elements)")
    # practical streaming ceiling: the library's plain copy kernel on 1 GiB (source and destination together are eight
    # times the 256 MB last-level cache, so this is an HBM figure)
    import ctypes as C
    ca = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cb = torch.empty_like(ca)
    cstream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    ms_copy = timed(lambda i: fcv2.lib().fcv2_stream_copy(C.c_void_p(ca.data_ptr()), C.c_void_p(cb.data_ptr()), ca.numel(), cstream), 20, 3)
    copy_gbs = 2 * ca.numel() / (ms_copy * 1e-3) / 1e9
    del ca, cb
    # the same copy kernel moving what quantize_pack / unpack_dequant move at the headline shape (41 MB): what a kernel
    # of that size can reach at all, launch ramp and tail included
    half = (ab["quantize_pack"] // 2 + 4095) // 4096 * 4096
    csets = [(torch.empty(half, dtype=torch.uint8, device=dev), torch.empty(half, dtype=torch.uint8, device=dev)) for _ in range(14)]
    ms_copy_small = timed(lambda i: fcv2.lib().fcv2_stream_copy(C.c_void_p(csets[i % 14][0].data_ptr()), C.c_void_p(csets[i % 14][1].data_ptr()),
                                                               half, cstream), 56, 14)
    copy_same_size = dict(bytes_moved=2 * half, us=round(ms_copy_small * 1e3, 2), gbs=round(2 * half / (ms_copy_small * 1e-3) / 1e9, 1))
    del csets
    # warm-cache figure for context: one buffer set, everything stays in the last-level cache
    ms_warm = run_steps(sets[:1], bits, args.steps, args.warmup)
    three = dict(step="quantize_pack + reduce_requant + unpack_dequant", ms_per_step=round(ms_step3, 5), algorithmic_bytes=total_bytes3,
                 gbs=round(total_bytes3 / (ms_step3 * 1e-3) / 1e9, 1), frac_of_hbm_peak=round(total_bytes3 / (ms_step3 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
    del sets
    torch.cuda.empty_cache()

    # ---- sweep over bit widths, and the dispatch workload -----------------------------------------------------
    sweep, dispatch, mixed_width = {}, None, None
    if not args.no_sweep:
        for b in (2, 3, 4, 5, 6, 7, 8):
            s = make_sets(b, n_sets_for(b))
            ms_b = run_steps(s, b, max(10, args.steps // 2), 3)
            k_b = run_kernels(s, b, max(10, args.steps // 2), 3)
            abb = algo_bytes(b)
            sweep[str(b)] = {k: dict(us=round(k_b[k] * 1e3, 2), gbs=round(abb[k] / (k_b[k] * 1e-3) / 1e9, 1),
                                     frac=round(abb[k] / (k_b[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)) for k in abb}
            sweep[str(b)]["step_gbs"] = round(sum(abb[k] for k in STEP) / (ms_b * 1e-3) / 1e9, 1)
            if b == 4:
                # peers at 4 bits, output at 3: the width-changing form of the call (a separate, simpler kernel)
                import ctypes as C
                f_in, f_out = fcv2._Fmt(4, group, SR), fcv2._Fmt(3, group, SR)
                st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
                ms_m = timed(lambda i: fcv2.lib().fcv2_reduce_requant(s[i % len(s)]["keep"][0], n_peers, n, C.byref(f_in), C.byref(f_out),
                                                                      C.c_void_p(s[i % len(s)]["r"].data_ptr()), None, st),
                             max(10, args.steps // 2), 3)
                mixed_bytes = n_peers * packed_bytes(n, 4, group) + packed_bytes(n, 3, group)
                mixed_width = dict(bits_in=4, bits_out=3, us=round(ms_m * 1e3, 2), algorithmic_bytes=mixed_bytes,
                                   gbs=round(mixed_bytes / (ms_m * 1e-3) / 1e9, 1))
            del s
            torch.cuda.empty_cache()
        w3 = W.WORKLOADS[3]
        T, H, E, K = w3["rows"], w3["cols"], w3["experts"], w3["topk"]
        x3 = bf16(W.tensor(3, 0).reshape(-1)).view(T, H)
        ids = torch.from_numpy(W.topk_routing(W.seed_for(3), T, E, K)).to(dev)
        L3 = fcv2.get_layout(H, 2, 128, SR, fcv2.ROW_ALIGN)
        bufs = [dict(send=torch.zeros((T * K, L3.total_bytes), dtype=torch.uint8, device=dev),
                     offs=torch.zeros(E + 1, dtype=torch.int32, device=dev),
                     src=torch.zeros(T * K, dtype=torch.int32, device=dev),
                     ws=torch.empty(fcv2.dispatch_workspace_bytes(T, K, E), dtype=torch.uint8, device=dev),
                     x=x3.clone()) for _ in range(4)]

        def disp(bf):
            fcv2.dispatch_quant(bf["x"], ids, E, 2, 128, SR, send_buf=bf["send"], expert_offsets=bf["offs"],
                                row_src=bf["src"], workspace=bf["ws"])

        for i in range(3):
            disp(bufs[i % 4])
        torch.cuda.synchronize()
        t0, t1 = ev(), ev()
        reps = max(10, args.steps // 4)
        t0.record()
        for i in range(reps):
            disp(bufs[i % 4])
        t1.record()
        torch.cuda.synchronize()
        ms_d = t0.elapsed_time(t1) / reps
        R = T * K
        bytes_d = 2 * T * H + 4 * T * K + R * packed_bytes(H, 2, 128) + 4 * (E + 1) + 4 * R
        dispatch = dict(workload=W.WORKLOADS[3]["name"], ms=round(ms_d, 4), algorithmic_bytes=bytes_d,
                        gbs=round(bytes_d / (ms_d * 1e-3) / 1e9, 1),
                        frac_of_hbm_peak=round(bytes_d / (ms_d * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
        del bufs, x3
        torch.cuda.empty_cache()

    # ---- the paper's default shape for the low widths (Section 4.1): groups of 32, spike reserving, and the integer
    # ---- scale and zero of Eq. 1 (Table 4, second row) against bf16 metadata ------------------------------------------
    low_bit = {}
    if not args.no_sweep:
        for b in (2, 3, 4):
            for name, fl, im in (("bf16_meta", SR, False), ("int_meta", SR | fcv2.F_META_INT, True)):
                per_set = 2 * n * 2 + (n_peers + 2) * packed_bytes(n, b, 32, True, im)
                s = make_sets(b, max(4, -(-3 * LLC_BYTES // per_set)), 32, fl)
                k_b = run_kernels(s, b, max(10, args.steps // 2), 3)
                abb = algo_bytes(b, 32, im)
                low_bit[f"b{b}_g32_{name}"] = dict(
                    record_bytes=packed_bytes(n, b, 32, True, im),
                    **{k: dict(us=round(k_b[k] * 1e3, 2), gbs=round(abb[k] / (k_b[k] * 1e-3) / 1e9, 1)) for k in abb})
                del s
                torch.cuda.empty_cache()

    # ---- quality proxy: signal-to-quantization-noise of plain RTN against spike reserving (direction of Tables 3, 7, 8) --
    quality = {}
    if not args.no_sweep:
        xf = xs[0].float()
        for b in (2, 3, 4, 5, 6, 8):
            row = {}
            for name, fl, g in (("rtn", 0, group), ("spike_reserving", SR, group), ("g32_spike_reserving", SR, 32),
                                ("g32_spike_reserving_int_meta", SR | fcv2.F_META_INT, 32)):
                v = fcv2.unpack_dequant(fcv2.quantize_pack(xs[0], b, g, fl), n, b, g, fl, torch.float32)
                row[name + "_sqnr_db"] = round(float(10 * torch.log10(xf.pow(2).sum() / (v - xf).pow(2).sum())), 2)
            quality[str(b)] = row
        del xf

    # ---- one rank's share of a whole two-step AllReduce over 8 ranks on the headline payload ------------------------
    two_step = None
    if not args.no_sweep:
        R = n_peers
        m = n // R
        send = [fcv2.quantize_pack_slices(x, R, 3, group, SR) for x in xs]          # what the 8 ranks would send
        mine = [[send[r][j] for r in range(R)] for j in range(R)]                    # copies of slice j, as received
        red = [fcv2.reduce_requant(mine[j], m, (3, group, SR)) for j in range(R)]    # what the 8 ranks would return
        out_t = torch.empty(n, dtype=torch.bfloat16, device=dev)
        sbuf = torch.zeros_like(send[0])

        import ctypes as C
        lib = fcv2.lib()
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        f3 = fcv2._Fmt(3, group, SR)
        arr_mine = [(C.c_void_p * R)(*[t.data_ptr() for t in mine[j]]) for j in range(R)]
        arr_red = (C.c_void_p * R)(*[t.data_ptr() for t in red])

        def rank_step(i):
            j = i % R
            lib.fcv2_quantize_pack_slices(C.c_void_p(xs[j].data_ptr()), n, R, C.byref(f3), C.c_void_p(sbuf.data_ptr()),
                                          sbuf.shape[1], st)                               # pack my payload as 8 slices
            lib.fcv2_reduce_requant(arr_mine[j], R, m, C.byref(f3), C.byref(f3), C.c_void_p(red[j].data_ptr()), None, st)
            lib.fcv2_unpack_dequant_slices(arr_red, R, n, C.byref(f3), C.c_void_p(out_t.data_ptr()), fcv2.DT_BF16, st)

        ms_ts = timed(rank_step, max(20, args.steps // 2), 3)
        P1 = packed_bytes(m, 3, group)
        bytes_ts = (2 * n + R * P1) + (R + 1) * P1 + (R * P1 + 2 * n)
        two_step = dict(ranks=R, us_per_rank=round(ms_ts * 1e3, 2), algorithmic_bytes=bytes_ts,
                        gbs=round(bytes_ts / (ms_ts * 1e-3) / 1e9, 1),
                        note="quantize_pack_slices(16M) + reduce_requant(2M x 8 peers) + unpack_dequant_slices(16M); "
                             "exchanges between ranks are not part of a one-GPU run")
        del send, mine, red, out_t, sbuf
        torch.cuda.empty_cache()

    # ---- micro-chunk pipelining (Section 3.4) in its one-GPU form: the chunks' quantize -> reduce -> unpack chains
    # ---- alternate between two streams, so one chunk's ramp-up and tail overlap the other's body ------------------------
    pipelined = None
    if not args.no_sweep:
        import ctypes as C
        lib = fcv2.lib()
        f3 = fcv2._Fmt(3, group, SR)
        n_chunks = 4
        mc = n // n_chunks
        Lc = fcv2.get_layout(mc, 3, group, SR)
        oth = [[fcv2.quantize_pack(x[c * mc:(c + 1) * mc], 3, group, SR) for c in range(n_chunks)] for x in xs[1:]]
        qc = [torch.zeros(Lc.total_bytes, dtype=torch.uint8, device=dev) for _ in range(n_chunks)]
        rc_ = [torch.zeros(Lc.total_bytes, dtype=torch.uint8, device=dev) for _ in range(n_chunks)]
        oc = torch.empty(n, dtype=torch.bfloat16, device=dev)
        arrs = [(C.c_void_p * n_peers)(qc[c].data_ptr(), *[o[c].data_ptr() for o in oth]) for c in range(n_chunks)]
        side = [torch.cuda.Stream(), torch.cuda.Stream()]
        main = torch.cuda.current_stream()

        def chunk_chain(c, st, xin):
            h = C.c_void_p(st.cuda_stream)
            lib.fcv2_quantize_pack(C.c_void_p(xin.data_ptr() + 2 * c * mc), mc, C.byref(f3), C.c_void_p(qc[c].data_ptr()), h)
            lib.fcv2_reduce_requant(arrs[c], n_peers, mc, C.byref(f3), C.byref(f3), C.c_void_p(rc_[c].data_ptr()), None, h)
            lib.fcv2_unpack_dequant(C.c_void_p(rc_[c].data_ptr()), mc, C.byref(f3), C.c_void_p(oc.data_ptr() + 2 * c * mc), fcv2.DT_BF16, h)

        def serial_chunks(i):
            for c in range(n_chunks):
                chunk_chain(c, main, xs[i % n_peers])

        def two_streams(i):
            e = torch.cuda.Event()
            e.record(main)
            for c in range(n_chunks):
                st = side[c % 2]
                if c < 2:
                    st.wait_event(e)
                chunk_chain(c, st, xs[i % n_peers])
            for st in side:
                main.wait_stream(st)

        # recorded as HIP graphs, so that host-side launch and event costs do not hide what the GPU does
        def record(body):
            body(0)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                body(0)
            return g

        def serial_in_capture(i):
            cur = torch.cuda.current_stream()
            for c in range(n_chunks):
                chunk_chain(c, cur, xs[0])

        def forked_in_capture(i):
            cur = torch.cuda.current_stream()
            for st in side:
                st.wait_stream(cur)
            for c in range(n_chunks):
                chunk_chain(c, side[c % 2], xs[0])
            for st in side:
                cur.wait_stream(st)

        def whole_in_capture(i):
            cur = torch.cuda.current_stream()
            h = C.c_void_p(cur.cuda_stream)
            s0 = whole_set
            lib.fcv2_quantize_pack(C.c_void_p(xs[0].data_ptr()), n, C.byref(f3), C.c_void_p(s0["q"].data_ptr()), h)
            lib.fcv2_reduce_requant(s0["arr"], n_peers, n, C.byref(f3), C.byref(f3), C.c_void_p(s0["r"].data_ptr()), None, h)
            lib.fcv2_unpack_dequant(C.c_void_p(s0["r"].data_ptr()), n, C.byref(f3), C.c_void_p(oc.data_ptr()), fcv2.DT_BF16, h)

        Lw = fcv2.get_layout(n, 3, group, SR)
        wp = [fcv2.quantize_pack(x, 3, group, SR) for x in xs]
        whole_set = dict(q=torch.zeros(Lw.total_bytes, dtype=torch.uint8, device=dev), r=torch.zeros(Lw.total_bytes, dtype=torch.uint8, device=dev))
        whole_set["arr"] = (C.c_void_p * n_peers)(whole_set["q"].data_ptr(), *[p.data_ptr() for p in wp[1:]])
        cnt = max(20, args.steps // 2)
        graphs = {k: record(f) for k, f in (("whole_payload", whole_in_capture), ("serial_chunks", serial_in_capture),
                                            ("two_streams", forked_in_capture))}
        pipelined = dict(chunks=n_chunks, chunk_elements=mc,
                         **{k + "_us": round(timed(lambda i, g=g: g.replay(), cnt, 3) * 1e3, 2) for k, g in graphs.items()},
                         eager_serial_chunks_us=round(timed(serial_chunks, cnt, 3) * 1e3, 2),
                         eager_two_streams_us=round(timed(two_streams, cnt, 3) * 1e3, 2),
                         note="one rank's quantize -> reduce(8) -> unpack on the 16M payload, whole or as 4 chunks; graph replays "
                              "of one fixed buffer set (cache-warm), so compare the three graph figures with each other only")
        del graphs, wp, whole_set
        del oth, qc, rc_, oc
        torch.cuda.empty_cache()

    # ---- decode-sized latency case (workload 5) and the large AllReduce payload (workload 4) --------------------
    latency, large = {}, {}
    if not args.no_sweep:
        import ctypes as C
        lib = fcv2.lib()
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        w5 = W.WORKLOADS[5]
        n5 = w5["rows"] * w5["cols"]
        x5 = bf16(W.tensor(5, 0).reshape(-1))
        peers5 = [bf16(W.tensor(5, p).reshape(-1)) for p in range(8)]
        for b in w5["bits"]:
            fmt5 = fcv2._Fmt(b, 128, SR)
            L5 = fcv2.get_layout(n5, b, 128, SR)
            q5 = torch.zeros(L5.total_bytes, dtype=torch.uint8, device=dev)
            o5 = torch.empty(n5, dtype=torch.bfloat16, device=dev)
            pk5 = [fcv2.quantize_pack(x, b, 128, SR) for x in peers5]
            arr5 = (C.c_void_p * 8)(*[p.data_ptr() for p in pk5])
            P5 = packed_bytes(n5, b, 128)
            calls = dict(
                quantize_pack=(lambda i: lib.fcv2_quantize_pack(C.c_void_p(x5.data_ptr()), n5, C.byref(fmt5), C.c_void_p(q5.data_ptr()), stream), 2 * n5 + P5),
                unpack_dequant=(lambda i: lib.fcv2_unpack_dequant(C.c_void_p(pk5[0].data_ptr()), n5, C.byref(fmt5), C.c_void_p(o5.data_ptr()), fcv2.DT_BF16, stream), 2 * n5 + P5),
                reduce_requant=(lambda i: lib.fcv2_reduce_requant(arr5, 8, n5, C.byref(fmt5), C.byref(fmt5), C.c_void_p(q5.data_ptr()), None, stream), 9 * P5))
            latency[str(b)] = {k: dict(us_per_call=round(timed(f, 1000, 20) * 1e3, 2)) for k, (f, _) in calls.items()}
            for k, (_, nbytes) in calls.items():
                latency[str(b)][k]["gbs"] = round(nbytes / (latency[str(b)][k]["us_per_call"] * 1e-6) / 1e9, 1)
            # the whole step (3 calls) eagerly and as a HIP graph of 20 recorded steps: launch overhead is what
            # bounds this size, and the library is capturable (kernel launches only)
            r5 = torch.zeros(L5.total_bytes, dtype=torch.uint8, device=dev)
            arr5s = (C.c_void_p * 8)(q5.data_ptr(), *[p.data_ptr() for p in pk5[1:]])

            def step5(st):
                lib.fcv2_quantize_pack(C.c_void_p(x5.data_ptr()), n5, C.byref(fmt5), C.c_void_p(q5.data_ptr()), st)
                lib.fcv2_reduce_requant(arr5s, 8, n5, C.byref(fmt5), C.byref(fmt5), C.c_void_p(r5.data_ptr()), None, st)
                lib.fcv2_unpack_dequant(C.c_void_p(r5.data_ptr()), n5, C.byref(fmt5), C.c_void_p(o5.data_ptr()), fcv2.DT_BF16, st)

            us_eager = timed(lambda i: step5(stream), 300, 20) * 1e3
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                cst = C.c_void_p(torch.cuda.current_stream().cuda_stream)
                for _ in range(20):
                    step5(cst)
            us_graph = timed(lambda i: gr.replay(), 30, 3) * 1e3 / 20
            latency[str(b)]["step_eager_us"] = round(us_eager, 2)
            latency[str(b)]["step_graph_us"] = round(us_graph, 2)
            del gr
        del x5, peers5
        w4 = W.WORKLOADS[4]
        n4 = w4["rows"] * w4["cols"]
        xs4 = [bf16(W.tensor(4, p).reshape(-1)) for p in range(8)]
        for b in w4["bits"]:
            for g in w4["groups"]:
                fmt4 = fcv2._Fmt(b, g, SR)
                L4 = fcv2.get_layout(n4, b, g, SR)
                pk4 = [fcv2.quantize_pack(x, b, g, SR) for x in xs4]
                q4 = torch.zeros(L4.total_bytes, dtype=torch.uint8, device=dev)
                arr4 = (C.c_void_p * 8)(*[p.data_ptr() for p in pk4])
                P4 = packed_bytes(n4, b, g)
                us_q = timed(lambda i: lib.fcv2_quantize_pack(C.c_void_p(xs4[i % 8].data_ptr()), n4, C.byref(fmt4), C.c_void_p(q4.data_ptr()), stream), 16, 2) * 1e3
                us_r = timed(lambda i: lib.fcv2_reduce_requant(arr4, 8, n4, C.byref(fmt4), C.byref(fmt4), C.c_void_p(q4.data_ptr()), None, stream), 16, 2) * 1e3
                large[f"b{b}_g{g}"] = dict(
                    quantize_pack=dict(us=round(us_q, 1), gbs=round((2 * n4 + P4) / us_q / 1e3, 1), frac=round((2 * n4 + P4) / us_q / 1e3 / HBM_PEAK_GBS, 4)),
                    reduce_requant=dict(us=round(us_r, 1), gbs=round(9 * P4 / us_r / 1e3, 1), frac=round(9 * P4 / us_r / 1e3 / HBM_PEAK_GBS, 4)))
                del pk4, q4
                torch.cuda.empty_cache()
        del xs4
        torch.cuda.empty_cache()

    # ---- the CPU oracle on the same workload, timed on the host -------------------------------------------------
    cpu = None
    if not args.no_cpu:
        import oracle as O
        fmt = (3, group, SR)
        reps = 8
        peers_o = [O.quantize_pack(x, *fmt) for x in xs_host]  # untimed set-up of the peer chunks
        t = time.perf_counter()
        for _ in range(reps):
            O.quantize_pack(xs_host[0], *fmt)
            O.reduce_requant(peers_o, n, fmt)
        dt = (time.perf_counter() - t) / reps
        cpu = dict(value=round(total_bytes / dt / 1e9, 4), unit="GB/s", cores=1, kind="oracle",
                   sample=f"{reps} full steps of the same workload (quantize_pack + reduce_requant N=8 "
                          f"on 4096x4096, 3-bit), {dt:.2f} s per step on one host thread")
        # the same oracle on all host cores: threads over disjoint row blocks (groups are independent; the calls
        # release the interpreter lock), each thread running the three calls on its block
        from concurrent.futures import ThreadPoolExecutor
        n_thr = max(1, min(16, len(os.sched_getaffinity(0))))
        while rows % n_thr:
            n_thr -= 1
        blk = n // n_thr
        xb = [[x[j * blk:(j + 1) * blk] for x in xs_host] for j in range(n_thr)]
        pb = [[O.quantize_pack(x, *fmt) for x in xb[j]] for j in range(n_thr)]  # untimed set-up

        def block_step(j):
            O.quantize_pack(xb[j][0], *fmt)
            O.reduce_requant(pb[j], blk, fmt)

        reps_mt = 8
        with ThreadPoolExecutor(n_thr) as pool:
            list(pool.map(block_step, range(n_thr)))
            t = time.perf_counter()
            for _ in range(reps_mt):
                list(pool.map(block_step, range(n_thr)))
            dt_mt = (time.perf_counter() - t) / reps_mt
        cpu["all_cores"] = dict(value=round(total_bytes / dt_mt / 1e9, 4), unit="GB/s", cores=n_thr,
                                sample=f"{reps_mt} steps, {n_thr} threads over row blocks, {dt_mt:.3f} s per step")
        # Direction of Table 3 on the CPU side (numpy forms of the two comparison methods next to the oracle's codec):
        # signal-to-noise in dB at 32 values per group on a 256 K-element slice of the same payload
        import oracle.quality as OQ
        t3 = OQ.table(xs_host[0][:64 * 4096], group=32)
        cpu["table3_direction_sqnr_db_g32"] = {f"int{b}": {k: round(v, 2) for k, v in row.items()} for b, row in t3.items()}

    out = {
        "metric": "effective HBM GB/s (and % of peak) for quantize_pack + reduce_requant, bits 2-8",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": W.WORKLOADS[2]["name"] + "_b3_g128_sr_N8", "elements": n, "bits": 3, "group": 128,
                   "spike_reserving": True, "peers": n_peers, "step": "quantize_pack + reduce_requant",
                   "buffer_sets_rotated": n_sets_for(3), "untimed_spin_up_steps": 600},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "warm_cache_gbs": round(total_bytes / (ms_warm * 1e-3) / 1e9, 1),  # the same two-call step on one buffer set
        "copy_ceiling_gbs": round(copy_gbs, 1), "copy_same_size_as_quantize_pack": copy_same_size,
        "three_call_step": three,
        "kernels": kernels, "roofline": roofline, "alu_roofline": alu_roofline, "cpu_baseline": cpu, "sweep_bits": sweep, "reduce_requant_4bit_in_3bit_out": mixed_width, "dispatch": dispatch,
        "quality_proxy_sqnr": quality, "low_bit_default_shape_g32": low_bit, "two_step_allreduce_rank_share": two_step, "micro_chunk_pipelining": pipelined, "decode_latency_64x7168": latency, "large_allreduce_8192x8192_N8": large,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
