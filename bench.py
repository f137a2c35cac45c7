#!/usr/bin/env python3
"""Benchmark of the HiKonv hot path on one MI355X.

A step is one pass of the packed 1-D convolution path (load of bit-dense inputs, packing,
one wide multiply per block, lane exchange, split, int32 store) over one batch of the
bitwidth sweep: 4096 independent rows of 65536 values, K = 3 taps, 4-bit unsigned, valid
outputs.  Inputs are resident in HBM before the timed region.  The JSON line also carries
the 1-bit and 8-bit cases, the unpacked one-product-per-multiply GPU kernel on the same
inputs, the two DNN-layer configurations (ALU-bound), the roofline of the dominant kernel
and the CPU oracle timed on a bounded sample.

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

ROWS, LENGTH, TAPS = 4096, 65536, 3
HBM_PEAK_GBS = 8000.0                      # MI355X published HBM3E bandwidth
VALU_LANE_RATE = 256 * 64 * 2.4e9          # lane-instructions/s at full rate: 256 CUs x 64 lanes x 2.4 GHz


def event_ms(fn, reps):
    """Average milliseconds per call of fn over reps back-to-back calls (events on torch's stream)."""
    import torch
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) / reps


def conv1d_case(hk, wl, bits, signed, taps=TAPS):
    """Device buffers and launch closures for one case of the sweep."""
    import torch
    TAPS = taps
    x, g = wl.conv1d_case(bits, signed, TAPS, ROWS, LENGTH)
    x_d8 = torch.from_numpy(x.view("uint8")).cuda()
    g_d = torch.from_numpy(g.view("uint8")).cuda()
    row_bytes = hk.hikonv_bitdense_row_bytes(LENGTH, bits)
    x_bd = torch.zeros(ROWS * row_bytes, dtype=torch.uint8, device="cuda")
    hk.hikonv_compact(x_d8, ROWS, LENGTH, bits, False, x_bd)
    del x_d8
    out_len = LENGTH - TAPS + 1
    y = torch.empty(ROWS * out_len, dtype=torch.int32, device="cuda")
    plan = hk.hikonv_plan_ex(bits_a=bits, bits_w=bits, a_signed=int(signed), w_signed=int(signed), L_A=32, L_B=32,
                             L_acc=64, mode=hk.MODE_CONV1D, taps=TAPS)

    def packed():
        hk.hikonv_conv1d(plan, x_bd, hk.FMT_BITDENSE, ROWS, LENGTH, g_d, TAPS, hk.OUT_VALID, y)

    def unpacked():
        hk.hikonv_conv1d_unpacked(bits, bits, hk.signedness(signed, signed), x_bd, hk.FMT_BITDENSE, ROWS, LENGTH, g_d,
                                  TAPS, hk.OUT_VALID, y)

    macs = ROWS * out_len * TAPS
    algo_bytes = ROWS * out_len * 4 + ROWS * row_bytes + TAPS
    return dict(x=x, g=g, y=y, plan=plan, packed=packed, unpacked=unpacked, macs=macs, bytes=algo_bytes,
                out_len=out_len, keep=(x_bd, g_d))


def cpu_baseline(x, g):
    """The oracle as it stands (int64 direct convolution, OpenMP over rows), timed on the host
    cores on the whole 4-bit case, plus one thread on a 256-row sample."""
    from oracle import direct
    direct.conv1d(x[:64], g, direct.VALID)                     # warm-up (page in the library)
    threads = direct.num_threads()
    best = float("inf")
    for _ in range(5):
        t0 = time.perf_counter()
        direct.conv1d(x, g, direct.VALID)
        best = min(best, time.perf_counter() - t0)
    macs = ROWS * (LENGTH - TAPS + 1) * TAPS
    direct.set_num_threads(1)
    t0 = time.perf_counter()
    direct.conv1d(x[:256], g, direct.VALID)
    one = time.perf_counter() - t0
    direct.set_num_threads(threads)
    return dict(value=2 * macs / best / 1e9, unit="GOPS", cores=threads, kind="oracle",
                sample="all %d rows of the same 4-bit case, best of 5 (%.1f ms); one thread on 256 rows: %.2f GOPS" %
                       (ROWS, best * 1e3, 2 * 256 * (LENGTH - TAPS + 1) * TAPS / one / 1e9))


def graph_replay_ms(fn, calls, reps):
    """Milliseconds per call of fn when `calls` calls are captured into one HIP graph and the
    graph is replayed (no host launch cost between the kernels); None if capture fails."""
    import torch
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(calls):
                fn()
        graph.replay()
        return event_ms(graph.replay, reps) / calls
    except Exception:                                          # graph capture is optional
        return None


def requant_extra(hk, wl, steps):
    """The same 1-D cases with the outputs requantised in the kernel and written bit-dense at the
    input's width: no int32 stream, so the integer VALUs bound it instead of HBM writes."""
    import torch
    report = {}
    for bits, signed in ((4, False), (1, False), (2, False), (4, True)):
        case = conv1d_case(hk, wl, bits, signed)
        x_bd, g_d = case["keep"]
        plan, out_len = case["plan"], case["out_len"]
        row_bytes = hk.hikonv_bitdense_row_bytes(out_len, bits)
        q = torch.empty(ROWS * row_bytes, dtype=torch.uint8, device="cuda")
        shift, qmax = max(0, 2 * bits - 3), (1 << bits) - 1 if bits < 8 else 127

        def packed():
            hk.hikonv_conv1d_requant(plan, x_bd, hk.FMT_BITDENSE, ROWS, LENGTH, g_d, TAPS, hk.OUT_VALID, shift, qmax,
                                     bits, q)

        def unpacked():
            hk.hikonv_conv1d_requant_unpacked(bits, bits, hk.signedness(signed, signed), x_bd, hk.FMT_BITDENSE, ROWS,
                                              LENGTH, g_d, TAPS, hk.OUT_VALID, shift, qmax, bits, q)

        event_ms(packed, 3)
        ms_p = event_ms(packed, steps)
        # the same call with the plan's own N, K, S instead of the container-aligned slices
        # (K = 1, N = 2, S = 16) that the library takes here by itself
        os.environ["HIKONV_REQUANT_KERNEL"] = "1"
        try:
            event_ms(packed, 3)
            ms_plan = event_ms(packed, steps)
        finally:
            del os.environ["HIKONV_REQUANT_KERNEL"]
        event_ms(unpacked, 3)
        ms_u = event_ms(unpacked, steps)
        algo = ROWS * (row_bytes + hk.hikonv_bitdense_row_bytes(LENGTH, bits)) + TAPS
        report["%d%s" % (bits, "s" if signed else "u")] = dict(
            ms=ms_p, gops=2 * case["macs"] / ms_p / 1e6, gbs=algo / ms_p / 1e6, unpacked_ms=ms_u,
            frac_of_unpacked_valu_peak=case["macs"] / (ms_p * 1e-3) / VALU_LANE_RATE,
            slices="container-aligned: N=2, K=1, S=16", plan_slices_ms=ms_plan,
            plan=dict(N=plan.N, K=plan.K, S=plan.S))
        del case, q
        torch.cuda.empty_cache()
    return report


def conv2d_extra(hk, wl, name, steps):
    """Packed vs unpacked DNN layer (ALU-bound configurations); returns a small report."""
    import torch
    if name == "c3":
        x, w = wl.config3()
        plan_kw = dict(bits_a=4, bits_w=4, a_signed=1, w_signed=1)
        sg, bits = hk.signedness(True, True), 4
    else:
        x, w = wl.config4()
        plan_kw = dict(bits_a=1, bits_w=1, bipolar=1)
        sg, bits = hk.BIPOLAR, 1
    n, c, h, wd = x.shape
    co, _, kh, kw = w.shape
    x_d = torch.from_numpy(x.view("uint8")).cuda()
    w_d = torch.from_numpy(w.view("uint8")).cuda()
    y = torch.empty(n * co * h * wd, dtype=torch.int32, device="cuda")
    macs = n * co * h * wd * c * kh * kw
    report = {"macs": macs}
    for label, width, acc, tight in (("wide32", 32, 64, 0), ("wide32_tight", 32, 64, 1), ("narrow24", 24, 32, 0)):
        try:
            plan = hk.hikonv_plan_ex(L_A=width, L_B=width, L_acc=acc, mode=hk.MODE_DNN, M=0, taps=kw, tight=tight,
                                     **plan_kw)
            if plan.N > 8:
                raise hk.HikonvError(hk.EUNSUPPORTED, "plan")
        except hk.HikonvError:
            continue
        ws = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, wd, co, kh, kw, 1, 1, True), dtype=torch.uint8,
                         device="cuda")
        pw = torch.empty(hk.hikonv_packed_weights_bytes(plan, co, c, kh, kw), dtype=torch.uint8, device="cuda")
        hk.hikonv_pack_weights(plan, w_d, co, c, kh, kw, pw)

        def run():
            hk.hikonv_conv2d_prepacked(plan, x_d, hk.FMT_INT8, n, c, h, wd, pw, co, kh, kw, 1, 1, ws, y)

        event_ms(run, 3)
        ms = event_ms(run, steps)
        graph_ms = graph_replay_ms(run, 20, max(3, steps // 4))
        # algorithmic VALU work of the packed layer: one multiply-accumulate per (block, channel, term)
        blocks = -(-(wd + 1) // plan.N)
        lane_mads = n * co * h * blocks * c * kh * plan.chunks
        report[label] = dict(ms=ms, gops=2 * macs / ms / 1e6, plan=dict(N=plan.N, K=plan.K, S=plan.S, M=plan.M),
                             graph_ms=graph_ms, graph_gops=(2 * macs / graph_ms / 1e6) if graph_ms else None,
                             frac_of_unpacked_valu_peak=macs / (ms * 1e-3) / VALU_LANE_RATE,
                             roofline={"bound": "alu", "achieved": lane_mads / (ms * 1e-3) / 1e12,
                                       "peak": VALU_LANE_RATE / 1e12, "unit": "T lane-instr/s",
                                       "frac": lane_mads / (ms * 1e-3) / VALU_LANE_RATE,
                                       "note": "packed multiply-accumulates only, whole call (input packing included)"})

    def run_unpacked():
        hk.hikonv_conv2d_unpacked(bits, bits, sg, x_d, n, c, h, wd, w_d, co, kh, kw, 1, 1, y)

    event_ms(run_unpacked, 3)
    ms = event_ms(run_unpacked, steps)
    report["unpacked"] = dict(ms=ms, gops=2 * macs / ms / 1e6, graph_ms=graph_replay_ms(run_unpacked, 20, max(3, steps // 4)))
    return report


def widened_extras(hk, steps):
    """The two widened layer forms on 4-bit signed data: a stride-2 3x3 layer (every column
    computed and every second stored, against the polyphase form) and a 3x3x3 volume layer."""
    import numpy as np
    import torch
    rng = np.random.default_rng(2208)
    out = {}
    kw_plan = dict(bits_a=4, bits_w=4, a_signed=1, w_signed=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=0)

    n, c, h, w, co = 8, 64, 56, 56, 128
    x_d = torch.from_numpy(rng.integers(-8, 8, (n, c, h, w), dtype=np.int8).view("uint8")).cuda()
    w_d = torch.from_numpy(rng.integers(-8, 8, (co, c, 3, 3), dtype=np.int8).view("uint8")).cuda()
    ho = wo = (h + 2 - 3) // 2 + 1
    y = torch.empty(n * co * ho * wo, dtype=torch.int32, device="cuda")
    macs = n * co * ho * wo * c * 9
    rep = {"shape": "8x64x56x56 -> 128, 3x3, stride 2, pad 1, int4", "macs": macs}
    for label, taps in (("decimate", 3), ("polyphase", 2)):
        plan = hk.hikonv_plan_ex(taps=taps, **kw_plan)
        ws = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, 3, 3, 2, 1, True), dtype=torch.uint8,
                         device="cuda")
        pw = torch.empty(hk.hikonv_packed_weights_bytes_ex(plan, co, c, 1, 3, 3, 2), dtype=torch.uint8, device="cuda")
        hk.hikonv_pack_weights_ex(plan, w_d, co, c, 1, 3, 3, 2, pw)
        run = lambda: hk.hikonv_conv2d_prepacked(plan, x_d, hk.FMT_INT8, n, c, h, w, pw, co, 3, 3, 2, 1, ws, y)
        event_ms(run, 3)
        ms = event_ms(run, steps)
        rep[label] = dict(ms=ms, gops=2 * macs / ms / 1e6, plan=dict(N=plan.N, K=plan.K, S=plan.S, M=plan.M))
    run_u = lambda: hk.hikonv_conv2d_unpacked(4, 4, hk.signedness(True, True), x_d, n, c, h, w, w_d, co, 3, 3, 2, 1, y)
    event_ms(run_u, 3)
    rep["unpacked_ms"] = event_ms(run_u, steps)
    out["conv2d_stride2"] = rep

    # the binarised layer shape at a batch that fills the chip (the configuration itself has 8 images)
    n, c, h, w, co = 64, 256, 28, 28, 256
    xb = (rng.integers(0, 2, (n, c, h, w), dtype=np.int8) * 2 - 1).astype(np.int8)
    wb = (rng.integers(0, 2, (co, c, 3, 3), dtype=np.int8) * 2 - 1).astype(np.int8)
    x_d = torch.from_numpy(xb.view("uint8")).cuda()
    w_d = torch.from_numpy(wb.view("uint8")).cuda()
    plan = hk.hikonv_plan_ex(L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=0, taps=3, bits_a=1, bits_w=1, bipolar=1)
    ws = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, 3, 3, 1, 1, True), dtype=torch.uint8,
                     device="cuda")
    pw = torch.empty(hk.hikonv_packed_weights_bytes(plan, co, c, 3, 3), dtype=torch.uint8, device="cuda")
    hk.hikonv_pack_weights(plan, w_d, co, c, 3, 3, pw)
    y = torch.empty(n * co * h * w, dtype=torch.int32, device="cuda")
    runb = lambda: hk.hikonv_conv2d_prepacked(plan, x_d, hk.FMT_INT8, n, c, h, w, pw, co, 3, 3, 1, 1, ws, y)
    event_ms(runb, 3)
    ms = event_ms(runb, steps)
    macs = n * co * h * w * c * 9
    lane_mads = n * co * h * (-(-(w + 1) // plan.N)) * c * 3 * plan.chunks
    out["conv2d_c4_batch64"] = dict(shape="64x256x28x28 -> 256, 3x3, stride 1, pad 1, {-1,+1}", macs=macs, ms=ms,
                                    gops=2 * macs / ms / 1e6, plan=dict(N=plan.N, K=plan.K, S=plan.S, M=plan.M),
                                    frac_of_unpacked_valu_peak=macs / (ms * 1e-3) / VALU_LANE_RATE,
                                    roofline={"bound": "alu", "achieved": lane_mads / (ms * 1e-3) / 1e12,
                                              "peak": VALU_LANE_RATE / 1e12, "unit": "T lane-instr/s",
                                              "frac": lane_mads / (ms * 1e-3) / VALU_LANE_RATE,
                                              "note": "packed multiply-accumulates only, whole call (input packing included)"})
    del x_d, w_d, ws, pw, y
    torch.cuda.empty_cache()

    n, c, d, h, w, co = 1, 16, 16, 56, 56, 32
    x_d = torch.from_numpy(rng.integers(-8, 8, (n, c, d, h, w), dtype=np.int8).view("uint8")).cuda()
    w_d = torch.from_numpy(rng.integers(-8, 8, (co, c, 3, 3, 3), dtype=np.int8).view("uint8")).cuda()
    y = torch.empty(n * co * d * h * w, dtype=torch.int32, device="cuda")
    macs = n * co * d * h * w * c * 27
    plan = hk.hikonv_plan_ex(taps=3, **kw_plan)
    ws = torch.empty(hk.hikonv_conv3d_workspace_bytes(plan, n, c, d, h, w, co, 3, 3, 3, 1, 1, True), dtype=torch.uint8,
                     device="cuda")
    pw = torch.empty(hk.hikonv_packed_weights_bytes_ex(plan, co, c, 3, 3, 3, 1), dtype=torch.uint8, device="cuda")
    hk.hikonv_pack_weights_ex(plan, w_d, co, c, 3, 3, 3, 1, pw)
    run3 = lambda: hk.hikonv_conv3d(plan, x_d, hk.FMT_INT8, n, c, d, h, w, pw, True, co, 3, 3, 3, 1, 1, ws, y)
    event_ms(run3, 3)
    ms = event_ms(run3, steps)
    out["conv3d"] = dict(shape="1x16x16x56x56 -> 32, 3x3x3, stride 1, pad 1, int4", macs=macs, ms=ms,
                         gops=2 * macs / ms / 1e6, plan=dict(N=plan.N, K=plan.K, S=plan.S, M=plan.M))
    return out


def small_extras(hk, wl, steps):
    """Latency-scale configurations: the 4096-value 1-D case and the nine-layer 4-bit CNN forward
    (eager launches and the same launches replayed from a captured HIP graph)."""
    import torch
    from paper_2208_00763_amd.cnn import PackedCnn
    out = {}
    x, g = wl.config1()
    plan = hk.hikonv_plan_ex(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3)
    x_d = torch.from_numpy(x).cuda()
    g_d = torch.from_numpy(g).cuda()
    x_bd = torch.zeros(hk.hikonv_bitdense_row_bytes(4096, 4), dtype=torch.uint8, device="cuda")
    hk.hikonv_compact(x_d, 1, 4096, 4, False, x_bd)
    y = torch.empty(4094, dtype=torch.int32, device="cuda")
    run1 = lambda: hk.hikonv_conv1d(plan, x_bd, hk.FMT_BITDENSE, 1, 4096, g_d, 3, hk.OUT_VALID, y)
    event_ms(run1, 10)
    out["conv1d_c1_us_per_call"] = event_ms(run1, 200) * 1e3
    g1 = graph_replay_ms(run1, 50, 10)
    out["conv1d_c1_graph_us_per_call"] = g1 * 1e3 if g1 else None

    xi, weights, specs = wl.config5()
    net = PackedCnn([torch.from_numpy(w.view("uint8")).cuda() for w in weights], specs)
    x5 = torch.zeros(3 * 160 * hk.hikonv_bitdense_row_bytes(320, 4), dtype=torch.uint8, device="cuda")
    hk.hikonv_compact(torch.from_numpy(xi).cuda(), 3 * 160, 320, 4, False, x5)
    shifts = [4, 6, 7, 7, 7, 7, 7, 7]
    fwd = lambda: net.forward(x5, 1, 160, 320, shifts)
    event_ms(fwd, 3)
    out["cnn_c5_eager_us"] = event_ms(fwd, steps) * 1e3
    macs = 0
    h, w = 160, 320
    for wt, spec in zip(weights, specs):
        macs += wt.shape[0] * wt.shape[1] * wt.shape[2] * wt.shape[3] * h * w
        if spec["pool"]:
            h, w = h // 2, w // 2
    out["cnn_c5_macs"] = macs
    g5 = graph_replay_ms(fwd, 1, steps)
    out["cnn_c5_graph_us"] = g5 * 1e3 if g5 else None
    # the same chain with separate epilogue and packing passes (bit-dense activations between layers)
    plain = PackedCnn([torch.from_numpy(w.view("uint8")).cuda() for w in weights], specs, fused=False)
    fwd_plain = lambda: plain.forward(x5, 1, 160, 320, shifts)
    g5p = graph_replay_ms(fwd_plain, 1, steps)
    out["cnn_c5_unfused_graph_us"] = g5p * 1e3 if g5p else None
    return out


def sweep(hk, wl, steps):
    """All 48 cases of the 1-D bitwidth sweep (1..8 bit, signed and unsigned, 3/5/7 taps, 4096 rows
    of 65536 values, valid outputs): packed and unpacked kernel time, effective GOPS, achieved
    algorithmic HBM bandwidth."""
    import torch
    rows = []
    for bits in range(1, 9):
        for signed in (False, True):
            for taps in (3, 5, 7):
                case = conv1d_case(hk, wl, bits, signed, taps)
                event_ms(case["packed"], 2)
                ms_p = min(event_ms(case["packed"], steps) for _ in range(2))
                event_ms(case["unpacked"], 2)
                ms_u = min(event_ms(case["unpacked"], steps) for _ in range(2))
                plan = case["plan"]
                rows.append(dict(bits=bits, signed=signed, taps=taps, N=plan.N, K=plan.K, S=plan.S, chunks=plan.chunks,
                                 packed_ms=ms_p, unpacked_ms=ms_u, gops=2 * case["macs"] / ms_p / 1e6,
                                 gbs=case["bytes"] / ms_p / 1e6, hbm_frac=case["bytes"] / ms_p / 1e6 / HBM_PEAK_GBS,
                                 speedup_vs_unpacked=ms_u / ms_p))
                del case
                torch.cuda.empty_cache()
    return rows


def microbench(hk):
    """Issue rates (10^12 lane-instructions/s over the whole chip) and HBM bandwidths (TB/s)."""
    import torch
    kinds = {"v_mad_u32_u24": hk.UB_MAD_U32_U24, "v_mad_i32_i24": hk.UB_MAD_I32_I24,
             "v_mad_u64_u32": hk.UB_MAD_U64_U32, "v_mad_i64_i32": hk.UB_MAD_I64_I32,
             "v_mul_lo_u32": hk.UB_MUL_LO_U32, "v_bfe_u32": hk.UB_BFE_U32, "v_lshrrev_b64": hk.UB_LSHR_B64,
             "v_lshl_add_u64": hk.UB_ADD_U64, "v_alignbit_b32": hk.UB_ALIGNBIT, "v_mov_b32_dpp wave_shr:1": hk.UB_DPP_MOV}
    blocks, iters = 256 * 32, 2000                       # 32 waves per CU, 64 instructions per iteration
    buf = torch.zeros(blocks * 256, dtype=torch.int32, device="cuda")
    out = {"valu_T_lane_instr_per_s": {}, "hbm_TB_per_s": {}, "nominal_valu_T": VALU_LANE_RATE / 1e12}
    for name, kind in kinds.items():
        full = min(event_ms(lambda: hk.hikonv_ubench(kind, iters, blocks, buf), 3) for _ in range(3))
        empty = min(event_ms(lambda: hk.hikonv_ubench(kind, 0, blocks, buf), 3) for _ in range(3))
        out["valu_T_lane_instr_per_s"][name] = blocks * 256 * iters * 64 / ((full - empty) * 1e-3) / 1e12
    big = torch.zeros(2 * 1024 ** 3 // 4, dtype=torch.int32, device="cuda")
    for name, kind in (("write", hk.UB_HBM_WRITE), ("write_nontemporal", hk.UB_HBM_WRITE_NT),
                       ("write_nontemporal_runs_per_wave", hk.UB_HBM_WRITE_RUNS),
                       ("copy_read_plus_write", hk.UB_HBM_COPY), ("read", hk.UB_HBM_READ)):
        best = min(event_ms(lambda: hk.hikonv_ubench(kind, 0, nb, big), 5) for nb in (4096, 16384, 32768, 65536, 89240))
        out["hbm_TB_per_s"][name] = big.numel() * 4 / (best * 1e-3) / 1e12
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extras", action="store_true", help="only the headline case and its roofline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--ubench", action="store_true",
                    help="print the measured issue rate of the integer VALU instructions the kernels use and the "
                         "HBM write / copy / read bandwidth (the two rooflines), then exit")
    ap.add_argument("--sweep", action="store_true",
                    help="time all 48 cases of the 1-D bitwidth sweep (packed and unpacked), print them as JSON "
                         "and as a table, then exit")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain copy kernel of known size (512 MiB read + 512 MiB written, 3 launches) "
                         "so that HBM byte counters collected by a profiler can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (every box has one); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2208_00763_amd as hk
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2

    if args.ubench:
        print(json.dumps(microbench(hk)))
        return 0

    if args.sweep:
        rows = sweep(hk, wl, max(3, args.steps // 5))
        print(json.dumps({"metric": "1-D bitwidth sweep, 4096 rows x 65536, valid, bit-dense input", "cases": rows}))
        print("bits signed taps  N  K  S chunks  packed_ms unpacked_ms  speedup   GOPS  GB/s  frac_of_8TB/s", file=sys.stderr)
        for r in rows:
            print("%4d %6s %4d %2d %2d %2d %6d %10.4f %11.4f %8.2f %6.0f %5.0f %8.3f" % (
                r["bits"], "s" if r["signed"] else "u", r["taps"], r["N"], r["K"], r["S"], r["chunks"], r["packed_ms"],
                r["unpacked_ms"], r["speedup_vs_unpacked"], r["gops"], r["gbs"], r["hbm_frac"]), file=sys.stderr)
        return 0

    if args.calibrate:
        cal = torch.zeros(1024 ** 3 // 4, dtype=torch.int32, device="cuda")
        for _ in range(3):
            hk.hikonv_ubench(hk.UB_HBM_COPY, 0, 32768, cal)
        torch.cuda.synchronize()
        del cal

    head = conv1d_case(hk, wl, 4, False)
    for _ in range(args.warmup):
        head["packed"]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_kernel = event_ms(head["packed"], args.steps)          # exactly K steps between two events
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    gops = 2 * head["macs"] / (ms_kernel * 1e-3) / 1e9
    achieved_gbs = head["bytes"] / (ms_kernel * 1e-3) / 1e9

    traffic = None
    traffic_file = os.path.join(ROOT, "profiles", "conv1d_packed_c2_b4u_k3_traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            traffic = json.load(fh).get("hbm_bytes_per_launch")

    line = {
        "metric": "effective low-bit MACs/s (GOPS) at 4-bit, packed 1-D convolution",
        "value": gops, "unit": "GOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_kernel, "wall_ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "1-D sweep case: 4096 rows x 65536, K=3, 4-bit unsigned, valid, bit-dense input",
                   "plan": {k: getattr(head["plan"], k) for k in ("N", "K", "S", "G_b", "chunks")}},
        "roofline": {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved_gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "k_conv1d_fast<N=3>", "algorithmic_bytes_per_launch": head["bytes"]},
    }

    extras = {}
    if not args.no_extras:
        ms_unp = event_ms(head["unpacked"], max(3, args.steps // 5))
        extras["unpacked_4bit"] = dict(ms=ms_unp, gops=2 * head["macs"] / ms_unp / 1e6)
        by_bits = {"4u": dict(ms=ms_kernel, gops=gops, gbs=achieved_gbs)}
        x_keep, g_keep = head["x"], head["g"]
        for key in ("packed", "unpacked", "y", "keep"):
            head.pop(key)
        torch.cuda.empty_cache()
        for bits, signed in ((1, False), (8, False), (4, True), (1, True), (8, True)):
            case = conv1d_case(hk, wl, bits, signed)
            event_ms(case["packed"], 3)
            ms_p = event_ms(case["packed"], max(3, args.steps // 5))
            ms_u = event_ms(case["unpacked"], max(3, args.steps // 5))
            by_bits["%d%s" % (bits, "s" if signed else "u")] = dict(
                ms=ms_p, gops=2 * case["macs"] / ms_p / 1e6, gbs=case["bytes"] / ms_p / 1e6, unpacked_ms=ms_u,
                plan=dict(N=case["plan"].N, K=case["plan"].K, S=case["plan"].S, chunks=case["plan"].chunks))
            del case
            torch.cuda.empty_cache()
        extras["conv1d_by_bits"] = by_bits
        extras["conv1d_requant_bitdense_out"] = requant_extra(hk, wl, max(3, args.steps // 5))
        for name in ("c3", "c4"):
            extras["conv2d_" + name] = conv2d_extra(hk, wl, name, max(5, args.steps // 2))
        extras["widened_layers"] = widened_extras(hk, max(5, args.steps // 2))
        extras["latency"] = small_extras(hk, wl, max(5, args.steps // 2))
        head["x"], head["g"] = x_keep, g_keep
    line["extras"] = extras

    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(head["x"], head["g"])
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
