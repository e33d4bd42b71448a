#!/usr/bin/env python3
"""Benchmark of the dual-PoT hot path on one MI355X.

Default workload (`c2_gemv`): the seven batch-1 GEMVs of a LLaMA-2-7B-shaped decoder block
(q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008), W3/A16, group 128, as ONE grouped
launch per step, cycling over >= 1 GiB of distinct packed copies so that neither L2 nor the
256 MiB Infinity Cache can hold the weights.  A step = one pass of the whole path (stream codes,
decode, both slab dot products, coefficient rescale, store) over one block.

Prints ONE JSON line: metric / value / unit per the build contract, plus
  roofline     achieved algorithmic GB/s of the GEMV launch against the 8 TB/s HBM peak
  cpu_baseline the CPU oracle (as it stands) timed on the host cores on the same workload
Inputs are synthetic (seeded canonical arrays with the code histogram the GEO quantizer produces
on N(0, 0.02^2) + Student-t weights); they stand in for the LLaMA-2 checkpoint.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import goq_inputs  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
MFMA_I8_PEAK_TOPS = 5000.0
FP64_VECTOR_PEAK_TFLOPS = 78.6


def gemv_bytes(bw, shapes, ybytes=4):
    """Algorithmic bytes of one pass: (bw + 0.75 + 0.25) bits per weight + x (fp16) + y."""
    tot = 0
    for _, out, inn in shapes:
        tot += out * inn * (bw + 1) // 8 + inn * 2 + out * ybytes
    return tot


def _event_pairs(torch, n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _stats_us(per_step_us):
    a = np.sort(np.asarray(per_step_us, dtype=np.float64))
    return {"mean": round(float(a.mean()), 3), "median": round(float(np.median(a)), 3), "min": round(float(a[0]), 3)}


def quantize_block_on_device(goq, torch, shapes, bw, config_id, dev):
    """Seeded fp16 weights -> goq_quantize (GEO mode, on the device) -> goq_pack.  Returns the packed
    buffers' sizes, the packed tensors and the host weights (for the cpu_baseline leg)."""
    packed, host_w = [], []
    for idx, (_, out, inn) in enumerate(shapes):
        w = goq_inputs.weights(out, inn, config_id=config_id, tensor_id=idx)
        host_w.append(w)
        wd = torch.from_numpy(w.view(np.int16)).to(dev)
        codes = torch.empty((out, inn), dtype=torch.uint8, device=dev)
        pat = torch.empty((out, inn // 8), dtype=torch.uint8, device=dev)
        sg = torch.empty((out, inn // 8), dtype=torch.uint8, device=dev)
        c1 = torch.empty((out, inn // 128), dtype=torch.int16, device=dev)
        c2 = torch.empty((out, inn // 128), dtype=torch.int16, device=dev)
        goq.quantize(bw, out, inn, wd, codes, pat, sg, c1, c2)
        pk = torch.empty(goq.packed_bytes(bw, out, inn), dtype=torch.uint8, device=dev)
        goq.pack(bw, out, inn, codes, pat, sg, c1, c2, pk)
        torch.cuda.synchronize()
        packed.append(pk)
        del wd, codes, pat, sg, c1, c2
    return packed, host_w


def bench_gemv(args, shapes, bw, name):
    """Batch-1 workloads.  A step = one pass of the whole path over one block (all its matrices).
    Steps are issued as goq_gemv_stream launches of up to `stream_blocks` blocks -- e.g. the 32
    decoder blocks of LLaMA-2-7B: one token through the model's projections -- every block with
    packed weights of its own, so one launch streams stream_blocks x (block bytes) of distinct
    weights from HBM.  The one-block-per-launch figure (goq_gemv_batch) is reported beside it."""
    import torch
    import paper_2605_26092_amd as goq
    from paper_2605_26092_amd import binding

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    alg_bytes = gemv_bytes(bw, shapes)
    weight_bytes = sum(goq.packed_bytes(bw, o, i) for _, o, i in shapes)
    # blocks per launch: the 32 decoder blocks of LLaMA-2-7B; otherwise about 3 GiB of distinct weights
    NB = args.stream_blocks if args.stream_blocks > 0 else (
        32 if [s[1:] for s in shapes] == [s[1:] for s in goq_inputs.LLAMA2_7B_BLOCK]
        else max(8, min(128, int(np.ceil((3 << 30) / weight_bytes)))))
    copies = NB

    t_setup = time.time()
    packed0, host_w = quantize_block_on_device(goq, torch, shapes, bw, 2, dev)
    # all copies in one allocation (block after block), so that the read probe can stream the very
    # bytes a launch streams
    big = torch.empty(copies * weight_bytes, dtype=torch.uint8, device=dev)
    all_packed, off = [], 0
    for c in range(copies):
        blk = []
        for pk in packed0:
            view = big[off:off + pk.numel()]
            view.copy_(pk)
            blk.append(view)
            off += pk.numel()
        all_packed.append(blk)
    xs, ys = [], []
    for idx, (nm, out, inn) in enumerate(shapes):
        x = goq_inputs.activations_a16(1, inn, config_id=2, tensor_id=100 + idx, outlier_frac=0.01)
        xs.append(torch.from_numpy(x.reshape(-1)).to(dev))
    ys = [[torch.zeros(out, dtype=torch.float32, device=dev) for _, out, _ in shapes] for _ in range(copies)]
    stream = torch.cuda.current_stream()

    def problems(c):
        return [(o, i, all_packed[c][k], xs[k], None, ys[c][k], goq.F32) for k, (_, o, i) in enumerate(shapes)]

    ws = torch.empty(goq.gemv_workspace_bytes() + 256, dtype=torch.uint8, device=dev)
    ws = ws[(-ws.data_ptr()) % 256:][:goq.gemv_workspace_bytes()]
    goq.gemv_workspace_init(ws, stream=stream)
    tables = {}

    def stream_launch(nblocks):
        """a bound goq_gemv_stream launch over the first `nblocks` copies"""
        if nblocks not in tables:
            probs = [p for c in range(nblocks) for p in problems(c)]
            th, nbytes = goq.gemv_stream_table(bw, goq.A16, probs)
            import ctypes
            raw = np.frombuffer((ctypes.c_ubyte * nbytes).from_address(ctypes.addressof(th)), dtype=np.uint8).copy()
            td = torch.from_numpy(raw).to(dev)
            tables[nblocks] = (th, td, binding.bind_gemv_stream(th, td, ws, stream))
        return tables[nblocks][2]

    def plan(nsteps):
        """launches (blocks each) that make up nsteps steps"""
        return [NB] * (nsteps // NB) + ([nsteps % NB] if nsteps % NB else [])

    for nb in set(plan(args.steps) + plan(args.warmup) + [NB]):
        stream_launch(nb)
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    # clock settle (part of set-up, untimed, echoed as effective warm-up): short runs end before the
    # GPU's clock governor has reacted to the load
    settle_steps = 0
    t_end = time.perf_counter() + args.settle_ms * 1e-3
    while time.perf_counter() < t_end:
        stream_launch(NB)()
        settle_steps += NB
        if settle_steps % (8 * NB) == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    for nb in plan(args.warmup):
        stream_launch(nb)()
    torch.cuda.synchronize()

    timed = plan(args.steps)
    ev = _event_pairs(torch, len(timed) + 1)
    t0 = time.perf_counter()
    ev[0].record(stream)
    for j, nb in enumerate(timed):
        stream_launch(nb)()
        ev[j + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / args.steps
    dev_ms = ev[0].elapsed_time(ev[-1]) / args.steps
    per_step_us = [ev[j].elapsed_time(ev[j + 1]) * 1e3 / nb for j, nb in enumerate(timed)]
    full_us = [ev[j].elapsed_time(ev[j + 1]) * 1e3 for j, nb in enumerate(timed) if nb == NB]

    # one block per launch (goq_gemv_batch), rotating over the copies: what a caller pays who launches
    # block by block
    single = [binding.bind_gemv_batch(bw, goq.A16, binding.make_descs(problems(c)), stream) for c in range(copies)]
    n1 = max(64, min(args.steps, 2000))
    for j in range(max(200, args.warmup)):
        single[j % copies]()
    torch.cuda.synchronize()
    chunk = 16                                           # events every 16 launches: median / min of those
    evs = _event_pairs(torch, n1 // chunk + 1)
    evs[0].record(stream)
    for j in range(n1 // chunk * chunk):
        single[j % copies]()
        if j % chunk == chunk - 1:
            evs[j // chunk + 1].record(stream)
    torch.cuda.synchronize()
    single_us = [evs[j].elapsed_time(evs[j + 1]) * 1e3 / chunk for j in range(n1 // chunk)]
    single_mean_us = evs[0].elapsed_time(evs[-1]) * 1e3 / (n1 // chunk * chunk)
    # the same copy every launch: cache-resident figure, labelled, not the headline
    for j in range(20):
        single[0]()
    torch.cuda.synchronize()
    evs[0].record(stream)
    for j in range(n1):
        single[0]()
    evs[1].record(stream)
    torch.cuda.synchronize()
    hot_us = evs[0].elapsed_time(evs[1]) * 1e3 / n1

    # each matrix as a launch of its own
    per_matrix = []
    if len(shapes) > 1:
        for k, (nm, o, i) in enumerate(shapes):
            one = [binding.bind_gemv_batch(bw, goq.A16, binding.make_descs([problems(c)[k]]), stream) for c in range(copies)]
            n2 = max(50, min(args.steps, 500))
            for j in range(50):
                one[j % copies]()
            torch.cuda.synchronize()
            evs[0].record(stream)
            for j in range(n2):
                one[j % copies]()
            evs[1].record(stream)
            torch.cuda.synchronize()
            us = evs[0].elapsed_time(evs[1]) / n2 * 1e3
            nbytes = o * i * (bw + 1) / 8.0 + 2.0 * i + 4.0 * o
            per_matrix.append({"name": nm, "out": o, "in": i, "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                               "kernel": gemv_kernel_name(bw, [(nm, o, i)])})

    # measured ceiling: a pure read stream over the bytes one full launch streams
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    nprobe = NB * weight_bytes
    for _ in range(2):
        goq.read_probe(big, nprobe, sink, stream=stream)
    torch.cuda.synchronize()
    pe = _event_pairs(torch, 6)
    pe[0].record(stream)
    for j in range(5):
        goq.read_probe(big, nprobe, sink, stream=stream)
        pe[j + 1].record(stream)
    torch.cuda.synchronize()
    probe_gbs = [nprobe / (pe[j].elapsed_time(pe[j + 1]) * 1e-3) / 1e9 for j in range(5)]

    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    launch_us = float(np.mean(full_us)) if full_us else dev_ms * 1e3 * timed[0]
    res = {
        "metric": "PoT GEMV GB/s (% HBM peak) and GEMM TOPS (% MFMA peak), LLaMA-2-7B shapes",
        "value": round(achieved, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dev_ms, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 x as eight 3-bit E5M2 digits of 24-bit block fixed point, E5M2 PoT weights, fp8 MFMA, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": name, "bw": bw, "act": "A16", "group": 128, "matrices": len(shapes),
                   "weights": int(sum(o * i for _, o, i in shapes)), "algorithmic_bytes_per_step": int(alg_bytes),
                   "weights_from": "seeded fp16 weights quantised by goq_quantize (GEO mode) on the device",
                   "launch": "goq_gemv_stream: up to %d blocks (steps) per launch, each block with packed weights of its own" % NB,
                   "stream_blocks": NB, "distinct_packed_bytes": int(copies * weight_bytes),
                   "launches_timed": len(timed), "blocks_per_launch": timed if len(timed) <= 4 else [timed[0], "...", timed[-1]],
                   "clock": "HIP events on the launch stream, first launch to last (value, ms_per_step, roofline use it)",
                   "wall_ms_per_step": round(wall_ms, 6),
                   "step_us": _stats_us(per_step_us),
                   "setup_s": round(setup_s, 1), "settle_ms": args.settle_ms,
                   "effective_warmup_steps": settle_steps + args.warmup,
                   "single_block_launch": {"entry": "goq_gemv_batch, one block per launch, rotating over the copies",
                                           "kernel": gemv_kernel_name(bw, shapes), "us": _stats_us(single_us),
                                           "GBps": round(alg_bytes / single_mean_us / 1e3, 1),
                                           "frac": round(alg_bytes / single_mean_us / 1e3 / HBM_PEAK_GBS, 4),
                                           "cache_resident_GBps": round(alg_bytes / hot_us / 1e3, 1)},
                   "per_matrix_launches": per_matrix,
                   "per_matrix_total_us": round(sum(m["us"] for m in per_matrix), 2) if per_matrix else None},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "gemv_stream_kernel<%d,0>" % bw, "avg_launch_us": round(launch_us, 3),
                     "units_per_launch": "%d blocks" % (NB if full_us else timed[0]),
                     "peak_measured": {"value": round(max(probe_gbs), 1), "mean": round(float(np.mean(probe_gbs)), 1), "unit": "GB/s",
                                       "what": "goq_read_probe: pure nontemporal read stream over the %d bytes one full launch streams, 512 x 512 threads" % nprobe}},
    }
    # HBM traffic per launch from the committed counter runs (FETCH_SIZE + WRITE_SIZE, scaled), if present
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json.txt")) as fh:
            t = json.load(fh)["gemv_stream_kernel<%d,0>" % bw]
            if t["workload"] == name and t["stream_blocks"] == NB:
                res["roofline"]["traffic"] = t["hbm_bytes_per_launch"]
                res["roofline"]["traffic_source"] = t["source"]
    except (OSError, KeyError, ValueError):
        pass
    if args.traffic_ref:
        # reference dispatches of known traffic for scaling FETCH_SIZE / WRITE_SIZE counter runs:
        # an elementwise add over 64 Mi int32 reads 256 MiB and writes 256 MiB
        src = torch.ones(64 << 20, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    if args.gemm_tokens > 0:
        res["gemm"] = bench_gemm_block(args, shapes, bw, goq.A16, packed0, args.gemm_tokens)
    res["cpu_baseline"] = cpu_baseline_gemv(host_w, shapes, bw, alg_bytes) if not args.no_cpu else None
    return res


def mfma_peak_measured(goq, torch, kind, stream):
    """goq_mfma_rate_probe: a loop of nothing but the matrix instruction (kind 0: f16 32x32x16, 1: i8
    32x32x32), four independent accumulators per wavefront, 4 wavefronts per SIMD on every CU."""
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    iters, wgs = 4096, 256 * 4
    goq.mfma_rate_probe(kind, wgs, 256, sink, stream=stream)
    torch.cuda.synchronize()
    best = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        ops = goq.mfma_rate_probe(kind, wgs, iters, sink, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        best = max(best, ops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return {"value": round(best, 1), "unit": "TFLOP/s" if kind == 0 else "TOP/s",
            "what": "goq_mfma_rate_probe: %s only, %d workgroups x 4 wavefronts x %d x 4 instructions, best of 3"
                    % ("v_mfma_f32_32x32x16_f16" if kind == 0 else "v_mfma_i32_32x32x32_i8", wgs, iters)}


def gemv_kernel_name(bw, shapes):
    """The kernel the library launches for these layers in one goq_gemv_batch call (goq_gemv_plan)."""
    import paper_2605_26092_amd as goq
    kernel, _ = goq.gemv_plan(bw, goq.A16, [(out, inn) for _, out, inn in shapes])
    return ("gemv_rows_kernel<%d,0>" if kernel == goq.GEMV_ROWS else "gemv_kernel<%d,0>") % bw


def bench_gemm_block(args, shapes, bw, act, packed, tokens, steps=10, warmup=2, folded=False):
    """The same block as many-token GEMMs (one goq_gemm_batch launch): issued ops = 4 M N K (two PoT
    bases), dense-equivalent = 2 M N K.  Reported next to the headline, not instead of it.
    folded: the ablation goq_gemm_folded (one contraction with the fp16 weight c1 b1 + c2 b2):
    issued = dense-equivalent = 2 M N K."""
    import torch
    import paper_2605_26092_amd as goq
    dev = torch.device("cuda:0")
    Xs, Ys, sxs = [], [], []
    for idx, (_, out, inn) in enumerate(shapes):
        if act == goq.A16:
            x = goq_inputs.activations_a16(tokens, inn, config_id=3, tensor_id=100 + idx, outlier_frac=0.01)
            sxs.append(None)
        elif act == goq.A8:
            x, sx = goq_inputs.activations_a8(tokens, inn, config_id=4, tensor_id=200 + idx)
            sxs.append(torch.from_numpy(sx).to(dev))
        elif act == goq.A6:
            x, sx = goq_inputs.activations_int(tokens, inn, 6, config_id=4, tensor_id=200 + idx)
            x = goq_inputs.pack_int6(x)
            sxs.append(torch.from_numpy(sx).to(dev))
        else:
            x, sx = goq_inputs.activations_int(tokens, inn, 4, config_id=4, tensor_id=200 + idx)
            x = goq_inputs.pack_int4(x)
            sxs.append(torch.from_numpy(sx).to(dev))
        Xs.append(torch.from_numpy(x).to(dev))
        Ys.append(torch.zeros((tokens, out), dtype=torch.float16, device=dev))
    stream = torch.cuda.current_stream()

    from paper_2605_26092_amd import binding
    descs = binding.make_gemm_descs([(tokens, out, inn, packed[k], Xs[k], sxs[k], Ys[k], goq.F16)
                                     for k, (_, out, inn) in enumerate(shapes)])

    def step():
        if folded:                   # the ablation has no batched entry point: one launch per matrix
            for k, (_, out, inn) in enumerate(shapes):
                goq.gemm_folded(bw, tokens, out, inn, packed[k], Xs[k], Ys[k], goq.F16, stream=stream)
        else:                        # the block's matrices as one grid (goq_gemm_batch)
            goq.gemm_batch(bw, act, descs, stream=stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    issued = (2.0 if folded else 4.0) * tokens * sum(o * i for _, o, i in shapes)
    # the peak of the matrix instruction the path runs on: fp16 for A16 and for bw = 4 with
    # integer activations (widened to fp16), int8 otherwise
    f16_path = act == goq.A16 or bw == 4
    peak = MFMA_F16_PEAK_TFLOPS if f16_path else MFMA_I8_PEAK_TOPS
    tops = issued / (ms * 1e-3) / 1e12
    measured = mfma_peak_measured(goq, torch, 0 if f16_path else 1, stream)
    # HBM traffic per launch (mean over the block's matrices) from the committed counter runs, if
    # they cover this workload: the 7B block at 2048 tokens, W3/A16
    traffic, traffic_source = None, None
    if bw == 3 and act == goq.A16 and tokens == 2048 and not folded and len(shapes) == 7 and shapes[0][1] == 4096:
        try:
            with open(os.path.join(ROOT, "profiles", "traffic.json.txt")) as fh:
                t = json.load(fh)["gemm_kernel<3,0,false>"]
                traffic, traffic_source = t["hbm_bytes_per_launch"], t.get("source")
        except (OSError, KeyError, ValueError):
            pass
    return {"workload": "same block as GEMMs, %d tokens, W%d/%s" % (tokens, bw, {goq.A16: "A16", goq.A8: "A8", goq.A4: "A4", goq.A6: "A6"}[act]),
            "ms_per_block": round(ms, 4), "issued_TOPS": round(tops, 1),
            "dense_equiv_TOPS": round(tops if folded else tops / 2, 1),
            "roofline": {"bound": "mfma", "achieved": round(tops, 1), "peak": peak, "unit": "TFLOP/s" if f16_path else "TOP/s",
                         "frac": round(tops / peak, 4), "traffic": traffic, "traffic_source": traffic_source,
                         "peak_measured": measured}}


def bench_gemm_only(args, shapes, bw, act_name, tokens, name, folded=False):
    """A GEMM workload on its own (BASELINE configs 3, 4 and the GEMM half of 5): the block's
    matrices in one goq_gemm_batch launch per step; value = issued TOPS (4 M N K per matrix)."""
    import torch
    import paper_2605_26092_amd as goq
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    act = {"A16": goq.A16, "A8": goq.A8, "A4": goq.A4, "A6": goq.A6}[act_name]
    packed, host_w = quantize_block_on_device(goq, torch, shapes, bw, 3, dev)
    g = bench_gemm_block(args, shapes, bw, act, packed, tokens, steps=max(3, min(args.steps, 20)), warmup=2,
                         folded=folded)
    res = {
        "metric": "PoT GEMV GB/s (% HBM peak) and GEMM TOPS (% MFMA peak), LLaMA-2-7B shapes",
        "value": g["issued_TOPS"], "unit": g["roofline"]["unit"], "n_gpus": 1, "steps": max(3, min(args.steps, 20)),
        "warmup": 2, "ms_per_step": g["ms_per_block"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if (act_name == "A16" or bw == 4) else "i8", "data": "synthetic",
        "config": {"workload": name, "bw": bw, "act": act_name, "group": 128, "tokens": tokens, "matrices": len(shapes),
                   "issued_ops_per_step": (2.0 if folded else 4.0) * tokens * sum(o * i for _, o, i in shapes),
                   "dense_equiv_TOPS": g["dense_equiv_TOPS"],
                   "weights_from": "seeded fp16 weights quantised by goq_quantize (GEO mode) on the device",
                   "clock": "HIP events on the launch stream around the timed launches"},
        "roofline": g["roofline"],
    }
    res["cpu_baseline"] = None if args.no_cpu else cpu_baseline_gemm(host_w[0], shapes, bw, act_name, tokens)
    return res


def bench_quantize(args, shapes, bw, name):
    """The GEO quantizer on the device (goq_quantize): a step quantizes every matrix of the block.
    Not the headline metric: reported in weights/s.  It is bound by vector-ALU issue (one lane per
    micro-block, everything in registers, fp64 arithmetic with exact sums), so the roofline is the
    fp64 vector peak against the method's real-arithmetic operations per weight; its HBM traffic
    (2 B read + 1 B codes + 0.25 B metadata + 4/128 B coefficients written per weight) is reported
    under config."""
    import torch
    import paper_2605_26092_amd as goq
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bufs = []
    for idx, (_, out, inn) in enumerate(shapes):
        w = goq_inputs.weights(out, inn, config_id=6, tensor_id=idx)
        bufs.append((out, inn, torch.from_numpy(w.view(np.int16)).to(dev),
                     torch.empty((out, inn), dtype=torch.uint8, device=dev),
                     torch.empty((out, inn // 8), dtype=torch.uint8, device=dev),
                     torch.empty((out, inn // 8), dtype=torch.uint8, device=dev),
                     torch.empty((out, inn // 128), dtype=torch.int16, device=dev),
                     torch.empty((out, inn // 128), dtype=torch.int16, device=dev), w))
    stream = torch.cuda.current_stream()
    steps, warmup = max(3, min(args.steps, 20)), 2

    def step():
        for out, inn, wd, c, p, sg, c1, c2, _ in bufs:
            goq.quantize(bw, out, inn, wd, c, p, sg, c1, c2, stream=stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    nw = sum(o * i for _, o, i in shapes)
    nbytes = nw * (2 + 1 + 0.25 + 4.0 / 128)
    gbs = nbytes / (ms * 1e-3) / 1e9
    # fp64 operations of the method per weight (Sec. 3.2 - 3.4, nearest state by midpoint compares):
    # |w| and max 2, midpoint compares 2^(bw-1) + 1, <w,b1> and ||b1||^2 4, residual 2, cross terms
    # 16 pairs x (2 mul, sub, abs, add) / 8 = 10, pair signs 2, <w,b2> and ||b2||^2 4
    flop_per_weight = 2 + ((1 << (bw - 1)) + 1) + 4 + 2 + 10 + 2 + 4
    tflops = nw * flop_per_weight / (ms * 1e-3) / 1e12
    res = {
        "metric": "GEO quantizer, weights/s (LLaMA-2-7B block shapes)", "value": round(nw / (ms * 1e-3) / 1e9, 2),
        "unit": "Gweights/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": name, "bw": bw, "group": 128, "matrices": len(shapes), "weights": int(nw),
                   "llama2_7b_32_blocks_s": round(32 * ms * 1e-3, 4), "hbm_GBps": round(gbs, 1),
                   "fp64_ops_per_weight": flop_per_weight},
        "roofline": {"bound": "alu", "achieved": round(tflops, 2), "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / FP64_VECTOR_PEAK_TFLOPS, 4), "traffic": None, "kernel": "quantize_kernel<%d>" % bw},
    }
    if args.no_cpu:
        res["cpu_baseline"] = None
    else:
        from oracle import goq_oracle as O
        threads = min(O.max_threads(), os.cpu_count() or 1)
        w = bufs[0][8][:1024]
        reps, t0 = 0, time.perf_counter()
        while True:
            O.quantize_geo(bw, w, threads=threads)
            reps += 1
            el = time.perf_counter() - t0
            if el > 10.0 or reps >= 5000:
                break
        res["cpu_baseline"] = {"value": round(w.size * reps / el / 1e9, 5), "unit": "Gweights/s", "cores": threads,
                               "kind": "oracle", "sample": "%d pass(es) over the first 1024 rows of the first matrix (%d weights), %.1f s"
                               % (reps, w.size, el)}
    return res


def bench_ref(args, shapes, bw, tokens, name):
    """REF-mode coefficients on the device (goq_ref_coefficients): a step re-solves (c1, c2) of every
    macro-block of every matrix of the block from `tokens` calibration rows.  Not the headline
    metric; fp64 arithmetic, so the roofline is the fp64 vector peak against the operations of the
    Gram-matrix formulation (2 T 128 in per matrix for the Gram matrices, 4 * 128^2 + 10 * 128 per
    output channel and macro-block for the two products and five dot products)."""
    import torch
    import paper_2605_26092_amd as goq
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bufs, flops = [], 0.0
    for idx, (_, out, inn) in enumerate(shapes):
        w = goq_inputs.weights(out, inn, config_id=7, tensor_id=idx)
        x = goq_inputs.activations_a16(tokens, inn, config_id=7, tensor_id=100 + idx, outlier_frac=0.01)
        gn = inn // 128
        wd = torch.from_numpy(w.view(np.int16)).to(dev)
        # bases from the GEO quantizer on the device (its coefficients are what REF mode replaces)
        codes = torch.empty((out, inn), dtype=torch.uint8, device=dev)
        pat = torch.empty((out, inn // 8), dtype=torch.uint8, device=dev)
        sg = torch.empty((out, inn // 8), dtype=torch.uint8, device=dev)
        g1 = torch.empty((out, gn), dtype=torch.int16, device=dev)
        g2 = torch.empty((out, gn), dtype=torch.int16, device=dev)
        goq.quantize(bw, out, inn, wd, codes, pat, sg, g1, g2)
        torch.cuda.synchronize()
        bufs.append((out, inn, wd, codes, pat, sg,
                     torch.from_numpy(x.view(np.int16)).to(dev),
                     torch.empty(goq.ref_workspace_bytes(inn), dtype=torch.uint8, device=dev),
                     torch.empty((out, gn), dtype=torch.int16, device=dev),
                     torch.empty((out, gn), dtype=torch.int16, device=dev), (w, x)))
        flops += 2.0 * tokens * 128 * inn + out * gn * (4.0 * 128 * 128 + 10 * 128)
    stream = torch.cuda.current_stream()
    steps, warmup = max(3, min(args.steps, 20)), 2

    def step():
        for out, inn, wd, c, p, sg, xd, ws, c1, c2, _ in bufs:
            goq.ref_coefficients(bw, tokens, out, inn, wd, c, p, sg, xd, 1e-4, ws, None, c1, c2, stream=stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    nw = sum(o * i for _, o, i in shapes)
    tflops = flops / (ms * 1e-3) / 1e12
    res = {
        "metric": "REF-mode coefficients, weights/s (LLaMA-2-7B block shapes)", "value": round(nw / (ms * 1e-3) / 1e9, 2),
        "unit": "Gweights/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": name, "bw": bw, "group": 128, "matrices": len(shapes), "weights": int(nw),
                   "calibration_tokens": tokens, "lambda": 1e-4, "fp64_ops_per_step": flops,
                   "llama2_7b_32_blocks_s": round(32 * ms * 1e-3, 4)},
        "roofline": {"bound": "alu", "achieved": round(tflops, 2), "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / FP64_VECTOR_PEAK_TFLOPS, 4), "traffic": None, "kernel": "ref_solve_kernel<%d>" % bw},
    }
    if args.no_cpu:
        res["cpu_baseline"] = None
    else:
        from oracle import goq_oracle as O
        threads = min(O.max_threads(), os.cpu_count() or 1)
        w, x = bufs[0][10]
        rows, tk = 64, 64
        qs = O.quantize_geo(bw, w[:rows], threads=threads)       # the oracle's own bases, untimed
        reps, t0 = 0, time.perf_counter()
        while True:
            O.ref_coefficients(qs, w[:rows], x[:tk], lam=1e-4, threads=threads)
            reps += 1
            el = time.perf_counter() - t0
            if el > 10.0 or reps >= 5000:
                break
        # weights/s at the benchmark's token count: the oracle's cost is linear in the tokens
        res["cpu_baseline"] = {"value": round(rows * w.shape[1] * reps / el / 1e9 * tk / tokens, 6), "unit": "Gweights/s",
                               "cores": threads, "kind": "oracle",
                               "sample": "%d pass(es) over the first %d rows of the first matrix with %d tokens (scaled to %d tokens), %.1f s"
                               % (reps, rows, tk, tokens, el)}
    return res


def cpu_baseline_gemm(w0, shapes, bw, act_name, tokens):
    """The oracle on a token slab of the first matrix (all outputs; the matrix quantised by the
    oracle's own GEO quantizer first, untimed), issued-op rate."""
    from oracle import goq_oracle as O
    threads = min(O.max_threads(), os.cpu_count() or 1)
    _, out, inn = shapes[0]
    canon = [O.quantize_geo(bw, w0, threads=threads)]
    slab = 32 if act_name == "A16" else 64
    if act_name == "A16":
        x = goq_inputs.activations_a16(slab, inn, config_id=3, tensor_id=100, outlier_frac=0.01)
    elif act_name == "A8":
        x, sx = goq_inputs.activations_a8(slab, inn, config_id=4, tensor_id=200)
    else:
        x, sx = goq_inputs.activations_int(slab, inn, 6 if act_name == "A6" else 4, config_id=4, tensor_id=200)
    reps, t0 = 0, time.perf_counter()
    while True:
        if act_name == "A16":
            O.gemm_a16(canon[0], x, threads=threads)
        else:
            O.gemm_a8(canon[0], x, sx, threads=threads)
        reps += 1
        el = time.perf_counter() - t0
        if el > 10.0 or reps >= 20000:
            break
    return {"value": round(4.0 * slab * out * inn * reps / el / 1e12, 5), "unit": "TOP/s (issued)", "cores": threads,
            "kind": "oracle", "sample": "%d pass(es) over a %d-token slab of the first matrix (%dx%d), all outputs, %.1f s"
            % (reps, slab, out, inn, el)}


def cpu_baseline_gemv(host_w, shapes, bw, alg_bytes):
    """The oracle, untuned, on the host cores: the same block of GEMVs (weights quantised by the
    oracle's own GEO quantizer first, untimed)."""
    from oracle import goq_oracle as O
    threads = min(O.max_threads(), os.cpu_count() or 1)
    canon = [O.quantize_geo(bw, w, threads=threads) for w in host_w]
    xs = [goq_inputs.activations_a16(1, inn, config_id=2, tensor_id=100 + k, outlier_frac=0.01)
          for k, (_, _, inn) in enumerate(shapes)]
    reps, t0 = 0, time.perf_counter()
    while True:
        for q, x in zip(canon, xs):
            O.gemm_a16(q, x, threads=threads)
        reps += 1
        el = time.perf_counter() - t0
        if el > 10.0 or reps >= 2000:
            break
    return {"value": round(alg_bytes * reps / el / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "%d pass(es) of the full block (all %d GEMVs, all rows), %.1f s" % (reps, len(shapes), el)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=192)
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="GEMV workloads: milliseconds of untimed launches before the warm-up that let the GPU clocks settle")
    ap.add_argument("--stream-blocks", type=int, default=0,
                    help="GEMV workloads: blocks per goq_gemv_stream launch (0 = by workload: 32 for the 7B block)")
    ap.add_argument("--workload", default="c2_gemv", choices=["c2_gemv", "c1_gemv", "c5_gemv", "c3_gemm_w3", "c3_gemm_w4", "c4_gemm_a8", "c4_gemm_a4", "c4_gemm_a6", "c4_gemm_w4a8", "c5_gemm", "q_geo_w3", "q_geo_w4", "ref_w3", "c3_gemm_folded", "c2_gemv_w4"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--traffic-ref", action="store_true",
                    help="also run a 256 MiB-in / 256 MiB-out elementwise kernel (reference for counter runs)")
    ap.add_argument("--gemm-tokens", type=int, default=2048,
                    help="also time the block as GEMMs with this many tokens (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of the path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.workload == "c2_gemv":
        res = bench_gemv(args, goq_inputs.LLAMA2_7B_BLOCK, 3, "llama2-7b decoder block, 7 GEMVs, W3/A16, batch 1")
    elif args.workload == "c2_gemv_w4":
        res = bench_gemv(args, goq_inputs.LLAMA2_7B_BLOCK, 4, "llama2-7b decoder block, 7 GEMVs, W4/A16, batch 1")
    elif args.workload == "c1_gemv":
        res = bench_gemv(args, [("l", 4096, 4096)], 3, "single 4096x4096 layer, W3/A16, batch 1")
    elif args.workload == "c5_gemv":
        res = bench_gemv(args, goq_inputs.LLAMA2_70B_LAYER, 3, "llama2-70b layer, 7 GEMVs, W3/A16, batch 1")
    elif args.workload in ("q_geo_w3", "q_geo_w4"):
        bw = 3 if args.workload == "q_geo_w3" else 4
        res = bench_quantize(args, goq_inputs.LLAMA2_7B_BLOCK, bw, "GEO quantization of a llama2-7b decoder block, W%d" % bw)
    elif args.workload == "ref_w3":
        res = bench_ref(args, goq_inputs.LLAMA2_7B_BLOCK, 3, 512, "REF coefficients of a llama2-7b decoder block, W3, 512 calibration tokens")
    elif args.workload == "c3_gemm_w3":
        res = bench_gemm_only(args, goq_inputs.LLAMA2_7B_BLOCK, 3, "A16", 2048, "llama2-7b block GEMMs, 2048 tokens, W3/A16")
    elif args.workload == "c3_gemm_folded":
        res = bench_gemm_only(args, goq_inputs.LLAMA2_7B_BLOCK, 3, "A16", 2048,
                              "ablation: llama2-7b block GEMMs, 2048 tokens, W3/A16, bases folded to one fp16 weight (2 M N K)",
                              folded=True)
    elif args.workload == "c3_gemm_w4":
        res = bench_gemm_only(args, goq_inputs.LLAMA2_7B_BLOCK, 4, "A16", 2048, "llama2-7b block GEMMs, 2048 tokens, W4/A16")
    elif args.workload == "c4_gemm_a8":
        res = bench_gemm_only(args, goq_inputs.VIT_B_BLOCK, 3, "A8", 197 * 64, "vit-b block GEMMs, 197x64 tokens, W3/A8")
    elif args.workload == "c4_gemm_a4":
        res = bench_gemm_only(args, goq_inputs.VIT_B_BLOCK, 3, "A4", 197 * 64, "vit-b block GEMMs, 197x64 tokens, W3/A4")
    elif args.workload == "c4_gemm_a6":
        res = bench_gemm_only(args, goq_inputs.VIT_B_BLOCK, 3, "A6", 197 * 64, "vit-b block GEMMs, 197x64 tokens, W3/A6 (packed int6)")
    elif args.workload == "c4_gemm_w4a8":
        res = bench_gemm_only(args, goq_inputs.VIT_B_BLOCK, 4, "A8", 197 * 64, "vit-b block GEMMs, 197x64 tokens, W4/A8")
    else:
        res = bench_gemm_only(args, goq_inputs.LLAMA2_70B_LAYER, 3, "A16", 512, "llama2-70b layer GEMMs, 512 tokens, W3/A16")
    print(json.dumps(res))


if __name__ == "__main__":
    main()
