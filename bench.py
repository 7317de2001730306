#!/usr/bin/env python3
"""ECF8 decode benchmark on one MI355X.

One step = one pass of the whole hot path over the workload: every tensor of the
stack is decoded from its resident compressed blob to exact FP8 bytes.  By
default the whole stack goes through ONE ecf8_decode_batched launch per step
(--launch stack); --launch layer issues one batched launch per layer/block
instead, on --streams streams round-robin.  Inputs are seeded synthetic
alpha-stable FP8 weights (recipe in paper_2510_02676_amd/synth.py); blobs and output buffers are resident
in HBM before the timed region starts.

With no --workload the headline is the largest single-GPU configuration, the
40-block diffusion-transformer stack (config3, 20.3 G weights); the same JSON
line carries the 8B-class LLM stack (config1, with its per-layer-launch rates)
and the 256-expert MoE layer (config2) under "configs", the LLM stack coded
with the plain Huffman code (no cap on the code length) under "plain_huffman",
each with its own roofline object, and the CPU oracle timed on a bounded sample,
on one core and on all of the machine's cores.  --workload configN times one
configuration alone (what the rocprofv3 summaries under profiles/ were made with).

Prints ONE JSON line: decoded FP8 GB/s as `value`, the roofline of the decode
kernel, and the extras above.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def algorithmic_bytes(h):
    """Bytes the method itself must move for one tensor: stream + nibble plane +
    lane/chunk metadata + header read, n_elem written."""
    rd = (h.stream_bits + 7) // 8 + (h.n_elem + 1) // 2 + 8 * (h.n_chunks + 1) + 2 * 64 * h.n_chunks + 256
    return rd, h.n_elem


def build_workload(name, seed, lane_syms, layers, launch="layer", group_chunks=0, max_code_len=0, cpu_encode=False, arena=False):
    from paper_2510_02676_amd import ecf8, synth
    if name == "config1":
        specs = synth.config1(seed, layers)
        group = lambda s: s["layer"]
        desc = "8B-class dense LLM stack, %d layers x 7 matrices" % layers
    elif name == "config3":
        specs = synth.config3(layers)
        group = lambda s: s["block"]
        desc = "14B-class DiT stack, %d blocks x 11 matrices" % layers
    elif name == "config2":
        specs = synth.config2(seed, layers)
        group = lambda s: 0 if "expert" in s else 1
        desc = "671B-class MoE layer, %d experts x 3 matrices + 2 attention projections" % layers
    elif name == "config0":
        specs = synth.config0()
        group = lambda s: 0
        desc = "single 1024x1024 matrix"
    else:
        raise SystemExit("unknown workload " + name)
    dev = "cuda:0"
    groups = {}
    t0 = time.time()
    for s in specs:
        w = synth.make(s, seed, device=dev)                       # uint8 (rows, cols) on the GPU
        if cpu_encode:
            blob = ecf8.ecf8_encode(w.cpu(), s["rows"], s["cols"], lane_syms=lane_syms, group_chunks=group_chunks,
                                    max_code_len=max_code_len)
            hdr, d_blob = blob.header, blob.to(dev)
        else:       # the device encoder writes the same container byte for byte (tests/test_gpu_encode.py), much faster
            hdr, big = ecf8.ecf8_encode_gpu(w, s["rows"], s["cols"], lane_syms=lane_syms, group_chunks=group_chunks,
                                            max_code_len=max_code_len)
            d_blob = big.clone()                                   # drops the encoder's worst-case allocation
            del big
        d_out = torch.empty((s["rows"], s["cols"]), dtype=torch.uint8, device=dev)
        groups.setdefault(group(s), []).append(dict(spec=s, w=w, hdr=hdr, d_blob=d_blob, d_out=d_out))
    if arena:
        # one allocation for all blobs and one for all outputs (tensors at multiples of 4 KiB inside them), the way a
        # serving process would hold a model, instead of one allocation per tensor
        al = lambda n: (n + 4095) // 4096 * 4096
        ts = [t for g in sorted(groups) for t in groups[g]]
        nb_all, no_all = sum(al(t["d_blob"].numel()) for t in ts), sum(al(t["d_out"].numel()) for t in ts)
        blobs = torch.empty(nb_all, dtype=torch.uint8, device=dev)
        outs = torch.empty(no_all, dtype=torch.uint8, device=dev)
        ob = oo = 0
        for t in ts:
            nb, no = t["d_blob"].numel(), t["d_out"].numel()
            blobs[ob:ob + nb].copy_(t["d_blob"])
            t["d_blob"] = blobs[ob:ob + nb]
            t["d_out"] = outs[oo:oo + no].view(t["d_out"].shape)
            ob, oo = ob + al(nb), oo + al(no)
        torch.cuda.empty_cache()
    if launch == "stack":      # every tensor of the stack in ONE ecf8_decode_batched launch
        groups = {0: [t for g in sorted(groups) for t in groups[g]]}
    batches = []
    for g in sorted(groups):
        ts = groups[g]
        batches.append((ecf8.Batch([t["hdr"] for t in ts], [t["d_blob"] for t in ts], [t["d_out"] for t in ts]), ts))
    return batches, desc, time.time() - t0


def cpu_baseline(batches, budget_syms=440_000_000):
    """The oracle's bit-serial tree-walk decoder on tensors of the workload: on one core (the first
    tensors, about 5 s of decoding), then on all of the machine's cores, one tensor per thread (tensors are
    independent; the C oracle runs outside the interpreter lock).  Only the decode is timed; preparing
    the oracle's inputs (its own encoder) takes about as long again."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    oracle.lib()

    def prepare(t):
        x = t["w"].cpu().numpy().reshape(-1)
        ln = oracle.huffman_lengths(oracle.histogram(x))
        stream, nbits = oracle.encode_exponents(x, ln, oracle.canonical_codes(ln), oracle.MSB_FIRST)
        return x, ln, stream, nbits, oracle.pack_nibbles_paper(x)

    def decode(p):
        x, ln, stream, nbits, packed = p
        t0 = time.perf_counter()
        out = oracle.decode_serial(stream, nbits, ln, packed, x.size, oracle.MSB_FIRST)
        dt = time.perf_counter() - t0
        if not np.array_equal(out, x):
            raise SystemExit("oracle round trip failed")
        return dt

    tensors = [t for _, ts in batches for t in ts]
    tot_syms, tot_t, names = 0, 0.0, []
    for t in tensors:
        if tot_syms >= budget_syms:
            break
        p = prepare(t)
        tot_t += decode(p)
        tot_syms += p[0].size
        names.append(t["spec"]["name"])
    single = {"value": round(tot_syms / tot_t / 1e9, 4), "unit": "GB/s decoded FP8", "cores": 1,
              "sample": "bit-serial decode of %d tensors (%s..%s), %d weights, %.1f s" % (
                  len(names), names[0], names[-1], tot_syms, tot_t)}
    # all cores: the box's share of the host is 16 cores per GPU, whatever the machine shows
    cores = max(1, min(16, os.cpu_count() or 1))
    big = sorted(tensors, key=lambda t: -t["w"].numel())[:cores]
    with ThreadPoolExecutor(max_workers=cores) as pool:
        prepared = list(pool.map(prepare, big))
        t0 = time.perf_counter()
        list(pool.map(decode, prepared))
        wall = time.perf_counter() - t0
    n_all = sum(p[0].size for p in prepared)
    try:
        model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
    except Exception:
        model = "unknown"
    return {"value": round(n_all / wall / 1e9, 4), "unit": "GB/s decoded FP8", "cores": cores, "kind": "oracle",
            "sample": "bit-serial decode of the %d largest tensors of the workload, one per thread, %d weights, %.1f s wall"
                      % (len(prepared), n_all, wall),
            "host": {"cpu_model": model, "cpu_count_seen": os.cpu_count()}, "single_core": single}


def profiled_traffic(workload, launch, hdrs, layers_full, kernel="ecf8_decode_kernel"):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this
    exact workload, or None when no summary covers it."""
    if not layers_full:
        return None
    key = "workload=%s launch=%s lane_syms=%d group_chunks=%d max_code_len=%d" % (
        workload, launch, hdrs[0].lane_syms, hdrs[0].group_chunks,
        max(h.max_code_len if hasattr(h, "max_code_len") else max(h.code_len) for h in hdrs))
    prefix = "%s_%s_%s" % (kernel, workload, launch)
    try:
        names = sorted(f for f in os.listdir(os.path.join(ROOT, "profiles")) if f.startswith(prefix) and f.endswith(".txt"))
    except OSError:
        return None
    for name in names:          # e.g. ..._config1_stack.txt (default cap) and ..._config1_stack_plain_huffman.txt
        text = open(os.path.join(ROOT, "profiles", name)).read()
        if key not in text:
            continue
        for line in text.splitlines():
            if line.startswith("traffic_bytes_per_launch="):
                return int(line.split("=")[1])
    return None


def per_layer_rates(tensors, alg_total, n_total, steps=10):
    """The same stack decoded with one batched launch per layer/block, on one stream and
    on two streams round-robin (the next layer's launch overlaps the previous one's tail)."""
    from paper_2510_02676_amd import ecf8
    key = "layer" if "layer" in tensors[0]["spec"] else "block" if "block" in tensors[0]["spec"] else "expert"
    groups = {}
    for t in tensors:
        groups.setdefault(t["spec"].get(key, -1), []).append(t)
    bs = [ecf8.Batch([t["hdr"] for t in ts], [t["d_blob"] for t in ts], [t["d_out"] for t in ts])
          for _, ts in sorted(groups.items())]
    res = {"launches_per_step": len(bs)}
    for ns in (1, 2):
        streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(ns - 1)]
        for it in range(2 + steps):
            if it == 2:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            for i, b in enumerate(bs):
                ecf8.ecf8_decode_batched(b, streams[i % ns])
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        res["streams_%d" % ns] = {"decoded_GBps": round(n_total / dt / 1e9, 2),
                                  "pct_of_hbm_peak": round(100 * alg_total / dt / 1e9 / HBM_PEAK_GBPS, 2),
                                  "us_per_launch": round(dt / len(bs) * 1e6, 2)}
    return res


def bench_config4(a):
    """configs[4]: W 14336 x 4096 decoded tile by tile into LDS and consumed by the FP8 matrix
    cores (ecf8_gemm_fp8), against the same GEMM on uncompressed W and against decode-then-GEMM."""
    from paper_2510_02676_amd import ecf8, synth

    def timeit(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e-3

    if a.copy_calibration:      # a kernel of known traffic for the profiler counters
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    spec = synth.config4()[0]
    w = synth.make(spec, a.seed, device="cuda:0")
    blob = ecf8.ecf8_encode(w.cpu(), spec["rows"], spec["cols"], lane_syms=64, tile_rows=16)
    h, d_blob, wout = blob.header, blob.to("cuda:0"), torch.empty_like(w)
    lin = ecf8.ecf8_encode(w.cpu(), spec["rows"], spec["cols"])     # default layout, for the decode-then-GEMM leg
    h_lin, d_lin = lin.header, lin.to("cuda:0")
    res = {}
    for M in (1, 16, 64):
        x = synth.activations(M, spec["cols"], seed=a.seed, device="cuda:0")
        y = torch.empty((M, spec["rows"]), dtype=torch.float32, device="cuda:0")
        y2 = torch.empty_like(y)
        ecf8.ecf8_gemm_fp8(h, d_blob, x, y)
        ecf8.ecf8_gemm_fp8_raw(w, x, y2)
        torch.cuda.synchronize()
        if not torch.equal(y, y2):
            raise SystemExit("fused GEMM differs from the GEMM on uncompressed weights at M=%d" % M)

        def two():
            ecf8.ecf8_decode(h_lin, d_lin, wout)
            ecf8.ecf8_gemm_fp8_raw(wout, x, y2)
        # the vendor library's FP8 GEMM on the same uncompressed operands, as context for the raw twin
        t_vendor = None
        try:
            mp = max(M, 16)
            xp = torch.zeros((mp, spec["cols"]), dtype=torch.uint8, device="cuda:0")
            xp[:M] = x
            one = torch.ones((), device="cuda:0", dtype=torch.float32)
            a8, b8 = xp.view(torch.float8_e4m3fn), w.view(torch.float8_e4m3fn).t()
            vend = lambda: torch._scaled_mm(a8, b8, scale_a=one, scale_b=one, out_dtype=torch.float32)
            if (vend()[:M] - y2).abs().max().item() <= 1e-4 * y2.abs().max().item():
                t_vendor = timeit(vend, a.steps, a.warmup)
        except Exception:
            t_vendor = None
        tf = timeit(lambda: ecf8.ecf8_gemm_fp8(h, d_blob, x, y), a.steps, a.warmup)
        tr = timeit(lambda: ecf8.ecf8_gemm_fp8_raw(w, x, y2), a.steps, a.warmup)
        # the same products on the F16 matrix cores (exact products, fp32 sums), and how far either kind of call
        # is from the fp64 product of the dequantised operands, as a fraction of sum |x w| per output
        # (the configuration asks for 1e-5; the reference here is torch's fp64 matmul on the device, the
        # oracle's own comparison is in tests/test_gpu_gemm.py)
        ye, ye2 = torch.empty_like(y), torch.empty_like(y)
        ecf8.ecf8_gemm_fp8_exact(h, d_blob, x, d_y=ye)
        ecf8.ecf8_gemm_fp8_raw_exact(w, x, d_y=ye2)
        ecf8.ecf8_gemm_fp8(h, d_blob, x, y)
        torch.cuda.synchronize()
        if not torch.equal(ye, ye2):
            raise SystemExit("exact fused GEMM differs from its twin on uncompressed weights at M=%d" % M)
        xd, wd_ = x.view(torch.float8_e4m3fn).double(), w.view(torch.float8_e4m3fn).double()
        yref, mag = xd @ wd_.t(), xd.abs() @ wd_.abs().t()
        err_fp8 = float(((y.double() - yref).abs() / mag).max())
        err_exact = float(((ye.double() - yref).abs() / mag).max())
        del xd, wd_, yref, mag
        te = timeit(lambda: ecf8.ecf8_gemm_fp8_exact(h, d_blob, x, d_y=ye), a.steps, a.warmup)
        ter = timeit(lambda: ecf8.ecf8_gemm_fp8_raw_exact(w, x, d_y=ye2), a.steps, a.warmup)
        t2 = timeit(two, a.steps, a.warmup)
        # with one scale per 128 x 128 block of W and per row of X
        ws = torch.rand((spec["rows"] // 128, spec["cols"] // 128), device="cuda:0") + 0.5
        xs = torch.rand((M,), device="cuda:0") + 0.5
        ecf8.ecf8_gemm_fp8_scaled(h, d_blob, x, ws, xs, y)
        ecf8.ecf8_gemm_fp8_raw_scaled(w, x, ws, xs, y2)
        torch.cuda.synchronize()
        if not torch.equal(y, y2):
            raise SystemExit("block-scaled fused GEMM differs from its twin on uncompressed weights at M=%d" % M)
        tfs = timeit(lambda: ecf8.ecf8_gemm_fp8_scaled(h, d_blob, x, ws, xs, y), a.steps, a.warmup)
        trs = timeit(lambda: ecf8.ecf8_gemm_fp8_raw_scaled(w, x, ws, xs, y2), a.steps, a.warmup)
        # ... and one scale per row of X and 128 columns (activations quantised in 1 x 128 groups)
        xg = torch.rand((M, spec["cols"] // 128), device="cuda:0") + 0.5
        ecf8.ecf8_gemm_fp8_scaled(h, d_blob, x, ws, xg, y)
        ecf8.ecf8_gemm_fp8_raw_scaled(w, x, ws, xg, y2)
        torch.cuda.synchronize()
        if not torch.equal(y, y2):
            raise SystemExit("group-scaled fused GEMM differs from its twin on uncompressed weights at M=%d" % M)
        tfg = timeit(lambda: ecf8.ecf8_gemm_fp8_scaled(h, d_blob, x, ws, xg, y), a.steps, a.warmup)
        res["M=%d" % M] = {"fused_us": round(tf * 1e6, 2), "raw_fp8_gemm_us": round(tr * 1e6, 2),
                           "fused_exact_us": round(te * 1e6, 2), "raw_exact_us": round(ter * 1e6, 2),
                           "max_err_over_sum_abs_fp8_core": float("%.3g" % err_fp8),
                           "max_err_over_sum_abs_exact": float("%.3g" % err_exact),
                           "meets_1e-5": {"fp8_core": err_fp8 <= 1e-5, "exact": err_exact <= 1e-5},
                           "fused_block_scaled_us": round(tfs * 1e6, 2), "raw_block_scaled_us": round(trs * 1e6, 2),
                           "fused_block_and_group_scaled_us": round(tfg * 1e6, 2),
                           "decode_then_gemm_us": round(t2 * 1e6, 2),
                           "vendor_fp8_gemm_us": None if t_vendor is None else round(t_vendor * 1e6, 2),
                           "fused_weight_GBps": round(w.numel() / tf / 1e9, 1)}
    # beyond the fused call's M: two calls of 64 rows against decoding W once and calling the vendor library's GEMM
    crossover = None
    if a.no_extra:
        return print_config4(a, spec, w, h, res, None, None, None, None)
    try:
        x128 = synth.activations(128, spec["cols"], seed=a.seed, device="cuda:0")
        y128 = torch.empty((128, spec["rows"]), dtype=torch.float32, device="cuda:0")
        one = torch.ones((), device="cuda:0", dtype=torch.float32)

        def fused_twice():
            ecf8.ecf8_gemm_fp8(h, d_blob, x128[:64], y128[:64])
            ecf8.ecf8_gemm_fp8(h, d_blob, x128[64:], y128[64:])

        def decode_then_vendor():
            ecf8.ecf8_decode(h_lin, d_lin, wout)
            return torch._scaled_mm(x128.view(torch.float8_e4m3fn), wout.view(torch.float8_e4m3fn).t(), scale_a=one,
                                    scale_b=one, out_dtype=torch.float32)
        fused_twice()
        ref = decode_then_vendor()
        torch.cuda.synchronize()
        if (ref - y128).abs().max().item() <= 1e-4 * y128.abs().max().item():
            crossover = {"M": 128, "fused_two_calls_us": round(timeit(fused_twice, a.steps, a.warmup) * 1e6, 2),
                         "decode_then_vendor_gemm_us": round(timeit(decode_then_vendor, a.steps, a.warmup) * 1e6, 2)}
            x64 = x128[:64].contiguous()
            v64 = lambda: (ecf8.ecf8_decode(h_lin, d_lin, wout), torch._scaled_mm(
                x64.view(torch.float8_e4m3fn), wout.view(torch.float8_e4m3fn).t(), scale_a=one, scale_b=one,
                out_dtype=torch.float32))
            crossover["decode_then_vendor_gemm_us_at_M64"] = round(timeit(v64, a.steps, a.warmup) * 1e6, 2)
    except Exception:
        crossover = None
    # the any-K kernels on the down projection of the same stack (4096 x 14336; X is fetched chunk by chunk)
    wd = synth.make_weight(4096, 14336, 1.7, 0.02, a.seed, tensor_id=400001, device="cuda:0")
    bd = ecf8.ecf8_encode(wd.cpu(), 4096, 14336, lane_syms=64, tile_rows=16)
    hd, d_bd = bd.header, bd.to("cuda:0")
    res_down = {}
    for M in (1, 16, 64):
        x = synth.activations(M, 14336, seed=a.seed, device="cuda:0")
        y = torch.empty((M, 4096), dtype=torch.float32, device="cuda:0")
        y2 = torch.empty_like(y)
        ecf8.ecf8_gemm_fp8(hd, d_bd, x, y)
        ecf8.ecf8_gemm_fp8_raw(wd, x, y2)
        torch.cuda.synchronize()
        if not torch.equal(y, y2):
            raise SystemExit("any-K fused GEMM differs from the GEMM on uncompressed weights at M=%d" % M)
        tf = timeit(lambda: ecf8.ecf8_gemm_fp8(hd, d_bd, x, y), a.steps, a.warmup)
        tr = timeit(lambda: ecf8.ecf8_gemm_fp8_raw(wd, x, y2), a.steps, a.warmup)
        res_down["M=%d" % M] = {"fused_us": round(tf * 1e6, 2), "raw_fp8_gemm_us": round(tr * 1e6, 2)}
    # split K on matrices of few rows (low-rank projections of 576 and 1536 rows, a 256-row slice of a down projection,
    # a grouped-query K/V projection): the plain calls against the split ones, fused and on uncompressed weights
    res_split = {}
    for rows, cols in ((256, 14336), (576, 7168), (1536, 7168), (1024, 4096)):
        ww = synth.make_weight(rows, cols, 1.7, 0.02, a.seed, tensor_id=400002, device="cuda:0")
        bb = ecf8.ecf8_encode(ww.cpu(), rows, cols, lane_syms=64, tile_rows=16, table_mode=1)
        hh, d_bb = bb.header, bb.to("cuda:0")
        entry = {"slices": ecf8.gemm_splitk_slices(rows, cols)}
        for M in (1, 16, 64):
            wsp = ecf8.gemm_splitk_workspace(rows, cols, M, "cuda:0")
            x = synth.activations(M, cols, seed=a.seed, device="cuda:0")
            y = torch.empty((M, rows), dtype=torch.float32, device="cuda:0")
            y2 = torch.empty_like(y)
            ecf8.ecf8_gemm_fp8_splitk(hh, d_bb, x, wsp, d_y=y)
            ecf8.ecf8_gemm_fp8_raw_splitk(ww, x, wsp, d_y=y2)
            torch.cuda.synchronize()
            if not torch.equal(y, y2):
                raise SystemExit("split-K fused GEMM differs from its twin on uncompressed weights at M=%d" % M)
            entry["M=%d" % M] = {
                "fused_us": round(timeit(lambda: ecf8.ecf8_gemm_fp8(hh, d_bb, x, y), a.steps, a.warmup) * 1e6, 2),
                "fused_split_us": round(timeit(lambda: ecf8.ecf8_gemm_fp8_splitk(hh, d_bb, x, wsp, d_y=y), a.steps, a.warmup) * 1e6, 2),
                "raw_us": round(timeit(lambda: ecf8.ecf8_gemm_fp8_raw(ww, x, y2), a.steps, a.warmup) * 1e6, 2),
                "raw_split_us": round(timeit(lambda: ecf8.ecf8_gemm_fp8_raw_splitk(ww, x, wsp, d_y=y2), a.steps, a.warmup) * 1e6, 2)}
        res_split["%dx%d" % (rows, cols)] = entry
    # a group of experts in one launch (config 2's shapes: 8 experts a token batch is routed to, gate / up 2048 x 7168
    # and down 7168 x 2048 each) against one call per matrix
    res_group = {}
    experts = []
    for e in range(8):
        for j, (rows, cols) in enumerate(((2048, 7168), (2048, 7168), (7168, 2048))):
            ww = synth.make_weight(rows, cols, 1.7, 0.02, a.seed, tensor_id=410000 + 3 * e + j, device="cuda:0")
            bb = ecf8.ecf8_encode(ww.cpu(), rows, cols, lane_syms=64, tile_rows=16)
            experts.append((ww, bb.header, bb.to("cuda:0")))
    for M in (1, 4, 16, 64):
        fused_m = [{"hdr": h_, "blob": b_, "x": synth.activations(M, h_.cols, seed=a.seed + i, device="cuda:0")}
                   for i, (w_, h_, b_) in enumerate(experts)]
        raw_m = [{"w": w_, "x": f_["x"]} for (w_, h_, b_), f_ in zip(experts, fused_m)]
        gf, gr = ecf8.GemmGroup(fused_m), ecf8.GemmGroup(raw_m)
        yf, yr = ecf8.ecf8_gemm_fp8_grouped(gf), ecf8.ecf8_gemm_fp8_grouped(gr)
        torch.cuda.synchronize()
        if not all(torch.equal(p_, q_) for p_, q_ in zip(yf, yr)):
            raise SystemExit("grouped fused GEMM differs from its twin on uncompressed weights at M=%d" % M)

        def singles_fused():
            for f_, y_ in zip(fused_m, yf):
                ecf8.ecf8_gemm_fp8(f_["hdr"], f_["blob"], f_["x"], y_)

        def singles_raw():
            for r_, y_ in zip(raw_m, yr):
                ecf8.ecf8_gemm_fp8_raw(r_["w"], r_["x"], y_)
        res_group["M=%d" % M] = {
            "grouped_fused_us": round(timeit(lambda: ecf8.ecf8_gemm_fp8_grouped(gf), a.steps, a.warmup) * 1e6, 2),
            "grouped_raw_us": round(timeit(lambda: ecf8.ecf8_gemm_fp8_grouped(gr), a.steps, a.warmup) * 1e6, 2),
            "24_fused_calls_us": round(timeit(singles_fused, a.steps, a.warmup) * 1e6, 2),
            "24_raw_calls_us": round(timeit(singles_raw, a.steps, a.warmup) * 1e6, 2)}
    res_group["weights"] = sum(w_.numel() for w_, _, _ in experts)
    del experts
    print_config4(a, spec, w, h, res, crossover, res_down, res_split, res_group)


def print_config4(a, spec, w, h, res, crossover, res_down, res_split, res_group):
    t16 = res["M=16"]["fused_us"] * 1e-6
    alg = int(h.total_size + 16 * (spec["cols"] + 4 * spec["rows"]))      # the blob and X read, Y written (M = 16)
    print(json.dumps({
        "metric": "decoded FP8 GB/s consumed by the fused decode+GEMM (M=16)", "value": round(w.numel() / t16 / 1e9, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(t16 * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8 x fp8 -> f32", "data": "synthetic",
        "config": {"workload": "config4: fused decode + FP8 MFMA GEMM, W 14336x4096, M in {1,16,64}", "seed": a.seed},
        "compression_ratio": round(h.total_size / w.numel(), 5), "bit_exact_vs_raw_weights_gemm": True,
        # the fused kernel reads the blob and X and writes Y: far from the memory roof, it is bound by the decode arithmetic
        "roofline": {"bound": "hbm", "kernel": "ecf8_gemm_kernel<1, 16, 64, 0>", "achieved": round(alg / t16 / 1e9, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(alg / t16 / 1e9 / HBM_PEAK_GBPS, 4),
                     "avg_launch_us": round(t16 * 1e6, 2), "algorithmic_bytes_per_launch": alg,
                     "traffic": profiled_gemm_traffic(h)},
        "gemm": res, "beyond_M64": crossover, "gemm_down_4096x14336_any_k": res_down, "split_k": res_split,
        "grouped_8_experts": res_group}))


def profiled_gemm_traffic(h):
    """HBM bytes of one fused M = 16 launch on config 4's W from the committed counter summary, or None."""
    try:
        text = open(os.path.join(ROOT, "profiles", "ecf8_gemm_kernel_config4_hbm_traffic.txt")).read()
    except OSError:
        return None
    if "blob_bytes=%d" % h.total_size not in text:
        return None
    for line in text.splitlines():
        if line.startswith("traffic_bytes_per_launch="):
            return int(line.split("=")[1])
    return None


def bench_jit(a):
    """Workload "jit" (paper Section 3.3): a forward pass over the config-1 stack with the weights
    decoded just in time into shared buffers (ecf8_jit_*).  The per-layer compute is a stand-in that
    reads every decoded byte once: the library's raw FP8 GEMM at M = 16 on each matrix (the
    4096 x 14336 down projection is read as 14336 x 4096).  Three timings per pass: compute on
    resident uncompressed weights; decode then compute on one stream and one buffer; decode of
    layer l+1 overlapped with the compute of layer l on two buffers."""
    from paper_2510_02676_amd import ecf8, synth
    dev = "cuda:0"
    layers = a.layers or 32
    specs = synth.config1(a.seed, layers)
    per_layer = {}
    t0 = time.time()
    for s in specs:
        w = synth.make(s, a.seed, device=dev)
        b = ecf8.ecf8_encode(w.cpu(), s["rows"], s["cols"])
        per_layer.setdefault(s["layer"], []).append((w, b.header, b.to(dev)))
    setup = time.time() - t0
    packed = [([t[1] for t in per_layer[l]], [t[2] for t in per_layer[l]]) for l in range(layers)]
    x = synth.activations(16, 4096, seed=a.seed, device=dev)
    y = torch.empty((16, 14336), dtype=torch.float32, device=dev)

    def gemm_stand_in(ws, stream):
        for w in ws:
            w2 = w if w.shape[1] == 4096 else w.view(-1, 4096)
            ecf8.ecf8_gemm_fp8_raw(w2, x, y[:, :w2.shape[0]], stream=stream)

    consumer = [gemm_stand_in]
    compute = lambda ws, stream: consumer[0](ws, stream)

    def timed(fn):
        for _ in range(a.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(a.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / a.steps

    main_stream = torch.cuda.current_stream()

    def resident_pass():
        for l in range(layers):
            compute([t[0] for t in per_layer[l]], main_stream)

    def make_pass(jit, overlap):
        def one_pass():
            jit.prefetch(0)
            for l in range(layers):
                if overlap and l + 1 < layers:
                    jit.prefetch(l + 1)
                ws = jit.acquire(l, main_stream)
                compute(ws, main_stream)
                jit.release(l, main_stream)
                if not overlap and l + 1 < layers:
                    jit.prefetch(l + 1)
        return one_pass

    # parity of what the consumer sees, once, before timing
    jit2 = ecf8.Jit(packed, n_buffers=2)
    jit2.prefetch(0)
    for l in range(layers):
        if l + 1 < layers:
            jit2.prefetch(l + 1)
        ws = jit2.acquire(l, main_stream)
        if not all(torch.equal(v, t[0]) for v, t in zip(ws, per_layer[l])):
            raise SystemExit("jit: layer %d differs from its weights" % l)
        jit2.release(l, main_stream)
    torch.cuda.synchronize()
    t_res = timed(resident_pass)
    jit1 = ecf8.Jit(packed, n_buffers=1)
    t_serial = timed(make_pass(jit1, False))
    t_jit = timed(make_pass(jit2, True))
    n_total = sum(t[0].numel() for l in range(layers) for t in per_layer[l])
    hidden = (t_serial - t_jit) / max(t_serial - t_res, 1e-9)

    # no buffer at all: the same GEMMs with the weights decoded inside them (ecf8_gemm_fp8 on row-tiled blobs)
    tiled = {}
    for l in range(layers):
        for w, _, _ in per_layer[l]:
            w2 = w if w.shape[1] == 4096 else w.view(-1, 4096)
            hdr_t, d_t = ecf8.ecf8_encode_gpu(w2, lane_syms=64, tile_rows=16)
            tiled.setdefault(l, []).append((hdr_t, d_t.clone(), w2))
    for hdr_t, d_t, w2 in tiled[0]:
        ya = ecf8.ecf8_gemm_fp8(hdr_t, d_t, x)
        yb = ecf8.ecf8_gemm_fp8_raw(w2, x)
        torch.cuda.synchronize()
        if not torch.equal(ya, yb):
            raise SystemExit("jit: fused GEMM differs from the GEMM on resident weights")

    def fused_pass():
        for l in range(layers):
            for hdr_t, d_t, w2 in tiled[l]:
                ecf8.ecf8_gemm_fp8(hdr_t, d_t, x, y[:, :w2.shape[0]], stream=main_stream)
    t_fused = timed(fused_pass)
    tiled_bytes = sum(h.total_size for l in tiled for h, _, _ in tiled[l])
    # one compressed copy for both regimes: the same row-tiled blobs decoded just in time into the two buffers
    jit_t = ecf8.Jit([([t[0] for t in tiled[l]], [t[1] for t in tiled[l]]) for l in range(layers)], n_buffers=2)
    jit_t.prefetch(0)
    ws = jit_t.acquire(0, main_stream)
    if not all(torch.equal(v.reshape(-1), t[2].reshape(-1)) for v, t in zip(ws, tiled[0])):
        raise SystemExit("jit: layer 0 decoded from row-tiled blobs differs from its weights")
    jit_t.release(0, main_stream)
    torch.cuda.synchronize()
    t_jit_tiled = timed(make_pass(jit_t, True))
    del jit_t
    del tiled
    # the way serving stacks hold these layers: Q, K, V as one matrix and gate, up as one (they share their input),
    # which fills the chip better with blocks of rows; resident and fused alike
    merged = {}
    y3 = torch.empty((16, 2 * 14336), dtype=torch.float32, device=dev)
    for l in range(layers):
        ws = [t[0] if t[0].shape[1] == 4096 else t[0].view(-1, 4096) for t in per_layer[l]]
        for grp in (torch.cat(ws[0:3]), ws[3], torch.cat(ws[4:6]), ws[6]):
            hdr_t, d_t = ecf8.ecf8_encode_gpu(grp, lane_syms=64, tile_rows=16)
            merged.setdefault(l, []).append((hdr_t, d_t.clone(), grp))

    def merged_resident_pass():
        for l in range(layers):
            for _, _, w2 in merged[l]:
                ecf8.ecf8_gemm_fp8_raw(w2, x, y3[:, :w2.shape[0]], stream=main_stream)

    def merged_fused_pass():
        for l in range(layers):
            for hdr_t, d_t, w2 in merged[l]:
                ecf8.ecf8_gemm_fp8(hdr_t, d_t, x, y3[:, :w2.shape[0]], stream=main_stream)
    t_res_m, t_fused_m = timed(merged_resident_pass), timed(merged_fused_pass)
    del merged

    # the same three timings with a compute-bound consumer (one bf16 4096^3 matmul per layer that does
    # not read the weights), and the decode confined to fewer workgroups so that the consumer's
    # kernels find free compute units while it runs
    ma = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
    mb = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
    mc = torch.empty_like(ma)
    consumer[0] = lambda ws, stream: torch.matmul(ma, mb, out=mc)
    mm = {"resident": round(timed(resident_pass), 4), "decode_then_compute_1_buffer": round(timed(make_pass(jit1, False)), 4)}
    for cap in (0, 192, 128, 64):
        jit2.set_decode_workgroups(cap)
        mm["jit_2_buffers_decode_workgroups_%s" % (cap or "all")] = round(timed(make_pass(jit2, True)), 4)
    jit2.set_decode_workgroups(0)
    consumer[0] = gemm_stand_in
    print(json.dumps({
        "metric": "decoded FP8 GB/s inside a just-in-time forward pass (decode of layer l+1 overlapped with compute of layer l)",
        "value": round(n_total / (t_jit * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(t_jit, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "jit: config-1 stack, %d layers, per-layer decode into 2 shared buffers + raw FP8 GEMM stand-in (M=16)" % layers,
                   "weights": n_total, "seed": a.seed},
        "bit_exact": True, "setup_s": round(setup, 1),
        "pass_ms": {"compute_on_resident_weights": round(t_res, 4), "decode_then_compute_1_buffer": round(t_serial, 4),
                    "jit_2_buffers_overlapped": round(t_jit, 4),
                    "fused_decode_gemm_no_buffer": round(t_fused, 4),
                    "jit_2_buffers_from_the_fused_calls_row_tiled_blobs": round(t_jit_tiled, 4),
                    "qkv_and_gate_up_merged": {"compute_on_resident_weights": round(t_res_m, 4),
                                               "fused_decode_gemm_no_buffer": round(t_fused_m, 4)}},
        "resident_compressed_bytes_row_tiled": tiled_bytes,
        "decode_time_hidden_frac": round(hidden, 3),
        "pass_ms_with_compute_bound_consumer": mm,
        "buffer_bytes_each": jit2.buffer_bytes, "resident_compressed_bytes": sum(h.total_size for hs, _ in packed for h in hs)}))


def bench_encode(a):
    """Workload "encode": the GPU-side encoder (ecf8_encode_gpu) on the matrices of one config-1 layer,
    each checked byte for byte against the CPU encoder's container, beside the CPU encoder's rate."""
    from paper_2510_02676_amd import ecf8, synth
    dev = "cuda:0"
    specs = synth.config1(a.seed, 1)
    rows = {}
    n_total, t_gpu_total, t_cpu_total = 0, 0.0, 0.0
    for s in specs:
        w = synth.make(s, a.seed, device=dev)
        t0 = time.time()
        ref = ecf8.ecf8_encode(w.cpu().numpy(), s["rows"], s["cols"])
        t_cpu = time.time() - t0
        hdr, d_blob = ecf8.ecf8_encode_gpu(w)
        torch.cuda.synchronize()
        if bytes(hdr) != bytes(ref.header) or not torch.equal(d_blob.cpu(), torch.from_numpy(ref.numpy())):
            raise SystemExit("GPU-encoded container of %s differs from the CPU encoder's" % s["name"])
        buf = torch.empty(d_blob.numel() + 4096, dtype=torch.uint8, device=dev)
        for _ in range(a.warmup):
            ecf8.ecf8_encode_gpu(w, d_blob=buf)
        torch.cuda.synchronize()
        t0 = time.time()
        for _ in range(a.steps):
            ecf8.ecf8_encode_gpu(w, d_blob=buf)
        torch.cuda.synchronize()
        t_gpu = (time.time() - t0) / a.steps
        rows[s["name"]] = {"weights": w.numel(), "gpu_encode_us": round(t_gpu * 1e6, 1),
                           "gpu_GBps": round(w.numel() / t_gpu / 1e9, 1), "cpu_encode_ms": round(t_cpu * 1e3, 1)}
        n_total += w.numel()
        t_gpu_total += t_gpu
        t_cpu_total += t_cpu
    print(json.dumps({
        "metric": "raw FP8 GB/s consumed by the GPU-side encoder (ecf8_encode_gpu)", "value": round(n_total / t_gpu_total / 1e9, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(t_gpu_total * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "encode: one config-1 layer (7 matrices), host wall clock incl. the one histogram read-back per tensor",
                   "weights": n_total, "seed": a.seed},
        "identical_to_cpu_encoder": True, "cpu_encoder_GBps": round(n_total / t_cpu_total / 1e9, 3), "tensors": rows}))


def bench_encode_wide(a):
    """Workloads "encode_bf16" / "encode_e5m2": the GPU-side encoder of the wide-alphabet codec on one
    14336 x 4096 matrix, checked byte for byte against the CPU encoder's container, beside the CPU encoder."""
    from paper_2510_02676_amd import ecfw, synth
    dev = "cuda:0"
    fmt = ecfw.FMT_BF16 if a.workload == "encode_bf16" else ecfw.FMT_E5M2
    make = synth.make_bf16 if fmt == ecfw.FMT_BF16 else synth.make_e5m2
    w = make(14336, 4096, 1.8, 0.02, a.seed, tensor_id=600000, device=dev)
    t0 = time.time()
    ref = ecfw.ecfw_encode(fmt, w.cpu(), 14336, 4096)
    t_cpu = time.time() - t0
    hdr, d_blob = ecfw.ecfw_encode_gpu(fmt, w)
    torch.cuda.synchronize()
    if bytes(hdr) != bytes(ref.header) or not torch.equal(d_blob.cpu(), torch.from_numpy(ref.numpy())):
        raise SystemExit("GPU-encoded container differs from the CPU encoder's")
    buf = torch.empty(d_blob.numel() + 4096, dtype=torch.uint8, device=dev)
    for _ in range(a.warmup):
        ecfw.ecfw_encode_gpu(fmt, w, d_blob=buf)
    torch.cuda.synchronize()
    t0 = time.time()
    for _ in range(a.steps):
        ecfw.ecfw_encode_gpu(fmt, w, d_blob=buf)
    torch.cuda.synchronize()
    t_gpu = (time.time() - t0) / a.steps
    raw = w.numel() * w.element_size()
    name = "BF16" if fmt == ecfw.FMT_BF16 else "E5M2"
    print(json.dumps({
        "metric": "raw %s GB/s consumed by the GPU-side encoder (ecfw_encode_gpu)" % name, "value": round(raw / t_gpu / 1e9, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(t_gpu * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16" if fmt == ecfw.FMT_BF16 else "u8",
        "data": "synthetic",
        "config": {"workload": "%s: one 14336x4096 matrix as %s, host wall clock incl. the histogram read-back" % (a.workload, name),
                   "elements": w.numel(), "seed": a.seed},
        "identical_to_cpu_encoder": True, "cpu_encoder_GBps": round(raw / t_cpu / 1e9, 3),
        "compression_ratio": round(hdr.total_size / raw, 5)}))


def bench_wide(a):
    """Workloads "wide_bf16" / "wide_e5m2": the wide-alphabet decoder on eight MLP-sized matrices
    (14336 x 4096) of the 8B-class stack in BF16 or E5M2: one ecfw_decode_batched launch per step, or with
    --launch layer one ecfw_decode launch per matrix."""
    from paper_2510_02676_amd import ecfw, synth
    import oracle
    dev = "cuda:0"
    fmt = ecfw.FMT_BF16 if a.workload == "wide_bf16" else ecfw.FMT_E5M2
    make = synth.make_bf16 if fmt == ecfw.FMT_BF16 else synth.make_e5m2
    eb = ecfw.ELEM_BYTES[fmt]
    n_mats = a.layers or 8
    t0 = time.time()
    mats = []
    for i in range(n_mats):
        alpha, scale = synth._drawn(a.seed, 600000 + i)
        w = make(14336, 4096, alpha, scale, a.seed, tensor_id=600000 + i, device=dev)
        blob = ecfw.ecfw_encode(fmt, w.cpu(), 14336, 4096, lane_syms=a.lane_syms, group_chunks=a.group_chunks,
                                max_code_len=a.max_code_len)
        h = blob.header
        d_out = torch.empty(h.n_elem * eb, dtype=torch.uint8, device=dev)
        mats.append(dict(w=w.view(torch.uint8).reshape(-1), hdr=h, d_blob=blob.to(dev), d_out=d_out, blob=blob if i == 0 else None))
    t_setup = time.time() - t0
    hdrs = [m["hdr"] for m in mats]
    n_total = sum(h.n_elem for h in hdrs)
    out_total = n_total * eb
    rd_total = sum((h.stream_bits + 7) // 8 + h.plane_bytes + h.sign_bytes + 8 * (h.n_chunks + 1) + 128 * h.n_chunks +
                   256 + 9 * h.n_alphabet for h in hdrs)
    alg_total = rd_total + out_total
    stream = torch.cuda.current_stream()

    batch = ecfw.WBatch(hdrs, [m["d_blob"] for m in mats], [m["d_out"] for m in mats])
    per_tensor = a.launch == "layer"          # --launch layer: one ecfw_decode launch per matrix instead

    def step():
        if per_tensor:
            for m in mats:
                ecfw.ecfw_decode(m["d_blob"], m["hdr"], m["d_out"], stream=stream)
        else:
            ecfw.ecfw_decode_batched(batch, stream)

    n_launch = n_mats if per_tensor else 1
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    if any(not torch.equal(m["d_out"], m["w"]) for m in mats):
        raise SystemExit("wide decode mismatch")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(a.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    sec_per_step = wall / a.steps
    launch_s = e0.elapsed_time(e1) * 1e-3 / (a.steps * n_launch)
    achieved = alg_total / n_launch / launch_s / 1e9
    name = "BF16" if fmt == ecfw.FMT_BF16 else "E5M2"
    out = {
        "metric": "decoded %s GB/s (exponent-coded container -> exact %s elements)" % (name, name),
        "value": round(out_total / sec_per_step / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16" if eb == 2 else "u8", "data": "synthetic",
        "config": {"workload": "%s: %d matrices 14336x4096 of the 8B-class stack as %s, %s"
                               % (a.workload, n_mats, name, "one ecfw_decode launch each" if per_tensor else
                                  "one ecfw_decode_batched launch"),
                   "launch": "tensor" if per_tensor else "batch",
                   "elements": n_total, "lane_syms": hdrs[0].lane_syms, "group_chunks": hdrs[0].group_chunks,
                   "max_code_len": max(h.max_code_len for h in hdrs), "seed": a.seed},
        "compression_ratio": round(sum(h.total_size for h in hdrs) / out_total, 5),
        "avg_code_bits": round(sum(h.stream_bits for h in hdrs) / n_total, 4),
        "total_moved_GBps": round(alg_total / sec_per_step / 1e9, 2), "bit_exact": True, "setup_s": round(t_setup, 1),
        "roofline": {"bound": "hbm", "kernel": "ecfw_decode_kernel", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "avg_launch_us": round(launch_s * 1e6, 2),
                     "algorithmic_bytes_per_launch": int(alg_total / n_launch),
                     "traffic": profiled_traffic(a.workload, "tensor" if per_tensor else "batch", hdrs, a.layers == 0,
                                                 "ecfw_decode_kernel")},
    }
    if fmt == ecfw.FMT_E5M2 and not per_tensor:
        # The same E5M2 bytes in the FP8 container: that codec never interprets its bytes, it codes bits 6..3 (here
        # the upper four of the five exponent bits) and keeps bits 7, 2, 1, 0 raw (sign, the lowest exponent bit,
        # the mantissa).  One exponent bit goes uncoded, and the pair-table kernels decode two symbols per lookup.
        from paper_2510_02676_amd import ecf8
        alt = []
        for m in mats:
            w8 = m["w"].view(14336, 4096)
            h8, big = ecf8.ecf8_encode_gpu(w8)
            alt.append((h8, big.clone(), torch.empty_like(w8), w8))
            del big
        b8 = ecf8.Batch([t[0] for t in alt], [t[1] for t in alt], [t[2] for t in alt])
        for _ in range(a.warmup):
            ecf8.ecf8_decode_batched(b8, stream)
        torch.cuda.synchronize()
        if any(not torch.equal(t[2], t[3]) for t in alt):
            raise SystemExit("E5M2 bytes through the FP8 container: decode mismatch")
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record(stream)
        for _ in range(a.steps):
            ecf8.ecf8_decode_batched(b8, stream)
        f1.record(stream)
        torch.cuda.synchronize()
        t8 = f0.elapsed_time(f1) * 1e-3 / a.steps
        alg8 = sum(algorithmic_bytes(t[0])[0] + t[0].n_elem for t in alt)
        out["same_bytes_in_the_fp8_container"] = {
            "decoded_GBps": round(out_total / t8 / 1e9, 2), "total_moved_GBps": round(alg8 / t8 / 1e9, 2),
            "pct_of_hbm_peak": round(100 * alg8 / t8 / 1e9 / HBM_PEAK_GBPS, 2), "launch_us": round(t8 * 1e6, 2),
            "compression_ratio": round(sum(t[0].total_size for t in alt) / out_total, 5), "bit_exact": True}
        del alt, b8
    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not a.no_cpu_baseline:
        # the oracle's bit-serial reader on the first 2^25 elements of the first matrix, re-encoded on their own
        # with the same code lengths
        x = mats[0]["w"][: (1 << 25) * eb].cpu().numpy()
        x = x.view(np.uint16) if eb == 2 else x
        part = oracle.w_container_encode(fmt, x, 1, x.size, hdrs[0].lane_syms, hdrs[0].group_chunks, mats[0]["blob"].code_len())
        t0 = time.perf_counter()
        dec, _ = oracle.w_container_decode(part)
        dt = time.perf_counter() - t0
        assert np.array_equal(dec, x)
        out["cpu_baseline"] = {"value": round(x.size * eb / dt / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "oracle container reader on the first 2^25 elements of matrix 0 (%.1f s)" % dt}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="all",
                    help="all (default): config3 headline with config1, config2 and plain Huffman beside it; or one of "
                         "config0..config4, jit, encode, wide_bf16, wide_e5m2, encode_bf16, encode_e5m2")
    ap.add_argument("--all-order", default="config3,config2,plain_huffman,config1", help="order of the parts of the default run")
    ap.add_argument("--arena", type=int, default=1,
                    help="1 (default): all blobs of a stack in one device allocation and all outputs in another, the way a serving "
                         "process holds a model; 0: one allocation per tensor (1-2 points of HBM peak slower)")
    ap.add_argument("--cpu-encode", action="store_true", help="set the stacks up with the CPU encoder instead of the device encoder")
    ap.add_argument("--layers", type=int, default=0, help="0 = the full stack of the workload")
    ap.add_argument("--lane-syms", type=int, default=0, help="0 = library default")
    ap.add_argument("--group-chunks", type=int, default=0, help="chunks interleaved per group, 0 = library default")
    ap.add_argument("--max-code-len", type=int, default=0, help="cap on the code length, 0 = library default (7), 15 = plain Huffman")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--launch", default="stack", choices=["layer", "stack"],
                    help="stack: the whole stack in one launch per step; "
                         "layer: one batched launch per layer/block (as a per-layer decode hook would)")
    ap.add_argument("--streams", type=int, default=1, help="streams for --launch layer (round-robin)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-layer-launch rates")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy (a kernel of known traffic for profiler counters); the stack "
                         "workloads always run and report it")
    a = ap.parse_args()
    if a.gpus != 1:
        raise SystemExit("this build runs on ONE GPU: tensors are independent and shard with no exchange "
                         "or collective; --gpus %d is not supported" % a.gpus)
    if not torch.cuda.is_available():
        raise SystemExit("no GPU visible: the decode path has no CPU fallback")
    from paper_2510_02676_amd import ecf8

    if a.workload == "config4":
        return bench_config4(a)
    if a.workload == "jit":
        return bench_jit(a)
    if a.workload == "encode":
        return bench_encode(a)
    if a.workload in ("wide_bf16", "wide_e5m2"):
        return bench_wide(a)
    if a.workload in ("encode_bf16", "encode_e5m2"):
        return bench_encode_wide(a)
    if a.workload != "all":
        out, batches = run_stack(a, a.workload, a.max_code_len, per_layer=not a.no_extra, copy_kernel=True)
        if not a.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(batches)
        print(json.dumps(out))
        return
    # default: headline on the largest configuration, the others beside it in the same line
    keep = ("value", "unit", "ms_per_step", "ms_per_step_median", "ms_per_step_min", "config", "compression_ratio",
            "memory_saving_pct", "avg_code_bits", "compressed_read_GBps", "total_moved_GBps", "pct_of_hbm_peak", "bit_exact",
            "setup_s", "roofline", "per_layer_launch")
    results, baseline = {}, None
    for part in a.all_order.split(","):
        if part == "config3":
            results[part], batches = run_stack(a, "config3", 0, per_layer=False, copy_kernel=True)
        elif part == "config2":
            results[part], batches = run_stack(a, "config2", 0, per_layer=False, copy_kernel=False)
        elif part == "plain_huffman":
            # the paper's own code (Section 3.1: the optimal Huffman code; its cap of 16 bits never binds on 16 symbols)
            results[part], batches = run_stack(a, "config1", 15, per_layer=False, copy_kernel=False)
        elif part == "config1":
            # the same stack under this library's default cap of 7 bits per codeword (a declared extension)
            results[part], batches = run_stack(a, "config1", 0, per_layer=not a.no_extra, copy_kernel=False)
            if not a.no_cpu_baseline:
                baseline = cpu_baseline(batches)
        else:
            raise SystemExit("unknown part " + part)
        del batches
        torch.cuda.empty_cache()
    out = results["config3"] if "config3" in results else dict(next(iter(results.values())))
    out["configs"] = {k: {f: results[k][f] for f in keep if f in results[k]} for k in ("config1", "config2") if k in results}
    if "plain_huffman" in results:
        out["plain_huffman"] = {f: results["plain_huffman"][f] for f in keep if f in results["plain_huffman"]}
    if baseline:
        out["cpu_baseline"] = baseline
    print(json.dumps(out))


def run_stack(a, workload, max_code_len, per_layer, copy_kernel):
    """Builds one stack workload, checks every decoded tensor against its input on the device, times a.steps
    steps after a.warmup warm-up steps.  Returns (the result object, the batches with their tensors)."""
    from paper_2510_02676_amd import ecf8
    layers = a.layers or {"config1": 32, "config2": 256, "config3": 40, "config0": 1}[workload]
    batches, desc, t_setup = build_workload(workload, a.seed, a.lane_syms, layers, a.launch, a.group_chunks, max_code_len,
                                            a.cpu_encode, a.arena)
    hdrs = [t["hdr"] for _, ts in batches for t in ts]
    n_total = sum(h.n_elem for h in hdrs)
    blob_total = sum(h.total_size for h in hdrs)
    rd_total = sum(algorithmic_bytes(h)[0] for h in hdrs)
    alg_total = rd_total + n_total

    stream = torch.cuda.current_stream()
    side = [stream] + [torch.cuda.Stream() for _ in range(max(0, a.streams - 1))]

    def step():
        for i, (b, _) in enumerate(batches):
            ecf8.ecf8_decode_batched(b, side[i % len(side)] if a.launch == "layer" else stream)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # parity of what the timed launches produce: exact bytes of every tensor
    bad = [t["spec"]["name"] for _, ts in batches for t in ts if not torch.equal(t["d_out"], t["w"])]
    if bad:
        raise SystemExit("decode mismatch on " + ", ".join(bad[:5]))

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    marks = []
    for _ in range(a.steps):
        step()
        if len(side) == 1 or a.launch == "stack":       # one event per step: median and fastest step beside the mean
            marks.append(torch.cuda.Event(enable_timing=True))
            marks[-1].record(stream)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_step = sorted(p.elapsed_time(q) for p, q in zip([e0] + marks[:-1], marks))
    dev_s = e0.elapsed_time(e1) * 1e-3 if len(side) == 1 or a.launch == "stack" else wall
    sec_per_step = wall / a.steps
    n_launch = len(batches) * a.steps
    launch_s = dev_s / n_launch                       # average duration of one decode launch (HIP events)
    alg_per_launch = alg_total / len(batches)
    achieved = alg_per_launch / launch_s / 1e9
    cap = max(max(h.code_len) for h in hdrs)

    out = {
        "metric": "decoded FP8 GB/s (ECF8 -> exact FP8 E4M3 bytes)",
        "value": round(n_total / sec_per_step / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4) if per_step else None,
        "ms_per_step_min": round(per_step[0], 4) if per_step else None,
        "config": {"workload": "%s: %s" % (workload, desc), "weights": n_total, "tensors": len(hdrs),
                   "launches_per_step": len(batches), "launch": a.launch, "lane_syms": hdrs[0].lane_syms,
                   "group_chunks": hdrs[0].group_chunks, "max_code_len": cap,
                   "code": "plain Huffman (the paper's code)" if max_code_len >= 15 else
                           "cheapest code with codewords of at most %d bits (this library's default)" % (max_code_len or 7),
                   "seed": a.seed},
        "compression_ratio": round(blob_total / n_total, 5),
        "memory_saving_pct": round(100 * (1 - blob_total / n_total), 2),
        "avg_code_bits": round(sum(h.stream_bits for h in hdrs) / n_total, 4),
        "compressed_read_GBps": round(rd_total / sec_per_step / 1e9, 2),
        "total_moved_GBps": round(alg_total / sec_per_step / 1e9, 2),
        "pct_of_hbm_peak": round(100 * alg_total / sec_per_step / 1e9 / HBM_PEAK_GBPS, 2),
        "bit_exact": True,
        "setup_s": round(t_setup, 1),
        "roofline": {"bound": "hbm", "kernel": "ecf8_decode_kernel<%d, %s>" % (hdrs[0].lane_syms, "pairs always fit" if 2 * cap <= 14 else "general"),
                     "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "avg_launch_us": round(launch_s * 1e6, 2),
                     "algorithmic_bytes_per_launch": int(alg_per_launch),
                     "traffic": profiled_traffic(workload, a.launch, hdrs, a.layers == 0)},
    }
    if a.launch == "stack" and per_layer and len(batches[0][1]) > 1:
        out["per_layer_launch"] = per_layer_rates(batches[0][1], alg_total, n_total)
    if copy_kernel:
        # the achievable ceiling on this machine: a plain device-to-device copy of 1 GiB (read + written bytes per second);
        # it doubles as the kernel of known traffic that the profiler counters are scaled by
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(5):
            dst.copy_(src)
        c1.record()
        torch.cuda.synchronize()
        copy_gbps = 5 * 2 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
        out["copy_kernel_GBps"] = round(copy_gbps, 1)
        out["pct_of_copy_kernel"] = round(100 * out["total_moved_GBps"] / copy_gbps, 1)
        del src, dst
    return out, batches


if __name__ == "__main__":
    main()
