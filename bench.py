#!/usr/bin/env python3
"""Benchmark of the T-MAN hot path on one MI355X.

Headline (the benchmark spec metric, configs[1]): decode mpGEMV weight GB/s on the 7B-style layer set,
uint2 weights, group 64, N = 1.  One step = one token through a 32-layer decoder built from that layer
set: 32 launches, one per layer, each layer with packed weights of its own (2 GB in all, so the 256 MB
Infinity Cache cannot serve them).  A launch takes the layer's activations in and gives its outputs: the
lookup-table precompute and the five table-lookup GEMVs (qkv, o, gate, up, down) run in one kernel whose
workgroups build the tables of their own K segment (the two-launch form, a table kernel followed by a
lookup kernel, is timed beside it).  All inputs are resident in HBM before timing.

The same JSON line carries: the error of the timed configuration against the fp64 CPU oracle; the prefill
mpGEMM figure (11008 x 4096 uint4 g64, N = 1024) with its error; `configs`, every other BASELINE
configuration timed briefly the same way with its error; the roofline fraction of the dominant kernel
(its average launch duration from HIP events that cut the timed region into runs of launches); and the
oracle timed on the host cores over a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
MFMA_I8_PEAK_TOPS = 5000.0

# HBM bytes per launch of the dominant kernels on the default workloads, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script scaled by a plain copy of known size (--calibration-copy); the counters
# cannot be read from inside the process.  Source: profiles/mpgemv_x_7b_w2g64_and_mpgemm_w4g64_hbm_traffic.txt.
MEASURED_TRAFFIC_BYTES = {
    ("mpgemv_x", "7b_w2g64", 1): 63_865_856 + 197_632,
    ("mpgemm", "prefill_w4g64", 1024): 92_651_315 + 22_544_384,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="7b_w2g64")
    ap.add_argument("--instances", type=int, default=0, help="copies of the layer set to rotate over (0 = workload default)")
    ap.add_argument("--prefill-tokens", type=int, default=1024)
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--event-every", type=int, default=50,
                    help="record a HIP event on the launch stream before every n-th launch of the dominant kernel; "
                         "the time between two events over n is the average launch duration of that run of launches "
                         "(an event around every single launch costs a few microseconds of stream time and spans the "
                         "dispatch, which distorts a 17 us kernel)")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the context figures (cache-resident, two-launch, device copy): under a profiler the "
                         "kernel statistics then cover the timed, cache-cold launches only")
    ap.add_argument("--table", action="store_true",
                    help="after the JSON line, print the same figures (headline, prefill, every other configuration) "
                         "as a table on stderr")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the `configs` array (every other BASELINE configuration, timed briefly and checked "
                         "against the oracle): under a profiler the statistics then cover the headline workloads only")
    ap.add_argument("--preroll", type=int, default=300,
                    help="untimed launches before the declared warm-up: clocks and caches reach their steady state, so "
                         "a short timed region reads what a long one reads")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device-to-device copy of 256 MiB before the timed region: under "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE its known traffic calibrates the counters")
    return ap.parse_args()


def decode_job(torch, tman, synth, dev, w, N, n_inst):
    """Everything one decode step of workload ``w`` needs, resident in HBM: ``n_inst`` packed copies of the
    layer set, their activations, table buffers, outputs, and per copy the two bound launches of a step."""
    shapes = [tman.Shape(l.M, l.K, w.bits, w.group, w.has_zero) for l in w.layers]
    acts = []  # distinct activation tags in order of first use
    for l in w.layers:
        if l.act not in acts:
            acts.append(l.act)
    act_of_layer = [acts.index(l.act) for l in w.layers]
    act_layer0 = [next(i for i, l in enumerate(w.layers) if l.act == a) for a in acts]

    blobs, xs, luts, ys, wss, descs = [], [], [], [], [], []
    weight_bytes_per_step = sum(tman.tman_packed_bytes(s) - 128 for s in shapes)
    for ai, li0 in enumerate(act_layer0):
        K = w.layers[li0].K
        luts.append(torch.empty(tman.tman_lut_bytes(N, K, w.group), dtype=torch.uint8, device=dev))
    for s in shapes:
        ys.append(torch.empty((N, s.M), dtype=torch.float16, device=dev))
        wss.append(torch.zeros(tman.tman_mpgemv_workspace_bytes(s, N), dtype=torch.uint8, device=dev))
    lut_of_layer = [luts[a] for a in act_of_layer]
    for inst in range(n_inst):
        bl = []
        for li, s in enumerate(shapes):
            q, sc, z = synth.layer_tensors(w, inst, li, device=dev)
            blob = torch.empty(tman.tman_packed_bytes(s), dtype=torch.uint8, device=dev)
            tman.tman_pack_weights(s, q, sc, z, blob)
            bl.append(blob)
            del q
        blobs.append(bl)
        xs.append([torch.from_numpy(synth.activation(w, inst, li0, N)).to(dev) for li0 in act_layer0])
        # one descriptor table per copy of the layer set: built once, reused by every step that visits it
        d = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev)
        tman.tman_mpgemv_batch_prepare(shapes, bl, lut_of_layer, N, ys, wss, d)
        descs.append(d)
    torch.cuda.synchronize()

    # per step: one launch builds the lookup tables of the step's activations, one launch runs all GEMVs
    stream = torch.cuda.current_stream().cuda_stream
    Ks = [w.layers[li0].K for li0 in act_layer0]
    lut_calls = [tman.bound_build_lut_batch(xs[inst], N, Ks, w.group, luts) for inst in range(n_inst)]
    gemv_calls = [tman.bound_mpgemv_batch_run(shapes, N, descs[inst]) for inst in range(n_inst)]
    # one token: the lookup kernel can build its tables itself, which makes the step a single launch
    x_calls, x_descs = None, []
    if N == 1:
        for inst in range(n_inst):
            d = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev)
            tman.tman_mpgemv_x_batch_prepare(shapes, blobs[inst], [xs[inst][a] for a in act_of_layer], ys, wss, d)
            x_descs.append(d)
        torch.cuda.synchronize()
        x_calls = [tman.bound_mpgemv_x_batch_run(shapes, x_descs[inst]) for inst in range(n_inst)]
    # integer tables (A_INT16 reading): a table launch that quantizes the activations, a lookup launch on int16 entries
    i16_luts = [torch.empty(tman.tman_lut_i16_bytes(N, w.layers[li0].K, w.group), dtype=torch.uint8, device=dev)
                for li0 in act_layer0]
    i16_descs = []
    for inst in range(n_inst):
        d = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev)
        tman.tman_mpgemv_batch_prepare(shapes, blobs[inst], [i16_luts[a] for a in act_of_layer], N, ys, wss, d)
        i16_descs.append(d)
    torch.cuda.synchronize()
    i16_lut_calls = [tman.bound_build_lut_i16_batch(xs[inst], N, Ks, w.group, i16_luts) for inst in range(n_inst)]
    i16_gemv_calls = [tman.bound_mpgemv_i16_batch_run(shapes, N, i16_descs[inst]) for inst in range(n_inst)]
    # a few tokens: the same product on the matrix cores (tman_mpgemm's small-batch kernel), one launch per layer set
    mm_calls, mm_keep = None, []
    if N > 1:
        mm_ws = []
        for s in shapes:
            need = tman.tman_mpgemm_workspace_bytes(s, N)
            mm_ws.append(torch.zeros(need, dtype=torch.uint8, device=dev) if need else None)
        for inst in range(n_inst):
            d = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev)
            tman.tman_mpgemm_batch_prepare(shapes, blobs[inst], [xs[inst][a] for a in act_of_layer], N, ys, mm_ws, d)
            mm_keep.append(d)
        torch.cuda.synchronize()
        mm_calls = [tman.bound_mpgemm_batch_run(shapes, N, mm_keep[inst]) for inst in range(n_inst)]
        mm_keep.append(mm_ws)
    return {"shapes": shapes, "acts": acts, "weight_bytes_per_step": weight_bytes_per_step, "ys": ys,
            "lut_calls": lut_calls, "gemv_calls": gemv_calls, "x_calls": x_calls, "mm_calls": mm_calls, "stream": stream,
            "i16_lut_calls": i16_lut_calls, "i16_gemv_calls": i16_gemv_calls,
            "keep": (blobs, xs, luts, wss, descs, x_descs, mm_keep, i16_luts, i16_descs)}  # the launches hold raw pointers into these


def timed_steps(torch, step, warm, steps):
    """Wall clock per step over `steps` calls of step(i) after `warm` untimed ones (device idle on both sides)."""
    for i in range(warm):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def decode_step_fn(job, n_inst, matrix_cores=False, integer_tables=False):
    stream = job["stream"]
    if integer_tables:  # activations quantized to integers, int16 tables, integer sums inside a quantization block
        def ints(i):
            job["i16_lut_calls"][i % n_inst](stream)
            job["i16_gemv_calls"][i % n_inst](stream)

        return ints
    if matrix_cores:  # a few tokens, dequantized in registers and multiplied on the matrix cores: one launch
        return lambda i: job["mm_calls"][i % n_inst](stream)
    if job["x_calls"] is not None:  # one token: one launch
        return lambda i: job["x_calls"][i % n_inst](stream)

    def two(i):
        job["lut_calls"][i % n_inst](stream)
        job["gemv_calls"][i % n_inst](stream)

    return two


def decode_error(torch, synth, oracle, w, job, N, inst=0, matrix_cores=False, integer_tables=False):
    """Largest row-normalised error of the outputs of the step on copy `inst` against the fp64 oracle (with integer
    tables: the oracle for the integer activations), and the oracle's time."""
    for y in job["ys"]:
        y.fill_(float("nan"))
    decode_step_fn(job, max(inst + 1, 1), matrix_cores, integer_tables)(inst)
    torch.cuda.synchronize()
    err, cpu_t, used = 0.0, 0.0, 1
    for li in range(len(job["shapes"])):
        q, sc, z = synth.layer_tensors(w, inst, li)
        xh = synth.activation(w, inst, li, N)
        c0 = time.perf_counter()
        if integer_tables:
            xq, ex = oracle.quantize_activations(xh)
            Y = oracle.matmul_real_x(q, sc, z, xq.astype(np.float64) * (2.0 ** ex.astype(np.float64))[:, None], w.bits, w.group)
        else:
            Y, used = oracle.matmul(q, sc, z, xh, w.bits, w.group, return_threads=True)
        cpu_t += time.perf_counter() - c0
        err = max(err, float(oracle.row_relative_error(job["ys"][li].cpu().numpy().astype(np.float64), Y).max()))
    return err, cpu_t, used


def whole_model_launch(torch, tman, dev, w, job):
    """BASELINE config 4 asks for the weight stream of a whole 32-layer decoder in one decode step, every GEMV
    with an activation of its own (nothing runs between the layers): all 32 x 5 GEMVs in ONE launch."""
    blobs, xs = job["keep"][0], job["keep"][1]
    acts = job["acts"]
    shapes, pk, xx, ys, wss = [], [], [], [], []
    for inst in range(w.instances):
        for li, l in enumerate(w.layers):
            sh = job["shapes"][li]
            shapes.append(sh); pk.append(blobs[inst][li]); xx.append(xs[inst][acts.index(l.act)])
            ys.append(torch.empty((1, sh.M), dtype=torch.float16, device=dev))
            wss.append(torch.zeros(tman.tman_mpgemv_workspace_bytes(sh, 1), dtype=torch.uint8, device=dev))
    desc = torch.empty(tman.tman_mpgemv_batch_desc_bytes(len(shapes)), dtype=torch.uint8, device=dev)
    tman.tman_mpgemv_x_batch_prepare(shapes, pk, xx, ys, wss, desc)
    call = tman.bound_mpgemv_x_batch_run(shapes, desc)
    return {"call": call, "ys": ys, "n_gemv": len(shapes), "keep": (wss, desc, pk, xx)}


def other_configs(args, torch, tman, synth, oracle, dev):
    """Every BASELINE configuration besides the two headline workloads, timed briefly with the headline protocol
    (rotating copies for decode, back-to-back calls for prefill) and checked against the oracle in the same run."""
    out = []

    def add(workload, sec, rate, unit, peak, err, checked):
        out.append({"workload": workload, "us": round(sec * 1e6, 2), "rate": round(rate, 1), "unit": unit,
                    "frac": round(rate / peak, 4), "max_err": float(f"{err:.3e}"), "checked": checked})

    for name in ("tiny_w4g64", "7b_w4g128", "3p8b_w2g64", "3p8b_w1g64"):
        w = synth.WORKLOADS[name]
        for N in w.tokens:
            job = decode_job(torch, tman, synth, dev, w, N, w.instances)
            step = decode_step_fn(job, w.instances)
            sec = timed_steps(torch, step, 100, 300)
            err, _, _ = decode_error(torch, synth, oracle, w, job, N)
            gbs = job["weight_bytes_per_step"] / sec / 1e9
            kind = "one launch per layer set" if job["x_calls"] is not None else "table launch + lookup launch per layer set"
            add(f"{name} N={N}, {w.instances} rotating copies, {kind}" + (" (cache-resident: correctness only)" if w.instances == 1 else ""),
                sec, gbs, "GB/s", HBM_PEAK_GBS, err, "all outputs of copy 0")
            if w.config == 2:  # integer activations and tables (the paper's A_INT16 configuration), same workload
                step = decode_step_fn(job, w.instances, integer_tables=True)
                sec = timed_steps(torch, step, 100, 300)
                err, _, _ = decode_error(torch, synth, oracle, w, job, N, integer_tables=True)
                add(f"{name} N={N}, {w.instances} rotating copies, integer tables (tman_build_lut_i16 launch + "
                    f"tman_mpgemv_i16 launch per layer set); error against the oracle for the integer activations, "
                    f"bound 1e-3", sec, job["weight_bytes_per_step"] / sec / 1e9, "GB/s", HBM_PEAK_GBS, err,
                    "all outputs of copy 0")
            if N > 1:  # the same tokens through the matrix-core kernel
                step = decode_step_fn(job, w.instances, matrix_cores=True)
                sec = timed_steps(torch, step, 100, 300)
                err, _, _ = decode_error(torch, synth, oracle, w, job, N, matrix_cores=True)
                add(f"{name} N={N}, {w.instances} rotating copies, one tman_mpgemm_batch launch per layer set "
                    f"(dequantization in registers + MFMA)", sec, job["weight_bytes_per_step"] / sec / 1e9, "GB/s",
                    HBM_PEAK_GBS, err, "all outputs of copy 0")
            if w.config == 4:  # the whole 32-layer weight stream as one launch of 160 GEMVs
                big = whole_model_launch(torch, tman, dev, w, job)
                stream = job["stream"]
                sec = timed_steps(torch, lambda i: big["call"](stream), 5, 40)
                err = 0.0
                for inst in (0, w.instances - 1):
                    for li in range(len(w.layers)):
                        q, sc, z = synth.layer_tensors(w, inst, li)
                        Y = oracle.matmul(q, sc, z, synth.activation(w, inst, li, 1), w.bits, w.group)
                        y = big["ys"][inst * len(w.layers) + li].cpu().numpy().astype(np.float64)
                        err = max(err, float(oracle.row_relative_error(y, Y).max()))
                total = job["weight_bytes_per_step"] * w.instances
                add(f"{name} N=1, all {w.instances} layers = {big['n_gemv']} GEMVs in one launch ({total / 1e6:.0f} MB)",
                    sec, total / sec / 1e9, "GB/s", HBM_PEAK_GBS, err, "all outputs of layers 0 and 31")
                del big
            del job, step
    pw = synth.WORKLOADS["prefill_w4g64"]
    spec = pw.layers[0]
    ps = tman.Shape(spec.M, spec.K, pw.bits, pw.group, True)
    q, sc, z = synth.layer_tensors(pw, 0, 0)
    pblob = torch.empty(tman.tman_packed_bytes(ps), dtype=torch.uint8, device=dev)
    tman.tman_pack_weights(ps, torch.from_numpy(q).to(dev), torch.from_numpy(sc).to(dev), torch.from_numpy(z).to(dev), pblob)
    for NP in pw.tokens:
        if NP == args.prefill_tokens:
            continue  # the headline prefill figure
        xh = synth.activation(pw, 0, 0, NP)
        px = torch.from_numpy(xh).to(dev)
        py = torch.empty((NP, spec.M), dtype=torch.float16, device=dev)
        sec = timed_steps(torch, lambda i: tman.tman_mpgemm(ps, pblob, px, NP, py, None), 40, 100)
        tf = 2.0 * NP * spec.M * spec.K / sec / 1e12
        err, rows = prefill_error(oracle, q, sc, z, xh, py, pw)
        add(f"{pw.name}: {spec.M}x{spec.K} uint4 g64, N={NP}", sec, tf, "TFLOP/s", MFMA_F16_PEAK_TFLOPS, err,
            f"{len(rows)} whole tokens (first, last, tile edges, seeded picks)")
    # per-tensor / per-channel formats on the integer matrix cores (Sec. 6.1 BitNet shapes; the prefill shape for scale)
    for (M, K, bits, label) in ((6912, 2560, 2, "BitNet-2B-style 6912x2560, ternary weights as 2-bit codes, one scale per tensor"),
                                (2560, 6912, 2, "BitNet-2B-style 2560x6912, ternary weights as 2-bit codes, one scale per tensor"),
                                (11008, 4096, 4, "11008x4096 uint4, one scale and zero per row")):
        NP, group = 1024, 64
        seed = 0x18000 + M
        q = synth.uniform_codes(seed, M * K, bits).reshape(M, K)
        if bits == 2:
            q = (q % 3).astype(np.uint8)
            rs, rz = np.full(M, np.float16(0.037)), np.ones(M, dtype=np.float16)
        else:
            rs, rz = synth.uniform_fp16(seed + 1, M, 0.005, 0.02), synth.uniform_fp16(seed + 2, M, 6.0, 9.0)
        xh = synth.normal_fp16(seed + 3, NP * K).reshape(NP, K)
        sh = tman.Shape(M, K, bits, group, True)
        blob = torch.empty(tman.tman_packed_bytes(sh), dtype=torch.uint8, device=dev)
        tman.tman_pack_weights(sh, torch.from_numpy(q).to(dev), torch.from_numpy(np.repeat(rs.reshape(M, 1), K // group, 1)).to(dev),
                               torch.from_numpy(np.repeat(rz.reshape(M, 1), K // group, 1)).to(dev), blob)
        px = torch.from_numpy(xh).to(dev)
        xq = torch.empty(tman.tman_act_i8_bytes(NP, K), dtype=torch.uint8, device=dev)
        py = torch.empty((NP, M), dtype=torch.float16, device=dev)
        tman.tman_quantize_act_i8(px, NP, K, xq)
        sec = timed_steps(torch, lambda i: tman.tman_mpgemm_i8(sh, blob, xq, NP, py, None), 40, 100)

        def both(i):
            tman.tman_quantize_act_i8(px, NP, K, xq)
            tman.tman_mpgemm_i8(sh, blob, xq, NP, py, None)

        sec_both = timed_steps(torch, both, 20, 100)
        rows = [0, 1, 127, 128, NP // 2, NP - 1] + np.random.default_rng(M).integers(0, NP, 10).tolist()
        xo, mo = oracle.quantize_activations_i8(xh[rows])
        _, Y = oracle.matmul_i8(q, rs, rz, xo, mo, bits)
        err = float(oracle.row_relative_error(py[rows].cpu().numpy().astype(np.float64), Y).max())
        tops = 2.0 * NP * M * K / sec / 1e12
        add(f"int8 matrix cores: {label}, N={NP} (tman_mpgemm_i8 alone; with the activation quantizer launch "
            f"{sec_both * 1e6:.1f} us); error against the oracle for the integer activations, bound 1e-3",
            sec, tops, "TOP/s", MFMA_I8_PEAK_TOPS, err, f"{len(rows)} whole tokens")
    return out


def prefill_error(oracle, q, sc, z, xh, py, pw):
    """Row-normalised error of a seeded sample of whole tokens (all output features of each) against the oracle."""
    NP = xh.shape[0]
    rng = np.random.default_rng(NP)
    rows = sorted(set([0, 1, 127, 128, NP // 2, NP - 129, NP - 128, NP - 1]) | set(rng.integers(0, NP, 16).tolist()))
    rows = [r for r in rows if 0 <= r < NP]
    Y = oracle.matmul(q, sc, z, xh[rows], pw.bits, pw.group)
    y = py[rows].cpu().numpy().astype(np.float64)
    return float(oracle.row_relative_error(y, Y).max()), rows



def print_table(out):
    rows = [("config", "GPU time (us)", "rate", "of vendor peak", "max err", "checked")]
    rows.append((out["config"]["workload"][:60] + "...", f"{out['ms_per_step'] * 1e3:.2f}", f"{out['value']:.0f} GB/s",
                 f"{out['value'] / HBM_PEAK_GBS:.1%}", f"{out['max_err']:.2e}", "all outputs of copy 0"))
    if "prefill" in out:
        p = out["prefill"]
        rows.append((p["config"]["workload"], f"{p['ms_per_call'] * 1e3:.1f}", f"{p['value']:.0f} TFLOP/s",
                     f"{p['roofline']['frac']:.1%}", f"{p['max_err']:.2e}", p["checked"]))
    for c in out.get("configs", []):
        rows.append((c["workload"], f"{c['us']:.2f}", f"{c['rate']:.0f} {c['unit']}", f"{c['frac']:.1%}",
                     f"{c['max_err']:.2e}", c["checked"]))
    for r in rows:
        print("| " + " | ".join(r) + " |", file=sys.stderr)
    if "cpu_baseline" in out:
        c = out["cpu_baseline"]
        print(f"oracle on the host: {c['value']} {c['unit']} on {c['cores']} cores ({c['sample']})", file=sys.stderr)


def context_figures(args, torch, dev, job, n_inst):
    """The step on one copy of the layer set (cache-resident), as two launches, and a plain device copy."""
    x_calls, lut_calls, gemv_calls, stream = job["x_calls"], job["lut_calls"], job["gemv_calls"], job["stream"]
    weight_bytes_per_step = job["weight_bytes_per_step"]
    steps = max(args.steps, 500)
    hot_value = weight_bytes_per_step / timed_steps(torch, lambda i: x_calls[0](stream), 100, steps) / 1e9

    # the same step as two launches (table precompute kernel, then the lookup kernel reading its tables)
    def two(i):
        lut_calls[i % n_inst](stream)
        gemv_calls[i % n_inst](stream)

    two_launch_value = weight_bytes_per_step / timed_steps(torch, two, 100, steps) / 1e9
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        cp_dst.copy_(cp_src)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2.0 * (1 << 30) / (time.perf_counter() - t0) / 1e9
    del cp_src, cp_dst

    return {"cache_resident_GBs": round(hot_value, 1), "two_launch_step_GBs": round(two_launch_value, 1),
            "device_copy_GBs_read_plus_write": round(copy_gbs, 1)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2511_11248_amd as tman
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.WORKLOADS[args.workload]
    n_inst = args.instances or w.instances
    N = 1
    job = decode_job(torch, tman, synth, dev, w, N, n_inst)
    shapes, acts, weight_bytes_per_step = job["shapes"], job["acts"], job["weight_bytes_per_step"]
    lut_calls, gemv_calls, x_calls, stream = job["lut_calls"], job["gemv_calls"], job["x_calls"], job["stream"]
    events = []

    # One step = one token through a 32-layer decoder of this layer set: the 32 copies in turn, one launch each
    # (activations in, outputs out: the table precompute and the lookups of all five GEMVs of a layer set).
    launches_per_step = n_inst

    def launch(j, record):
        if record:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            events.append((j, e))
        x_calls[j % n_inst](stream)

    def step(i, timed):
        for j in range(i * launches_per_step, (i + 1) * launches_per_step):
            launch(j, timed and j % args.event_every == 0)

    if args.calibration_copy:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.preroll):  # clocks and caches to their steady state, before the declared warm-up
        launch(i, False)
    torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, True)
    e = torch.cuda.Event(enable_timing=True)
    e.record()
    events.append((args.steps * launches_per_step, e))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps
    weight_bytes_per_launch = weight_bytes_per_step
    weight_bytes_per_step = weight_bytes_per_launch * launches_per_step
    value = weight_bytes_per_step / sec_per_step / 1e9

    # dominant kernel: the table-lookup GEMV (one launch per step covers the whole layer set); its average
    # launch duration comes from the HIP events that cut the timed region into runs of launches
    runs = [(i1 - i0, e0.elapsed_time(e1)) for (i0, e0), (i1, e1) in zip(events[:-1], events[1:])]
    n_launch = sum(n for n, _ in runs)
    avg_launch_s = sum(ms for _, ms in runs) / 1e3 / n_launch
    gemv_ms = sorted(ms / n for n, ms in runs)  # per-launch averages of the runs
    bytes_per_launch = weight_bytes_per_launch
    achieved = bytes_per_launch / avg_launch_s / 1e9
    roofline = {
        "bound": "hbm", "kernel": "mpgemv_x_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(("mpgemv_x", w.name, N)),
        "launches": n_launch, "event_runs": len(runs), "avg_launch_us": round(avg_launch_s * 1e6, 3),
        "median_run_avg_us": round(gemv_ms[len(gemv_ms) // 2] * 1e3, 3),
        "fastest_run_avg_us": round(gemv_ms[0] * 1e3, 3),
        "algorithmic_bytes_per_launch": int(bytes_per_launch),
    }

    # context figures (not the headline): the same step on ONE copy of the layer set (63 MB: served by the
    # 256 MB Infinity Cache), the bit-plane bytes alone, and what a plain device copy moves on this machine
    codes_bytes = sum(s.M * s.K * w.bits // 8 for s in shapes) * launches_per_step
    context = {}
    if not args.no_context:
        context = context_figures(args, torch, dev, job, n_inst)

    # the same step on copy 0 against the fp64 oracle, every output of the five GEMVs
    import oracle

    oracle.build()
    max_err, _, _ = decode_error(torch, synth, oracle, w, job, N)

    out = {
        "metric": "decode mpGEMV weight GB/s", "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "max_err": float(f"{max_err:.3e}"), "tolerance": 2e-3,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{w.name}: decode of one token (N=1) through {n_inst} layers of the 7B-style layer set "
                               f"(qkv 12288x4096, o 4096x4096, gate/up 11008x4096, down 4096x11008), uint{w.bits} "
                               f"g{w.group}, every layer with weights of its own ({weight_bytes_per_step / 1e9:.2f} GB per "
                               f"step); one launch per layer: every workgroup builds the lookup tables of its K "
                               f"segment from the layer's {len(acts)} activations, then does its lookups",
                   "launches_per_step": launches_per_step, "us_per_launch": round(sec_per_step / launches_per_step * 1e6, 3),
                   "weight_bytes_per_step": int(weight_bytes_per_step), "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
                   "codes_only_GBs": round(value * codes_bytes / weight_bytes_per_step, 1), **context},
        "roofline": roofline,
    }

    # ------------------------------------------------------------------ prefill (secondary figure)
    if not args.no_prefill:
        pw = synth.WORKLOADS["prefill_w4g64"]
        spec = pw.layers[0]
        ps = tman.Shape(spec.M, spec.K, pw.bits, pw.group, True)
        q, sc, z = synth.layer_tensors(pw, 0, 0, device=dev)
        pblob = torch.empty(tman.tman_packed_bytes(ps), dtype=torch.uint8, device=dev)
        tman.tman_pack_weights(ps, q, sc, z, pblob)
        del q
        NP = args.prefill_tokens
        px = torch.from_numpy(synth.activation(pw, 0, 0, NP)).to(dev)
        py = torch.empty((NP, spec.M), dtype=torch.float16, device=dev)
        for _ in range(40):  # the clocks need a few milliseconds of this load to settle
            tman.tman_mpgemm(ps, pblob, px, NP, py, None)
        torch.cuda.synchronize()
        runs_p, per_run = 10, 10  # events cut 100 back-to-back calls into runs of ten
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(runs_p + 1)]
        for r in range(runs_p):
            pe[r].record()
            for _ in range(per_run):
                tman.tman_mpgemm(ps, pblob, px, NP, py, None)
        pe[runs_p].record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) / per_run for a, b in zip(pe[:-1], pe[1:]))
        avg_ms = sum(ts) / len(ts)
        flops = 2.0 * NP * spec.M * spec.K
        tf = flops / (avg_ms / 1e3) / 1e12
        qh, sh, zh = synth.layer_tensors(pw, 0, 0)
        perr, prow = prefill_error(oracle, qh, sh, zh, synth.activation(pw, 0, 0, NP), py, pw)
        out["prefill"] = {
            "metric": "prefill mpGEMM TFLOPS", "value": round(tf, 1), "unit": "TFLOP/s",
            "max_err": float(f"{perr:.3e}"), "checked": f"{len(prow)} whole tokens",
            "config": {"workload": f"{pw.name}: {spec.M}x{spec.K} uint4 g64, N={NP}"},
            "ms_per_call": round(avg_ms, 4), "fastest_run_ms_per_call": round(ts[0], 4),
            "roofline": {"bound": "mfma", "kernel": "mpgemm_kernel", "achieved": round(tf, 1),
                         "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_F16_PEAK_TFLOPS, 4),
                         "traffic": MEASURED_TRAFFIC_BYTES.get(("mpgemm", pw.name, NP))},
        }
        del pblob, px, py

    # ------------------------------------------------------------------ every other BASELINE configuration
    del job, lut_calls, gemv_calls, x_calls
    if not args.no_configs:
        out["configs"] = other_configs(args, torch, tman, synth, oracle, dev)

    # ------------------------------------------------------------------ CPU oracle on the host cores
    if not args.no_cpu_baseline:
        done_bytes, cpu_t, cores, used = 0, 0.0, os.cpu_count(), 1
        sample = []
        inst = 0
        while cpu_t < args.cpu_seconds:
            for li, s in enumerate(shapes):
                q, sc, z = synth.layer_tensors(w, inst % n_inst, li, device=dev)
                qh, sh, zh = q.cpu().numpy(), sc.cpu().numpy(), (z.cpu().numpy() if z is not None else None)
                xh = synth.activation(w, inst % n_inst, li, N)
                c0 = time.perf_counter()
                _, used = oracle.matmul(qh, sh, zh, xh, w.bits, w.group, return_threads=True)
                cpu_t += time.perf_counter() - c0
                done_bytes += tman.tman_packed_bytes(s) - 128
                sample.append(f"{inst % n_inst}:{w.layers[li].name}")
                if cpu_t >= args.cpu_seconds:
                    break
            inst += 1
        out["cpu_baseline"] = {
            "value": round(done_bytes / cpu_t / 1e9, 3), "unit": "GB/s", "cores": int(used), "kind": "oracle",
            "sample": f"{len(sample)} GEMVs of the same workload (layer sets 0..{min(inst, n_inst) - 1}, revisited "
                      f"in order if exhausted), {cpu_t:.1f} s of fp64 "
                      f"dequantize-then-multiply; weight bytes counted as for the GPU",
        }

    print(json.dumps(out), flush=True)
    if args.table:
        print_table(out)


if __name__ == "__main__":
    main()
