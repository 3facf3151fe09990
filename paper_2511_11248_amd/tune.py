#!/usr/bin/env python3
"""Measured search for the library's tiling on the device it runs on (Sec. 4.1 "Unified tiling strategy": tile
sizes are searched per machine under the constraints of Eq. 1-4).

The shared tile block is fixed by the packed layout; what is searched is how many tile blocks a workgroup takes
(`tman_tiling_t`, include/tman.h).  Candidates that violate the constraints are refused by tman_set_tiling (the
tables of a one-token K segment must fit the workgroup's LDS, the prefill stage ring must fit 160 KB), every
admissible candidate is timed on synthetic layers of the benchmark shapes with rotating weight copies, and the
best value of each parameter is printed beside the built-in default.

    python -m paper_2511_11248_amd.tune [--copies 8] [--steps 200]
"""
from __future__ import annotations

import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--copies", type=int, default=8, help="rotating copies of a layer set (8 x 63 MB exceeds the 256 MB cache)")
    ap.add_argument("--steps", type=int, default=200)
    args = ap.parse_args()

    import torch

    import bench
    import paper_2511_11248_amd as tman
    import synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    default = tman.tman_default_tiling()

    def with_tiling(**kw):
        t = tman.tman_default_tiling()
        for k, v in kw.items():
            setattr(t, k, v)
        try:
            tman.tman_set_tiling(t)
        except tman.TmanError:
            return False  # violates a constraint: not a candidate
        return True

    def time_decode(workload, N, matrix_cores=False):
        w = synth.WORKLOADS[workload]
        job = bench.decode_job(torch, tman, synth, dev, w, N, args.copies)
        sec = bench.timed_steps(torch, bench.decode_step_fn(job, args.copies, matrix_cores=matrix_cores), 50, args.steps)
        del job
        return sec * 1e6

    def time_prefill(N):
        pw = synth.WORKLOADS["prefill_w4g64"]
        spec = pw.layers[0]
        ps = tman.Shape(spec.M, spec.K, pw.bits, pw.group, True)
        q, sc, z = synth.layer_tensors(pw, 0, 0, device=dev)
        blob = torch.empty(tman.tman_packed_bytes(ps), dtype=torch.uint8, device=dev)
        tman.tman_pack_weights(ps, q, sc, z, blob)
        x = torch.from_numpy(synth.activation(pw, 0, 0, N)).to(dev)
        y = torch.empty((N, spec.M), dtype=torch.float16, device=dev)
        return bench.timed_steps(torch, lambda i: tman.tman_mpgemm(ps, blob, x, N, y, None), 40, 100) * 1e6

    def time_prefill_i8(N):
        pw = synth.WORKLOADS["prefill_w4g64"]
        spec = pw.layers[0]
        ps = tman.Shape(spec.M, spec.K, pw.bits, pw.group, True)
        q, sc, z = synth.layer_tensors(pw, 0, 0, device=dev)
        sc = sc[:, :1].expand(-1, spec.K // pw.group).contiguous()  # one scale and zero per row
        z = z[:, :1].expand(-1, spec.K // pw.group).contiguous()
        blob = torch.empty(tman.tman_packed_bytes(ps), dtype=torch.uint8, device=dev)
        tman.tman_pack_weights(ps, q, sc, z, blob)
        x = torch.from_numpy(synth.activation(pw, 0, 0, N)).to(dev)
        xq = torch.empty(tman.tman_act_i8_bytes(N, spec.K), dtype=torch.uint8, device=dev)
        tman.tman_quantize_act_i8(x, N, spec.K, xq)
        y = torch.empty((N, spec.M), dtype=torch.float16, device=dev)
        return bench.timed_steps(torch, lambda i: tman.tman_mpgemm_i8(ps, blob, xq, N, y, None), 40, 100) * 1e6

    def sweep(title, param, values, measure):
        print(f"\n{title}\n  {param}: time per step (us)", flush=True)
        best = None
        for v in values:
            if not with_tiling(**{param: v}):
                print(f"    {v:>7}: refused (constraint)", flush=True)
                continue
            t = measure()
            mark = " (default)" if v == getattr(default, param) else ""
            print(f"    {v:>7}: {t:8.2f}{mark}", flush=True)
            if best is None or t < best[1]:
                best = (v, t)
        print(f"  best {param} = {best[0]} ({best[1]:.2f} us)", flush=True)
        tman.tman_set_tiling(default)
        return best

    t0 = time.time()
    print("built-in tiling:", default.as_dict())
    sweep("one-token decode, 7B layer set uint2 g64: workgroups numbered for equal work per compute unit (1) or a plain grid (0)",
          "decode_balance", [0, 1], lambda: time_decode("7b_w2g64", 1))
    sweep("one-token decode, 3.8B layer set uint2 g64: the same",
          "decode_balance", [0, 1], lambda: time_decode("3p8b_w2g64", 1))
    sweep("one-token decode, 7B layer set uint2 g64 (K = 4096 and 11008): segments of a K that needs cutting",
          "decode_x_long_seg_tiles", [15, 16, 17, 18, 20, 22, 24, 29, 32, 40], lambda: time_decode("7b_w2g64", 1))
    sweep("one-token decode, 7B layer set uint4 g128: the same",
          "decode_x_long_seg_tiles", [15, 17, 20, 22, 24, 32], lambda: time_decode("7b_w4g128", 1))
    sweep("one-token decode, 7B layer set uint4 g128: bytes of packed weights per row block up to which K stays one segment",
          "decode_x_whole_bytes", [40960, 81920, 163840], lambda: time_decode("7b_w4g128", 1))
    sweep("one-token decode, 3.8B layer set uint2 g64 (K = 3072 and 8192)",
          "decode_x_long_seg_tiles", [15, 17, 20, 22, 24, 32], lambda: time_decode("3p8b_w2g64", 1))
    sweep("8 tokens through the lookup kernel, 7B layer set uint4 g128",
          "decode_seg_tiles_many", [16, 20, 24, 28, 32], lambda: time_decode("7b_w4g128", 8))
    sweep("8 tokens through the small-batch matrix-core kernel, 7B layer set uint4 g128",
          "small_seg_tiles", [16, 22, 24, 32, 43, 86], lambda: time_decode("7b_w4g128", 8, matrix_cores=True))
    for N in (256, 1024, 2048):
        sweep(f"prefill 11008 x 4096 uint4 g64, N = {N}: tile blocks in M per workgroup (0 = the launcher's rule)",
              "prefill_row_blocks", [0, 1, 2, 3, 4, 5], lambda: time_prefill(N))
    for N in (128, 256):
        sweep(f"prefill 11008 x 4096 uint4 g64, N = {N}: 1 = the tiled kernel, 2 / 3 = the kernel whose waves split K with its "
              "64 x 256 / 128 x 128 tile (0 = the launcher's rule)",
              "prefill_k_split", [0, 1, 2, 3], lambda: time_prefill(N))
    for N in (256, 512, 1024, 2048):
        sweep(f"int8 prefill 11008 x 4096 uint4 per row, N = {N}: 1 = 128 x 128 tiles, 3 / 4 / 7 = 256 rows x 96 / 128 / 224 "
              "tokens dequantized in registers, 9 = waves split K (0 = the launcher's rule, 2 does not exist)",
              "i8_token_blocks", [0, 1, 2, 3, 4, 7, 9], lambda: time_prefill_i8(N))
    print(f"\nsearch took {time.time() - t0:.0f} s")


if __name__ == "__main__":
    main()
