#!/usr/bin/env python3
"""Benchmark of the GraSS compression hot path on one MI355X.

Headline workload ("mlp_mask_sjlt"): n = 4,096 per-sample gradients of an MLP
784-1024-1024-10 (p = 1,863,690 fp32, ReLU-style zeros), Random Mask to
k' = 65,536, SJLT to k = 4,096 with s = 1, fused (Sec. 3.3.1).  A step is one
call of grass_sjlt with the mask indices over the whole batch, inputs resident
in HBM.  Prints ONE JSON line: value = n / time per step; roofline.achieved =
algorithmic bytes per launch (n (4k' + 4k) + 4k') / kernel time measured with
HIP events; roofline.traffic = HBM bytes per launch from the rocprofv3 counter
runs summarised under profiles/; cpu_baseline = the CPU oracle on the same rows.

The other paths (s = 4, the plain gather, ResNet-scale SJLT, FactGraSS, score
GEMM) are timed briefly afterwards and reported under "extras".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
MFMA_PEAK_F32_TFLOPS = 157.3     # MI355X published dense fp32 matrix rate
MFMA_PEAK_BF16_TFLOPS = 2500.0

# HBM traffic per launch of the headline kernel comes from the rocprofv3 --pmc summary under profiles/ (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size).  The summary ends in a
# "traffic_record:" line naming the kernel instantiation, launch grid and workload it was taken on; the figure is
# used only if the library reports the same instantiation and grid for this run, otherwise traffic is null.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "sjlt_fused_mlp_pmc.txt")


def _traffic_record(path):
    """Parses 'traffic_record: key=value ...' from a profile summary; None if the file or the line is missing."""
    try:
        with open(path) as fh:
            lines = [ln for ln in fh if ln.startswith("traffic_record:")]
    except OSError:
        return None
    if not lines:
        return None
    rec = {}
    for tok in lines[-1].split()[1:]:
        key, _, val = tok.partition("=")
        rec[key] = val
    return rec


def _touched_lines(idx, elem_bytes, row_bytes, base_mod, rows):
    """Number of distinct 128-byte lines that `rows` rows touch when every row reads the elements `idx` (element size
    elem_bytes) and consecutive rows start row_bytes apart, the first at an address congruent to base_mod mod 128."""
    import numpy as np
    off = idx.astype(np.int64) * elem_bytes
    period = 128 // np.gcd(row_bytes % 128, 128) if row_bytes % 128 else 1
    per_phase = [np.unique((off + (base_mod + r * row_bytes) % 128) // 128).size for r in range(min(period, rows))]
    total = 0
    for r, cnt in enumerate(per_phase):
        total += cnt * ((rows - r + period - 1) // period)
    return total


def _timed(fn, steps, warmup, torch, indexed=False, per_call=False):
    """HIP events on torch's current stream (the stream the binding launches on) around the timed calls.
    per_call=True also brackets every call (used for the headline kernel; an event record between two calls of a few
    tens of microseconds would show up in their time, so the short paths are timed as one region).
    indexed=True hands fn the running call number (warm-up included) so that it can rotate its inputs."""
    for w in range(warmup):
        fn(w) if indexed else fn()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        fn(warmup + i) if indexed else fn()
        if per_call or i == steps - 1:
            evs[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)] if per_call else []
    total_ms = evs[0].elapsed_time(evs[steps])
    return total_ms, per, wall_ms


def _roof(bound, achieved, peak, unit, **more):
    """A roofline object in the shape of the headline's, for one of the extra paths."""
    d = {"bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit, "frac": round(achieved / peak, 4)}
    d.update(more)
    return d


def bench_single_layer(grass, synth, torch, dev, seed, extras):
    """FactGraSS, the LoGra baseline and the other factorised compressors on one 4096 x 4096 linear layer
    (n = 32 sequences of 512 tokens, masks 64/64, k = 1,024), inputs rotated through five tensor pairs."""
    # FactGraSS on one 4096 x 4096 linear layer.  Five (x, g) pairs of 268 MB each are rotated so that no call
    # finds its inputs in the 256 MB last-level cache (the resident figure is reported next to it)
    n4, T4, d4, kf, k4, NPAIR = 32, 512, 4096, 64, 1024, 5
    pairs = [synth.linear_layer_factors(n4, T4, d4, d4, seed=1004 + 50 * q, device=dev) for q in range(NPAIR)]
    x4, go4 = pairs[0]
    ii = grass.grass_mask_indices(seed, 16, d4, kf, device=dev)
    io = grass.grass_mask_indices(seed, 17, d4, kf, device=dev)
    o4 = torch.empty((n4, k4), dtype=torch.float32, device=dev)
    w4 = torch.empty(max(grass.factgrass_linear_workspace_bytes(n4, T4, kf, kf, k4, 1), 1), dtype=torch.uint8,
                     device=dev)
    # 128-byte lines a token touches in x and in g (rows of 8,192 bytes start on a line), the floor for a gather
    ii_h, io_h = ii.cpu().numpy(), io.cpu().numpy()
    lines4 = _touched_lines(ii_h, 2, d4 * 2, 0, 1) + _touched_lines(io_h, 2, d4 * 2, 0, 1)
    line_bytes4 = n4 * T4 * lines4 * 128 + n4 * k4 * 4 + 2 * w4.numel()
    t, _, _ = _timed(lambda: grass.factgrass_linear(x4, go4, ii, io, k4, 1, seed, 18, out=o4, ws=w4), 20, 3, torch)
    resident_ms = t / 20
    t, _, _ = _timed(lambda c: grass.factgrass_linear(pairs[c % NPAIR][0], pairs[c % NPAIR][1], ii, io, k4, 1, seed, 18,
                                                      out=o4, ws=w4), 40, NPAIR, torch, indexed=True)
    fg_ms = t / 40
    extras["factgrass_linear_4096"] = {"ms": round(fg_ms, 4), "ms_inputs_resident": round(resident_ms, 4),
                                       "rotating_input_pairs": NPAIR,
                                       "samples_per_s": round(n4 / (fg_ms * 1e-3), 1),
                                       "tokens_per_s": round(n4 * T4 / (fg_ms * 1e-3), 1),
                                       "useful_GBps": round(2 * n4 * T4 * 2 * kf / (fg_ms * 1e-3) / 1e9, 2),
                                       "lines_per_token": int(lines4),
                                       "roofline": _roof("hbm", line_bytes4 / (fg_ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s",
                                                         traffic_model_bytes=int(line_bytes4),
                                                         note="touched 128-byte lines of the gathered columns (counted "
                                                              "from the indices) + partial sums + output")}
    # LoGra baseline (dense factorised projection to 64 x 64) on the same layer, for the speed ratio
    Pi = grass.grass_to_bf16(grass.grass_gauss_matrix(seed, 40, d4, kf, 0, d4, device=dev))
    Po = grass.grass_to_bf16(grass.grass_gauss_matrix(seed, 41, d4, kf, 0, d4, device=dev))
    ol = torch.empty((n4, kf * kf), dtype=torch.float32, device=dev)
    wl = torch.empty(max(grass.logra_linear_workspace_bytes(n4, T4, kf, kf), 1), dtype=torch.uint8, device=dev)
    tl, _, _ = _timed(lambda c: grass.logra_linear(pairs[c % NPAIR][0], pairs[c % NPAIR][1], Pi, Po, out=ol, ws=wl),
                      40, NPAIR, torch, indexed=True)
    lg_ms = tl / 40
    lg_bytes = 2 * n4 * T4 * d4 * 2 + n4 * kf * kf * 4 + 2 * wl.numel()
    extras["logra_linear_4096"] = {"ms": round(lg_ms, 4), "tokens_per_s": round(n4 * T4 / (lg_ms * 1e-3), 1),
                                   "rotating_input_pairs": NPAIR,
                                   "factgrass_speedup": round(lg_ms / fg_ms, 2),
                                   "roofline": _roof("hbm", lg_bytes / (lg_ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s",
                                                     algorithmic_bytes=int(lg_bytes),
                                                     note="every column of x and g is read once")}
    # the other factorised compressors of the paper's Table 2 on the same layer (64 x 64 -> 4,096 outputs)
    wm = torch.empty(max(grass.factmask_linear_workspace_bytes(n4, T4, kf, kf), 1), dtype=torch.uint8, device=dev)
    tm, _, _ = _timed(lambda c: grass.factmask_linear(pairs[c % NPAIR][0], pairs[c % NPAIR][1], ii, io, out=ol, ws=wm),
                      40, NPAIR, torch, indexed=True)
    Si = grass.grass_to_bf16(grass.grass_projection_matrix(seed, 40, d4, kf, 1, device=dev))
    So = grass.grass_to_bf16(grass.grass_projection_matrix(seed, 41, d4, kf, 1, device=dev))
    ts, _, _ = _timed(lambda c: grass.logra_linear(pairs[c % NPAIR][0], pairs[c % NPAIR][1], Si, So, out=ol, ws=wl),
                      40, NPAIR, torch, indexed=True)
    extras["table2_style_4096_layer_ms"] = {"mask_kin_x_kout": round(tm / 40, 4), "sjlt_kin_x_kout": round(ts / 40, 4),
                                            "factgrass": round(fg_ms, 4), "logra_gauss_kin_x_kout": round(lg_ms, 4),
                                            "rotating_input_pairs": NPAIR}
    del pairs, x4, go4, o4, w4, Pi, Po, ol, wl, wm, Si, So
    torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extras", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="SJLT (s = 1) against the dense Gaussian projection at p = 131,072 over target dimensions and "
                         "input sparsity levels (the setting of the paper's SJLT benchmark figure); prints one JSON object")
    ap.add_argument("--full-score", action="store_true",
                    help="run only the attribute-stage GEMM over all 112 concatenated layer blocks (K = 458,752, bf16)")
    ap.add_argument("--single-layer-only", action="store_true",
                    help="run only the 4096 x 4096 linear-layer paths (FactGraSS, LoGra, factorised baselines) on rotating "
                         "inputs; for counter runs of these kernels alone")
    ap.add_argument("--accumulators", action="store_true",
                    help="ResNet-scale and MLP-scale SJLT with the two LDS accumulator policies (fp64 atomic add, fp32 "
                         "compare-and-swap) forced through the per-call tuning argument")
    ap.add_argument("--copy-reference", action="store_true",
                    help="run only a plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--probe", action="store_true",
                    help="run only the memory-system probe: pseudo-random 128-byte line reads over 16 GiB, alone and with "
                         "the write stream of the plain mask gather (what the chip sustains for the gather's pattern)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (samples are independent: more GPUs would compress "
              "disjoint row ranges with identical tables and exchange nothing); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2505_18976_amd as grass
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    grass.load_library()          # fails loudly if libgrass.so was not built

    if args.copy_reference:
        nbytes = 1 << 30
        a = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
        b = torch.empty_like(a)
        t, _, _ = _timed(lambda: b.copy_(a), 5, 2, torch)
        print(json.dumps({"copy_reference_bytes_read": nbytes, "copy_reference_bytes_written": nbytes,
                          "ms": round(t / 5, 4), "GBps_read_plus_write": round(2 * nbytes / (t / 5 * 1e-3) / 1e9, 1)}))
        return 0

    if args.probe:
        blocks, reads = 65536, 16
        src = torch.zeros((16 << 30) // 4, dtype=torch.float32, device=dev)
        dst = torch.empty(blocks * 256 * reads, dtype=torch.float32, device=dev)
        lines = blocks * 256 * reads
        out = {"probe": "random_line_reads", "footprint_GiB": 16, "lines_per_launch": lines}
        for mode, name in ((0, "reads_nontemporal"), (1, "reads_nontemporal_plus_gather_write_stream"), (2, "reads_plain")):
            t, _, _ = _timed(lambda c: grass.grass_probe_line_reads(src, dst, mode, 100 + c, blocks), 5, 2, torch, indexed=True)
            nbytes = lines * 128 + (lines * 4 if mode == 1 else 0)
            out[name] = {"ms": round(t / 5, 3), "G_lines_per_s": round(lines / (t / 5 * 1e-3) / 1e9, 2),
                         "line_plus_write_GBps": round(nbytes / (t / 5 * 1e-3) / 1e9, 1)}
        sblocks = (16 << 30) // (64 << 10)                      # one pass over the buffer
        t, _, _ = _timed(lambda: grass.grass_probe_line_reads(src, dst, 3, 0, sblocks), 5, 2, torch)
        out["sequential_stream_nontemporal"] = {"ms": round(t / 5, 3), "GBps": round((16 << 30) / (t / 5 * 1e-3) / 1e9, 1)}
        print(json.dumps(out))
        return 0

    if args.single_layer_only:
        extras = {}
        bench_single_layer(grass, synth, torch, dev, 0, extras)
        print(json.dumps({"workload": "single_linear_layer_4096", "extras": extras}))
        return 0

    if args.accumulators:
        out_rows = []
        n3, p3, k3 = 1024, 11173962, 8192
        g3 = synth.laplace_sparse(n3, p3, 0.3, 1e-3, seed=1003, device=dev)
        o3 = torch.empty((n3, k3), dtype=torch.float32, device=dev)
        for acc, name in ((3, "fp64 LDS atomic add"), (2, "fp32 compare-and-swap")):
            tun = dict(sjlt_accumulator=acc)
            w3 = torch.empty(max(grass.grass_sjlt_workspace_bytes(n3, p3, 0, k3, 1, tun), 1), dtype=torch.uint8, device=dev)
            t, _, _ = _timed(lambda: grass.grass_sjlt(g3, k3, 1, 0, 1, out=o3, ws=w3, tuning=tun), 10, 2, torch)
            out_rows.append({"workload": "resnet_sjlt_s1", "accumulator": name, "ms": round(t / 10, 4),
                             "launch": grass.grass_sjlt_describe(n3, p3, g3.stride(0), 0, k3, 1, g=g3, tuning=tun)})
            del w3
        del g3, o3
        torch.cuda.empty_cache()
        n, p, kp, k = 4096, synth.mlp_num_params(), 65536, 4096
        g = synth.mlp_relu_gradients(n, seed=1002, device=dev)
        idx = grass.grass_mask_indices(0, 0, p, kp, device=dev)
        out = torch.empty((n, k), dtype=torch.float32, device=dev)
        for acc, name in ((3, "fp64 LDS atomic add"), (2, "fp32 compare-and-swap")):
            tun = dict(sjlt_accumulator=acc)
            w = torch.empty(max(grass.grass_sjlt_workspace_bytes(n, p, kp, k, 1, tun), 1), dtype=torch.uint8, device=dev)
            t, _, _ = _timed(lambda: grass.grass_sjlt(g, k, 1, 0, 1, idx=idx, out=out, ws=w, tuning=tun), 10, 2, torch)
            out_rows.append({"workload": "mlp_mask_sjlt_s1", "accumulator": name, "ms": round(t / 10, 4),
                             "launch": grass.grass_sjlt_describe(n, p, g.stride(0), kp, k, 1, g=g, tuning=tun)})
        print(json.dumps({"accumulator_policy": out_rows}))
        return 0

    if args.full_score:
        # the attribute stage of the Llama-style configuration at its full width: 65,536 train rows and 1,024 test
        # rows of 112 x 4,096 = 458,752 compressed coordinates, kept in bf16 (60 GB; fp32 would be 120 GB)
        N5, M5, K5 = 65536, 1024, 112 * 4096
        trb = torch.empty((N5, K5), dtype=torch.bfloat16, device=dev)
        for r0 in range(0, N5, 4096):
            trb[r0:r0 + 4096] = synth.dense_normal(4096, K5, seed=1400 + r0, device=dev).to(torch.bfloat16)
        teb = synth.dense_normal(M5, K5, seed=1399, device=dev).to(torch.bfloat16)
        sc = torch.empty((M5, N5), dtype=torch.float32, device=dev)
        t, _, _ = _timed(lambda: grass.grass_score_bf16(trb, teb, out=sc), 1, 0, torch)
        tf = 2.0 * N5 * M5 * K5 / (t * 1e-3) / 1e12
        # spot check of four entries against fp64 inner products of the same bf16 values
        worst = 0.0
        for (mi, ni) in ((0, 0), (1023, 65535), (517, 40000), (3, 12345)):
            ref = float((teb[mi].double() * trb[ni].double()).sum().item())
            worst = max(worst, abs(float(sc[mi, ni].item()) - ref) / (abs(ref) + K5 ** 0.5))
        print(json.dumps({"workload": "score_gemm_full_width_bf16", "N": N5, "M": M5, "K": K5, "ms": round(t, 1),
                          "TFLOPs": round(tf, 1), "frac_of_mfma_peak": round(tf / MFMA_PEAK_BF16_TFLOPS, 4),
                          "spot_check_rel_err": worst}))
        return 0

    if args.sweep:
        ns, ps, seed = 1024, 131072, 0
        rows = []
        for zero_frac in (0.0, 0.5, 0.9, 0.99):
            gs = synth.bernoulli_sparse_normal(ns, ps, zero_frac, 1.0, seed=1300, device=dev)
            sub = gs[:256]
            d_exact = torch.cdist(sub.double(), sub.double())
            mask = ~torch.eye(256, dtype=torch.bool, device=dev)
            for ks in (64, 256, 1024, 4096, 16384):
                o = torch.empty((ns, ks), dtype=torch.float32, device=dev)
                w = torch.empty(max(grass.grass_sjlt_workspace_bytes(ns, ps, 0, ks, 1), 1), dtype=torch.uint8, device=dev)
                t, _, _ = _timed(lambda: grass.grass_sjlt(gs, ks, 1, seed, 1, out=o, ws=w), 20, 3, torch)
                d = torch.cdist(o[:256].double(), o[:256].double())
                err_s = float(((d[mask] / d_exact[mask]) - 1).abs().mean().item())
                wg = torch.empty(grass.grass_gauss_project_workspace_bytes(ns, ps, ks, 32768), dtype=torch.uint8, device=dev)
                tg, _, _ = _timed(lambda: grass.grass_gauss_project(gs, ks, seed, 2, 32768, compute_mode=0, out=o, ws=wg),
                                  3, 1, torch)
                d = torch.cdist(o[:256].double(), o[:256].double())
                err_g = float(((d[mask] / d_exact[mask]) - 1).abs().mean().item())
                rows.append({"zero_frac": zero_frac, "k": ks, "sjlt_ms": round(t / 20, 4), "gauss_fp32_ms": round(tg / 3, 3),
                             "sjlt_rel_dist_err": round(err_s, 4), "gauss_rel_dist_err": round(err_g, 4)})
                del o, w, wg
            del gs
            torch.cuda.empty_cache()
        print(json.dumps({"sweep": "sjlt_vs_gaussian", "n": ns, "p": ps, "s": 1,
                          "note": "Gaussian time includes generating P chunk by chunk; errors are the mean relative "
                                  "pairwise-distance error over the first 256 rows", "rows": rows}))
        return 0

    # ------------------------------------------------------------ headline
    n, p, kp, k, s, seed = 4096, synth.mlp_num_params(), 65536, 4096, 1, 0
    g = synth.mlp_relu_gradients(n, seed=1002, device=dev)
    idx = grass.grass_mask_indices(seed, 0, p, kp, device=dev)
    out = torch.empty((n, k), dtype=torch.float32, device=dev)
    ws_bytes = grass.grass_sjlt_workspace_bytes(n, p, kp, k, s)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev)

    def step():
        grass.grass_sjlt(g, k, s, seed, 1, idx=idx, out=out, ws=ws)

    total_ms, per, _ = _timed(step, args.steps, args.warmup, torch, per_call=True)
    ms_per_step = total_ms / args.steps
    kernel_ms = float(np.mean(per))       # one launch per step when the workspace query is 0
    samples_per_s = n / (ms_per_step * 1e-3)

    alg_bytes = n * (4 * kp + 4 * k) + 4 * kp          # useful reads + writes + the index vector once
    achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
    launched = grass.grass_sjlt_describe(n, p, g.stride(0), kp, k, s, g=g, with_workspace=True)
    roofline = {"bound": "hbm", "kernel": launched.split()[0], "launch": launched, "achieved": round(achieved, 2),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": None, "kernel_ms": round(kernel_ms, 4),
                "algorithmic_bytes_per_launch": alg_bytes, "launches_per_step": 1 if ws_bytes == 0 else 2}
    # what the launch really moves: a kept 4-byte entry costs its whole 128-byte line, and one coordinate in 28
    # touches 68 % of the lines of every row.  Counted here on the host from the actual indices, row distance and
    # base alignment (lines read once each + the output rows + idx), and taken from the counter run if that run was
    # made on this very kernel instantiation, grid and workload.
    idx_np = idx.cpu().numpy()
    lines = _touched_lines(idx_np, 4, g.stride(0) * 4, g.data_ptr() % 128, n)
    expected = lines * 128 + n * k * 4 + kp * 4
    roofline["expected_line_traffic"] = int(expected)
    roofline["expected_line_traffic_GBps"] = round(expected / (kernel_ms * 1e-3) / 1e9, 1)
    roofline["expected_line_traffic_frac_of_peak"] = round(expected / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    rec = _traffic_record(TRAFFIC_PROFILE)
    want = {"kernel": launched.split()[0], "grid": launched.split()[1].split("=")[1], "n": str(n), "p": str(p),
            "kprime": str(kp), "k": str(k), "s": str(s)}
    if rec and all(rec.get(key) == val for key, val in want.items()):
        traffic = int(rec["bytes_per_launch"])
        roofline["traffic"] = traffic
        roofline["traffic_source"] = "profiles/" + os.path.basename(TRAFFIC_PROFILE)
        roofline["traffic_GBps"] = round(traffic / (kernel_ms * 1e-3) / 1e9, 1)
        roofline["traffic_frac_of_peak"] = round(traffic / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    else:
        roofline["traffic_source"] = ("no counter record for this kernel instantiation, grid and workload under profiles/"
                                      if rec else "profiles/ summary not found")

    result = {
        "metric": "compressed per-sample gradients/sec at 1 GPU",
        "value": round(samples_per_s, 1), "unit": "samples/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "mlp_mask_sjlt_s1", "n": n, "p": p, "kprime": kp, "k": k, "s": s,
                   "zeros": "ReLU dead-neuron runs, ~50%", "fused": True},
        "roofline": roofline,
    }

    # --------------------------------------------------------- CPU baseline
    if not args.no_cpu_baseline:
        from oracle import grass_oracle as orc
        idx_h = idx.cpu().numpy()
        rows_done, t_used, batch = 0, 0.0, 32
        err = 0.0
        while t_used < 12.0 and rows_done < n:
            rows = slice(rows_done, min(n, rows_done + batch))
            gh = g[rows].cpu().numpy()
            t0 = time.perf_counter()
            ref = orc.grass(gh, idx_h, k, s, seed, 1)
            t_used += time.perf_counter() - t0
            err = max(err, orc.max_rel_err(out[rows].cpu().numpy(), ref))
            rows_done += gh.shape[0]
        result["cpu_baseline"] = {"value": round(rows_done / t_used, 2), "unit": "samples/s", "cores": 1,
                                  "kind": "oracle", "sample": f"first {rows_done} of {n} rows, NumPy float64, 1 thread",
                                  "host_cores_visible": os.cpu_count(), "gpu_vs_oracle_max_rel_err": err}

    # --------------------------------------------------------------- extras
    if not args.no_extras:
        extras = {}
        st = max(5, min(args.steps, 20))
        # s = 4 on the same batch
        ws4 = torch.empty(max(grass.grass_sjlt_workspace_bytes(n, p, kp, k, 4), 1), dtype=torch.uint8, device=dev)
        t, _, _ = _timed(lambda: grass.grass_sjlt(g, k, 4, seed, 1, idx=idx, out=out, ws=ws4), st, 2, torch)
        extras["mlp_mask_sjlt_s4"] = {"ms": round(t / st, 4), "samples_per_s": round(n / (t / st * 1e-3), 1)}
        # the same batch stored as bf16 (half the lines: 64 columns per 128-byte line)
        g16 = g.to(torch.bfloat16)
        t, _, _ = _timed(lambda: grass.grass_sjlt_bf16(g16, k, s, seed, 1, idx=idx, out=out, ws=ws), st, 2, torch)
        extras["mlp_mask_sjlt_s1_bf16_input"] = {"ms": round(t / st, 4), "samples_per_s": round(n / (t / st * 1e-3), 1)}
        del g16
        # plain gather
        gm = torch.empty((n, kp), dtype=torch.float32, device=dev)
        t, _, _ = _timed(lambda: grass.grass_mask(g, idx, out=gm), st, 2, torch)
        gather_bytes = lines * 128 + n * kp * 4 + kp * 4
        extras["mlp_mask_gather"] = {"ms": round(t / st, 4), "useful_GBps": round(2 * n * kp * 4 / (t / st * 1e-3) / 1e9, 1),
                                     "roofline": _roof("hbm", gather_bytes / (t / st * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s",
                                                       traffic_model_bytes=int(gather_bytes),
                                                       note="touched 128-byte lines (counted from the indices) + the "
                                                            "n x k' output")}
        # mask index generation (one-time set-up)
        t, _, _ = _timed(lambda: grass.grass_mask_indices(seed, 0, p, kp, device=dev), 5, 1, torch)
        extras["mask_indices_p1863690"] = {"ms": round(t / 5, 4)}
        del gm, out, ws, ws4
        torch.cuda.empty_cache()
        # one Selective Mask training step (objective + gradient) on the same batch of gradients, 256 test rows
        msm = 256
        gt_sm = synth.mlp_relu_gradients(msm, seed=1012, device=dev)
        s_sm = synth.dense_normal(1, p, seed=1013, device=dev).reshape(-1).contiguous()
        a_sm = grass.grass_score(g, gt_sm, compute_mode=0)
        w_sm = torch.empty(grass.grass_selective_mask_grad_workspace_bytes(n, msm, p), dtype=torch.uint8, device=dev)
        gr_sm = torch.empty(p, dtype=torch.float32, device=dev)
        ob_sm = torch.empty(1, dtype=torch.float64, device=dev)
        t, _, _ = _timed(lambda: grass.grass_selective_mask_grad(g, gt_sm, a_sm, s_sm, 1e-6, 1.0, grad=gr_sm, objective=ob_sm,
                                                                 ws=w_sm), 2, 1, torch)
        tf = 2 * 2.0 * n * msm * p / (t / 2 * 1e-3) / 1e12
        extras["selective_mask_grad_mlp"] = {"ms": round(t / 2, 2), "TFLOPs": round(tf, 1), "train_rows": n, "test_rows": msm}
        # the same step on the same gradients stored with the row distance rounded up to a multiple of 4 elements
        # (p = 1,863,690 is not one): 16-byte aligned rows take the direct-to-LDS GEMM in both contractions and the
        # backward one reads G in place instead of through transposed copies
        gpad = torch.empty((n, (p + 3) // 4 * 4), dtype=torch.float32, device=dev)
        gpad[:, :p].copy_(g)
        gtpad = torch.empty((msm, (p + 3) // 4 * 4), dtype=torch.float32, device=dev)
        gtpad[:, :p].copy_(gt_sm)
        t, _, _ = _timed(lambda: grass.grass_selective_mask_grad(gpad[:, :p], gtpad[:, :p], a_sm, s_sm, 1e-6, 1.0, grad=gr_sm,
                                                                 objective=ob_sm, ws=w_sm), 2, 1, torch)
        extras["selective_mask_grad_mlp_aligned_rows"] = {"ms": round(t / 2, 2),
                                                          "TFLOPs": round(2 * 2.0 * n * msm * p / (t / 2 * 1e-3) / 1e12, 1),
                                                          "row_distance": gpad.shape[1]}
        del gpad, gtpad
        t, _, _ = _timed(lambda: grass.grass_selective_mask_indices(s_sm, kp), 3, 1, torch)
        extras["selective_mask_indices_top_k"] = {"ms": round(t / 3, 3)}
        del g, gt_sm, s_sm, a_sm, w_sm, gr_sm, ob_sm
        torch.cuda.empty_cache()
        # Selective Mask training end to end on gradients with 2,048 planted informative coordinates among 65,536:
        # 60 device-side ascent steps with a decreasing temperature, exact-k extraction, and the first term of Eq. (1)
        # (correlation between exact and masked GradDot scores) of the trained mask against Random Masks of equal size
        nt, mt, pt, kt_ = 2048, 128, 65536, 2048
        Gp, Gtp, planted = synth.planted_gradients(nt, mt, pt, kt_, seed=3700, device=dev)
        Ap = grass.grass_score(Gp, Gtp, compute_mode=0)
        Sp = synth.dense_normal(1, pt, seed=3701, device=dev, std=0.1).reshape(-1).contiguous()
        wtr = torch.empty(grass.grass_selective_mask_train_workspace_bytes(nt, mt, pt), dtype=torch.uint8, device=dev)
        sched = np.geomspace(1.0, 0.6, 60)
        S_run = Sp.clone()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, objs = grass.grass_selective_mask_train(Gp, Gtp, Ap, S_run, 3e-4 / 16, 4800.0, sched, ws=wtr)
        torch.cuda.synchronize()
        train_ms = (time.perf_counter() - t0) * 1e3

        def _mask_corr(ix):
            Y = grass.grass_score(grass.grass_mask(Gp, ix), grass.grass_mask(Gtp, ix), compute_mode=0)
            return float(grass.grass_score_correlation(Ap, Y).item())
        sel = grass.grass_selective_mask_indices(S_run, kt_)
        hits = int(torch.isin(sel.long(), planted.to(dev)).sum().item())
        rand_corr = [_mask_corr(grass.grass_mask_indices(sd, 0, pt, kt_, device=dev)) for sd in range(3)]
        extras["selective_mask_training_planted"] = {
            "train_rows": nt, "test_rows": mt, "p": pt, "k": kt_, "steps": len(sched), "ms_per_step": round(train_ms / len(sched), 3),
            "TFLOPs": round(2 * 2.0 * nt * mt * pt * len(sched) / (train_ms * 1e-3) / 1e12, 1),
            "objective_first_last": [round(float(objs[0].item()), 4), round(float(objs[-1].item()), 4)],
            "planted_coordinates_recovered": hits, "correlation_selective_mask": round(_mask_corr(sel), 4),
            "correlation_random_masks": [round(c, 4) for c in rand_corr]}
        del Gp, Gtp, Ap, Sp, wtr, S_run
        torch.cuda.empty_cache()

        # ResNet-scale unmasked SJLT
        n3, p3, k3 = 1024, 11173962, 8192
        g3 = synth.laplace_sparse(n3, p3, 0.3, 1e-3, seed=1003, device=dev)
        o3 = torch.empty((n3, k3), dtype=torch.float32, device=dev)
        w3 = torch.empty(max(grass.grass_sjlt_workspace_bytes(n3, p3, 0, k3, 1), 1), dtype=torch.uint8, device=dev)
        t, _, _ = _timed(lambda: grass.grass_sjlt(g3, k3, 1, seed, 1, out=o3, ws=w3), 10, 2, torch)
        gbps = n3 * (4 * p3 + 4 * k3) / (t / 10 * 1e-3) / 1e9
        extras["resnet_sjlt_s1"] = {"ms": round(t / 10, 4), "samples_per_s": round(n3 / (t / 10 * 1e-3), 1),
                                    "algorithmic_GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBS, 4),
                                    "launch": grass.grass_sjlt_describe(n3, p3, g3.stride(0), 0, k3, 1, g=g3),
                                    "roofline": _roof("hbm", gbps, HBM_PEAK_GBS, "GB/s",
                                                      note="algorithmic bytes n (4p + 4k): every input byte must be read once")}
        # the dense Gaussian baseline on the same full input (P is 366 GB as a matrix: it is generated chunk by chunk
        # inside the call and never stored); one call per mode, 1.87e17 FLOP each
        wg3 = torch.empty(grass.grass_gauss_project_workspace_bytes(n3, p3, k3, 32768), dtype=torch.uint8, device=dev)
        for mode in (1, 0):
            t, _, _ = _timed(lambda: grass.grass_gauss_project(g3, k3, seed, 2, 32768, compute_mode=mode, out=o3, ws=wg3),
                             1, 0, torch)
            extras[f"resnet_gauss_project_full_p_mode{mode}"] = {
                "ms": round(t, 1), "samples_per_s": round(n3 / (t * 1e-3), 1),
                "TFLOPs_incl_generation": round(2.0 * n3 * p3 * k3 / (t * 1e-3) / 1e12, 1),
                "sjlt_speedup": round(t / extras["resnet_sjlt_s1"]["ms"], 1)}
        del wg3
        g3h = g3.to(torch.bfloat16)
        del g3
        t, _, _ = _timed(lambda: grass.grass_sjlt_bf16(g3h, k3, 1, seed, 1, out=o3, ws=w3), 10, 2, torch)
        gbps = n3 * (2 * p3 + 4 * k3) / (t / 10 * 1e-3) / 1e9
        extras["resnet_sjlt_s1_bf16_input"] = {"ms": round(t / 10, 4), "samples_per_s": round(n3 / (t / 10 * 1e-3), 1),
                                               "algorithmic_GBps": round(gbps, 1)}
        del g3h, o3, w3
        torch.cuda.empty_cache()

        bench_single_layer(grass, synth, torch, dev, seed, extras)

        # FactGraSS over a Llama-style 1.2B model: 16 blocks x 7 linears, n = 8 sequences x 1,024 tokens,
        # every layer with its own activations and gradients (12.3 GB in total, so nothing is served from
        # cache), per-layer masks and SJLT streams, outputs concatenated
        n5, T5, kl, kf = 8, 1024, 4096, 64
        layers = []
        for layer in range(16 * 7):
            name, d_in, d_out = synth.LLAMA_BLOCK_LINEARS[layer % 7]
            layers.append((synth.linear_layer_factors(n5, T5, d_in, d_out, seed=2000 + layer, device=dev),
                           grass.grass_mask_indices(seed, 16 + 4 * layer, d_in, kf, device=dev),
                           grass.grass_mask_indices(seed, 17 + 4 * layer, d_out, kf, device=dev), 18 + 4 * layer))
        cat = torch.empty((n5, kl * len(layers)), dtype=torch.float32, device=dev)
        w5 = torch.empty(max(grass.factgrass_linear_workspace_bytes(n5, T5, kf, kf, kl, 1), 1), dtype=torch.uint8,
                         device=dev)

        def llama_pass():
            for l, ((xl, gl), a_in, a_out, stream_id) in enumerate(layers):
                grass.factgrass_linear(xl, gl, a_in, a_out, kl, 1, seed, stream_id, out=cat[:, l * kl:(l + 1) * kl], ws=w5)

        t, _, wall = _timed(llama_pass, 5, 2, torch)
        extras["factgrass_llama_112_layers"] = {"ms": round(t / 5, 4), "tokens_per_s": round(n5 * T5 / (t / 5 * 1e-3), 1),
                                                "layer_calls_per_pass": len(layers)}
        batched = [(xl, gl, a_in, a_out, stream_id) for ((xl, gl), a_in, a_out, stream_id) in layers]
        wb = torch.empty(max(grass.factgrass_layers_workspace_bytes(len(layers), n5, T5, kf, kf, kl, 1), 1),
                         dtype=torch.uint8, device=dev)
        t, _, wall = _timed(lambda: grass.factgrass_layers(batched, kl, 1, seed, cat, ws=wb), 5, 2, torch)
        lines5 = 0
        for ((xl, gl), a_in, a_out, _sid) in layers:
            lines5 += (_touched_lines(a_in.cpu().numpy(), 2, xl.shape[2] * 2, 0, 1)
                       + _touched_lines(a_out.cpu().numpy(), 2, gl.shape[2] * 2, 0, 1))
        line_bytes5 = n5 * T5 * lines5 * 128 + n5 * kl * len(layers) * 4
        extras["factgrass_llama_112_layers_one_launch"] = {
            "ms": round(t / 5, 4), "tokens_per_s": round(n5 * T5 / (t / 5 * 1e-3), 1),
            "roofline": _roof("hbm", line_bytes5 / (t / 5 * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s",
                              traffic_model_bytes=int(line_bytes5),
                              note="touched 128-byte lines of the gathered columns of all 112 layers (12.3 GB of "
                                   "distinct inputs) + output")}
        del wb, batched
        del layers, cat, w5
        torch.cuda.empty_cache()

        # dense Gaussian projection baseline on a 131,072-column slice of the ResNet-scale problem
        ng, pg, kg = 1024, 131072, 8192
        gg = synth.laplace_sparse(ng, pg, 0.3, 1e-3, seed=1003, device=dev)
        og = torch.empty((ng, kg), dtype=torch.float32, device=dev)
        wg = torch.empty(grass.grass_gauss_project_workspace_bytes(ng, pg, kg, 32768), dtype=torch.uint8, device=dev)
        for mode, peak in ((0, MFMA_PEAK_F32_TFLOPS), (1, MFMA_PEAK_BF16_TFLOPS)):
            t, _, _ = _timed(lambda: grass.grass_gauss_project(gg, kg, seed, 2, 32768, compute_mode=mode, out=og, ws=wg),
                             3, 1, torch)
            tf = 2.0 * ng * pg * kg / (t / 3 * 1e-3) / 1e12
            extras[f"gauss_project_slice_mode{mode}"] = {"ms": round(t / 3, 3), "TFLOPs_incl_generation": round(tf, 2),
                                                          "samples_per_s_extrapolated_to_p_11173962":
                                                              round(ng / (t / 3 * 1e-3) * pg / 11173962, 1)}
        del gg, og, wg
        torch.cuda.empty_cache()

        # tiny config: n = 64, p = 65,536, k' = 8,192, k = 1,024 (launch-latency bound)
        g1 = synth.bernoulli_sparse_normal(64, 65536, 0.8, 1.0, seed=1001, device=dev)
        i1 = grass.grass_mask_indices(seed, 0, 65536, 8192, device=dev)
        o1 = torch.empty((64, 1024), dtype=torch.float32, device=dev)
        w1 = torch.empty(max(grass.grass_sjlt_workspace_bytes(64, 65536, 8192, 1024, 1), 1), dtype=torch.uint8, device=dev)
        t, _, _ = _timed(lambda: grass.grass_sjlt(g1, 1024, 1, seed, 1, idx=i1, out=o1, ws=w1), 50, 5, torch)
        extras["tiny_mask_sjlt"] = {"ms": round(t / 50, 4), "samples_per_s": round(64 / (t / 50 * 1e-3), 1)}
        # the same call over a rotating set of 40 input buffers (671 MB > the 256 MB last-level cache), so that the
        # 16.8 MB input does not stay cache-resident between launches
        ring = [synth.bernoulli_sparse_normal(64, 65536, 0.8, 1.0, seed=1100 + i, device=dev) for i in range(40)]
        turn = [0]

        def tiny_rotating():
            grass.grass_sjlt(ring[turn[0] % 40], 1024, 1, seed, 1, idx=i1, out=o1, ws=w1)
            turn[0] += 1
        t, _, _ = _timed(tiny_rotating, 80, 40, torch)
        extras["tiny_mask_sjlt_rotating_inputs"] = {"ms": round(t / 80, 4), "samples_per_s": round(64 / (t / 80 * 1e-3), 1),
                                                    "buffers": 40}
        # the 40 calls over the rotating buffers captured once into a HIP graph and replayed (the entry points only
        # enqueue kernels, so a caller with a launch-bound loop can do this)
        outs = torch.empty((40, 64, 1024), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(40):
                grass.grass_sjlt(ring[i], 1024, 1, seed, 1, idx=i1, out=outs[i], ws=w1)
        t, _, _ = _timed(graph.replay, 5, 2, torch)
        extras["tiny_mask_sjlt_graph_replay"] = {"ms_per_call": round(t / 5 / 40, 4),
                                                 "samples_per_s": round(64 * 40 / (t / 5 * 1e-3), 1), "calls_per_graph": 40}
        del ring, outs, graph

        # reference points measured in the same process: a plain 1 GiB device copy and a square bf16 GEMM from the
        # vendor library (context for the roofline fractions, not part of the library)
        ca = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        cb = torch.empty_like(ca)
        t, _, _ = _timed(lambda: cb.copy_(ca), 5, 2, torch)
        extras["reference_device_copy"] = {"GBps_read_plus_write": round(2 * (1 << 30) / (t / 5 * 1e-3) / 1e9, 1)}
        del ca, cb
        ma = synth.dense_normal(8192, 8192, seed=1200, device=dev).to(torch.bfloat16)
        mb = synth.dense_normal(8192, 8192, seed=1201, device=dev).to(torch.bfloat16)
        t, _, _ = _timed(lambda: torch.matmul(ma, mb.t()), 5, 2, torch)
        extras["reference_vendor_bf16_gemm_8192"] = {"TFLOPs": round(2.0 * 8192 ** 3 / (t / 5 * 1e-3) / 1e12, 1)}
        del ma, mb
        torch.cuda.empty_cache()

        # score GEMM, one layer block of compressed gradients
        N5, M5, K5 = 65536, 1024, 4096
        tr = synth.dense_normal(N5, K5, seed=1005, device=dev)
        te = synth.dense_normal(M5, K5, seed=1006, device=dev)
        sc = torch.empty((M5, N5), dtype=torch.float32, device=dev)
        for mode, peak in ((0, MFMA_PEAK_F32_TFLOPS), (1, MFMA_PEAK_BF16_TFLOPS)):
            wsc = torch.empty(max(grass.grass_score_workspace_bytes(N5, M5, K5, mode), 1), dtype=torch.uint8, device=dev)
            t, _, _ = _timed(lambda: grass.grass_score(tr, te, compute_mode=mode, out=sc, ws=wsc), 5, 1, torch)
            tf = 2.0 * N5 * M5 * K5 / (t / 5 * 1e-3) / 1e12
            extras[f"score_gemm_mode{mode}"] = {"ms": round(t / 5, 4), "TFLOPs": round(tf, 2),
                                                "frac_of_mfma_peak": round(tf / peak, 4),
                                                "roofline": _roof("mfma", tf, peak, "TFLOP/s", target_frac=0.5,
                                                                  target_met=bool(tf / peak >= 0.5))}
            del wsc
        t, _, _ = _timed(lambda: grass.grass_score(tr, te, compute_mode=1, out=sc, ws=None), 5, 1, torch)
        extras["score_gemm_mode1_no_workspace"] = {"ms": round(t / 5, 4),
                                                   "TFLOPs": round(2.0 * N5 * M5 * K5 / (t / 5 * 1e-3) / 1e12, 2)}
        # 16 layer blocks wide (K = 65,536): the fraction of the roofline does not depend on K once K is a few thousand
        tr16 = synth.dense_normal(N5, 16 * K5, seed=1007, device=dev)
        te16 = synth.dense_normal(M5, 16 * K5, seed=1008, device=dev)
        t, _, _ = _timed(lambda: grass.grass_score(tr16, te16, compute_mode=0, out=sc, ws=None), 2, 1, torch)
        tf = 2.0 * N5 * M5 * 16 * K5 / (t / 2 * 1e-3) / 1e12
        extras["score_gemm_mode0_K65536"] = {"ms": round(t / 2, 3), "TFLOPs": round(tf, 2),
                                             "frac_of_mfma_peak": round(tf / MFMA_PEAK_F32_TFLOPS, 4),
                                             "roofline": _roof("mfma", tf, MFMA_PEAK_F32_TFLOPS, "TFLOP/s", target_frac=0.5,
                                                               target_met=bool(tf / MFMA_PEAK_F32_TFLOPS >= 0.5))}
        tr16b, te16b = grass.grass_to_bf16(tr16), grass.grass_to_bf16(te16)
        del tr16, te16
        t, _, _ = _timed(lambda: grass.grass_score_bf16(tr16b, te16b, out=sc), 3, 1, torch)
        tf = 2.0 * N5 * M5 * 16 * K5 / (t / 3 * 1e-3) / 1e12
        extras["score_gemm_bf16_inputs_K65536"] = {"ms": round(t / 3, 3), "TFLOPs": round(tf, 2),
                                                   "frac_of_mfma_peak": round(tf / MFMA_PEAK_BF16_TFLOPS, 4),
                                                   "roofline": _roof("mfma", tf, MFMA_PEAK_BF16_TFLOPS, "TFLOP/s",
                                                                     target_frac=0.5,
                                                                     target_met=bool(tf / MFMA_PEAK_BF16_TFLOPS >= 0.5))}
        del tr16b, te16b
        trb, teb = grass.grass_to_bf16(tr), grass.grass_to_bf16(te)
        t, _, _ = _timed(lambda: grass.grass_score_bf16(trb, teb, out=sc), 10, 2, torch)
        tf = 2.0 * N5 * M5 * K5 / (t / 10 * 1e-3) / 1e12
        extras["score_gemm_bf16_inputs"] = {"ms": round(t / 10, 4), "TFLOPs": round(tf, 2),
                                            "frac_of_mfma_peak": round(tf / MFMA_PEAK_BF16_TFLOPS, 4),
                                            "roofline": _roof("mfma", tf, MFMA_PEAK_BF16_TFLOPS, "TFLOP/s", target_frac=0.5,
                                                              target_met=bool(tf / MFMA_PEAK_BF16_TFLOPS >= 0.5))}
        t, _, _ = _timed(lambda: grass.grass_to_bf16(tr, out=trb), 5, 1, torch)
        extras["to_bf16_train_rows"] = {"ms": round(t / 5, 4)}
        del trb, teb, te, sc

        # cache stage after compression on the same block: FIM, damped inverse, iFVP of all train rows
        Fm = torch.empty((K5, K5), dtype=torch.float32, device=dev)
        Wm = torch.empty((K5, K5), dtype=torch.float32, device=dev)
        wf = torch.empty(grass.grass_fim_workspace_bytes(N5, K5), dtype=torch.uint8, device=dev)
        wi = torch.empty(grass.grass_fim_inverse_workspace_bytes(K5), dtype=torch.uint8, device=dev)
        pre = torch.empty((N5, K5), dtype=torch.float32, device=dev)
        t, _, _ = _timed(lambda: grass.grass_fim(tr, out=Fm, ws=wf), 3, 1, torch)
        tf = 2.0 * N5 * K5 * K5 / (t / 3 * 1e-3) / 1e12
        tiles = K5 // 256
        tf_exec = tf * (tiles * (tiles + 1) / 2) / (tiles * tiles)
        extras["fim_65536x4096"] = {"ms": round(t / 3, 3), "TFLOPs_full_product": round(tf, 2),
                                    "note": "only tiles on or below the diagonal are computed",
                                    "roofline": _roof("mfma", tf_exec, MFMA_PEAK_F32_TFLOPS, "TFLOP/s",
                                                      note="flops of the executed lower 256 x 256 tiles")}
        t, _, _ = _timed(lambda: grass.grass_fim_inverse(Fm, 1e-3, out=Wm, ws=wi), 3, 1, torch)
        extras["fim_inverse_4096"] = {"ms": round(t / 3, 3), "fp64_GFLOPs_at_k3": round(K5 ** 3 / (t / 3 * 1e-3) / 1e9, 1),
                                      "roofline": _roof("mfma", K5 ** 3 / (t / 3 * 1e-3) / 1e12, 78.6, "TFLOP/s",
                                                        note="k^3 flops (k^3/3 factorisation + k^3/3 triangular inverse "
                                                             "+ k^3/3 product) against the fp64 matrix rate")}
        t, _, _ = _timed(lambda: grass.grass_ifvp(tr, Wm, out=pre), 3, 1, torch)
        tf = 2.0 * N5 * K5 * K5 / (t / 3 * 1e-3) / 1e12
        extras["ifvp_65536x4096"] = {"ms": round(t / 3, 3), "TFLOPs": round(tf, 2),
                                     "frac_of_mfma_peak": round(tf / MFMA_PEAK_F32_TFLOPS, 4),
                                     "roofline": _roof("mfma", tf, MFMA_PEAK_F32_TFLOPS, "TFLOP/s")}
        del Fm, Wm, wf, wi, pre, tr
        result["extras"] = extras

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
