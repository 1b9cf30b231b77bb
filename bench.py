#!/usr/bin/env python3
"""Benchmark of the whole coding path on one MI355X.

One step = pcc_encode followed by pcc_decode of the 768x512 workload (all
pixels through gather, network, mixture CDF, row-rANS, stream assembly, then the
wavefront decoder), inputs and outputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline]
                  [--network workload|paper|diagonal|<ablation shape>] [--image WxH]

--network paper runs the paper's own network shape (12-pixel neighbourhood, 36-128x4-36, LeakyReLU, K=3,
delay 3) instead of the measured workloads' one, --network diagonal the same shape in the diagonal decoding
order (passes r + c, three inputs copied), --network fewer_layers | more_layers | fewer_filters | more_filters |
more_mixtures | most_mixtures one of the shapes of the paper's ablation study (Sec. IV-E); --image 512x512 gives
the image size of the paper's run-time table.  None of these is the headline: the driver's default run is
config 1 with the workload network.
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

# 2 * multiply-accumulates per pixel: 30-160-160-128-60 (58,560) and 36-128-128-128-128-36 (58,368)
FLOP_PER_PIXEL_BY_NET = {"workload": 117120, "paper": 116736, "diagonal": 116736}
NET_NAME = {"workload": "He-init 30-160-160-128-60 network, ReLU, K=5, 10-pixel neighbourhood",
            "paper": "He-init 36-128-128-128-128-36 network, LeakyReLU, K=3, 12-pixel neighbourhood",
            "diagonal": "He-init 36-128-128-128-128-36 network, LeakyReLU, K=3, 12-pixel neighbourhood with the three "
                        "undecoded inputs copied, diagonal order"}
# the shapes of the paper's ablation study (Sec. IV-E): name -> (K, C, L), as paper_2212_01185_amd.synth lists them
ABLATION_SHAPES = {"fewer_layers": (3, 128, 4), "fewer_filters": (3, 64, 5), "more_mixtures": (5, 128, 5),
                   "most_mixtures": (7, 128, 5), "more_layers": (3, 128, 6), "more_filters": (3, 192, 5)}
for _name, (_k, _c, _l) in ABLATION_SHAPES.items():
    _dims = (36,) + (_c,) * (_l - 1) + (12 * _k,)
    FLOP_PER_PIXEL_BY_NET[_name] = 2 * sum(a * b for a, b in zip(_dims[:-1], _dims[1:]))
    NET_NAME[_name] = "He-init %s network, LeakyReLU, K=%d, 12-pixel neighbourhood" % ("-".join(str(d) for d in _dims), _k)
# paper, Table II: 512x512, diagonal order: encode 3.08 s, decode 27.22 s
PAPER_512_DIAGONAL_STEP_SECONDS = 3.08 + 27.22
# paper, Table II: 512x512, wavefront, RTX 2080 + i7-9700: encode 3.10 s, decode 26.26 s
PAPER_512_STEP_SECONDS = 3.10 + 26.26
PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch of the encode kernel at 768x512 from rocprofv3 FETCH_SIZE / WRITE_SIZE,
# scaled by what the same counters read for a plain 64 MiB copy (summary under profiles/).  The kernel of
# this workload hands its symbols to a row coder running beside it as 8-byte tagged words: 3 B/pixel in,
# 24 B/pixel out (12 B/pixel out when the row coder runs after it: 2.88e6 fetched, 4.72e6 written).
ENCODE_KERNEL_TRAFFIC_768x512 = {"fetch_bytes": 2.87e6, "write_bytes": 9.44e6, "algorithmic_bytes": 27 * 393216}


def cpu_baseline(blob, imgs, rows):
    """The oracle as it stands, single thread, on the first `rows` rows of image 0: encode + raster decode."""
    import numpy as np
    from oracle import pcc_oracle as po
    orc = po.Oracle(blob)
    strip = np.ascontiguousarray(imgs[:1, :rows])
    n, h, w, _ = strip.shape
    t0 = time.perf_counter()
    stream, _ = orc.encode(strip, po.MODE_EXACT, want_bits=False)
    t1 = time.perf_counter()
    out = orc.decode(stream, n, h, w, po.MODE_EXACT, po.ORDER_RASTER)
    t2 = time.perf_counter()
    assert np.array_equal(out, strip)
    px = h * w
    return {
        "value": px / (t2 - t0) / 1e6, "unit": "MPix/s", "cores": 1, "kind": "oracle",
        "sample": "first %d rows (%d pixels) of the same %dx%d image, encode + raster decode, fp64" % (rows, px, w, imgs.shape[1]),
        "encode_MPix_s": px / (t1 - t0) / 1e6, "decode_MPix_s": px / (t2 - t1) / 1e6,
        "seconds": t2 - t0,
    }


def cpu_baseline_batch(blob, imgs, rows, threads):
    """The same oracle on a batch, one image per thread (the oracle's library keeps no state outside its model object,
    and ctypes releases the interpreter lock during a call): encode + raster decode of the first `rows` rows of each image."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import pcc_oracle as po
    n = imgs.shape[0]
    threads = max(1, min(threads, n))
    strips = [np.ascontiguousarray(imgs[i:i + 1, :rows]) for i in range(n)]

    def one(strip):
        orc = po.Oracle(blob)
        _, h, w, _ = strip.shape
        stream, _ = orc.encode(strip, po.MODE_EXACT, want_bits=False)
        return np.array_equal(orc.decode(stream, 1, h, w, po.MODE_EXACT, po.ORDER_RASTER), strip)

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        ok = list(pool.map(one, strips))
    dt = time.perf_counter() - t0
    assert all(ok)
    px = n * strips[0].shape[1] * strips[0].shape[2]
    return {"value": px / dt / 1e6, "unit": "MPix/s", "cores": threads, "kind": "oracle",
            "sample": "first %d rows of each of the %d images of the 24 x 768x512 workload (%d pixels), one image per thread, "
                      "encode + raster decode, fp64" % (rows, n, px),
            "seconds": dt}


def host_description():
    """CPU model and logical core count of the machine the oracle baseline runs on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"cpu_model": model, "nproc": os.cpu_count()}


PHASE_NAMES = ("gather", "layer 1", "layer 2", "layer 3", "layer 4", "layer 5", "layer 6", "layer 7", "mixtures",
               "search R", "search G", "search B", "publish", "fetch at step end", "end barrier", "loop top")


def phase_profile(codec, d_img, d_stream, d_out, n, h, w):
    """Cycles per decode step and phase, per wave of the workgroup that decoded ticket 8 (or the last one), from the
    build with -DPCC_PHASE_TIMING.  Each of the 13 marks of a step costs that build about 56 cycles (what an empty
    phase reads) and keeps the compiler from moving instructions across it: the sum is above the product's step."""
    import ctypes
    import torch
    from paper_2212_01185_amd import binding
    lib = binding.load()
    if not hasattr(lib, "pcc_debug_phase_cycles"):
        sys.exit("bench.py --phase-profile: %s was not built with -DPCC_PHASE_TIMING" % binding.LIB_PATH)
    codec.pcc_set_profiling(True)
    s = codec.pcc_encode(d_img, out=d_stream)
    for _ in range(4):
        codec.pcc_decode(s, n, h, w, out=d_out)
    torch.cuda.synchronize()
    assert torch.equal(d_out, d_img)
    ms = codec.pcc_last_timings()["decode"]
    arr = (ctypes.c_ulonglong * (4 * 17))()
    lib.pcc_debug_phase_cycles.argtypes = [ctypes.c_void_p]
    assert lib.pcc_debug_phase_cycles(arr) == 0
    steps = float(arr[16])
    print("decode %.3f ms, %.3f us per wavefront step (%d); the profiled band ran %d steps" %
          (ms, ms * 1e3 / binding.pcc_wavefront_steps(h, w, codec.delay), binding.pcc_wavefront_steps(h, w, codec.delay), steps))
    print("| phase | wave 0 | wave 1 | wave 2 | wave 3 |\n|---|---|---|---|---|")
    tot = [0.0] * 4
    for k, name in enumerate(PHASE_NAMES):
        row = [arr[wv * 17 + k] / steps for wv in range(4)]
        if any(row):
            print("| %s | %s |" % (name, " | ".join("%.0f" % v for v in row)))
            tot = [a + b for a, b in zip(tot, row)]
    print("| sum | %s |" % " | ".join("%.0f" % v for v in tot))


def measure_workload(codec, imgs, steps, warmup, flop_per_pixel):
    """Encode + decode `steps` times (after `warmup` untimed ones), inputs and outputs resident in HBM: the figures
    of one workload for the all_configs table.  The round trip is checked."""
    import torch
    from paper_2212_01185_amd import binding
    n, h, w, _ = imgs.shape
    pixels = n * h * w
    d_img = torch.from_numpy(imgs).cuda()
    d_stream = torch.empty(binding.pcc_stream_bound(n, h, w), dtype=torch.uint8, device="cuda")
    d_out = torch.empty_like(d_img)
    for _ in range(warmup):
        s = codec.pcc_encode(d_img, out=d_stream)
        codec.pcc_decode(s, n, h, w, out=d_out)
    torch.cuda.synchronize()
    t_enc = t_dec = pix_ms = dec_ms = 0.0
    for _ in range(steps):
        a = time.perf_counter()
        s = codec.pcc_encode(d_img, out=d_stream)
        b = time.perf_counter()
        pix_ms += codec.pcc_last_timings()["encode_pixels"]
        b2 = time.perf_counter()
        codec.pcc_decode(s, n, h, w, out=d_out)
        c = time.perf_counter()
        dec_ms += codec.pcc_last_timings()["decode"]
        t_enc += b - a
        t_dec += c - b2
    torch.cuda.synchronize()
    assert torch.equal(d_out, d_img), "round trip is not lossless"
    steps_wave = binding.pcc_wavefront_steps(h, w, codec.delay)
    return {
        "workload": "%d x %dx%d" % (n, w, h), "pixels": pixels, "steps": steps,
        "encode_MPix_s": pixels / (t_enc / steps) / 1e6, "decode_MPix_s": pixels / (t_dec / steps) / 1e6,
        "roundtrip_MPix_s": pixels / ((t_enc + t_dec) / steps) / 1e6,
        "decode_us_per_step": dec_ms / steps * 1e3 / steps_wave, "wavefront_steps": steps_wave,
        "encode_frac": flop_per_pixel * pixels / (pix_ms / steps * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "bpsp": 8.0 * int(s.numel()) / (3 * pixels),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, help="workload id 0..4 (1 = 768x512, the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the three-step runs of workloads 0, 2, 3, 4 that follow the timed headline")
    ap.add_argument("--cpu-rows", type=int, default=256, help="rows of image 0 the oracle baseline codes (about 13 s)")
    ap.add_argument("--network", choices=("workload", "paper", "diagonal") + tuple(ABLATION_SHAPES), default="workload")
    ap.add_argument("--image", default=None, help="WxH of one synthetic image instead of a numbered config")
    ap.add_argument("--phase-profile", action="store_true",
                    help="needs PCC_LIBRARY to name a build made with -DPCC_PHASE_TIMING: decode the workload and print "
                         "the cycles per decode step and phase that the waves of one workgroup counted, no JSON")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs: three encodes + decodes and one plain "
                         "64 MiB device copy of known traffic, no timing, no JSON")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2212_01185_amd import binding, synth

    FLOP_PER_PIXEL = FLOP_PER_PIXEL_BY_NET[args.network]
    if args.network in ABLATION_SHAPES:
        blob = synth.make_ablation_blob(*ABLATION_SHAPES[args.network])
    else:
        blob = {"workload": synth.make_blob, "paper": synth.make_paper_blob, "diagonal": synth.make_diagonal_blob}[args.network](0)
    if args.image:
        iw, ih = (int(v) for v in args.image.lower().split("x"))
        imgs = synth.make_image(0, synth.ImageSpec(iw, ih, 32, 8.0, 64.0))[None]
        wl_name = "1 x %dx%d" % (iw, ih)
    else:
        imgs = synth.make_batch(args.config)
        wl_name = "config %d: %d x %dx%d" % (args.config, imgs.shape[0], imgs.shape[2], imgs.shape[1])
    n, h, w, _ = imgs.shape
    pixels = n * h * w
    codec = binding.Codec(blob, 0)
    d_img = torch.from_numpy(imgs).cuda()
    d_stream = torch.empty(binding.pcc_stream_bound(n, h, w), dtype=torch.uint8, device="cuda")
    d_out = torch.empty_like(d_img)
    if args.phase_profile:
        phase_profile(codec, d_img, d_stream, d_out, n, h, w)
        return
    if args.traffic_probe:
        src = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            s = codec.pcc_encode(d_img, out=d_stream)
            codec.pcc_decode(s, n, h, w, out=d_out)
            dst.copy_(src)          # calibration: reads 64 MiB, writes 64 MiB
            torch.cuda.synchronize()    # every step starts on an idle stream, as in the timed loop
        torch.cuda.synchronize()
        return
    codec.pcc_set_profiling(True)

    for _ in range(args.warmup):
        s = codec.pcc_encode(d_img, out=d_stream)
        codec.pcc_decode(s, n, h, w, out=d_out)
    torch.cuda.synchronize()
    assert torch.equal(d_out, d_img), "round trip is not lossless"

    acc = {k: 0.0 for k in binding.TIMING_NAMES}
    t_enc = t_dec = 0.0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        a = time.perf_counter()
        s = codec.pcc_encode(d_img, out=d_stream)        # synchronises the stream before returning
        b = time.perf_counter()
        tm = codec.pcc_last_timings()
        for k in ("encode_pixels", "encode_rans", "encode_scan", "encode_compact"):
            acc[k] += tm[k]
        b2 = time.perf_counter()
        codec.pcc_decode(s, n, h, w, out=d_out)          # synchronises too
        c = time.perf_counter()
        acc["decode"] += codec.pcc_last_timings()["decode"]
        t_enc += b - a
        t_dec += c - b2
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert torch.equal(d_out, d_img), "round trip is not lossless"

    # the third entry point of the boundary, outside the step: raw head outputs and bits of every pixel
    # (3 B read, 4 * (head outputs + 1) B written per pixel; an HBM-side figure)
    d_params = torch.empty((n, h, w, codec.head_outputs), dtype=torch.float32, device="cuda")
    d_bits = torch.empty((n, h, w), dtype=torch.float32, device="cuda")
    lib = binding.load()
    st = torch.cuda.current_stream().cuda_stream
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    probs_reps = max(1, min(10, args.steps))
    for i in range(probs_reps + 1):
        if i == 1:
            ev0.record()
        rc = lib.pcc_encode_probs(codec._h, d_img.data_ptr(), n, h, w, d_params.data_ptr(), d_bits.data_ptr(), st)
        assert rc == 0, rc
    ev1.record()
    torch.cuda.synchronize()
    probs_ms = ev0.elapsed_time(ev1) / probs_reps
    probs_bytes = pixels * (3 + 4 * (codec.head_outputs + 1))

    # The pixel kernel of a small job leaves compute units to the row coder that runs beside it.  For reference:
    # the same kernel with the whole chip, the row coder after it (a second context, not part of the step).
    os.environ["PCC_ENCODE_OVERLAP"] = "0"
    plain = binding.Codec(blob, 0)
    del os.environ["PCC_ENCODE_OVERLAP"]
    plain.pcc_set_profiling(True)
    plain_reps, plain_pix_ms = max(1, min(10, args.steps)), 0.0
    for i in range(plain_reps + 2):
        plain.pcc_encode(d_img, out=d_stream)
        if i >= 2:
            plain_pix_ms += plain.pcc_last_timings()["encode_pixels"] / plain_reps
    plain.close()

    k = args.steps
    ms_per_step = (t1 - t0) / k * 1e3
    kern = {name: acc[name] / k for name in acc}       # ms per launch
    stream_bytes = int(s.numel())
    steps_wave = binding.pcc_wavefront_steps(h, w, codec.delay)
    headline = args.network == "workload" and not args.image and args.config == 1
    paper_case = args.network in ("paper", "diagonal") and (n, h, w) == (1, 512, 512)
    paper_seconds = PAPER_512_STEP_SECONDS if args.network == "paper" else PAPER_512_DIAGONAL_STEP_SECONDS

    enc_tflops = FLOP_PER_PIXEL * pixels / (kern["encode_pixels"] * 1e-3) / 1e12
    result = {
        "metric": "decode MPix/s (wavefront) + encode MPix/s at 768x512 RGB; MFMA util % of peak",
        "value": pixels / (ms_per_step * 1e-3) / 1e6,
        "unit": "MPix/s (one step = encode + wavefront decode of every pixel)",
        "n_gpus": 1, "steps": k, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak",
        # only the paper's own case (its network shape, its 512x512 image size; its machine was an RTX 2080)
        "vs_baseline": (pixels / (ms_per_step * 1e-3)) / (512 * 512 / paper_seconds) if paper_case else None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s RGB uint8, seeded blobs+gradient+noise, %s" % (wl_name, NET_NAME[args.network]),
                   "pixels": pixels, "wavefront_steps": steps_wave, "stream_bytes": stream_bytes,
                   "bpsp": 8.0 * stream_bytes / (3 * pixels)},
        "encode_MPix_s": pixels / (t_enc / k) / 1e6,
        "decode_MPix_s": pixels / (t_dec / k) / 1e6,
        "encode_ms": t_enc / k * 1e3, "decode_ms": t_dec / k * 1e3,
        "kernel_ms": kern,
        "decode_us_per_wavefront_step": kern["decode"] * 1e3 / steps_wave,
        "roofline": {
            "kernel": "encode_kernel (gather + network on MFMA + mixture CDF, all pixels)",
            "bound": "mfma", "achieved": enc_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": enc_tflops / PEAK_BF16_TFLOPS,
            # HBM bytes per launch (fetched + written, rocprofv3 counters scaled by a plain copy's reading)
            "traffic": (ENCODE_KERNEL_TRAFFIC_768x512["fetch_bytes"] + ENCODE_KERNEL_TRAFFIC_768x512["write_bytes"])
                       if headline else None,
            "traffic_detail": ENCODE_KERNEL_TRAFFIC_768x512 if headline else None,
            # the same kernel when the row coder runs after it and it has every compute unit
            "whole_chip": {"kernel_ms": plain_pix_ms,
                           "frac": FLOP_PER_PIXEL * pixels / (plain_pix_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        },
        "roofline_decode": {
            "kernel": "decode_kernel (persistent wavefront)", "bound": "dependency chain",
            "achieved_TFLOP_s": FLOP_PER_PIXEL * pixels / (kern["decode"] * 1e-3) / 1e12,
            "frac_of_mfma_peak": FLOP_PER_PIXEL * pixels / (kern["decode"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        },
        "encode_probs": {"ms": probs_ms, "MPix_s": pixels / (probs_ms * 1e-3) / 1e6, "bytes": probs_bytes,
                         "GB_s": probs_bytes / (probs_ms * 1e-3) / 1e9,
                         "frac_of_hbm_peak": probs_bytes / (probs_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "paper_context": "paper, 512x512 on RTX 2080 + i7-9700: wavefront encode 3.10 s, decode 26.26 s (0.0846 / 0.00998 MPix/s); "
                         "diagonal 3.08 s / 27.22 s",
    }
    if headline and not args.no_all_configs:
        # the other four workloads, three steps each, outside the timed region of the headline
        table = {"1": {"workload": "1 x 768x512", "pixels": pixels, "steps": k,
                       "encode_MPix_s": result["encode_MPix_s"], "decode_MPix_s": result["decode_MPix_s"],
                       "roundtrip_MPix_s": result["value"], "decode_us_per_step": result["decode_us_per_wavefront_step"],
                       "wavefront_steps": steps_wave, "encode_frac": result["roofline"]["frac"],
                       "bpsp": result["config"]["bpsp"]}}
        del d_params, d_bits, d_img, d_out, d_stream
        for cfg in (0, 2, 3, 4):
            table[str(cfg)] = measure_workload(codec, synth.make_batch(cfg), 3, 1, FLOP_PER_PIXEL)
            torch.cuda.empty_cache()
        result["all_configs"] = dict(sorted(table.items()))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(blob, imgs, min(args.cpu_rows, h))
        result["cpu_baseline"]["host"] = host_description()
        if headline and not args.no_all_configs:
            # the batch workload with the host's cores: one image per thread (16 threads is the GPU machine's CPU share)
            result["cpu_baseline"]["batch"] = cpu_baseline_batch(blob, synth.make_batch(2), 16,
                                                                 min(16, os.cpu_count() or 1))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
