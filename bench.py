#!/usr/bin/env python3
"""Benchmark of the transform codec hot path on one MI355X.

One step = fmtc_encode followed by fmtc_decode of one batch of synthetic
activations (the ResNet-18 stage-2 shape: N=32, C=128, 28x28, fp32, NHWC, b=6,
4096-symbol chunks; basis fitted offline on a separate 8-image calibration
batch).  Inputs are resident in HBM before the timed region; the step rotates
through enough buffer sets that the working set exceeds the 256 MB last-level
cache.  Prints ONE JSON line (see the fields below).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--bits 6] [--workload NAME]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense f16 matrix rate (the projections run as split-f16 contractions)

# HBM traffic per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script scaled by what the
# same counters read for the 64 MiB yardstick copy (profiles/*_pmc.txt has the numbers and the commands), keyed
# by (workload, bits, kernel).  None where no counter run exists.
MEASURED_TRAFFIC_BYTES = {
    ("resnet18_stage2_c128_28", 6, "k_project_quantize"): 17242931,
    ("resnet18_stage2_c128_28", 6, "k_pack"): 7290675,
    ("resnet18_stage2_c128_28", 6, "k_decode"): 15311667,
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--bits", type=int, default=6)
    ap.add_argument("--workload", default="resnet18_stage2_c128_28")
    ap.add_argument("--layout", default="nhwc", choices=["nhwc", "nchw"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hot", action="store_true", help="one buffer set only (cache-hot figure)")
    ap.add_argument("--keep", type=int, default=0, help="truncate the basis to this many components (0: all)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a one-GPU codec; run it with --gpus 1 "
                 "(no multi-GPU path exists: the codec shards over pixels, each GPU coding its own share)")

    import numpy as np
    import torch

    from paper_1905_10830_amd import binding as fmtc
    from paper_1905_10830_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: needs a GPU")
    torch.cuda.set_device(0)
    lib = fmtc.load_library()

    wl = synth.WORKLOADS[args.workload]
    bits = args.bits
    layout = fmtc.NHWC if args.layout == "nhwc" else fmtc.NCHW
    calib, data = synth.workload(args.workload, seed=0)
    xs = synth.to_layout(data, layout)
    N, C, H, W = wl["N"], wl["C"], wl["H"], wl["W"]
    P, V = N * H * W, N * H * W * C
    in_bytes = 4 * V

    # ---- offline: fit the basis on the calibration batch (GPU moments + host eigensolver) ----
    basis = fmtc.fit_basis(torch.from_numpy(synth.to_layout(calib, layout)).cuda(), layout)
    if args.keep:
        basis = basis.truncate(args.keep)

    # ---- buffer sets ----
    cap = fmtc.encode_bound(P, C, bits)
    ws_bytes = fmtc.workspace_size(P, C, bits)
    per_set = 2 * in_bytes + cap + ws_bytes
    R = 1 if args.hot else max(2, int(np.ceil(320e6 / per_set)))
    x0 = torch.from_numpy(xs).cuda()
    sets = []
    for r in range(R):
        sets.append(dict(
            x=x0.clone(), stream=torch.empty(cap, dtype=torch.uint8, device="cuda"),
            nbytes=torch.zeros(1, dtype=torch.int64, device="cuda"),
            ws=torch.empty(ws_bytes, dtype=torch.uint8, device="cuda"),
            xhat=torch.empty_like(x0), err=torch.zeros(1, dtype=torch.int32, device="cuda")))
    stream_h = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def enc_args(s):
        return (basis._h, s["x"].data_ptr(), N, C, H, W, layout, bits, 4096, s["stream"].data_ptr(), cap,
                s["nbytes"].data_ptr(), s["ws"].data_ptr(), ws_bytes, stream_h)

    def dec_args(s):
        return (basis._h, s["stream"].data_ptr(), cap, s["xhat"].data_ptr(), N, C, H, W, layout, bits,
                s["err"].data_ptr(), stream_h)

    ea = [enc_args(s) for s in sets]
    da = [dec_args(s) for s in sets]

    def step(i):
        r = i % R
        st = lib.fmtc_encode(*ea[r])
        st |= lib.fmtc_decode(*da[r])
        return st

    def run(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        bad = 0
        for i in range(n):
            bad |= fn(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if bad:
            raise RuntimeError("a library call failed: " + lib.fmtc_last_error().decode())
        return dt

    run(step, args.warmup)
    dt = run(step, args.steps)
    ms_per_step = 1e3 * dt / args.steps
    # encode and decode alone (same buffers; streams are valid from the runs above)
    dt_enc = run(lambda i: lib.fmtc_encode(*ea[i % R]), args.steps)
    dt_dec = run(lambda i: lib.fmtc_decode(*da[i % R]), args.steps)
    # the same step on one buffer set only (inputs and outputs stay in the last-level cache): labelled as such
    dt_hot = run(lambda i: lib.fmtc_encode(*ea[0]) | lib.fmtc_decode(*da[0]), args.steps) if R > 1 else dt
    for s in sets:
        assert int(s["err"].item()) == 0, "decoder flagged its own stream"

    # ---- the same steps as two independent chains on two HIP streams (default priority): step i runs encode then
    # decode of buffer set i on stream i % 2, so the kernels of neighbouring steps overlap.  Reported beside
    # `value`, which stays the one-stream figure. ----
    dt_two = None
    if R >= 2 and os.environ.get("FMTC_EXCLUSIVE_DEVICE", "0")[:1] != "1":  # (that setting promises one stream)
        side = [torch.cuda.Stream(), torch.cuda.Stream()]
        hs = [ctypes.c_void_p(st.cuda_stream) for st in side]
        ea2 = [[a[:-1] + (h,) for a in ea] for h in hs]
        da2 = [[a[:-1] + (h,) for a in da] for h in hs]
        Re = R - (R % 2)  # an even number of sets: a set always stays on the same stream

        def step2(i):
            r, q = i % Re, i % 2
            return lib.fmtc_encode(*ea2[q][r]) | lib.fmtc_decode(*da2[q][r])

        run(step2, args.warmup)
        dt_two = run(step2, args.steps)
        for s in sets:
            assert int(s["err"].item()) == 0, "decoder flagged its own stream"

    # ---- rate and distortion of the coded batch ----
    info = fmtc.stream_info(sets[0]["stream"][:64].cpu().numpy())
    R_payload = info["payload_bits"] / V
    R_container = 8.0 * info["stream_bytes"] / V
    mse = float(((sets[0]["xhat"] - sets[0]["x"]) ** 2).mean().item())

    # ---- per-kernel durations over one more pass of the same steps (HIP events on the launch stream) ----
    fmtc.profile_enable(args.steps)
    run(step, args.steps)
    prof = fmtc.profile_read()
    fmtc.profile_enable(0)

    flops = 2.0 * C * V  # one direction of the dense C x C projection, as the method defines it
    stream_bytes = float(info["stream_bytes"])
    # Per launch: algorithmic HBM bytes, and the matrix flops the kernel issues for the method's 2*C*V (the fp32
    # contraction runs as 3 (forward) or 2 (inverse) f16 products).  A kernel is held against the roof that takes
    # longer at peak: bytes / 8 TB/s or issued flops / 2.5 PFLOP/s.
    alg = {
        # projection: reads the activations once, writes one symbol byte per value
        "k_project_quantize": (4.0 * V + V, 3.0 * flops),
        # coder: reads the symbols once, writes the container
        "k_pack": (V + stream_bytes, 0.0),
        # decoder: reads the container, writes the activations
        "k_decode": (stream_bytes + 4.0 * V, 2.0 * flops),
    }
    kernels = {}
    for name, (avg_ms, min_ms, n) in prof.items():
        entry = {"avg_us": round(1e3 * avg_ms, 3), "min_us": round(1e3 * min_ms, 3), "launches": n}
        if name in alg:
            hbm_bytes, mfma_flops = alg[name]
            t = avg_ms * 1e-3
            t_hbm, t_mfma = hbm_bytes / (HBM_PEAK_GBS * 1e9), mfma_flops / (MFMA_F16_PEAK_TFLOPS * 1e12)
            if t_hbm >= t_mfma:
                bound, ach, peak, unit = "hbm", hbm_bytes / t / 1e9, HBM_PEAK_GBS, "GB/s"
            else:
                bound, ach, peak, unit = "mfma", mfma_flops / t / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s"
            entry.update(bound=bound, achieved=round(ach, 3), peak=peak, unit=unit, frac=round(ach / peak, 4),
                         hbm_bytes_algorithmic=int(hbm_bytes), hbm_GBps_algorithmic=round(hbm_bytes / t / 1e9, 1),
                         mfma_f16_flops_issued=mfma_flops, mfma_TFLOPps=round(mfma_flops / t / 1e12, 2))
        kernels[name] = entry
    dominant = max((k for k in kernels if k in alg), key=lambda k: kernels[k]["avg_us"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"], "peak": dk["peak"],
                "unit": dk["unit"], "frac": dk["frac"],
                "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, bits, dominant)),
                "avg_us": dk["avg_us"], "hbm_bytes_algorithmic": dk["hbm_bytes_algorithmic"]}

    # ---- the encoder with a code table fixed at calibration time (reported beside `value`, not part of it) ----
    table = fmtc.fit_table(basis, torch.from_numpy(synth.to_layout(calib, layout)).cuda(), bits, layout)
    scap = fmtc.encode_static_bound(table, P, C)
    sstreams = [torch.empty(scap, dtype=torch.uint8, device="cuda") for _ in sets]
    sa = [(basis._h, table._h, s["x"].data_ptr(), N, C, H, W, layout, 4096, st.data_ptr(), scap,
           s["nbytes"].data_ptr(), s["ws"].data_ptr(), ws_bytes, stream_h) for s, st in zip(sets, sstreams)]
    run(lambda i: lib.fmtc_encode_static(*sa[i % R]), args.warmup)
    dt_static = run(lambda i: lib.fmtc_encode_static(*sa[i % R]), args.steps)
    fmtc.profile_enable(args.steps)
    run(lambda i: lib.fmtc_encode_static(*sa[i % R]), args.steps)
    sprof = fmtc.profile_read()
    fmtc.profile_enable(0)
    sinfo = fmtc.stream_info(sstreams[0][:64].cpu().numpy())
    static = {"encode_GBps": round(in_bytes / (dt_static / args.steps) / 1e9, 3),
              "us_per_encode": round(1e6 * dt_static / args.steps, 2),
              "bits_per_value": round(sinfo["payload_bits"] / V, 4),
              "container_bits_per_value": round(8.0 * sinfo["stream_bytes"] / V, 4),
              "kernels": {k: round(1e3 * v[0], 3) for k, v in sprof.items()},
              "note": "projection, quantizer and packing as one kernel for 32/64/128 channels and at most 4 chunks per compute unit, else two kernels without histogram and table"}
    xh2, err2 = fmtc.decode(basis, sstreams[0], xs.shape, bits, layout)
    assert int(err2.item()) == 0 and torch.equal(xh2, sets[0]["xhat"]), "the two encoders disagree on the symbols"
    # ... and the decoder with ready-made tables, and the two together as a step
    sda = [(basis._h, table._h, st.data_ptr(), scap, s["xhat"].data_ptr(), N, C, H, W, layout, s["err"].data_ptr(),
            stream_h) for s, st in zip(sets, sstreams)]
    run(lambda i: lib.fmtc_encode_static(*sa[i % R]) | lib.fmtc_decode_static(*sda[i % R]), args.warmup)
    dt_sstep = run(lambda i: lib.fmtc_encode_static(*sa[i % R]) | lib.fmtc_decode_static(*sda[i % R]), args.steps)
    dt_sdec = run(lambda i: lib.fmtc_decode_static(*sda[i % R]), args.steps)
    fmtc.profile_enable(args.steps)
    run(lambda i: lib.fmtc_decode_static(*sda[i % R]), args.steps)
    sdprof = fmtc.profile_read()
    fmtc.profile_enable(0)
    for s in sets:
        assert int(s["err"].item()) == 0, "decoder flagged its own stream"
    assert torch.equal(sets[0]["xhat"], xh2), "the decoder with ready-made tables differs"
    static["decode_GBps"] = round(in_bytes / (dt_sdec / args.steps) / 1e9, 3)
    static["us_per_decode"] = round(1e6 * dt_sdec / args.steps, 2)
    static["decode_kernel_us"] = round(1e3 * sdprof["k_decode"][0], 3)
    static["encode_decode_GBps"] = round(in_bytes / (dt_sstep / args.steps) / 1e9, 3)
    static["us_per_step"] = round(1e6 * dt_sstep / args.steps, 2)

    # ---- the 8-bit path: unsigned 8-bit activations, 8-bit basis, integer matrix cores (reported beside `value`) ----
    sx = float(x0.max().item()) / 255.0
    xq0 = torch.clamp(torch.round(x0 / sx), 0, 255).to(torch.uint8)
    b8 = fmtc.Basis8(basis, sx)
    usets = [dict(xq=xq0.clone(), out=torch.empty_like(xq0), ws=torch.empty(V, dtype=torch.uint8, device="cuda"))
             for _ in sets]
    ua = [(b8._h, u["xq"].data_ptr(), N, C, H, W, layout, bits, 4096, s["stream"].data_ptr(), cap,
           s["nbytes"].data_ptr(), s["ws"].data_ptr(), ws_bytes, stream_h) for s, u in zip(sets, usets)]
    uda = [(b8._h, s["stream"].data_ptr(), cap, u["out"].data_ptr(), N, C, H, W, layout, bits, s["err"].data_ptr(),
            u["ws"].data_ptr(), V, stream_h) for s, u in zip(sets, usets)]
    run(lambda i: lib.fmtc_encode_u8(*ua[i % R]) | lib.fmtc_decode_u8(*uda[i % R]), args.warmup)
    dt_u8 = run(lambda i: lib.fmtc_encode_u8(*ua[i % R]) | lib.fmtc_decode_u8(*uda[i % R]), args.steps)
    fmtc.profile_enable(args.steps)
    run(lambda i: lib.fmtc_encode_u8(*ua[i % R]) | lib.fmtc_decode_u8(*uda[i % R]), args.steps)
    uprof = fmtc.profile_read()
    fmtc.profile_enable(0)
    for s in sets:
        assert int(s["err"].item()) == 0, "decoder flagged its own stream"
    uinfo = fmtc.stream_info(sets[0]["stream"][:64].cpu().numpy())
    u8 = {"us_per_step": round(1e6 * dt_u8 / args.steps, 2),
          "encode_decode_Gvalues_per_s": round(V / (dt_u8 / args.steps) / 1e9, 3),
          "bits_per_value": round(uinfo["payload_bits"] / V, 4),
          "mse": float((((usets[0]["out"].float() - usets[0]["xq"].float()) * sx) ** 2).mean().item()),
          "kernels": {k: round(1e3 * v[0], 3) for k, v in uprof.items()},
          "note": "1 byte per value in and out; projection (with histogram) and reconstruction (inside the chunk "
                  "decoder up to 128 channels) on the integer matrix cores, exact; table and packing by the fp32 "
                  "path's pack kernel"}

    # ---- yardstick for the memory counters: one plain copy of known size (not timed) ----
    ysrc = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    ydst = torch.empty_like(ysrc)
    fmtc.profile_copy(ydst, ysrc)
    torch.cuda.synchronize()

    # ---- the oracle on this machine's host cores, same tensors ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        T, mu, eig, A = basis.export()
        d = oracle.delta(A, bits)
        reps, t_cpu = 0, 0.0
        while t_cpu < 12.0 and reps < 200:
            t0 = time.perf_counter()
            enc = oracle.encode(xs, T, mu, d, bits, layout)
            oracle.decode(enc["stream"], xs.shape, T, mu, bits, layout)
            t_cpu += time.perf_counter() - t0
            reps += 1
        cpu = {"value": round(in_bytes / (t_cpu / reps) / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"the full batch ({N} images), encode+decode, mean of {reps} runs ({t_cpu:.1f} s), "
                         "single thread"}

    out = {
        "metric": "encode+decode throughput of fp32 activations (input GB/s)",
        "value": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 3),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "shape_NCHW": [N, C, H, W], "layout": args.layout, "bits": bits,
                   "chunk_syms": 4096, "keep": args.keep or C, "buffer_sets": R, "cache": "hot" if args.hot else "cold (rotating > 256 MB)"},
        "arithmetic": "fp32 in/out; projections as split-f16 matrix products with fp32 accumulation, fp64 where a "
                      "rounding decision is close",
        "cache_hot_value": round(in_bytes / (dt_hot / args.steps) / 1e9, 3),
        "two_stream_value": None if dt_two is None else round(in_bytes / (dt_two / args.steps) / 1e9, 3),
        "encode_GBps": round(in_bytes / (dt_enc / args.steps) / 1e9, 3),
        "decode_GBps": round(in_bytes / (dt_dec / args.steps) / 1e9, 3),
        "bits_per_value": round(R_payload, 4),
        "container_bits_per_value": round(R_container, 4),
        "mse": mse,
        "roofline": roofline,
        "kernels": kernels,
        "static_table_codec": static,
        "u8_codec": u8,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
