#!/usr/bin/env python3
"""Benchmark of the transform codec hot path on one MI355X.

One step = fmtc_encode followed by fmtc_decode of one batch of synthetic activations.  The headline workload is the
largest single-GPU configuration of the benchmark definition: the first ResNet-18 post-block map at N = 256
(resnet18_n256_c64_56: C = 64, 56 x 56, fp32, NHWC, 205 MB), b = 6, 4096-symbol chunks, basis fitted offline on a
separate 8-image calibration batch.  Inputs are resident in HBM before the timed region; the step rotates through
enough buffer sets that the working set exceeds the 256 MB last-level cache.  Prints ONE JSON line; the other seven
shapes of the benchmark definition are timed after it, with fewer steps, and reported as `other_shapes`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--bits 6] [--workload NAME] [--main-only]

A second mode turns rocprofv3 output of this script into the text summary kept under profiles/ (from which
`roofline.traffic` is read back):

    python bench.py --summarize STATS_DIR FETCH_DIR WRITE_DIR [--workload NAME] [--bits B]
"""
import argparse
import csv
import ctypes
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense f16 matrix rate (the projections run as split-f16 contractions)
YARDSTICK_BYTES = 64 << 20   # the plain copy the memory counters are scaled with

# (workload, bits) of the benchmark definition's configurations; the first is the headline
SHAPES = [("resnet18_n256_c64_56", 6), ("resnet18_n256_c128_28", 6), ("resnet18_n256_c256_14", 4),
          ("resnet18_n256_c512_7", 4), ("mbv2_c144_56", 5), ("mbv2_c960_7", 5), ("resnet18_stage2_c128_28", 6),
          ("resnet18_stage3_c256_14", 4), ("resnet18_stage4_c512_7", 4), ("cfg0_c64_56", 8)]

# rocprofv3 kernel names -> the names fmtc_profile_* reports
KERNEL_FAMILIES = [("k_project_quantize", "k_project_quantize"), ("k_huffman_table", "k_huffman_table"),
                   ("k_chunk_bits", "k_chunk_bits"), ("k_pack", "k_pack"), ("k_decode", "k_decode"),
                   ("k_quantize_u8", "k_quantize_u8"), ("k_int8_tiles", "k_quantize_u8"), ("k_copy", "k_copy")]


def family(kernel_name):
    for needle, fam in KERNEL_FAMILIES:
        if needle in kernel_name:
            return fam
    return None


def profile_path(workload, bits):
    return os.path.join(ROOT, "profiles", f"{workload}_b{bits}_profile.txt")


def read_traffic(workload, bits):
    """HBM bytes per launch, per kernel family, from the committed rocprofv3 summary of this workload (None if absent)."""
    out = {}
    try:
        for line in open(profile_path(workload, bits)):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes":
                out[f[1]] = int(f[2])
    except OSError:
        pass
    return out


def summarize(args):
    """rocprofv3 csv output (kernel stats; FETCH_SIZE run; WRITE_SIZE run) -> profiles/<workload>_b<bits>_profile.txt"""
    stats_dir, fetch_dir, write_dir = args.summarize

    def one(d, suffix):
        hits = glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True)
        if not hits:
            sys.exit(f"no *{suffix} under {d}")
        return hits[0]

    rows = []
    for r in csv.DictReader(open(one(stats_dir, "kernel_stats.csv"))):
        if "fmtc::" in r["Name"]:
            rows.append((r["Name"], int(r["Calls"]), float(r["AverageNs"]), int(r["MinNs"]), int(r["MaxNs"])))

    def counter(d):
        acc = {}
        for r in csv.DictReader(open(one(d, "counter_collection.csv"))):
            if "fmtc::" in r["Kernel_Name"]:
                a = acc.setdefault(r["Kernel_Name"], [0, 0.0])
                a[0] += 1
                a[1] += float(r["Counter_Value"])
        return {k: (n, s / n) for k, (n, s) in acc.items()}

    fetch, write = counter(fetch_dir), counter(write_dir)
    ycopy = [k for k in fetch if "k_copy" in k]
    if not ycopy or ycopy[0] not in write:
        sys.exit("the yardstick copy (fmtc::k_copy) is missing from the counter runs")
    f_scale = (YARDSTICK_BYTES / 1024.0) / fetch[ycopy[0]][1]
    w_scale = (YARDSTICK_BYTES / 1024.0) / write[ycopy[0]][1]
    cmd = f"python3 bench.py --workload {args.workload} --bits {args.bits} --main-only"
    out = [f"rocprofv3 summary: bench.py --main-only on workload {args.workload}, b = {args.bits}, fp32 NHWC, "
           "4096-symbol chunks, one MI355X.",
           "Commands (from the repository root, on the GPU box; the summary is written by",
           f"  python3 bench.py --summarize STATS FETCH WRITE --workload {args.workload} --bits {args.bits}):",
           f"  rocprofv3 --kernel-trace --stats -d STATS -o run --output-format csv -- {cmd} --steps 100 --warmup 10",
           f"  rocprofv3 --kernel-trace --pmc FETCH_SIZE -d FETCH -o run --output-format csv -- {cmd} --steps 10 --warmup 2",
           f"  rocprofv3 --kernel-trace --pmc WRITE_SIZE -d WRITE -o run --output-format csv -- {cmd} --steps 10 --warmup 2",
           "", "kernel statistics (kernel_stats.csv, library kernels):",
           f"{'kernel':78s} {'calls':>6s} {'avg_ns':>9s} {'min_ns':>8s} {'max_ns':>8s}"]
    for name, calls, avg, mn, mx in rows:
        out.append(f"{name[:78]:78s} {calls:6d} {avg:9.0f} {mn:8d} {mx:8d}")
    out += ["", f"memory counters (KiB per dispatch, mean over the dispatches; yardstick: the {YARDSTICK_BYTES >> 20} MiB copy "
            f"fmtc::k_copy reads FETCH_SIZE {fetch[ycopy[0]][1]:.1f}, WRITE_SIZE {write[ycopy[0]][1]:.1f} "
            f"-> scale factors {f_scale:.4f}, {w_scale:.4f}):",
            f"{'kernel':78s} {'n':>4s} {'FETCH KiB':>11s} {'WRITE KiB':>11s} {'HBM bytes':>12s}"]
    fam_bytes = {}
    for k in sorted(fetch):
        if k not in write:
            continue
        b = int(1024.0 * (fetch[k][1] * f_scale + write[k][1] * w_scale))
        out.append(f"{k[:78]:78s} {fetch[k][0]:4d} {fetch[k][1]:11.1f} {write[k][1]:11.1f} {b:12d}")
        fam = family(k)
        if fam and fam != "k_copy":
            a = fam_bytes.setdefault(fam, [0, 0])
            a[0] += fetch[k][0]
            a[1] += b * fetch[k][0]
    out += ["", "HBM bytes per launch by kernel family (read back by bench.py as roofline.traffic):"]
    for fam, (n, tot) in sorted(fam_bytes.items()):
        out.append(f"traffic_bytes {fam} {tot // n}")
    path = profile_path(args.workload, args.bits)
    open(path, "w").write("\n".join(out) + "\n")
    print(path)


class Bench:
    def __init__(self, args):
        import numpy as np
        import torch

        from paper_1905_10830_amd import binding as fmtc
        from paper_1905_10830_amd import synth

        self.np, self.torch, self.fmtc, self.synth = np, torch, fmtc, synth
        self.lib = fmtc.load_library()
        self.args = args
        self.stream_h = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def run(self, fn, n):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        bad = 0
        for i in range(n):
            bad |= fn(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if bad:
            raise RuntimeError("a library call failed: " + self.lib.fmtc_last_error().decode())
        return dt

    def kernel_times(self, fn, n):
        """Per-kernel durations over n more calls of fn (HIP events attached to the dispatches, on the launch stream)."""
        self.fmtc.profile_enable(n)
        self.run(fn, n)
        prof = self.fmtc.profile_read()
        self.fmtc.profile_enable(0)
        return prof

    def measure(self, workload, bits, steps, warmup, detail):
        np, torch, fmtc, synth, lib, args = self.np, self.torch, self.fmtc, self.synth, self.lib, self.args
        wl = synth.WORKLOADS[workload]
        layout = fmtc.NHWC if args.layout == "nhwc" else fmtc.NCHW
        calib, data = synth.workload(workload, seed=0)
        xs = synth.to_layout(data, layout)
        N, C, H, W = wl["N"], wl["C"], wl["H"], wl["W"]
        P, V = N * H * W, N * H * W * C
        in_bytes = 4 * V
        stream_h = self.stream_h

        # ---- offline: fit the basis on the calibration batch (GPU moments + host eigensolver) ----
        calib_d = torch.from_numpy(synth.to_layout(calib, layout)).cuda()
        basis = fmtc.fit_basis(calib_d, layout)
        if args.keep and detail:
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
                x=x0 if r == 0 else x0.clone(), stream=torch.empty(cap, dtype=torch.uint8, device="cuda"),
                nbytes=torch.zeros(1, dtype=torch.int64, device="cuda"),
                ws=torch.empty(ws_bytes, dtype=torch.uint8, device="cuda"),
                xhat=torch.empty_like(x0), err=torch.zeros(1, dtype=torch.int32, device="cuda")))

        ea = [(basis._h, s["x"].data_ptr(), N, C, H, W, layout, bits, 4096, s["stream"].data_ptr(), cap,
               s["nbytes"].data_ptr(), s["ws"].data_ptr(), ws_bytes, stream_h) for s in sets]
        da = [(basis._h, s["stream"].data_ptr(), cap, s["xhat"].data_ptr(), N, C, H, W, layout, bits,
               s["err"].data_ptr(), stream_h) for s in sets]

        def step(i):
            r = i % R
            return lib.fmtc_encode(*ea[r]) | lib.fmtc_decode(*da[r])

        def check_err():
            for s in sets:
                assert int(s["err"].item()) == 0, "decoder flagged its own stream"

        self.run(step, warmup)
        dt = self.run(step, steps)
        ms_per_step = 1e3 * dt / steps
        # encode and decode alone (same buffers; streams are valid from the runs above)
        dt_enc = self.run(lambda i: lib.fmtc_encode(*ea[i % R]), steps)
        dt_dec = self.run(lambda i: lib.fmtc_decode(*da[i % R]), steps)
        check_err()

        # ---- rate and distortion of the coded batch ----
        info = fmtc.stream_info(sets[0]["stream"][:64].cpu().numpy())
        R_payload = info["payload_bits"] / V
        R_container = 8.0 * info["stream_bytes"] / V
        mse = float(((sets[0]["xhat"] - sets[0]["x"]) ** 2).mean().item())

        # ---- per-kernel durations over one more pass of the same steps ----
        prof = self.kernel_times(step, steps)
        flops = 2.0 * C * V  # one direction of the dense C x C projection, as the method defines it
        stream_bytes = float(info["stream_bytes"])
        n_chunks = float(info["n_chunks"])
        # Per launch (one launch = the whole tensor): algorithmic HBM bytes, and the matrix flops the kernel issues
        # for the method's 2*C*V (the fp32 contraction runs as 3 (forward) or 2 (inverse) f16 products).  A kernel is
        # held against the roof that takes longer at peak: bytes / 8 TB/s or issued flops / 2.5 PFLOP/s.
        alg = {
            # projection: reads the activations once, writes one symbol byte per value
            "k_project_quantize": (4.0 * V + V, 3.0 * flops),
            # code bits of every chunk: reads the symbols, writes 4 bytes per chunk
            "k_chunk_bits": (V + 4.0 * n_chunks, 0.0),
            # coder: reads the symbols once, writes the container
            "k_pack": (V + stream_bytes, 0.0),
            # decoder: reads the container, writes the activations
            "k_decode": (stream_bytes + 4.0 * V, 2.0 * flops),
        }
        traffic = read_traffic(workload, bits)
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
                             t_roof_us=round(1e6 * max(t_hbm, t_mfma), 3),
                             hbm_bytes_algorithmic=int(hbm_bytes), hbm_frac=round(t_hbm / t, 4),
                             mfma_f16_flops_issued=mfma_flops, mfma_frac=round(t_mfma / t, 4),
                             traffic=traffic.get(name))
            kernels[name] = entry
        dominant = max((k for k in kernels if k in alg), key=lambda k: kernels[k]["avg_us"])
        dk = kernels[dominant]
        roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"], "peak": dk["peak"],
                    "unit": dk["unit"], "frac": dk["frac"], "traffic": dk["traffic"],
                    "avg_us": dk["avg_us"], "hbm_bytes_algorithmic": dk["hbm_bytes_algorithmic"]}
        # the whole encoder and the whole decoder against the method's bytes (survey: 6 + R/8 and R/8 + 4 per value)
        enc_alg, dec_alg = 6.0 * V + stream_bytes, stream_bytes + 4.0 * V
        res = {
            "workload": workload, "shape_NCHW": [N, C, H, W], "bits": bits, "steps": steps,
            "us_per_step": round(1e3 * ms_per_step, 2),
            "value_GBps": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 3),
            "encode_GBps": round(in_bytes / (dt_enc / steps) / 1e9, 3),
            "decode_GBps": round(in_bytes / (dt_dec / steps) / 1e9, 3),
            "encode_hbm_frac": round(enc_alg / (dt_enc / steps) / (HBM_PEAK_GBS * 1e9), 4),
            "decode_hbm_frac": round(dec_alg / (dt_dec / steps) / (HBM_PEAK_GBS * 1e9), 4),
            "bits_per_value": round(R_payload, 4), "container_bits_per_value": round(R_container, 4), "mse": mse,
            "kernels": kernels,
        }
        if not detail:
            return res
        res["roofline"] = roofline
        res["ms_per_step"] = ms_per_step
        res["buffer_sets"] = R
        res["in_bytes"] = in_bytes
        if args.main_only:
            return res

        # the same step on one buffer set only (inputs and outputs stay in the last-level cache): labelled as such
        dt_hot = self.run(lambda i: lib.fmtc_encode(*ea[0]) | lib.fmtc_decode(*da[0]), steps) if R > 1 else dt
        res["cache_hot_value"] = round(in_bytes / (dt_hot / steps) / 1e9, 3)

        # ---- the same steps as two independent chains on two HIP streams (default priority): step i runs encode
        # then decode of buffer set i on stream i % 2, so the kernels of neighbouring steps overlap.  Reported
        # beside `value`, which stays the one-stream figure. ----
        res["two_stream_value"] = None
        if R >= 2:
            side = [torch.cuda.Stream(), torch.cuda.Stream()]
            hs = [ctypes.c_void_p(st.cuda_stream) for st in side]
            ea2 = [[a[:-1] + (h,) for a in ea] for h in hs]
            da2 = [[a[:-1] + (h,) for a in da] for h in hs]
            Re = R - (R % 2)  # an even number of sets: a set always stays on the same stream

            def step2(i):
                r, q = i % Re, i % 2
                return lib.fmtc_encode(*ea2[q][r]) | lib.fmtc_decode(*da2[q][r])

            self.run(step2, warmup)
            dt_two = self.run(step2, steps)
            check_err()
            res["two_stream_value"] = round(in_bytes / (dt_two / steps) / 1e9, 3)

        # ---- the encoder with a code table fixed at calibration time (reported beside `value`, not part of it) ----
        table = fmtc.fit_table(basis, calib_d, bits, layout)
        scap = fmtc.encode_static_bound(table, P, C)
        sstreams = [torch.empty(scap, dtype=torch.uint8, device="cuda") for _ in sets]
        sa = [(basis._h, table._h, s["x"].data_ptr(), N, C, H, W, layout, 4096, st.data_ptr(), scap,
               s["nbytes"].data_ptr(), s["ws"].data_ptr(), ws_bytes, stream_h) for s, st in zip(sets, sstreams)]
        sda = [(basis._h, table._h, st.data_ptr(), scap, s["xhat"].data_ptr(), N, C, H, W, layout,
                s["err"].data_ptr(), stream_h) for s, st in zip(sets, sstreams)]
        self.run(lambda i: lib.fmtc_encode_static(*sa[i % R]), warmup)
        dt_static = self.run(lambda i: lib.fmtc_encode_static(*sa[i % R]), steps)
        sprof = self.kernel_times(lambda i: lib.fmtc_encode_static(*sa[i % R]), steps)
        sinfo = fmtc.stream_info(sstreams[0][:64].cpu().numpy())
        static = {"encode_GBps": round(in_bytes / (dt_static / steps) / 1e9, 3),
                  "us_per_encode": round(1e6 * dt_static / steps, 2),
                  "bits_per_value": round(sinfo["payload_bits"] / V, 4),
                  "container_bits_per_value": round(8.0 * sinfo["stream_bytes"] / V, 4),
                  "kernels": {k: round(1e3 * v[0], 3) for k, v in sprof.items()}}
        xh2, err2 = fmtc.decode(basis, sstreams[0], xs.shape, bits, layout)
        assert int(err2.item()) == 0 and torch.equal(xh2, sets[0]["xhat"]), "the two encoders disagree on the symbols"
        del xh2
        step_s = lambda i: lib.fmtc_encode_static(*sa[i % R]) | lib.fmtc_decode_static(*sda[i % R])  # noqa: E731
        self.run(step_s, warmup)
        dt_sstep = self.run(step_s, steps)
        dt_sdec = self.run(lambda i: lib.fmtc_decode_static(*sda[i % R]), steps)
        sdprof = self.kernel_times(lambda i: lib.fmtc_decode_static(*sda[i % R]), steps)
        check_err()
        static["decode_GBps"] = round(in_bytes / (dt_sdec / steps) / 1e9, 3)
        static["us_per_decode"] = round(1e6 * dt_sdec / steps, 2)
        static["decode_kernel_us"] = round(1e3 * sdprof["k_decode"][0], 3)
        static["encode_decode_GBps"] = round(in_bytes / (dt_sstep / steps) / 1e9, 3)
        static["us_per_step"] = round(1e6 * dt_sstep / steps, 2)
        res["static_table_codec"] = static
        del sstreams

        # ---- the 8-bit path: unsigned 8-bit activations, 8-bit basis, integer matrix cores (beside `value`) ----
        sx = float(x0.max().item()) / 255.0
        xq0 = torch.clamp(torch.round(x0 / sx), 0, 255).to(torch.uint8)
        b8 = fmtc.Basis8(basis, sx)
        usets = [dict(xq=xq0 if i == 0 else xq0.clone(), out=torch.empty_like(xq0),
                      ws=torch.empty(V, dtype=torch.uint8, device="cuda")) for i in range(len(sets))]
        ua = [(b8._h, u["xq"].data_ptr(), N, C, H, W, layout, bits, 4096, s["stream"].data_ptr(), cap,
               s["nbytes"].data_ptr(), s["ws"].data_ptr(), ws_bytes, stream_h) for s, u in zip(sets, usets)]
        uda = [(b8._h, s["stream"].data_ptr(), cap, u["out"].data_ptr(), N, C, H, W, layout, bits,
                s["err"].data_ptr(), u["ws"].data_ptr(), V, stream_h) for s, u in zip(sets, usets)]
        step_u = lambda i: lib.fmtc_encode_u8(*ua[i % R]) | lib.fmtc_decode_u8(*uda[i % R])  # noqa: E731
        self.run(step_u, warmup)
        dt_u8 = self.run(step_u, steps)
        uprof = self.kernel_times(step_u, steps)
        check_err()
        uinfo = fmtc.stream_info(sets[0]["stream"][:64].cpu().numpy())
        res["u8_codec"] = {
            "us_per_step": round(1e6 * dt_u8 / steps, 2),
            "encode_decode_Gvalues_per_s": round(V / (dt_u8 / steps) / 1e9, 3),
            "bits_per_value": round(uinfo["payload_bits"] / V, 4),
            "mse": float((((usets[0]["out"].float() - usets[0]["xq"].float()) * sx) ** 2).mean().item()),
            "kernels": {k: round(1e3 * v[0], 3) for k, v in uprof.items()},
            "note": "1 byte per value in and out; projection and reconstruction on the integer matrix cores, exact"}
        del usets

        # ---- the oracle on this machine's host cores: a slab of the same batch ----
        if not args.no_cpu_baseline:
            res["cpu_baseline"], res["cpu_baseline_all_cores"] = self.cpu_baseline(basis, xs, N, bits, layout)
        return res

    def cpu_baseline(self, basis, xs, N, bits, layout):
        """The oracle as it stands, encode + decode, on a slab of the batch: one thread, then one slab per core."""
        import concurrent.futures as cf

        import oracle

        fmtc = self.fmtc
        T, mu, eig, A = basis.export()
        d = oracle.delta(A, bits)
        n_slab = max(1, min(N, int(round(3.2e6 / (xs.size // N)))))  # about 3 M values: a fraction of a second a run
        slab = self.np.ascontiguousarray(xs[:n_slab])
        slab_bytes = 4 * slab.size

        def once(x):
            enc = oracle.encode(x, T, mu, d, bits, layout)
            oracle.decode(enc["stream"], x.shape, T, mu, bits, layout)

        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 200:
            t0 = time.perf_counter()
            once(slab)
            t_cpu += time.perf_counter() - t0
            reps += 1
        one = {"value": round(slab_bytes / (t_cpu / reps) / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"the first {n_slab} of the batch's {N} images as one tensor, encode+decode, mean of {reps} "
                         f"runs ({t_cpu:.1f} s), single thread; the full batch is {N // n_slab} such slabs"}
        # every host core codes a slab of its own (the oracle itself stays single-threaded: the ctypes call
        # releases the interpreter lock, so the threads run side by side)
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)), N // n_slab, 64))
        slabs = [self.np.ascontiguousarray(xs[i * n_slab:(i + 1) * n_slab]) for i in range(cores)]
        rounds = max(1, int(8.0 / (t_cpu / reps)))
        with cf.ThreadPoolExecutor(cores) as ex:
            t0 = time.perf_counter()
            list(ex.map(lambda x: [once(x) for _ in range(rounds)], slabs))
            t_all = time.perf_counter() - t0
        many = {"value": round(cores * rounds * slab_bytes / t_all / 1e9, 5), "unit": "GB/s", "cores": cores,
                "kind": "oracle",
                "sample": f"{cores} threads, each coding its own {n_slab}-image slab of the batch {rounds} times "
                          f"({t_all:.1f} s): the batch sharded over the host cores, one code table per slab"}
        del fmtc
        return one, many


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--bits", type=int, default=0, help="0: the bit depth the workload is listed with")
    ap.add_argument("--workload", default=SHAPES[0][0])
    ap.add_argument("--layout", default="nhwc", choices=["nhwc", "nchw"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--main-only", action="store_true",
                    help="the headline step and its kernels only (the form the rocprofv3 summaries are made from)")
    ap.add_argument("--no-other-shapes", action="store_true")
    ap.add_argument("--hot", action="store_true", help="one buffer set only (cache-hot figure)")
    ap.add_argument("--keep", type=int, default=0, help="truncate the basis to this many components (0: all)")
    ap.add_argument("--summarize", nargs=3, metavar=("STATS_DIR", "FETCH_DIR", "WRITE_DIR"))
    args = ap.parse_args()
    if not args.bits:
        args.bits = dict(SHAPES).get(args.workload, 6)
    if args.summarize:
        return summarize(args)
    if args.gpus != 1:
        sys.exit("bench.py: this build is a one-GPU codec; run it with --gpus 1 "
                 "(no multi-GPU path exists: the codec shards over pixels, each GPU coding its own share)")

    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py: needs a GPU")
    torch.cuda.set_device(0)
    b = Bench(args)
    res = b.measure(args.workload, args.bits, args.steps, args.warmup, detail=True)
    wl = b.synth.WORKLOADS[args.workload]

    others = None
    if not (args.main_only or args.no_other_shapes):
        others = []
        for name, bits in SHAPES:
            if name == args.workload:
                continue
            torch.cuda.empty_cache()
            others.append(b.measure(name, bits, min(args.steps, 50), min(args.warmup, 10), detail=False))

    # ---- yardstick for the memory counters: one plain copy of known size (not timed) ----
    ysrc = torch.empty(YARDSTICK_BYTES, dtype=torch.uint8, device="cuda")
    ydst = torch.empty_like(ysrc)
    b.fmtc.profile_copy(ydst, ysrc)
    torch.cuda.synchronize()

    out = {
        "metric": "encode+decode throughput of fp32 activations (input GB/s)",
        "value": round(res["in_bytes"] / (res["ms_per_step"] * 1e-3) / 1e9, 3),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "shape_NCHW": [wl["N"], wl["C"], wl["H"], wl["W"]],
                   "layout": args.layout, "bits": args.bits, "chunk_syms": 4096, "keep": args.keep or wl["C"],
                   "buffer_sets": res["buffer_sets"], "cache": "hot" if args.hot else "cold (rotating > 256 MB)"},
        "arithmetic": "fp32 in/out; projections as split-f16 matrix products with fp32 accumulation, fp64 where a "
                      "rounding decision is close",
        "roofline": res["roofline"],
    }
    for k in ("encode_GBps", "decode_GBps", "encode_hbm_frac", "decode_hbm_frac", "bits_per_value",
              "container_bits_per_value", "mse", "cache_hot_value", "two_stream_value", "kernels",
              "static_table_codec", "u8_codec"):
        if k in res:
            out[k] = res[k]
    if others is not None:
        out["other_shapes"] = others
    out["cpu_baseline"] = res.get("cpu_baseline")
    if "cpu_baseline_all_cores" in res:
        out["cpu_baseline_all_cores"] = res["cpu_baseline_all_cores"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
