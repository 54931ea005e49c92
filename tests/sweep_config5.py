#!/usr/bin/env python3
"""The inference-shaped sweep of the benchmark definition: the four ResNet-18 post-block maps at N = 256, every bit
depth b in {8, 6, 4, 3, 2}, encoded and decoded end to end by the HIP path, rate against distortion reported -- and
every cell held against the CPU oracle on the same tensor:

  * the container equals the oracle's packing (histogram, Huffman lengths, canonical codes, offsets, run sizes,
    payload) of the symbols it carries, byte for byte, and its header's bit count is the oracle's;
  * the symbols against the oracle's fp64 quantizer under the boundary rule (differences only within 1e-4 steps
    of a rounding boundary, rate <= 1e-6), on the first `check_images` images;
  * the decoded tensor within 1e-4 of the oracle's fp64 reconstruction of the same symbols, on those images;
  * the rate obeys H <= R < H + 1 (section 3.1 "Variable length coding").

    python tests/sweep_config5.py [--images N] [--check-images K] [--markdown FILE]

Prints one line per cell; --markdown writes the table that the design doc quotes.  tests/test_gpu_config5.py runs the
same function on a few images per shape.
"""
import argparse
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

SHAPES = ["resnet18_n256_c64_56", "resnet18_n256_c128_28", "resnet18_n256_c256_14", "resnet18_n256_c512_7"]
BITS = (8, 6, 4, 3, 2)
SYM_MARGIN, SYM_RATE, RECON_TOL = 1e-4, 1e-6, 1e-4


def run(images=None, check_images=8, shapes=SHAPES, bits_list=BITS, log=print):
    import torch

    import oracle
    from paper_1905_10830_amd import binding as fmtc
    from paper_1905_10830_amd import synth

    oracle.build()
    rows = []
    for name in shapes:
        wl = synth.WORKLOADS[name]
        C, hw = wl["C"], wl["H"] * wl["W"]
        calib, x = synth.workload(name, seed=0, n_override=images)
        T, mu, _, A = oracle.fit(calib)
        basis = fmtc.basis_import(T, mu, A)
        x_d = torch.from_numpy(x).cuda()
        P, V = x.size // C, x.size
        k = min(check_images, x.shape[0])
        y_k = oracle.project(x[:k], T, mu)
        for bits in bits_list:
            t0 = time.time()
            d = oracle.delta(A, bits)
            stream, nbytes = fmtc.encode(basis, x_d, bits)
            xhat, err = fmtc.decode(basis, stream, x.shape, bits)
            torch.cuda.synchronize()
            assert int(err.item()) == 0
            n = int(nbytes.item())
            got = stream[:n].cpu().numpy()
            info = fmtc.stream_info(got[:64])
            mse_gpu = float(((xhat - x_d).double() ** 2).mean().item())
            # the oracle on the same symbols
            sym, d2, pbits = oracle.unpack(got, P, C, bits)
            assert d2 == d
            h = oracle.histogram(sym, bits)
            ln = oracle.huffman_lengths(h[: 1 << bits])
            again = oracle.pack(sym, C, bits, d, ln, oracle.canonical_codes(ln))
            assert len(again) == n and (got == again).all(), f"{name} b={bits}: container differs from the oracle's"
            assert pbits == info["payload_bits"] == int((h[: 1 << bits] * ln.astype(np.uint64)).sum())
            H = oracle.entropy(h[: 1 << bits])
            R = pbits / V
            assert H - 1e-9 <= R < H + 1, f"{name} b={bits}: H={H} R={R}"
            # symbols and reconstruction against the fp64 definitions, first k images
            ref_sym, margin = oracle.quantize(y_k, d, bits, want_margin=True)
            diff = sym[: k * hw] != ref_sym
            n_bad = int(diff.sum())
            if n_bad:
                assert margin[diff].max() <= SYM_MARGIN, f"{name} b={bits}: symbol off a boundary differs"
                assert n_bad <= max(1, int(SYM_RATE * ref_sym.size)), f"{name} b={bits}: {n_bad} symbols differ"
            ref_hat = oracle.reconstruct(sym[: k * hw], x[:k].shape, T, mu, d, bits)
            worst = float(np.abs(xhat[:k].cpu().numpy().astype(np.float64) - ref_hat).max())
            assert worst <= RECON_TOL, f"{name} b={bits}: reconstruction off by {worst:.3e}"
            mse_ref = float(((ref_hat - x[:k].astype(np.float64)) ** 2).mean())
            mse_gpu_k = float(((xhat[:k] - x_d[:k]).double() ** 2).mean().item())
            rows.append(dict(workload=name, N=x.shape[0], C=C, bits=bits, delta=float(d), entropy=H, rate=R,
                             container=8.0 * n / V, mse=mse_gpu, mse_first=mse_gpu_k, mse_oracle_first=mse_ref,
                             psnr=10.0 * math.log10(float(x.max()) ** 2 / mse_gpu) if mse_gpu > 0 else float("inf"),
                             sym_diffs=n_bad, recon_err=worst))
            log(f"{name} N={x.shape[0]} b={bits}: H {H:.4f} R {R:.4f} container {8.0 * n / V:.4f} bits/value, "
                f"mse {mse_gpu:.4e} (first {k} images: GPU {mse_gpu_k:.6e}, oracle {mse_ref:.6e}), "
                f"{n_bad} boundary symbols, recon err {worst:.2e}  [{time.time() - t0:.1f} s]")
        del x_d, basis
    return rows


def markdown(rows):
    out = ["| map (N = 256) | b | entropy H | rate R (bits/value) | container bits/value | MSE (GPU, whole batch) | "
           "MSE first images: GPU / oracle fp64 | PSNR dB |", "|---|---|---|---|---|---|---|---|"]
    for r in rows:
        out.append(f"| {r['workload']} | {r['bits']} | {r['entropy']:.4f} | {r['rate']:.4f} | {r['container']:.4f} | "
                   f"{r['mse']:.4e} | {r['mse_first']:.5e} / {r['mse_oracle_first']:.5e} | {r['psnr']:.2f} |")
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--images", type=int, default=None, help="images per shape (default: the workload's 256)")
    ap.add_argument("--check-images", type=int, default=8)
    ap.add_argument("--markdown", default=None)
    a = ap.parse_args()
    rows = run(a.images, a.check_images, log=lambda s: print(s, flush=True))
    if a.markdown:
        open(a.markdown, "w").write(markdown(rows))
