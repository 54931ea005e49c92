"""Rate-distortion sweep of the codec on the GPU (section 3: rate = average code bits per value, distortion =
mean squared error of the reconstruction; the paper's rate-distortion figures sweep the quantizer step).

Utilities around the library's entry points, nothing more: for every bit depth the tensor is encoded and decoded
by the HIP kernels; the entropy of the symbols (the bound section 3.1 compares the Huffman code with,
H <= R < H + 1) is computed on the host from the GPU's histogram.
"""
import math

from . import binding as fmtc


def entropy_bits(hist):
    """-sum p log2 p of a histogram (any iterable of counts)."""
    total = float(sum(int(h) for h in hist))
    if total <= 0:
        return 0.0
    return -sum((int(h) / total) * math.log2(int(h) / total) for h in hist if int(h) > 0)


def sweep(basis, x, bits_list=(8, 7, 6, 5, 4, 3, 2), layout=fmtc.NHWC):
    """x: device fp32 tensor.  -> list of dicts, one per bit depth:
    bits, delta, entropy (bits/value), rate (Huffman payload bits/value), container (all stream bits/value),
    mse, psnr (dB against the tensor's peak magnitude)."""
    import torch

    T, mu, eig, A = basis.export()
    V = x.numel()
    peak = float(x.abs().max().item())
    out = []
    for bits in bits_list:
        sym, hist = fmtc.quantize(basis, x, bits, layout)
        stream, nbytes = fmtc.encode(basis, x, bits, layout)
        xhat, err = fmtc.decode(basis, stream, tuple(x.shape), bits, layout)
        torch.cuda.synchronize()
        if int(err.item()):
            raise RuntimeError("decoder flagged its own stream")
        info = fmtc.stream_info(stream[:64].cpu().numpy())
        mse = float(((xhat - x) ** 2).mean().item())
        out.append({
            "bits": bits,
            "delta": fmtc.delta(A, bits),
            "entropy": entropy_bits(hist.cpu().tolist()),
            "rate": info["payload_bits"] / V,
            "container": 8.0 * info["stream_bytes"] / V,
            "mse": mse,
            "psnr": (10.0 * math.log10(peak * peak / mse)) if mse > 0 and peak > 0 else float("inf"),
        })
    return out


def truncation_sweep(basis, x, bits, keeps, layout=fmtc.NHWC):
    """Rate and distortion against the number of principal components kept (section 4 "Ablation study": dropping
    the least significant components trades projection work against rate and error).  -> list of dicts with keep,
    work (share of the projection's multiply-adds that the kept rows need) and the fields of sweep()."""
    out = []
    C = basis.C
    for keep in keeps:
        t = basis.truncate(keep)
        row = sweep(t, x, (bits,), layout)[0]
        t.close()
        row["keep"] = keep
        row["work"] = keep / C
        out.append(row)
    return out


def main():
    import argparse

    import torch

    from . import synth

    ap = argparse.ArgumentParser(description="rate-distortion table of a synthetic workload")
    ap.add_argument("--workload", default="resnet18_stage2_c128_28", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--truncate-at", type=int, default=0, metavar="BITS",
                    help="also print the table over the number of components kept, at this bit depth")
    args = ap.parse_args()
    calib, data = synth.workload(args.workload, seed=0)
    basis = fmtc.fit_basis(torch.from_numpy(calib).cuda())
    print(f"{args.workload}: bits  delta      H       R   container   mse        psnr")
    for r in sweep(basis, torch.from_numpy(data).cuda()):
        print(f"  {r['bits']:4d}  {r['delta']:.5f}  {r['entropy']:.4f}  {r['rate']:.4f}  {r['container']:.4f}  "
              f"{r['mse']:.4e}  {r['psnr']:.2f}")
    if args.truncate_at:
        C = basis.C
        keeps = sorted({max(1, C * k // 8) for k in range(1, 9)})
        print(f"{args.workload}, {args.truncate_at} bits: keep  work    H       R   container   mse        psnr")
        for r in truncation_sweep(basis, torch.from_numpy(data).cuda(), args.truncate_at, keeps):
            print(f"  {r['keep']:4d}  {r['work']:.3f}  {r['entropy']:.4f}  {r['rate']:.4f}  {r['container']:.4f}  "
                  f"{r['mse']:.4e}  {r['psnr']:.2f}")


if __name__ == "__main__":
    main()
