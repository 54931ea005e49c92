"""Seeded synthetic feature maps (stand-ins for CNN activations).

Holds none of the codec's arithmetic: it only draws inputs.  Both the GPU
tests/benchmark and the CPU oracle's tests take their tensors from here.

Recipe (one stream per seed, draw order fixed):
    rng  = numpy Generator(PCG64(seed))
    M    = rng.standard_normal((C, r)) / sqrt(r)        mixing matrix, rank r
    beta = 0.5 * rng.standard_normal(C)                 per-channel offset (std 0.5)
    then for every image in turn:
        z   = rng.standard_normal((H*W, r))
        eps = rng.standard_normal((H*W, C))
        x   = act(z @ M.T + beta + 0.1 * eps)           act = ReLU or ReLU6
Images are produced channels-last ([N, H, W, C], fp32); `to_layout` gives the
NCHW-contiguous copy.  A calibration batch is the first images of the stream,
the data batch the images after it.
"""
import numpy as np

NCHW, NHWC = 0, 1


class FeatureMapStream:
    def __init__(self, C, H, W, rank, act="relu", seed=0):
        self.C, self.H, self.W, self.rank, self.act = int(C), int(H), int(W), int(rank), act
        self.rng = np.random.Generator(np.random.PCG64(seed))
        self.M = self.rng.standard_normal((self.C, self.rank)) / np.sqrt(self.rank)
        self.beta = 0.5 * self.rng.standard_normal(self.C)

    def images(self, n):
        """Next n images of the stream, [n, H, W, C] fp32."""
        out = np.empty((n, self.H, self.W, self.C), np.float32)
        hw = self.H * self.W
        for i in range(n):
            z = self.rng.standard_normal((hw, self.rank))
            eps = self.rng.standard_normal((hw, self.C))
            pre = z @ self.M.T + self.beta + 0.1 * eps
            if self.act == "relu":
                np.maximum(pre, 0.0, out=pre)
            elif self.act == "relu6":
                np.clip(pre, 0.0, 6.0, out=pre)
            elif self.act != "none":
                raise ValueError(self.act)
            out[i] = pre.reshape(self.H, self.W, self.C)
        return out


def to_layout(x_nhwc, layout):
    """Storage array for a layout: NHWC -> as is, NCHW -> contiguous permuted copy."""
    if layout == NHWC:
        return np.ascontiguousarray(x_nhwc)
    return np.ascontiguousarray(np.transpose(x_nhwc, (0, 3, 1, 2)))


# The workloads named by the benchmark definition: (name, N, C, H, W, rank, act, bits, calib images)
WORKLOADS = {
    "cfg0_c64_56": dict(N=1, C=64, H=56, W=56, rank=16, act="relu", bits=(8,), calib=0),
    "resnet18_stage2_c128_28": dict(N=32, C=128, H=28, W=28, rank=32, act="relu", bits=(6, 4), calib=8),
    "resnet18_stage3_c256_14": dict(N=64, C=256, H=14, W=14, rank=64, act="relu", bits=(4,), calib=8),
    "resnet18_stage4_c512_7": dict(N=64, C=512, H=7, W=7, rank=128, act="relu", bits=(4,), calib=8),
    "mbv2_c144_56": dict(N=64, C=144, H=56, W=56, rank=18, act="relu6", bits=(5,), calib=8),
    "mbv2_c960_7": dict(N=64, C=960, H=7, W=7, rank=120, act="relu6", bits=(5,), calib=8),
    # inference-shaped sweep: the four ResNet-18 post-block shapes at N = 256
    "resnet18_n256_c64_56": dict(N=256, C=64, H=56, W=56, rank=16, act="relu", bits=(8, 6, 4, 3, 2), calib=8),
    "resnet18_n256_c128_28": dict(N=256, C=128, H=28, W=28, rank=32, act="relu", bits=(8, 6, 4, 3, 2), calib=8),
    "resnet18_n256_c256_14": dict(N=256, C=256, H=14, W=14, rank=64, act="relu", bits=(8, 6, 4, 3, 2), calib=8),
    "resnet18_n256_c512_7": dict(N=256, C=512, H=7, W=7, rank=128, act="relu", bits=(8, 6, 4, 3, 2), calib=8),
}


def workload(name, seed=0, n_override=None):
    """-> (calibration batch, data batch), both [*, H, W, C] fp32.  With calib == 0
    the basis is fitted on the data itself (calibration batch is the data batch)."""
    w = WORKLOADS[name]
    s = FeatureMapStream(w["C"], w["H"], w["W"], w["rank"], w["act"], seed)
    n = w["N"] if n_override is None else n_override
    if w["calib"] == 0:
        data = s.images(n)
        return data, data
    calib = s.images(w["calib"])
    data = s.images(n)
    return calib, data
