"""Seeded synthetic inputs for the RMSMP hot path.

Serves both the CPU oracle (tests) and the HIP library (tests, bench).  It holds
shapes, distributions and seeds only -- no quantizer, no GEMM, no packing.  The
paper trained on ImageNet / GLUE with ResNet-18 / BERT weights; neither data nor
weights are available here, so tensors with the same shapes and the value
distributions below stand in for them.

Seed rule: numpy PCG64(211100153 + 1000*config + layer).
"""
import numpy as np

FIXED4, POT4, FIXED8 = 0, 1, 2
SEED_BASE = 211100153


def rng_for(config, layer=0):
    return np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * int(config) + int(layer)))


def weights_rowscaled(rng, M, K, std_lo=0.01, std_hi=0.1):
    """fp32 M x K, row r ~ N(0, s_r^2) with s_r ~ U(std_lo, std_hi)."""
    s = rng.uniform(std_lo, std_hi, size=(M, 1))
    return (rng.standard_normal((M, K)) * s).astype(np.float32)


def weights_bert(rng, M, K, std=0.02):
    """fp32 M x K, row r ~ N(0, (std*j_r)^2) with j_r ~ U(0.5, 1.5)."""
    j = rng.uniform(0.5, 1.5, size=(M, 1))
    return (rng.standard_normal((M, K)) * (std * j)).astype(np.float32)


def act_codes_u4(rng, shape):
    """Unsigned 4-bit activation codes, uniform on {0..15}, one per uint8."""
    return rng.integers(0, 16, size=shape, dtype=np.uint8)


def act_codes_i8(rng, shape):
    """Signed 8-bit activation codes, uniform on {-127..127}, one per int8."""
    return rng.integers(-127, 128, size=shape, dtype=np.int8)


def scheme_permutation(rng, counts):
    """Per-row scheme codes: counts = (n_fixed4, n_pot4, n_fixed8) in a seeded random order."""
    n4, np4, n8 = (int(c) for c in counts)
    s = np.concatenate([np.full(n4, FIXED4, np.uint8), np.full(np4, POT4, np.uint8),
                        np.full(n8, FIXED8, np.uint8)])
    return s[rng.permutation(s.size)]


def affine_u4_from_float(x):
    """Shift a signed float tensor to a non-negative 4-bit code range with one per-tensor
    scale: s = (max-min)/15, z = clamp(rint(-min/s), 0, 15), code = clamp(rint(x/s)+z, 0, 15).
    Returns (codes uint8, s float, z int).  Input preparation only (BERT-shaped config)."""
    x = np.asarray(x, dtype=np.float32)
    lo, hi = float(x.min()), float(x.max())
    s = np.float32((hi - lo) / 15.0) if hi > lo else np.float32(1.0)
    z = int(np.clip(np.rint(-lo / s), 0, 15))
    codes = np.clip(np.rint(x / s) + z, 0, 15).astype(np.uint8)
    return codes, float(s), z


def symmetric_i8_from_float(x):
    """Signed 8-bit codes with s = max|x|/127 (first-layer image input).  Returns (codes int8, s)."""
    x = np.asarray(x, dtype=np.float32)
    m = float(np.abs(x).max())
    s = np.float32(m / 127.0) if m > 0 else np.float32(1.0)
    codes = np.clip(np.rint(x / s), -127, 127).astype(np.int8)
    return codes, float(s)


# ResNet-18 convolution stack at 224x224 (standard topology).  Each entry:
# (name, C_in, M_out, kernel, stride, pad, H_in).  Output size = (H + 2p - k)//s + 1.
RESNET18_CONVS = [
    ("conv1", 3, 64, 7, 2, 3, 224),
    ("layer1.0.conv1", 64, 64, 3, 1, 1, 56),
    ("layer1.0.conv2", 64, 64, 3, 1, 1, 56),
    ("layer1.1.conv1", 64, 64, 3, 1, 1, 56),
    ("layer1.1.conv2", 64, 64, 3, 1, 1, 56),
    ("layer2.0.conv1", 64, 128, 3, 2, 1, 56),
    ("layer2.0.conv2", 128, 128, 3, 1, 1, 28),
    ("layer2.0.downsample", 64, 128, 1, 2, 0, 56),
    ("layer2.1.conv1", 128, 128, 3, 1, 1, 28),
    ("layer2.1.conv2", 128, 128, 3, 1, 1, 28),
    ("layer3.0.conv1", 128, 256, 3, 2, 1, 28),
    ("layer3.0.conv2", 256, 256, 3, 1, 1, 14),
    ("layer3.0.downsample", 128, 256, 1, 2, 0, 28),
    ("layer3.1.conv1", 256, 256, 3, 1, 1, 14),
    ("layer3.1.conv2", 256, 256, 3, 1, 1, 14),
    ("layer4.0.conv1", 256, 512, 3, 2, 1, 14),
    ("layer4.0.conv2", 512, 512, 3, 1, 1, 7),
    ("layer4.0.downsample", 256, 512, 1, 2, 0, 14),
    ("layer4.1.conv1", 512, 512, 3, 1, 1, 7),
    ("layer4.1.conv2", 512, 512, 3, 1, 1, 7),
]
RESNET18_FC = ("fc", 512, 1000)


def conv_out(h, k, s, p):
    return (h + 2 * p - k) // s + 1


def resnet18_macs_per_image():
    """Multiply-accumulates of the 20 convolutions plus the FC layer for one 224x224 image."""
    total = 0
    for _, c, m, k, s, p, h in RESNET18_CONVS:
        o = conv_out(h, k, s, p)
        total += m * c * k * k * o * o
    total += RESNET18_FC[1] * RESNET18_FC[2]
    return total


# The five benchmark configurations.  ratio = (pct_pot4, pct_fixed4, pct_fixed8).
CONFIGS = {
    0: dict(kind="gemm", M=64, K=576, N=256, ratio=(35, 60, 5), s_x=0.05),
    1: dict(kind="conv", B=32, C=256, M=256, H=14, W=14, KH=3, KW=3, stride=1, pad=1,
            ratio=(35, 60, 5), s_x=0.05),
    2: dict(kind="gemm_bert", M=3072, K=768, N=4096, ratio=(35, 60, 5)),
    3: dict(kind="resnet18", B=64, ratio=(35, 60, 5)),
    4: dict(kind="gemm", M=4096, K=4096, N=(1, 8, 64), ratio=(40, 50, 10), s_x=0.05),
}
