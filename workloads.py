"""Seeded synthetic inputs for the layer-quantization path.

This module only *makes inputs*: weight matrices W (d_row x d_col, fp32),
calibration inputs X (d_col x N, fp32) and the shape lists of the benchmark
configurations.  It holds none of the method's arithmetic (no Hessian, no
quantizer, no ordering) and is the one piece of code that both the CPU oracle's
tests and the GPU path's tests/bench import, so that both sides see identical
bits.

The inputs stand in for the trained ResNet / YOLOv5 weights and the ImageNet /
COCO calibration activations of the paper's experiments (Section 6.1), which are
not available offline: shapes follow the public architectures, values are
He-normal weights and ReLU(N(0,1)) activations.

Random numbers come from a counter-based generator defined here (so that any
element can be produced independently of the others and the result does not
depend on chunking): element n of stream s under seed k is

    h   = mix64(mix64(k * GOLDEN + s) + n * GOLDEN)        (64-bit, wrapping)
    u1  = ((h >> 32) + 1) / 2^32        in (0, 1]
    u2  = (h & 0xffffffff) / 2^32       in [0, 1)
    z   = sqrt(-2 ln u1) * cos(2 pi u2)                     (fp64, Box-Muller)

and the fp32 value is float32(std * z).
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
import os
from typing import Dict, List, Optional, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22

STREAM_W = 1
STREAM_ACT = 2


def _mix64(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function (Steele, Lea, Flood 2014), vectorised."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _GOLDEN + np.uint64(stream)
        return _mix64(np.asarray(k, dtype=np.uint64))[()]


def normal_f64(count: int, seed: int, stream: int, offset: int = 0) -> np.ndarray:
    """`count` standard normals (fp64) for counters offset..offset+count-1.  Chunks are filled by a few
    threads (every element depends on its own counter only, so the result does not depend on the split)."""
    out = np.empty(count, dtype=np.float64)
    key = _stream_key(seed, stream)
    two_pi = 2.0 * np.pi
    inv32 = 1.0 / 4294967296.0

    def fill(lo: int) -> None:
        hi = min(count, lo + _CHUNK)
        with np.errstate(over="ignore"):
            n = np.arange(offset + lo, offset + hi, dtype=np.uint64)
            h = _mix64(key + n * _GOLDEN)
            u1 = ((h >> np.uint64(32)).astype(np.float64) + 1.0) * inv32
            u2 = (h & np.uint64(0xFFFFFFFF)).astype(np.float64) * inv32
            out[lo:hi] = np.sqrt(-2.0 * np.log(u1)) * np.cos(two_pi * u2)

    starts = range(0, count, _CHUNK)
    if len(starts) <= 1:
        for lo in starts:
            fill(lo)
    else:
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, starts))
    return out


def normal_f32(shape, std: float, seed: int, stream: int) -> np.ndarray:
    count = int(np.prod(shape))
    out = np.empty(count, dtype=np.float32)
    piece = 1 << 27                         # bounds the fp64 temporary to 1 GiB
    for lo in range(0, count, piece):
        n = min(piece, count - lo)
        out[lo:lo + n] = (normal_f64(n, seed, stream, offset=lo) * std).astype(np.float32)
    return out.reshape(shape)


def relu_normal_f32(shape, seed: int, stream: int) -> np.ndarray:
    """max(N(0,1), 0) in fp32."""
    a = normal_f32(shape, 1.0, seed, stream)
    np.maximum(a, 0.0, out=a)
    return a


def device_normal_f32(shape, std: float, seed: int, stream: int, relu: bool, device="cuda"):
    """The generator above evaluated with torch ops on `device` (for inputs too large to draw on the host
    in reasonable time): the same counters, mixing function and Box-Muller formula in fp64, rounded to fp32.
    The integer part is bit-identical to the numpy version; log / sqrt / cos are the device's, so an element
    can differ from the numpy generator's in its last fp32 bit.  Inputs that both the oracle and the GPU
    path must see identically are therefore always drawn with the numpy functions."""
    import torch

    def i64(v: int) -> int:                       # two's-complement view of a 64-bit constant
        v &= 0xFFFFFFFFFFFFFFFF
        return v - (1 << 64) if v >= (1 << 63) else v

    def lsr(z, k: int):                           # logical shift right on int64
        return (z >> k) & ((1 << (64 - k)) - 1)

    def mix(z):
        z = (z ^ lsr(z, 30)) * i64(int(_M1))
        z = (z ^ lsr(z, 27)) * i64(int(_M2))
        return z ^ lsr(z, 31)

    count = int(np.prod(shape))
    key = i64(int(_stream_key(seed, stream)))
    out = torch.empty(count, dtype=torch.float32, device=device)
    step = 1 << 26
    for lo in range(0, count, step):
        hi = min(count, lo + step)
        n = torch.arange(lo, hi, dtype=torch.int64, device=device)
        h = mix(n * i64(int(_GOLDEN)) + key)
        u1 = (lsr(h, 32).to(torch.float64) + 1.0) * (1.0 / 4294967296.0)
        u2 = (h & 0xFFFFFFFF).to(torch.float64) * (1.0 / 4294967296.0)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * np.pi) * u2)
        v = (z * std).to(torch.float32)
        out[lo:hi] = torch.clamp_min(v, 0.0) if relu else v
    return out.reshape(shape)


def im2col(maps: np.ndarray, k: int, stride: int, pad: int) -> np.ndarray:
    """Unfold feature maps into the (d_col x N) input matrix of a k x k conv.

    maps: (images, H, W, C) fp32.  Returns X with
      row index    = c * k*k + ky * k + kx
      column index = image * Ho*Wo + y * Wo + x
    and zeros where the window leaves the map (zero padding).
    """
    n, h, w, c = maps.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    padded = np.zeros((n, h + 2 * pad, w + 2 * pad, c), dtype=maps.dtype)
    padded[:, pad:pad + h, pad:pad + w, :] = maps
    x = np.empty((c, k, k, n, ho, wo), dtype=maps.dtype)
    for ky in range(k):
        for kx in range(k):
            win = padded[:, ky:ky + stride * ho:stride, kx:kx + stride * wo:stride, :]
            x[:, ky, kx] = np.transpose(win, (3, 0, 1, 2))
    return x.reshape(c * k * k, n * ho * wo)


@dataclasses.dataclass(frozen=True)
class LayerSpec:
    """One layer-quantization problem: shapes, quantizer settings, input recipe."""
    name: str
    d_row: int
    d_col: int
    n: int                       # calibration columns N
    bits: int = 4
    group: int = 0               # 0 = one grid per row
    damp: float = 0.01
    w_std: Optional[float] = None  # None = He-normal sqrt(2 / d_col)
    conv: Optional[Tuple[int, int, int, int, int]] = None  # (images, side, channels, k, pad): input maps of a conv
    stride: int = 1              # stride of that convolution
    seed: int = 0
    layer_index: int = 0

    @property
    def weights(self) -> int:
        return self.d_row * self.d_col

    def make_w(self) -> np.ndarray:
        std = self.w_std if self.w_std is not None else float(np.sqrt(2.0 / self.d_col))
        return normal_f32((self.d_row, self.d_col), std, self.seed,
                          STREAM_W + 16 * self.layer_index)

    def make_maps(self) -> np.ndarray:
        """Input feature maps (images, side, side, channels) of a conv recipe."""
        assert self.conv is not None
        images, side, ch, _k, _pad = self.conv
        return relu_normal_f32((images, side, side, ch), self.seed, STREAM_ACT + 16 * self.layer_index)

    def make_w_device(self, device="cuda"):
        """make_w on the device (torch tensor); see device_normal_f32."""
        std = self.w_std if self.w_std is not None else float(np.sqrt(2.0 / self.d_col))
        return device_normal_f32((self.d_row, self.d_col), std, self.seed, STREAM_W + 16 * self.layer_index,
                                 relu=False, device=device)

    def make_input_device(self, device="cuda"):
        """The layer's calibration input on the device: the feature maps (images, side, side, channels)
        of a conv recipe, else X (d_col x n).  Same recipe as make_maps / make_x."""
        stream = STREAM_ACT + 16 * self.layer_index
        if self.conv is not None:
            images, side, ch, _k, _pad = self.conv
            return device_normal_f32((images, side, side, ch), 1.0, self.seed, stream, relu=True, device=device)
        return device_normal_f32((self.d_col, self.n), 1.0, self.seed, stream, relu=True, device=device)

    def make_x(self, n: Optional[int] = None) -> np.ndarray:
        """X (d_col x n).  For conv recipes n must be the full N."""
        stream = STREAM_ACT + 16 * self.layer_index
        if self.conv is not None:
            _images, _side, _ch, k, pad = self.conv
            maps = self.make_maps()
            x = im2col(maps, k, self.stride, pad)
            assert x.shape == (self.d_col, self.n), (x.shape, self.d_col, self.n)
            return x
        n = self.n if n is None else n
        return relu_normal_f32((self.d_col, n), self.seed, stream)


def configs() -> Dict[str, LayerSpec]:
    """The benchmark configurations (layer shapes of the evaluation models)."""
    c: Dict[str, LayerSpec] = {}
    c["c1_tiny"] = LayerSpec("c1_tiny", 64, 128, 512, bits=4, w_std=0.05)
    # 3x3 conv 256->256 on 14x14 maps, 128 images -> X = 2304 x 25088
    c["c2_resnet50_3x3"] = LayerSpec("c2_resnet50_3x3", 256, 2304, 25088, bits=4,
                                     conv=(128, 14, 256, 3, 1))
    c["c3a_expand_w8"] = LayerSpec("c3a_expand_w8", 2048, 512, 25088, bits=8, layer_index=1)
    c["c3a_expand_w4"] = LayerSpec("c3a_expand_w4", 2048, 512, 25088, bits=4, layer_index=1)
    c["c3b_fc_w8"] = LayerSpec("c3b_fc_w8", 1000, 2048, 1024, bits=8, layer_index=2)
    c["c3b_fc_w4"] = LayerSpec("c3b_fc_w4", 1000, 2048, 1024, bits=4, layer_index=2)
    c["c5_large_d"] = LayerSpec("c5_large_d", 2048, 4608, 49152, bits=3, group=128, layer_index=3)
    return c


# Shape classes of the whole-model sweep: (count, d_row, d_col, N) with 128 images.
RESNET50_CLASSES: List[Tuple[int, int, int, int]] = [
    (1, 64, 147, 1605632),
    (1, 64, 64, 401408), (3, 64, 576, 401408), (4, 256, 64, 401408),
    (2, 64, 256, 401408), (1, 128, 256, 401408),
    (4, 128, 1152, 100352), (4, 512, 128, 100352), (1, 512, 256, 100352),
    (3, 128, 512, 100352), (1, 256, 512, 100352),
    (6, 256, 2304, 25088), (6, 1024, 256, 25088), (1, 1024, 512, 25088),
    (5, 256, 1024, 25088), (1, 512, 1024, 25088),
    (3, 512, 4608, 6272), (3, 2048, 512, 6272), (1, 2048, 1024, 6272),
    (2, 512, 2048, 6272),
    (1, 1000, 2048, 128),
]

YOLOV5S_CLASSES: List[Tuple[int, int, int, int]] = [
    (1, 32, 108, 13107200),
    (1, 64, 288, 3276800), (2, 32, 64, 3276800), (1, 64, 64, 3276800),
    (1, 32, 32, 3276800), (1, 32, 288, 3276800),
    (1, 128, 576, 819200), (2, 64, 128, 819200), (2, 128, 128, 819200),
    (3, 64, 64, 819200), (3, 64, 576, 819200), (2, 64, 256, 819200),
    (1, 255, 128, 819200),
    (1, 256, 1152, 204800), (5, 128, 256, 204800), (3, 256, 256, 204800),
    (5, 128, 128, 204800), (6, 128, 1152, 204800), (2, 128, 512, 204800),
    (1, 255, 256, 204800),
    (1, 512, 2304, 51200), (6, 256, 512, 51200), (2, 512, 512, 51200),
    (2, 256, 256, 51200), (3, 256, 2304, 51200), (1, 512, 1024, 51200),
    (1, 255, 512, 51200),
]


def _resnet50_geometry():
    """(d_row, d_col, in_side, in_channels, k, stride, pad) of the 53 convolutions of a ResNet-50-shaped network
    on 224 x 224 inputs (bottleneck blocks 3-4-6-3, the stride of a stage on its 3x3 convolution), then the
    classifier as a 1 x 1 layer on a 1 x 1 map."""
    g = [(64, 3 * 49, 224, 3, 7, 2, 3)]
    side, cin = 56, 64                      # after the 3 x 3 max-pool
    for width, blocks, stride in ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)):
        for b in range(blocks):
            st = stride if b == 0 else 1
            g.append((width, cin, side, cin, 1, 1, 0))
            g.append((width, width * 9, side, width, 3, st, 1))
            out_side = side // st
            g.append((4 * width, width, out_side, width, 1, 1, 0))
            if b == 0:
                g.append((4 * width, cin, side, cin, 1, st, 0))     # projection shortcut
            side, cin = out_side, 4 * width
    g.append((1000, 2048, 1, 2048, 1, 1, 0))
    return g


def _yolov5s_geometry():
    """The 60 convolutions of a YOLOv5s-shaped network (6 x 6 stem, C3 stages of 1 / 2 / 3 / 1 bottlenecks,
    SPPF, the up- and down-sampling neck, three 255-channel detection heads) on 640 x 640 inputs."""
    g = []

    def conv(cout, cin, side, k, st):
        g.append((cout, cin * k * k, side, cin, k, st, k // 2 if k > 1 else 0))
        return side // st

    def c3(cin, cout, n, side):
        h = cout // 2
        conv(h, cin, side, 1, 1)
        conv(h, cin, side, 1, 1)
        for _ in range(n):
            conv(h, h, side, 1, 1)
            conv(h, h, side, 3, 1)
        conv(cout, 2 * h, side, 1, 1)

    g.append((32, 108, 640, 3, 6, 2, 2))
    side = 320
    side = conv(64, 32, side, 3, 2);   c3(64, 64, 1, side)       # 160
    side = conv(128, 64, side, 3, 2);  c3(128, 128, 2, side)     # 80
    side = conv(256, 128, side, 3, 2); c3(256, 256, 3, side)     # 40
    side = conv(512, 256, side, 3, 2); c3(512, 512, 1, side)     # 20
    conv(256, 512, 20, 1, 1); conv(512, 1024, 20, 1, 1)          # SPPF
    conv(256, 512, 20, 1, 1)                                     # neck, top-down
    c3(512, 256, 1, 40)
    conv(128, 256, 40, 1, 1)
    c3(256, 128, 1, 80)
    conv(128, 128, 80, 3, 2)                                     # neck, bottom-up
    c3(256, 256, 1, 40)
    conv(256, 256, 40, 3, 2)
    c3(512, 512, 1, 20)
    conv(255, 128, 80, 1, 1); conv(255, 256, 40, 1, 1); conv(255, 512, 20, 1, 1)   # detection heads
    return g


def sweep_layers(model: str, images: int = 128) -> List[LayerSpec]:
    """Per-layer list of the whole-model sweep (4-bit, per-row grids), each with the geometry of its
    convolution.  A k x k or strided convolution carries `conv` (its input maps are drawn, X is their
    unfolding); a 1 x 1 convolution of stride 1 and the classifier take X (d_col x N) directly: with
    independent activations a channel-major map is the same thing as X."""
    geo = {"resnet50": _resnet50_geometry, "yolov5s": _yolov5s_geometry}[model]()
    out: List[LayerSpec] = []
    idx = 100 if model == "resnet50" else 300
    seen: Dict[str, int] = {}
    for r, d, side, cin, k, st, pad in geo:
        so = (side + 2 * pad - k) // st + 1
        n = images * so * so
        key = f"{model}_{r}x{d}_n{n}"
        rep = seen.get(key, 0)
        seen[key] = rep + 1
        conv = (images, side, cin, k, pad) if (k > 1 or st > 1) else None
        out.append(LayerSpec(f"{key}_{rep}", r, d, n, bits=4, layer_index=idx, conv=conv, stride=st))
        idx += 1
    return out
