"""Random-init int8 networks serialised as ISRM model blobs.

Blob format (all fields little-endian 32-bit unless noted):

    header   : magic 'ISRM', version=1, in_C, in_H, in_W, num_classes,
               n_tensors, n_ops
    tensors  : n_tensors x {C, H, W, zero_point(i32)}; tensor 0 is the network
               input in the signed domain (pixel - 128, zero-point 0)
    ops      : n_ops x {type, payload_bytes, payload}
        CONV    (1): in, out, k, stride, pad, relu,
                     w int8[Cout][Cin][k][k] (zero-padded to 4 bytes),
                     bias i32[Cout], M0 i32[Cout], shift i32[Cout]
        ADD     (2): a, b, out, Ma, Mb, shift, relu
        MAXPOOL (3): in, out, k, stride, pad
        GAP     (4): in, out, M0, shift
        FC      (5): in, out, w int8[Cout][Cin] (padded to 4), bias i32[Cout]

The architectures are the standard ones named by the workload list: a tiny
two-conv net, CIFAR ResNet-20/110 (3 stages of basic blocks, 1x1 stride-2
projection on the shortcut where the shape changes) and ResNet-50 (bottleneck
3-4-6-3, stride on the 3x3, projection at the first block of each stage).

Weights are round(N(0, std 40)) clamped to [-127, 127], biases uniform in
[-512, 512], multipliers M0 uniform in [2^30, 2^31).  For the tiny net the
shifts are uniform in 8..11; for the deep nets each layer's shift is chosen
from its fan-in so that activations neither collapse nor saturate (bookkeeping
on a predicted RMS only; no forward pass is run here).
"""
from __future__ import annotations

import math
import struct
from dataclasses import dataclass, field

import numpy as np

MAGIC = 0x4D525349  # 'ISRM'
OP_CONV, OP_ADD, OP_MAXPOOL, OP_GAP, OP_FC = 1, 2, 3, 4, 5

TARGET_STD = 40.0   # aimed pre-activation standard deviation of conv outputs
M0_RMS = math.sqrt(7.0 / 12.0)  # rms of U[0.5, 1)


@dataclass
class _Tensor:
    C: int
    H: int
    W: int
    zp: int
    rms: float = 0.0  # predicted rms of (q - zp); bookkeeping for shift choice


@dataclass
class NetBuilder:
    rng: np.random.Generator
    in_shape: tuple
    num_classes: int
    tensors: list = field(default_factory=list)
    ops: list = field(default_factory=list)
    macs: int = 0
    fixed_shift_range: tuple | None = None

    def tensor(self, C, H, W, zp, rms=0.0):
        self.tensors.append(_Tensor(C, H, W, zp, rms))
        return len(self.tensors) - 1

    # -- ops ---------------------------------------------------------------
    def conv(self, tin, cout, k, stride, pad, relu, w=None, bias=None, m0=None, sh=None, zp_out=None):
        """Append a convolution; explicit w/bias/m0/sh/zp_out override the random draw."""
        ti = self.tensors[tin]
        cin = ti.C
        ho = (ti.H + 2 * pad - k) // stride + 1
        wo = (ti.W + 2 * pad - k) // stride + 1
        fan_in = cin * k * k
        given = dict(w=w, bias=bias, m0=m0, sh=sh)
        w = np.clip(np.rint(self.rng.normal(0.0, 40.0, size=(cout, cin, k, k))), -127, 127).astype(np.int8)
        bias = self.rng.integers(-512, 513, size=cout, dtype=np.int64).astype(np.int32)
        m0 = self.rng.integers(1 << 30, 1 << 31, size=cout, dtype=np.int64).astype(np.int32)
        if self.fixed_shift_range is not None:
            lo, hi = self.fixed_shift_range
            sh = self.rng.integers(lo, hi + 1, size=cout, dtype=np.int64).astype(np.int32)
            gain = M0_RMS * 40.0 * ti.rms * math.sqrt(fan_in) * float(np.mean(2.0 ** (-sh.astype(np.float64))))
        else:
            raw = M0_RMS * 40.0 * max(ti.rms, 1.0) * math.sqrt(fan_in)
            s = int(round(math.log2(raw / TARGET_STD)))
            s = min(max(s, 1), 24)
            sh = np.full(cout, s, dtype=np.int32)
            gain = raw * 2.0 ** (-s)
        if given["w"] is not None:
            w = np.asarray(given["w"], dtype=np.int8).reshape(cout, cin, k, k)
        if given["bias"] is not None:
            bias = np.asarray(given["bias"], dtype=np.int32).reshape(cout)
        if given["m0"] is not None:
            m0 = np.broadcast_to(np.asarray(given["m0"], dtype=np.int32), (cout,)).copy()
        if given["sh"] is not None:
            sh = np.broadcast_to(np.asarray(given["sh"], dtype=np.int32), (cout,)).copy()
        if zp_out is None:
            zp_out = -128 if relu else 0
        rms_out = gain / math.sqrt(2.0) if relu else gain
        tout = self.tensor(cout, ho, wo, zp_out, min(rms_out, 120.0))
        wbytes = w.tobytes()
        wbytes += b"\0" * ((-len(wbytes)) % 4)
        payload = struct.pack("<6i", tin, tout, k, stride, pad, int(relu)) + wbytes \
            + bias.tobytes() + m0.tobytes() + sh.tobytes()
        self.ops.append((OP_CONV, payload))
        self.macs += cout * ho * wo * fan_in
        return tout

    def add(self, ta, tb, relu=True, ma=None, mb=None, sh=20, zp_out=None):
        a, b = self.tensors[ta], self.tensors[tb]
        assert (a.C, a.H, a.W) == (b.C, b.H, b.W)
        if ma is None:
            ma = int(self.rng.integers(int(0.65 * (1 << sh)), int(0.85 * (1 << sh))))
        if mb is None:
            mb = int(self.rng.integers(int(0.65 * (1 << sh)), int(0.85 * (1 << sh))))
        if zp_out is None:
            zp_out = -128 if relu else 0
        tout = self.tensor(a.C, a.H, a.W, zp_out, 0.8 * TARGET_STD)
        self.ops.append((OP_ADD, struct.pack("<7i", ta, tb, tout, ma, mb, sh, int(relu))))
        return tout

    def maxpool(self, tin, k, stride, pad):
        ti = self.tensors[tin]
        ho = (ti.H + 2 * pad - k) // stride + 1
        wo = (ti.W + 2 * pad - k) // stride + 1
        tout = self.tensor(ti.C, ho, wo, ti.zp, ti.rms * 1.6)
        self.ops.append((OP_MAXPOOL, struct.pack("<5i", tin, tout, k, stride, pad)))
        return tout

    def gap(self, tin, m0=None, sh=None):
        ti = self.tensors[tin]
        hw = ti.H * ti.W
        if m0 is None:
            # multiplier ~ 1/(H*W) as M0 * 2^-(31+shift) with M0 in [2^30, 2^31)
            sh = 0
            while (1 << (31 + sh)) // hw < (1 << 30):
                sh += 1
            m0 = (1 << (31 + sh)) // hw
            if m0 == (1 << 31):
                m0, sh = ((1 << 30), sh - 1) if sh > 0 else ((1 << 31) - 1, 0)
            assert (1 << 30) <= m0 < (1 << 31)
        tout = self.tensor(ti.C, 1, 1, ti.zp, ti.rms)
        self.ops.append((OP_GAP, struct.pack("<4i", tin, tout, m0, sh)))
        return tout

    def fc(self, tin, cout, w=None, bias=None):
        ti = self.tensors[tin]
        cin = ti.C * ti.H * ti.W
        if w is None:
            w = np.clip(np.rint(self.rng.normal(0.0, 40.0, size=(cout, cin))), -127, 127).astype(np.int8)
        else:
            w = np.asarray(w, dtype=np.int8).reshape(cout, cin)
        if bias is None:
            bias = self.rng.integers(-512, 513, size=cout, dtype=np.int64).astype(np.int32)
        else:
            bias = np.asarray(bias, dtype=np.int32).reshape(cout)
        tout = self.tensor(cout, 1, 1, 0)
        wbytes = w.tobytes()
        wbytes += b"\0" * ((-len(wbytes)) % 4)
        self.ops.append((OP_FC, struct.pack("<2i", tin, tout) + wbytes + bias.tobytes()))
        self.macs += cout * cin
        return tout

    # -- serialise ---------------------------------------------------------
    def blob(self) -> bytes:
        c, h, w = self.in_shape
        out = [struct.pack("<8I", MAGIC, 1, c, h, w, self.num_classes, len(self.tensors), len(self.ops))]
        for t in self.tensors:
            out.append(struct.pack("<3Ii", t.C, t.H, t.W, t.zp))
        for typ, payload in self.ops:
            assert len(payload) % 4 == 0
            out.append(struct.pack("<2I", typ, len(payload)))
            out.append(payload)
        return b"".join(out)


def _input_rms():
    # (pixel - 128) for roughly uniform pixels
    return 74.0


def _tiny(b: NetBuilder):
    x = b.tensor(3, 32, 32, 0, _input_rms())
    t = b.conv(x, 16, 3, 1, 1, True)
    t = b.conv(t, 32, 3, 2, 1, True)
    t = b.gap(t)
    b.fc(t, b.num_classes)


def _cifar_resnet(b: NetBuilder, blocks_per_stage: int):
    x = b.tensor(3, 32, 32, 0, _input_rms())
    t = b.conv(x, 16, 3, 1, 1, True)
    for si, ch in enumerate((16, 32, 64)):
        for bi in range(blocks_per_stage):
            stride = 2 if (si > 0 and bi == 0) else 1
            u = b.conv(t, ch, 3, stride, 1, True)
            u = b.conv(u, ch, 3, 1, 1, False)
            if stride != 1 or b.tensors[t].C != ch:
                s = b.conv(t, ch, 1, stride, 0, False)
            else:
                s = t
            t = b.add(s, u, True)
    t = b.gap(t)
    b.fc(t, b.num_classes)


def _resnet50(b: NetBuilder, size: int = 224):
    x = b.tensor(3, size, size, 0, _input_rms())
    t = b.conv(x, 64, 7, 2, 3, True)
    t = b.maxpool(t, 3, 2, 1)
    for si, (width, nblocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3))):
        for bi in range(nblocks):
            stride = 2 if (si > 0 and bi == 0) else 1
            u = b.conv(t, width, 1, 1, 0, True)
            u = b.conv(u, width, 3, stride, 1, True)
            u = b.conv(u, width * 4, 1, 1, 0, False)
            if bi == 0:
                s = b.conv(t, width * 4, 1, stride, 0, False)
            else:
                s = t
            t = b.add(s, u, True)
    t = b.gap(t)
    b.fc(t, b.num_classes)


# name -> (architecture, input shape, classes); index = workload config number
CONFIGS = {
    0: dict(name="tiny", arch="tiny", shape=(3, 32, 32), classes=10,
            sigmas=(32,), n0=100, n=1000, images=1),
    1: dict(name="resnet20", arch="resnet20", shape=(3, 32, 32), classes=10,
            sigmas=(32, 64, 128), n0=100, n=100000, images=100),
    2: dict(name="resnet110", arch="resnet110", shape=(3, 32, 32), classes=10,
            sigmas=(64,), n0=100, n=100000, images=500),
    3: dict(name="resnet50", arch="resnet50", shape=(3, 224, 224), classes=101,
            sigmas=(64, 128), n0=100, n=10000, images=20),
    4: dict(name="resnet50-sweep", arch="resnet50", shape=(3, 224, 224), classes=101,
            sigmas=(32, 64, 128, 256), n0=100, n=100000, images=10),
}


def _make_builder(config: int, arch: str | None = None, size: int | None = None) -> NetBuilder:
    cfg = CONFIGS[config]
    arch = arch or cfg["arch"]
    rng = np.random.Generator(np.random.PCG64(1000 * config + 0))
    shape = cfg["shape"] if size is None else (3, size, size)
    b = NetBuilder(rng=rng, in_shape=shape, num_classes=cfg["classes"])
    if arch == "tiny":
        b.fixed_shift_range = (8, 11)
        _tiny(b)
    elif arch == "resnet20":
        _cifar_resnet(b, 3)
    elif arch == "resnet110":
        _cifar_resnet(b, 18)
    elif arch == "resnet50":
        _resnet50(b, shape[1])
    else:
        raise ValueError(arch)
    return b


def build_model(config: int, size: int | None = None) -> bytes:
    """Model blob for workload `config` (0..4).  `size` overrides the input
    height/width (used by small parity cases of the ResNet-50 architecture)."""
    return _make_builder(config, size=size).blob()


def model_macs(config: int, size: int | None = None) -> int:
    """Algorithmic multiply-accumulates of one forward pass (conv + FC)."""
    return _make_builder(config, size=size).macs
