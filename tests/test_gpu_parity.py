"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer results (noisy copies, layer tensors,
logits, argmax, votes) must be bit-exact; radii agree to 1e-9 relative."""
import numpy as np
import pytest

import oracle
import synth
from synth.models import NetBuilder

pytestmark = pytest.mark.gpu

ALPHA = 0.001


@pytest.fixture(scope="module")
def isr():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2108_09413_amd as lib
    return lib


def _load(isr, blob, chunk):
    m = isr.isr_load_model(blob)
    isr.isr_set_workspace(m, chunk)
    return m


def _say(msg):
    print(msg, flush=True)


def _oracle_at(om, x, sigma, seed, image, phase, indices):
    """Oracle logits and argmax of scattered sample indices, one host thread per index."""
    from concurrent.futures import ThreadPoolExecutor
    import os

    def one(i):
        lg, am, _ = om.mc(x, sigma, seed, image, phase, int(i), 1, threads=1)
        return lg[0], int(am[0])
    with ThreadPoolExecutor(max_workers=min(os.cpu_count() or 1, 16)) as ex:
        out = list(ex.map(one, indices))
    return np.stack([o[0] for o in out]), np.array([o[1] for o in out])


# ---- S2: noise -------------------------------------------------------------

@pytest.mark.parametrize("sigma", [1, 32, 64, 128, 256, 1024])
def test_noisy_copies_cifar_shape(isr, sigma):
    _say(f"noise parity 32x32 sigma={sigma}")
    m = _load(isr, synth.build_model(0), 64)
    x = synth.make_image(0, 1)
    for seed, image, phase, begin, count in ((0, 0, 0, 0, 5), (0x0123456789ABCDEF, 7, 1, 99990, 10)):
        got = isr.isr_debug_noisy(m, x, sigma, seed, image, phase, begin, count)
        for s in range(count):
            want = oracle.noisy(x, sigma, seed, image, phase, begin + s)
            assert np.array_equal(got[s], want), (sigma, seed, s)
    m.close()


def test_noisy_copies_224_shape_and_extreme_pixels(isr):
    _say("noise parity 224x224")
    m = _load(isr, synth.build_model(3), 4)
    x = synth.make_image(3, 1)
    x[0, :8, :] = 0
    x[1, :8, :] = 255
    for sigma in (64, 256):
        got = isr.isr_debug_noisy(m, x, sigma, 5, 3, 1, 12345, 2)
        for s in range(2):
            assert np.array_equal(got[s], oracle.noisy(x, sigma, 5, 3, 1, 12345 + s))
    m.close()


@pytest.mark.parametrize("sigma", [1, 32, 256, 1024])
def test_stored_training_noise_bank(isr, sigma):
    """Unsaturated int16 draws for noise sampled ahead of training: bit-exact against
    the oracle for a range of tensors that does not start at 0, a tensor size that
    leaves the last workgroup ragged, and a tiny tensor."""
    _say(f"noise bank parity sigma={sigma}")
    for seed, bank, first, count, d in ((3, 2, 4094, 5, 3 * 32 * 32), (0xFFFFFFFF00000001, 9, 0, 3, 12)):
        got = isr.isr_noise_bank(sigma, seed, bank, first, count, d).cpu().numpy()
        want = oracle.noise_bank(sigma, seed, bank, first, count, d)
        assert got.dtype == np.int16 and np.array_equal(got, want), (sigma, seed)
    import ctypes
    import torch
    buf = torch.empty(64, dtype=torch.int16, device="cuda")
    for bad_sigma, bad_d in ((0, 8), (1025, 8), (sigma, 6), (sigma, 0)):
        rc = isr.lib().isr_noise_bank(bad_sigma, ctypes.c_uint64(0), 0, 0, 1, bad_d, ctypes.c_void_p(buf.data_ptr()), None)
        assert rc == isr.ISR_ERR_ARG
    assert isr.lib().isr_noise_bank(sigma, ctypes.c_uint64(0), 0, 0, 1, 8, None, None) == isr.ISR_ERR_ARG


@pytest.mark.parametrize("sigma", [2, 32])
def test_device_sampler_law_at_scale(isr, sigma):
    """1.5e8 draws of the device sampler (a full stored-noise bank) against Def. 3.3 itself:
    mean, variance and a chi-square over 50 cells with the exact cell probabilities
    (50-digit arithmetic) -- a property of the law, not of the oracle's code."""
    import mpmath as mp
    import torch
    _say(f"sampler law at scale sigma={sigma}")
    count, d = 50000, 3072
    bank = isr.isr_noise_bank(sigma, 12345, 7, 0, count, d)
    n = count * d
    x = bank.to(torch.float64)
    mean, var = float(x.mean()), float(x.var(unbiased=False))
    assert abs(mean) < 5 * sigma / np.sqrt(n)
    assert abs(var / sigma ** 2 - 1) < 5 * np.sqrt(2.0 / n) + 1e-9      # the discrete law's variance is sigma^2 to < 1e-13 for sigma >= 2
    mp.mp.dps = 50
    K = 12 * sigma
    w = [mp.e ** (-(mp.mpf(k) ** 2) / (2 * mp.mpf(sigma) ** 2)) for k in range(0, K + 1)]
    Z = w[0] + 2 * sum(w[1:])
    pmf = lambda k: w[abs(k)] / Z if abs(k) <= K else mp.mpf(0)
    step = max(1, sigma // 8)
    edges = list(range(-3 * sigma, 3 * sigma + 1, step))                 # cells [e_i, e_{i+1}) plus the two tails
    obs = torch.histc(x, bins=len(edges) - 1, min=edges[0] - 0.5, max=edges[-1] - 0.5).cpu().numpy()
    lo_tail = float((x < edges[0] - 0.5).sum()); hi_tail = float((x > edges[-1] - 0.5).sum())
    obs = np.concatenate([[lo_tail], obs, [hi_tail]])
    probs = [float(sum(pmf(k) for k in range(-K, edges[0])))]
    probs += [float(sum(pmf(k) for k in range(a, b))) for a, b in zip(edges, edges[1:])]
    probs += [float(sum(pmf(k) for k in range(edges[-1], K + 1)))]
    assert abs(sum(probs) - 1) < 1e-12 and int(obs.sum()) == n
    exp = np.array(probs) * n
    chi2 = float(((obs - exp) ** 2 / exp).sum())
    assert chi2 < 110.0, chi2          # 49 degrees of freedom: P[chi2 > 110] ~ 1e-6


# ---- S3-S6: layer tensors ----------------------------------------------------

def _check_all_tensors(isr, blob, x, sigma, seed=3, image=1, phase=1, sample=17, chunk=4, min_fused=0, fusion=1):
    """Every tensor of one noisy copy against the oracle.  With fusion on (the default) a tensor that
    a fused kernel stores is that kernel's own output; a tensor that no fused kernel stores (the
    output of a convolution folded into a residual add, the 112x112 first-layer output under the
    pooling fusion, the middle tensors of a block kernel) is served by the op-by-op kernels, so that
    comparison checks those kernels and not the fused ones -- isr_debug_tensor_source says which.
    The fused kernels are covered by the tensors they do store (block outputs), by the logits of
    this copy below, and by the multi-copy logits check that follows every fused-kernel test.
    min_fused: at least that many tensors must come from fused kernels (guards the test's premise)."""
    m = _load(isr, blob, chunk)
    isr.isr_set_fusion(m, fusion)
    om = oracle.Model(blob)
    a0 = oracle.noisy(x, sigma, seed, image, phase, sample)
    logits, tensors = om.forward(a0)
    n_fused = 0
    for tid in sorted(tensors):
        c, h, w, _ = om.tensor_shape(tid)
        got = isr.isr_debug_tensor(m, x, sigma, seed, image, phase, sample, tid, (c, h, w))
        bad = np.argwhere(got != tensors[tid])
        src = "fused" if isr.isr_debug_tensor_source(m, tid) else "op-by-op"
        n_fused += src == "fused"
        assert bad.size == 0, f"tensor {tid} ({src} plan) shape {(c, h, w)}: {len(bad)} mismatches, first at {bad[0]}"
    assert n_fused >= min_fused, (n_fused, min_fused)
    gl, ga, gc = isr.isr_debug_forward(m, x, sigma, seed, image, phase, sample, 1)
    assert np.array_equal(gl[0], logits)
    m.close()


def test_layer_tensors_tiny(isr):
    _say("layer parity tiny")
    _check_all_tensors(isr, synth.build_model(0), synth.make_image(0, 1), 32)


def test_layer_tensors_resnet20(isr):
    _say("layer parity resnet20")
    _check_all_tensors(isr, synth.build_model(1), synth.make_image(1, 1), 64)


def test_layer_tensors_resnet50_small(isr):
    _say("layer parity resnet50 at 64x64")
    _check_all_tensors(isr, synth.build_model(3, size=64), synth.make_image(3, 1, shape=(3, 64, 64)), 128)


def test_layer_tensors_odd_shapes(isr):
    """Channel counts that are not multiples of 16, 5x5 / 7x7 / 1x1 kernels,
    strides, shifts of 0 and 31, non-trivial zero-points, both add signs."""
    _say("layer parity odd shapes")
    rng = np.random.default_rng(11)
    b = NetBuilder(rng=np.random.default_rng(12), in_shape=(3, 20, 12), num_classes=7)
    t0 = b.tensor(3, 20, 12, 0, 74.0)
    t1 = b.conv(t0, 5, 5, 1, 2, True, sh=rng.integers(6, 10, size=5))
    t2 = b.conv(t1, 40, 3, 2, 1, False, zp_out=9, sh=rng.integers(5, 9, size=40))
    t3 = b.conv(t2, 40, 1, 1, 0, True, sh=rng.integers(4, 8, size=40), zp_out=-100)
    t4 = b.add(t2, t3, False, ma=-600000, mb=900000, sh=20, zp_out=-5)
    t5 = b.conv(t4, 70, 3, 1, 1, True, sh=np.concatenate([[0, 31], rng.integers(5, 9, size=68)]))
    t6 = b.maxpool(t5, 3, 2, 1)
    t7 = b.conv(t6, 130, 1, 2, 0, False, sh=rng.integers(4, 8, size=130))
    t8 = b.conv(t7, 64, 1, 1, 0, True, sh=rng.integers(5, 9, size=64))
    t9 = b.conv(t8, 64, 1, 1, 0, True, sh=rng.integers(5, 9, size=64))   # Cin 64: flat 1x1 path
    t10 = b.maxpool(t9, 2, 1, 0)
    g = b.gap(t10)
    b.fc(g, 7)
    x = np.random.default_rng(5).integers(0, 256, size=(3, 20, 12)).astype(np.uint8)
    _check_all_tensors(isr, b.blob(), x, 64)


def test_first_layer_7x7_stride2(isr):
    _say("layer parity 7x7 stem")
    b = NetBuilder(rng=np.random.default_rng(21), in_shape=(3, 36, 28), num_classes=4)
    t0 = b.tensor(3, 36, 28, 0, 74.0)
    t1 = b.conv(t0, 24, 7, 2, 3, True)
    t2 = b.maxpool(t1, 3, 2, 1)
    b.fc(b.gap(t2), 4)
    x = np.random.default_rng(6).integers(0, 256, size=(3, 36, 28)).astype(np.uint8)
    _check_all_tensors(isr, b.blob(), x, 32)


@pytest.mark.parametrize("shape", [(32, 32), (48, 16), (7, 64)])
def test_first_layer_3x3_into_16_channels(isr, shape):
    """The LDS-resident first layer of the narrow nets (3x3, stride 1, pad 1, 16 stored
    channels): 13 real channels, ReLU off with a non-trivial output zero-point, one variant
    with power-of-two multipliers (rounding ties), 6 copies (ragged against 4 images per
    workgroup); image sizes with one, two and four 16-pixel strips."""
    h, w = shape
    _say(f"layer parity first 3x3 layer {h}x{w}")
    for pow2 in (False, True):
        b = NetBuilder(rng=np.random.default_rng(91), in_shape=(3, h, w), num_classes=4)
        kw = dict(m0=np.full(13, 1 << 30, dtype=np.int64), sh=np.full(13, 7)) if pow2 else {}
        t1 = b.conv(b.tensor(3, h, w, 0, 74.0), 13, 3, 1, 1, pow2, zp_out=-128 if pow2 else 9, **kw)
        t2 = b.conv(t1, 32, 3, 2, 1, True)
        b.fc(b.gap(t2), 4)
        blob = b.blob()
        x = np.random.default_rng(13).integers(0, 256, size=(3, h, w)).astype(np.uint8)
        _check_all_tensors(isr, blob, x, 64, sample=1, chunk=3)
        m = _load(isr, blob, 6)
        om = oracle.Model(blob)
        lg, am, cnt = isr.isr_debug_forward(m, x, 128, 5, 2, 0, 7, 6)
        olg, oam, ocnt = om.mc(x, 128, 5, 2, 0, 7, 6)
        assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
        m.close()


@pytest.mark.parametrize("shape", [(224, 224), (64, 64), (37, 28), (30, 44), (9, 8)])
def test_first_layer_fused_with_max_pooling(isr, shape):
    """7x7/2 convolution into 64 channels followed by 3x3/2 max pooling (one fused kernel):
    every tensor against the oracle, at the full 224 x 224 size, sizes with odd row
    counts, ragged last bands and images narrower than one fragment row."""
    h, w = shape
    _say(f"layer parity fused stem + pool {h}x{w}")
    b = NetBuilder(rng=np.random.default_rng(31), in_shape=(3, h, w), num_classes=5)
    t0 = b.tensor(3, h, w, 0, 74.0)
    t1 = b.conv(t0, 61, 7, 2, 3, True, zp_out=-100)
    t2 = b.maxpool(t1, 3, 2, 1)
    t3 = b.conv(t2, 64, 1, 1, 0, True)
    b.fc(b.gap(t3), 5)
    x = np.random.default_rng(7).integers(0, 256, size=(3, h, w)).astype(np.uint8)
    _check_all_tensors(isr, b.blob(), x, 64, sample=3, chunk=5)


def test_identity_residual_blocks_in_one_kernel(isr):
    """conv3x3 -> conv3x3 -> add with the block input, at the three shapes that run as one
    LDS-resident kernel (16 channels at 32x32, 32 at 16x16, 64 at 8x8): non-trivial zero-points
    on every tensor, ReLU on and off, power-of-two multipliers (rounding ties) in one block,
    7 copies (ragged against 2 and 4 images per workgroup)."""
    _say("layer parity fused identity blocks")
    rng = np.random.default_rng(71)
    b = NetBuilder(rng=np.random.default_rng(72), in_shape=(3, 32, 32), num_classes=6)
    t = b.conv(b.tensor(3, 32, 32, 0, 74.0), 16, 3, 1, 1, True)
    def block(t, ch, relu1, relu_out, z1, z2, zo, pow2=False):
        m0 = np.full(ch, 1 << 30, dtype=np.int64) if pow2 else None
        u = b.conv(t, ch, 3, 1, 1, relu1, zp_out=z1, m0=m0, sh=np.full(ch, 9) if pow2 else None)
        u = b.conv(u, ch, 3, 1, 1, False, zp_out=z2)
        if pow2:
            return b.add(t, u, relu_out, ma=1 << 19, mb=1 << 19, sh=20, zp_out=zo)
        return b.add(t, u, relu_out, zp_out=zo)
    t = block(t, 16, True, True, -128, 0, -128)
    t = block(t, 16, False, False, 7, -5, 3)
    t = block(t, 16, True, True, -100, 9, -120, pow2=True)
    t = b.conv(t, 32, 3, 2, 1, True)
    t = block(t, 32, True, False, -128, 4, -2)
    t = block(t, 32, False, True, 11, 0, -128, pow2=True)
    t = b.conv(t, 64, 3, 2, 1, True)
    t = block(t, 64, True, True, -128, 0, -128)
    t = block(t, 64, False, False, -9, 13, 6)
    b.fc(b.gap(t), 6)
    blob = b.blob()
    x = np.random.default_rng(11).integers(0, 256, size=(3, 32, 32)).astype(np.uint8)
    _check_all_tensors(isr, blob, x, 64, sample=4, chunk=3)
    m = _load(isr, blob, 7)
    om = oracle.Model(blob)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 2, 1, 1, 100, 7)
    olg, oam, ocnt = om.mc(x, 64, 2, 1, 1, 100, 7)
    assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
    m.close()


def test_downsampling_residual_blocks_in_one_kernel(isr):
    """conv3x3 stride 2 -> conv3x3 with a 1x1 stride-2 projection shortcut and the add, at
    the two shapes that run as one LDS-resident kernel (16 -> 32 channels at 32x32 -> 16x16,
    32 -> 64 at 16x16 -> 8x8): zero-points on every tensor, ReLU on and off, a variant with
    power-of-two multipliers (rounding ties), 5 copies (ragged against 2 images per workgroup)."""
    _say("layer parity fused down-sampling blocks")
    for pow2 in (False, True):
        b = NetBuilder(rng=np.random.default_rng(101), in_shape=(3, 32, 32), num_classes=6)
        t = b.conv(b.tensor(3, 32, 32, 0, 74.0), 16, 3, 1, 1, True, zp_out=-128 if not pow2 else -90)
        def down(x, ch, z1, z2, zp, zo, relu1, relu_out):
            kw = dict(m0=np.full(ch, 1 << 30, dtype=np.int64), sh=np.full(ch, 8)) if pow2 else {}
            u = b.conv(x, ch, 3, 2, 1, relu1, zp_out=z1, **kw)
            u = b.conv(u, ch, 3, 1, 1, False, zp_out=z2, **kw)
            r = b.conv(x, ch, 1, 2, 0, False, zp_out=zp)
            if pow2:
                return b.add(u, r, relu_out, ma=1 << 19, mb=1 << 19, sh=20, zp_out=zo)
            return b.add(u, r, relu_out, zp_out=zo)
        t = down(t, 32, -128, 0, 0, -128, True, True)
        t = down(t, 64, 11, -7, 5, 3, False, False)
        b.fc(b.gap(t), 6)
        blob = b.blob()
        x = np.random.default_rng(14).integers(0, 256, size=(3, 32, 32)).astype(np.uint8)
        _check_all_tensors(isr, blob, x, 64, sample=3, chunk=3)
        m = _load(isr, blob, 5)
        om = oracle.Model(blob)
        lg, am, cnt = isr.isr_debug_forward(m, x, 32, 6, 1, 1, 40, 5)
        olg, oam, ocnt = om.mc(x, 32, 6, 1, 1, 40, 5)
        assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
        m.close()


@pytest.mark.parametrize("shape", [(30, 20), (28, 28), (5, 40)])
def test_bottleneck_blocks_in_one_kernel(isr, shape):
    """conv1x1 -> conv3x3 (64 middle channels) [-> conv1x1 + add with the block input] as one
    kernel working on 14 x 14 pixel tiles: images that leave ragged tiles in both directions,
    one exactly two tiles wide and one lower than a tile; block widths 64 / 128 / 256 (one to
    four K steps); zero-points on every tensor, ReLU on and off, a block with power-of-two
    multipliers (rounding ties), a block whose residual comes from a projection (head only)."""
    h, w = shape
    _say(f"layer parity fused bottleneck blocks {h}x{w}")
    b = NetBuilder(rng=np.random.default_rng(81), in_shape=(3, h, w), num_classes=5)
    t = b.conv(b.tensor(3, h, w, 0, 74.0), 64, 3, 1, 1, True)
    def block(x, cx, z1, z2, z3, zo, relu12=True, relu_out=True, pow2=False, project=False):
        kw = dict(m0=np.full(64, 1 << 30, dtype=np.int64), sh=np.full(64, 9)) if pow2 else {}
        u = b.conv(x, 64, 1, 1, 0, relu12, zp_out=z1, **kw)
        u = b.conv(u, 64, 3, 1, 1, relu12, zp_out=z2, **kw)
        if project:
            r = b.conv(x, cx, 1, 1, 0, False, zp_out=5)
            u = b.conv(u, cx, 1, 1, 0, False, zp_out=z3)
            return b.add(r, u, relu_out, zp_out=zo)
        u = b.conv(u, cx, 1, 1, 0, False, zp_out=z3)
        if pow2:
            return b.add(x, u, relu_out, ma=1 << 19, mb=1 << 19, sh=20, zp_out=zo)
        return b.add(x, u, relu_out, zp_out=zo)
    t = block(t, 64, -128, -128, 0, -128)
    t = block(t, 256, -100, 7, 3, -128, project=True)
    t = block(t, 256, -128, -128, 0, -128)
    t = block(t, 256, 9, -20, -6, 11, relu12=False, relu_out=False)
    t = block(t, 256, -128, -128, 4, -128, pow2=True)
    t = b.conv(t, 128, 1, 1, 0, True)
    t = block(t, 128, -128, -90, 0, -128)
    b.fc(b.gap(t), 5)
    blob = b.blob()
    x = np.random.default_rng(12).integers(0, 256, size=(3, h, w)).astype(np.uint8)
    _check_all_tensors(isr, blob, x, 64, sample=2, chunk=3)
    m = _load(isr, blob, 5)
    om = oracle.Model(blob)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 3, 1, 1, 50, 5)
    olg, oam, ocnt = om.mc(x, 64, 3, 1, 1, 50, 5)
    assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
    m.close()


@pytest.mark.parametrize("shape", [(30, 20), (28, 28), (5, 40)])
def test_bottleneck_blocks_with_128_middle_channels_in_one_kernel(isr, shape):
    """conv1x1 -> conv3x3 (128 middle channels) -> conv1x1 + add with the block input as one kernel on
    14 x 14 pixel tiles: images with ragged tiles in both directions, one exactly two tiles wide, one
    lower than a tile; block widths 512 / 256 / 192 (eight, four and three K steps; 192 leaves the
    last round of output-channel passes to two of the four waves); zero-points on every tensor, ReLU
    on and off, a block with power-of-two multipliers (rounding ties)."""
    h, w = shape
    _say(f"layer parity fused bottleneck blocks, 128 middle channels, {h}x{w}")
    b = NetBuilder(rng=np.random.default_rng(83), in_shape=(3, h, w), num_classes=5)
    t = b.conv(b.tensor(3, h, w, 0, 74.0), 64, 3, 1, 1, True)
    t = b.conv(t, 512, 1, 1, 0, True)
    def block(x, cx, z1, z2, z3, zo, relu12=True, relu_out=True, pow2=False):
        kw = dict(m0=np.full(128, 1 << 30, dtype=np.int64), sh=np.full(128, 9)) if pow2 else {}
        u = b.conv(x, 128, 1, 1, 0, relu12, zp_out=z1, **kw)
        u = b.conv(u, 128, 3, 1, 1, relu12, zp_out=z2, **kw)
        u = b.conv(u, cx, 1, 1, 0, False, zp_out=z3)
        if pow2:
            return b.add(x, u, relu_out, ma=1 << 19, mb=1 << 19, sh=20, zp_out=zo)
        return b.add(x, u, relu_out, zp_out=zo)
    t = block(t, 512, -128, -128, 0, -128)
    t = block(t, 512, 9, -20, -6, 11, relu12=False, relu_out=False)
    t = block(t, 512, -128, -128, 4, -128, pow2=True)
    t = b.conv(t, 256, 1, 1, 0, True)
    t = block(t, 256, -100, 7, 3, -128)
    t = b.conv(t, 192, 1, 1, 0, True)
    t = block(t, 192, -128, -90, 0, -128)
    b.fc(b.gap(t), 5)
    blob = b.blob()
    x = np.random.default_rng(15).integers(0, 256, size=(3, h, w)).astype(np.uint8)
    _check_all_tensors(isr, blob, x, 64, sample=2, chunk=3, min_fused=5, fusion=2)
    m = _load(isr, blob, 5)
    isr.isr_set_fusion(m, 2)
    om = oracle.Model(blob)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 3, 1, 1, 50, 5)
    olg, oam, ocnt = om.mc(x, 64, 3, 1, 1, 50, 5)
    assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
    isr.isr_set_fusion(m, False)
    lg2, _, _ = isr.isr_debug_forward(m, x, 64, 3, 1, 1, 50, 5)
    assert np.array_equal(lg2, olg)
    m.close()


def test_residual_computed_by_a_second_convolution(isr):
    """Projection-shortcut pattern: the residual of an add is the output of a 1x1
    convolution issued right before the add's other convolution; the fused plan then
    computes both in one kernel and never stores the residual.  Main convolution 3x3
    (gather), 1x1 stride 2 (gather) and 1x1 stride 1 (plain GEMM); channel counts that
    leave a ragged last M tile; K of the two convolutions different; 29 copies."""
    _say("layer parity dual-convolution residual add")
    rng = np.random.default_rng(61)
    b = NetBuilder(rng=np.random.default_rng(62), in_shape=(3, 12, 12), num_classes=8)
    t0 = b.tensor(3, 12, 12, 0, 74.0)
    t1 = b.conv(t0, 64, 3, 1, 1, True)
    t2 = b.conv(t1, 192, 1, 1, 0, False, zp_out=11)          # residual producer (K = 64)
    t3 = b.conv(t1, 192, 3, 1, 1, False, zp_out=-9)          # main, K = 576
    t4 = b.add(t2, t3, True)
    u = b.conv(t4, 128, 3, 2, 1, True)                       # 6 x 6
    r = b.conv(u, 320, 1, 1, 0, False)                       # residual producer (K = 128)
    mn = b.conv(t4, 320, 1, 2, 0, False)                     # main: 1x1 stride 2, K = 192
    t5 = b.add(mn, r, True)                                  # residual is the second operand here
    r2 = b.conv(t5, 64, 1, 1, 0, False)                      # 64 output channels: the 64 x 256 tile
    m2 = b.conv(t5, 64, 1, 1, 0, True)
    t6 = b.add(r2, m2, False, ma=-500000, mb=800000, sh=20)
    b.fc(b.gap(t6), 8)
    blob = b.blob()
    x = np.random.default_rng(10).integers(0, 256, size=(3, 12, 12)).astype(np.uint8)
    _check_all_tensors(isr, blob, x, 64, sample=1, chunk=3)
    m = _load(isr, blob, 29)
    om = oracle.Model(blob)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 1, 1, 1, 0, 29)
    olg, oam, ocnt = om.mc(x, 64, 1, 1, 1, 0, 29)
    assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
    isr.isr_set_fusion(m, False)
    lg2, _, _ = isr.isr_debug_forward(m, x, 64, 1, 1, 1, 0, 29)
    assert np.array_equal(lg2, olg)
    m.close()


def test_exact_halves_in_both_requantisations(isr):
    """Power-of-two multipliers make acc * M0 and the residual sum land on exact halves
    all the time (negative ones included), so the rounding's sign correction decides
    results: layers that cannot take the tie-free shortcut, next to ones that can."""
    _say("layer parity with rounding ties")
    rng = np.random.default_rng(41)
    b = NetBuilder(rng=np.random.default_rng(42), in_shape=(3, 16, 16), num_classes=6)
    t0 = b.tensor(3, 16, 16, 0, 74.0)
    m_pow2 = np.full(64, 1 << 30, dtype=np.int64)
    m_mixed = np.where(np.arange(64) % 2 == 0, 1 << 30, (1 << 30) + 12345).astype(np.int64)
    t1 = b.conv(t0, 64, 3, 1, 1, True, m0=m_pow2, sh=np.full(64, 9))
    t2 = b.conv(t1, 64, 3, 1, 1, False, m0=m_mixed, sh=np.full(64, 10), zp_out=3)
    t3 = b.conv(t2, 64, 1, 1, 0, False, m0=m_pow2, sh=np.full(64, 8), zp_out=-7)
    t4 = b.add(t2, t3, True, ma=1 << 19, mb=1 << 19, sh=20, zp_out=-20)      # ties in the fused add
    t5 = b.conv(t4, 128, 1, 1, 0, False, sh=rng.integers(6, 9, size=128))
    t6 = b.conv(t5, 128, 3, 1, 1, False, m0=np.full(128, 3 << 29, dtype=np.int64), sh=np.full(128, 9))
    t7 = b.add(t5, t6, False, ma=700001, mb=-(1 << 20), sh=20, zp_out=5)
    b.fc(b.gap(t7), 6)
    x = np.random.default_rng(8).integers(0, 256, size=(3, 16, 16)).astype(np.uint8)
    _check_all_tensors(isr, b.blob(), x, 64, sample=2, chunk=3)


# ---- S6-S8: logits, votes, decisions -----------------------------------------

def test_config0_full_certify_and_predict(isr):
    _say("config 0 full certify")
    blob, x = synth.build_model(0), synth.make_image(0, 1)
    om = oracle.Model(blob)
    m = _load(isr, blob, 300)
    res, c0, c1 = isr.isr_certify(m, x, 32, 100, 1000, ALPHA, seed=0, image_id=0)
    cls, rad, p_l, k, oc0, oc1 = oracle.certify(om, x, 32, 100, 1000, ALPHA, seed=0, image=0)
    assert np.array_equal(c0, oc0) and np.array_equal(c1, oc1)
    assert res.cls == cls and res.n_top == k
    assert res.p_lower == pytest.approx(p_l, rel=1e-12)
    assert res.radius == pytest.approx(rad, rel=1e-9)
    # integer-only tail (Thm 3.2, proof steps 2-3) from the device tallies, in the same call
    assert (res.cls, res.radius_int, res.radius_sq_int) == oracle.stats.certify_decision_integer(oc0, oc1, 32, 1000, ALPHA)
    assert res.radius_int > 0 and res.radius_sq_int == res.radius_int ** 2 and res.radius_int <= res.radius
    lg, am, cnt = isr.isr_debug_forward(m, x, 32, 0, 0, 1, 0, 1000)
    olg, oam, ocnt = om.mc(x, 32, 0, 0, 1, 0, 1000)
    assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
    assert np.array_equal(cnt, c1)
    pres, pc = isr.isr_predict(m, x, 32, 1000, ALPHA, seed=9, image_id=2)
    pcls, pv, n_a, n_b, opc = oracle.predict(om, x, 32, 1000, ALPHA, seed=9, image=2)
    assert np.array_equal(pc, opc) and (pres.cls, pres.n_top, pres.n_second) == (pcls, n_a, n_b)
    assert pres.p_lower == pytest.approx(pv, rel=1e-9, abs=1e-300)
    m.close()


def test_votes_invariant_to_chunk_size_and_ragged_tail(isr):
    _say("chunk invariance")
    blob, x = synth.build_model(0), synth.make_image(0, 1)
    ref = None
    for chunk in (1, 7, 64, 257, 1000):
        m = _load(isr, blob, chunk)
        lg, am, cnt = isr.isr_debug_forward(m, x, 128, 4, 5, 0, 3, 333)
        cur = (lg.copy(), am.copy(), cnt.copy())
        if ref is None:
            ref = cur
            om = oracle.Model(blob)
            olg, oam, ocnt = om.mc(x, 128, 4, 5, 0, 3, 333)
            assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
        else:
            assert all(np.array_equal(a, b) for a, b in zip(ref, cur))
        assert np.array_equal(np.bincount(am, minlength=m.classes).astype(np.uint32), cnt)
        m.close()


def test_fused_and_unfused_kernels_agree(isr):
    """Residual adds folded into the convolution epilogue vs one kernel per op:
    identical logits, and both equal the oracle."""
    _say("fusion on/off")
    for cfg, size, sigma in ((1, None, 64), (3, 64, 128)):
        blob = synth.build_model(cfg, size=size)
        shape = (3, size, size) if size else None
        x = synth.make_image(cfg, 2, shape=shape)
        m = _load(isr, blob, 16)
        a = isr.isr_debug_forward(m, x, sigma, 8, 2, 1, 40, 24)
        isr.isr_set_fusion(m, False)
        b = isr.isr_debug_forward(m, x, sigma, 8, 2, 1, 40, 24)
        isr.isr_set_fusion(m, True)
        assert all(np.array_equal(u, v) for u, v in zip(a, b))
        om = oracle.Model(blob)
        olg, oam, ocnt = om.mc(x, sigma, 8, 2, 1, 40, 24)
        assert np.array_equal(a[0], olg) and np.array_equal(a[1], oam) and np.array_equal(a[2], ocnt)
        m.close()


@pytest.mark.parametrize("item,sigma", [(1, 32), (1, 64), (1, 128), (2, 32), (2, 64), (2, 128)])
def test_resnet20_logits_and_votes(isr, item, sigma):
    """Two images at the three noise levels of the CIFAR-shaped workload: every selection sample
    (n0 = 100), the first 5000 and the last 300 estimation samples of an n = 100000 run --
    per-sample logits, argmax and tallies against the oracle."""
    _say(f"resnet20 logits parity image {item} sigma {sigma}")
    blob = synth.build_model(1)
    om = oracle.Model(blob)
    m = _load(isr, blob, 2048)
    x = synth.make_image(1, item)
    for phase, begin, count in ((0, 0, 100), (1, 0, 5000), (1, 99700, 300)):
        lg, am, cnt = isr.isr_debug_forward(m, x, sigma, 0, item, phase, begin, count)
        olg, oam, ocnt = om.mc(x, sigma, 0, item, phase, begin, count)
        assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
    m.close()


def test_resnet20_certify_and_predict_end_to_end(isr):
    """Alg. 1 and Alg. 2 as whole calls on ResNet-20 (n0 = 100, n = 1500; chunk 700 leaves a
    ragged last chunk): tallies, selected class, bound and radius against the oracle."""
    _say("resnet20 end-to-end certify / predict")
    blob = synth.build_model(1)
    om = oracle.Model(blob)
    m = _load(isr, blob, 700)
    x = synth.make_image(1, 4)
    res, c0, c1 = isr.isr_certify(m, x, 64, 100, 1500, ALPHA, seed=11, image_id=4)
    cls, rad, p_l, k, oc0, oc1 = oracle.certify(om, x, 64, 100, 1500, ALPHA, seed=11, image=4)
    assert np.array_equal(c0, oc0) and np.array_equal(c1, oc1)
    assert res.cls == cls and res.n_top == k
    assert res.p_lower == pytest.approx(p_l, rel=1e-12)
    assert res.radius == pytest.approx(rad, rel=1e-9)
    assert (res.cls, res.radius_int, res.radius_sq_int) == oracle.stats.certify_decision_integer(oc0, oc1, 64, 1500, ALPHA)
    pres, pc = isr.isr_predict(m, x, 128, 333, ALPHA, seed=12, image_id=4)
    pcls, pv, n_a, n_b, opc = oracle.predict(om, x, 128, 333, ALPHA, seed=12, image=4)
    assert np.array_equal(pc, opc) and (pres.cls, pres.n_top, pres.n_second) == (pcls, n_a, n_b)
    assert pres.p_lower == pytest.approx(pv, rel=1e-9, abs=1e-300)
    m.close()


def test_resnet110_logits(isr):
    """1000 noisy copies of the deep narrow net inside bench.py's chunk of 4096 (the block-chain
    kernels with every workgroup full and a ragged last one): logits, argmax, tallies."""
    _say("resnet110 logits parity")
    blob = synth.build_model(2)
    om = oracle.Model(blob)
    m = _load(isr, blob, 4096)
    x = synth.make_image(2, 1)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 0, 1, 1, 500, 1000)
    olg, oam, ocnt = om.mc(x, 64, 0, 1, 1, 500, 1000)
    assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
    m.close()


@pytest.mark.parametrize("sigma", [32, 64, 128, 256])
def test_resnet50_full_size_logits(isr, sigma):
    """ResNet-50 at 224x224, 101 classes: 64 sample indices per noise level in four disjoint
    ranges -- the selection loop, the start, the middle and the last indices of a
    100000-sample estimation loop -- on two images."""
    _say(f"resnet50 224 logits parity sigma {sigma}")
    blob = synth.build_model(4)
    om = oracle.Model(blob)
    m = _load(isr, blob, 16)
    for item, phase, begin, count in ((1, 0, 0, 16), (1, 1, 0, 16), (2, 1, 50000, 16), (2, 1, 99984, 16)):
        x = synth.make_image(4, item)
        lg, am, cnt = isr.isr_debug_forward(m, x, sigma, 0, item, phase, begin, count)
        olg, oam, ocnt = om.mc(x, sigma, 0, item, phase, begin, count)
        assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
    m.close()


# copies of a 668-copy chunk that sit on the boundaries of the kernels' pixel tiles: first and last
# copy, both sides of the 64-, 128- and 256-copy marks (whole tiles at 7x7 ... 56x56 pixels per
# copy), the middle of the chunk (second round of workgroups), and the ragged end
CHUNK668_COPIES = (0, 1, 2, 31, 32, 63, 64, 65, 127, 128, 191, 192, 255, 256, 257, 300, 333, 334, 335, 400,
                   447, 448, 511, 512, 513, 575, 576, 639, 640, 665, 666, 667)


@pytest.mark.parametrize("sigma,item", [(32, 1), (256, 3)])
def test_resnet50_chunk_668_sampled_copies(isr, sigma, item):
    """bench.py's launch configuration (chunks of 668 copies, library-chosen tiles) at the
    smallest and the largest noise level of the headline sweep: 32 copies spread over the
    chunk, chosen on tile and workgroup-round boundaries, against the oracle one by one."""
    _say(f"resnet50 224 parity at chunk 668, sigma {sigma}")
    blob = synth.build_model(4)
    om = oracle.Model(blob)
    m = _load(isr, blob, 668)
    x = synth.make_image(4, item)
    begin = 99332                                # the last full chunk of an n = 100000 run
    lg, am, cnt = isr.isr_debug_forward(m, x, sigma, 0, item, 1, begin, 668)
    assert int(cnt.sum()) == 668 and np.array_equal(np.bincount(am, minlength=len(cnt)), cnt)
    olg, oam = _oracle_at(om, x, sigma, 0, item, 1, [begin + i for i in CHUNK668_COPIES])
    for j, i in enumerate(CHUNK668_COPIES):
        assert np.array_equal(lg[i], olg[j]) and am[i] == oam[j], i
    m.close()


def test_resnet50_in_the_benchmarked_launch_configuration(isr):
    """bench.py's configuration: chunks of 668 noisy copies, library-chosen tiles
    (256x256, 128x256, 128x128 and the fused first layer all occur).  One full chunk
    on the device; the oracle checks sampled copies one by one, the vote counts must
    add up, and forcing each tile must not change a single logit."""
    _say("resnet50 224 parity at chunk 668")
    blob = synth.build_model(4)
    om = oracle.Model(blob)
    m = _load(isr, blob, 668)
    x = synth.make_image(4, 2)
    lg, am, cnt = isr.isr_debug_forward(m, x, 128, 0, 2, 1, 20000, 668)
    assert int(cnt.sum()) == 668 and np.array_equal(np.bincount(am, minlength=len(cnt)), cnt)
    assert np.array_equal(am, np.argmax(lg, axis=1))
    picks = (0, 100, 255, 256, 333, 334, 512, 667)
    olg, oam = _oracle_at(om, x, 128, 0, 2, 1, [20000 + i for i in picks])
    for j, i in enumerate(picks):
        assert np.array_equal(lg[i], olg[j]) and am[i] == oam[j], i
    for tile in (1, 2, 3, 4, 5, 6, 7):
        _say(f"  forced tile {tile}")
        isr.isr_set_conv_tile(m, tile)
        lg2, am2, cnt2 = isr.isr_debug_forward(m, x, 128, 0, 2, 1, 20000, 668)
        assert np.array_equal(lg2, lg) and np.array_equal(cnt2, cnt)
    m.close()


@pytest.mark.parametrize("cfg,chunk", [(1, 8192), (2, 4096)])
def test_cifar_nets_in_the_benchmarked_launch_configuration(isr, cfg, chunk):
    """bench.py's configuration for the narrow nets: one full chunk (8192 / 4096 noisy
    copies) through the LDS-resident block kernels.  Votes must add up, sampled copies
    (first, last, and a few in between) are checked by the oracle one by one, and the
    op-by-op plan must give the same logits for the whole chunk."""
    _say(f"config {cfg} parity at chunk {chunk}")
    blob = synth.build_model(cfg)
    om = oracle.Model(blob)
    m = _load(isr, blob, chunk)
    x = synth.make_image(cfg, 3)
    begin = 100000 - chunk                      # the last chunk of an n = 100000 run
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 0, 3, 1, begin, chunk)
    assert int(cnt.sum()) == chunk and np.array_equal(np.bincount(am, minlength=len(cnt)), cnt)
    assert np.array_equal(am, np.argmax(lg, axis=1))
    for i in (0, 1, 4095, chunk // 2 + 1, chunk - 2, chunk - 1):
        olg, oam, _ = om.mc(x, 64, 0, 3, 1, begin + i, 1)
        assert np.array_equal(lg[i], olg[0]) and am[i] == oam[0], i
    isr.isr_set_fusion(m, False)
    lg2, am2, cnt2 = isr.isr_debug_forward(m, x, 64, 0, 3, 1, begin, chunk)
    assert np.array_equal(lg2, lg) and np.array_equal(cnt2, cnt)
    m.close()


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5, 6, 7])
def test_every_conv_tile_against_the_oracle(isr, tile):
    """Layers deep enough for 128-byte K steps and for every output tile of the
    direct-to-LDS kernel, channel counts that leave a ragged last M tile, a ragged
    last pixel tile (37 copies of a 12x12 image), strides; tile forced through the C ABI."""
    _say(f"conv tile {tile} parity")
    rng = np.random.default_rng(51)
    b = NetBuilder(rng=np.random.default_rng(52), in_shape=(3, 12, 12), num_classes=9)
    t0 = b.tensor(3, 12, 12, 0, 74.0)
    t1 = b.conv(t0, 128, 3, 1, 1, True)
    t2 = b.conv(t1, 128, 3, 1, 1, True)                 # K = 1152
    t3 = b.conv(t2, 256, 1, 1, 0, True)                 # K = 128
    t4 = b.conv(t3, 256, 3, 1, 1, True)                 # K = 2304, 128-byte steps
    t5 = b.conv(t4, 512, 1, 1, 0, False)                # K = 256
    t6 = b.conv(t5, 272, 1, 1, 0, True)                 # K = 512, ragged M
    t7 = b.conv(t6, 320, 3, 2, 1, True)                 # K = 2448 (not a multiple of 128), stride 2, ragged M
    t8 = b.conv(t7, 1024, 1, 1, 0, True)                # K = 320
    t9 = b.conv(t8, 256, 1, 1, 0, True)                 # K = 1024, 128-byte steps, 1x1
    b.fc(b.gap(t9), 9)
    blob = b.blob()
    x = np.random.default_rng(9).integers(0, 256, size=(3, 12, 12)).astype(np.uint8)
    m = _load(isr, blob, 37)
    isr.isr_set_conv_tile(m, tile)
    om = oracle.Model(blob)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 1, 1, 1, 5, 37)
    olg, oam, ocnt = om.mc(x, 64, 1, 1, 1, 5, 37)
    assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
    m.close()
    if tile == 4:
        _check_all_tensors(isr, blob, x, 64)


@pytest.mark.parametrize("in_shape,stride,copies", [((28, 28), 2, 37), ((28, 28), 4, 150), ((28, 28), 1, 11), ((12, 20), 2, 61),
                                                    ((36, 124), 4, 13), ((10, 4), 2, 333)])
def test_3x3_layers_with_staged_pixel_rows_against_the_oracle(isr, in_shape, stride, copies):
    """The 3x3 kernel that stages a tile's pixel rows once per channel slice (forced tile 7) and addresses the
    nine taps as shifted rows: its tiles of 256 consecutive pixels straddle image rows and whole images, so
    every border case of the shift arithmetic occurs -- square and non-square maps, the widest map its staging
    buffer takes (31), a map narrower than the kernel, a ragged last tile.  128-channel (64-byte slices, two
    slices) and 256-channel tiles (128-byte slices; one and two slices; a ragged second M tile).  The final
    layer is fully connected over all pixels, so one wrong activation anywhere changes the logits."""
    h, w = in_shape                                     # maps of 14x14, 7x7, 28x28, 6x10, 9x31, 5x2 behind the strided first layer
    _say(f"staged-rows 3x3 parity, input {h}x{w} stride {stride}, {copies} copies")
    b = NetBuilder(rng=np.random.default_rng(77 + h), in_shape=(3, h, w), num_classes=9)
    t0 = b.tensor(3, h, w, 0, 74.0)
    t1 = b.conv(t0, 128, 3, stride, 1, True)
    t2 = b.conv(t1, 128, 3, 1, 1, True, zp_out=-100)    # 128-channel tile, K = 1152
    t3 = b.conv(t2, 256, 3, 1, 1, False, zp_out=7)      # 256-channel tile, one slice of 128 channels
    t4 = b.conv(t3, 272, 3, 1, 1, True)                 # two slices, ragged second M tile
    t5 = b.conv(t4, 16, 1, 1, 0, True)
    b.fc(t5, 9)
    blob = b.blob()
    x = np.random.default_rng(h * 100 + w).integers(0, 256, size=(3, h, w)).astype(np.uint8)
    om = oracle.Model(blob)
    olg, oam, ocnt = om.mc(x, 64, 2, 1, 1, 3, copies)
    m = _load(isr, blob, copies)
    for tile in (7, 0):
        isr.isr_set_conv_tile(m, tile)
        lg, am, cnt = isr.isr_debug_forward(m, x, 64, 2, 1, 1, 3, copies)
        assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt), tile
    m.close()


def test_expand_add_and_next_reduce_in_one_kernel(isr):
    """The kernels that run a block's closing 1x1 (128 -> 512) + residual add and the next block's opening 1x1
    (512 -> 128, or 256 for the first block of a next stage) on pixel tiles of all 512 channels.  Seven such pairs in a row (the last two with the 14x14 stage's 256 / 1024 channels): a first block whose residual is
    a stride-2 projection of the 256-channel block input issued after the closing convolution (the order of a
    ResNet-50), two identity blocks (the second with an add that meets exact halves, i.e. the other template
    instance; residual as first and as second operand), a projection block in the other order (projection
    first, stride 1), and an identity block followed by a 256-channel opening convolution.  Every tensor of one copy; then 1001 copies of a 6x6 map = 1127 tiles of 32 pixels for 512
    (256) persistent workgroups -- three and more tiles each, so the counted waits of the steady state run --
    with a ragged last tile, logits of a layer that is fully connected over all pixels, against the oracle.
    The timing report must name the kernels."""
    _say("expand + add + next reduce in one kernel")
    rng = np.random.default_rng(61)
    b = NetBuilder(rng=np.random.default_rng(62), in_shape=(3, 24, 24), num_classes=7)
    t0 = b.tensor(3, 24, 24, 0, 74.0)
    ta = b.conv(t0, 256, 3, 2, 1, True)                        # block input: 256 channels on 12x12
    u = b.conv(ta, 128, 1, 1, 0, True)
    u = b.conv(u, 128, 3, 2, 1, True)                          # 6x6
    u = b.conv(u, 512, 1, 1, 0, False, sh=rng.integers(7, 10, size=512))
    s_ = b.conv(ta, 512, 1, 2, 0, False, zp_out=-9)            # projection, stride 2, issued right before the add
    t1 = b.add(s_, u, True)
    t2 = b.conv(t1, 128, 1, 1, 0, True)                        # pair 0: projection + expand + add + t2
    t3 = b.conv(t2, 128, 3, 1, 1, True)
    t4 = b.conv(t3, 512, 1, 1, 0, False, zp_out=4, sh=rng.integers(7, 10, size=512))
    t5 = b.add(t1, t4, True)                                   # residual first
    t6 = b.conv(t5, 128, 1, 1, 0, True)                        # pair 1: t4 + add + t6
    t7 = b.conv(t6, 128, 3, 1, 1, True)
    t8 = b.conv(t7, 512, 1, 1, 0, False, sh=rng.integers(7, 10, size=512))
    t9 = b.add(t8, t5, True, ma=1 << 19, mb=1 << 19, sh=20, zp_out=-30)   # ties in the add, residual second
    t10 = b.conv(t9, 128, 1, 1, 0, True)                       # pair 2
    tb = b.conv(t10, 256, 1, 1, 0, True)                       # a block input of 256 channels on 6x6
    v = b.conv(tb, 128, 1, 1, 0, True)
    v = b.conv(v, 128, 3, 1, 1, True)
    s2 = b.conv(tb, 512, 1, 1, 0, False)                       # projection first ...
    v = b.conv(v, 512, 1, 1, 0, False, zp_out=11)              # ... the closing convolution right before the add
    t11 = b.add(v, s2, True, ma=1 << 19, mb=3 << 18, sh=20)
    t12 = b.conv(t11, 128, 1, 1, 0, True)                      # pair 3
    w_ = b.conv(t12, 128, 3, 1, 1, True)
    w_ = b.conv(w_, 512, 1, 1, 0, False)
    t13 = b.add(t11, w_, True)
    t14 = b.conv(t13, 256, 1, 1, 0, True)                      # pair 4: the next block has 256 middle channels
    # the 14 x 14 stage's shapes: 256 middle, 1024 block channels
    tc = b.conv(t14, 1024, 1, 1, 0, True)
    w_ = b.conv(tc, 256, 1, 1, 0, True)
    w_ = b.conv(w_, 256, 3, 1, 1, True)
    w_ = b.conv(w_, 1024, 1, 1, 0, False, zp_out=-3)
    t15 = b.add(tc, w_, True)
    t16 = b.conv(t15, 256, 1, 1, 0, True)                      # pair 5
    w_ = b.conv(t16, 256, 3, 1, 1, True)
    w_ = b.conv(w_, 1024, 1, 1, 0, False)
    t17 = b.add(w_, t15, True, ma=1 << 19, mb=1 << 19, sh=20)  # ties in the add
    t18 = b.conv(t17, 256, 1, 1, 0, True)                      # pair 6
    t19 = b.conv(t18, 16, 1, 1, 0, True)
    b.fc(t19, 7)
    blob = b.blob()
    x = np.random.default_rng(63).integers(0, 256, size=(3, 24, 24)).astype(np.uint8)
    _check_all_tensors(isr, blob, x, 64, sample=5, chunk=3)
    copies = 1001
    om = oracle.Model(blob)
    olg, oam, ocnt = om.mc(x, 64, 3, 2, 1, 7, copies)
    m = _load(isr, blob, copies)
    isr.isr_profile(m, 1)
    lg, am, cnt = isr.isr_debug_forward(m, x, 64, 3, 2, 1, 7, copies)
    assert np.array_equal(lg, olg) and np.array_equal(am, oam) and np.array_equal(cnt, ocnt)
    stats = {s["name"]: s["launches"] for s in isr.isr_profile_read(m)}
    assert stats.get("expand_reduce_kernel<128, 512, 128>", 0) == 2, stats
    assert stats.get("proj_expand_reduce_kernel<256, 128, 512, 128>", 0) == 2, stats
    assert stats.get("expand_reduce_kernel<128, 512, 256>", 0) == 1, stats
    assert stats.get("expand_reduce_kernel<256, 1024, 256>", 0) == 2, stats
    isr.isr_set_fusion(m, 0)                                   # one kernel per op gives the same
    lg0, am0, cnt0 = isr.isr_debug_forward(m, x, 64, 3, 2, 1, 7, copies)
    assert np.array_equal(lg0, olg) and np.array_equal(cnt0, ocnt)
    m.close()


# ---- many (image, sigma) pairs in one pass -------------------------------------

def _check_batch_against_oracle(isr, m, om, xs, items, n0, n, seed):
    res, c0, c1 = isr.isr_certify_batch(m, xs, items, n0, n, ALPHA, seed=seed)
    want = oracle.certify_batch(om, xs, items, n0, n, ALPHA, seed=seed)
    for i, (cls, rad, p_l, k, oc0, oc1) in enumerate(want):
        assert np.array_equal(c0[i], oc0) and np.array_equal(c1[i], oc1), (i, items[i])
        assert res[i].cls == cls and res[i].n_top == k
        assert res[i].p_lower == pytest.approx(p_l, rel=1e-12)
        assert res[i].radius == pytest.approx(rad, rel=1e-9)
        assert (res[i].cls, res[i].radius_int, res[i].radius_sq_int) == \
            oracle.stats.certify_decision_integer(oc0, oc1, items[i][1], n, ALPHA), (i, items[i])
    pres, pc = isr.isr_predict_batch(m, xs, items, n, ALPHA, seed=seed + 1)
    pwant = oracle.predict_batch(om, xs, items, n, ALPHA, seed=seed + 1)
    for i, (cls, pv, n_a, n_b, opc) in enumerate(pwant):
        assert np.array_equal(pc[i], opc), (i, items[i])
        assert (pres[i].cls, pres[i].n_top, pres[i].n_second) == (cls, n_a, n_b)
        assert pres[i].p_lower == pytest.approx(pv, rel=1e-9, abs=1e-300)
    return res, c0, c1


@pytest.mark.parametrize("chunk", [64, 1000])
def test_batched_pairs_config0(isr, chunk):
    """Six (image, sigma) pairs over five images, four noise levels, one image used
    twice: chunks smaller than a pair's run (64) and chunks spanning several pairs
    (1000), n0 and n no multiples of either.  Every pair against the oracle, and
    against the single-pair entry point."""
    _say(f"batched certify / predict, tiny net, chunk {chunk}")
    blob = synth.build_model(0)
    om = oracle.Model(blob)
    m = _load(isr, blob, chunk)
    xs = np.stack([synth.make_image(0, i) for i in range(1, 6)])
    items = [(0, 32, 0), (1, 64, 7), (0, 128, 3), (4, 32, 9), (2, 1024, 11), (3, 64, 0)]
    res, c0, c1 = _check_batch_against_oracle(isr, m, om, xs, items, 37, 250, seed=5)
    for i, (img, sigma, image_id) in enumerate(items):
        one, s0, s1 = isr.isr_certify(m, xs[img], sigma, 37, 250, ALPHA, seed=5, image_id=image_id)
        assert np.array_equal(s0, c0[i]) and np.array_equal(s1, c1[i])
        assert (one.cls, one.n_top, one.radius, one.p_lower) == (res[i].cls, res[i].n_top, res[i].radius, res[i].p_lower)
    m.close()


def test_batched_pairs_resnet20_small_n(isr):
    """Prediction-sized runs (n = 100) of eight pairs in chunks of 512 on ResNet-20:
    five pairs share a chunk; a second call with fewer pairs reuses the buffers."""
    _say("batched certify / predict, resnet20")
    blob = synth.build_model(1)
    om = oracle.Model(blob)
    m = _load(isr, blob, 512)
    xs = np.stack([synth.make_image(1, i) for i in range(1, 5)])
    items = [(i % 4, (32, 64, 128)[i % 3], i) for i in range(8)]
    _check_batch_against_oracle(isr, m, om, xs, items, 20, 100, seed=0)
    _check_batch_against_oracle(isr, m, om, xs, items[5:7], 10, 33, seed=2)
    m.close()


@pytest.mark.parametrize("chunk", [16, 200])
def test_batched_pairs_with_the_noise_drawn_inside_the_first_layer(isr, chunk):
    """A net whose first layer is the 7x7/2 convolution + max pooling kernel, which draws the noisy
    input rows itself (no separate noise launch, the noisy copy is never stored): batched pairs over
    four images and three noise levels, chunks that split a pair's run (16) and chunks that span
    several pairs (200); every pair against the oracle and against the single-pair call; per-sample
    logits of a range against the oracle with and without the fusions."""
    _say(f"batched certify / predict, noise drawn in the first layer, chunk {chunk}")
    b = NetBuilder(rng=np.random.default_rng(33), in_shape=(3, 36, 28), num_classes=5)
    t1 = b.conv(b.tensor(3, 36, 28, 0, 74.0), 61, 7, 2, 3, True, zp_out=-100)
    t3 = b.conv(b.maxpool(t1, 3, 2, 1), 64, 1, 1, 0, True)
    b.fc(b.gap(t3), 5)
    blob = b.blob()
    om = oracle.Model(blob)
    m = _load(isr, blob, chunk)
    xs = np.stack([np.random.default_rng(40 + i).integers(0, 256, size=(3, 36, 28)).astype(np.uint8) for i in range(4)])
    items = [(0, 32, 0), (1, 64, 7), (3, 256, 3), (2, 32, 9), (0, 64, 11)]
    res, c0, c1 = _check_batch_against_oracle(isr, m, om, xs, items, 13, 57, seed=6)
    for i, (img, sigma, image_id) in enumerate(items):
        one, s0, s1 = isr.isr_certify(m, xs[img], sigma, 13, 57, ALPHA, seed=6, image_id=image_id)
        assert np.array_equal(s0, c0[i]) and np.array_equal(s1, c1[i])
    lg, am, cnt = isr.isr_debug_forward(m, xs[1], 128, 9, 4, 1, 99990, 37)
    olg, oam, ocnt = om.mc(xs[1], 128, 9, 4, 1, 99990, 37)
    assert np.array_equal(lg, olg) and np.array_equal(cnt, ocnt)
    isr.isr_set_fusion(m, False)
    lg2, _, _ = isr.isr_debug_forward(m, xs[1], 128, 9, 4, 1, 99990, 37)
    assert np.array_equal(lg2, olg)
    # the noisy copy itself is still available through the debug hook (the separate noise kernel)
    isr.isr_set_fusion(m, True)
    got = isr.isr_debug_noisy(m, xs[2], 64, 6, 9, 1, 5, 3)
    for s in range(3):
        assert np.array_equal(got[s], oracle.noisy(xs[2], 64, 6, 9, 1, 5 + s))
    m.close()


def test_batched_call_argument_errors(isr):
    blob = synth.build_model(0)
    m = _load(isr, blob, 32)
    xs = np.stack([synth.make_image(0, i) for i in range(1, 3)])
    for items in ([(2, 32, 0)], [(0, 0, 0)], [(0, 1025, 0)], [(0, s, 0) for s in range(1, 10)]):
        with pytest.raises(isr.IsrError) as e:
            isr.isr_predict_batch(m, xs, items, 10, ALPHA)
        assert e.value.status == isr.ISR_ERR_ARG
    with pytest.raises(isr.IsrError):
        isr.isr_certify_batch(m, xs, [(0, 32, 0)], 0, 10, ALPHA)
    # eight distinct noise levels are the limit and work
    res, c = isr.isr_predict_batch(m, xs, [(1, s, 3) for s in (1, 2, 3, 4, 5, 6, 7, 8)], 40, ALPHA)
    assert all(int(row.sum()) == 40 for row in c)
    m.close()


# ---- argument handling --------------------------------------------------------

def test_error_paths(isr):
    blob, x = synth.build_model(0), synth.make_image(0, 1)
    m = isr.isr_load_model(blob)
    with pytest.raises(isr.IsrError) as e:
        isr.isr_certify(m, x, 32, 10, 10, ALPHA)
    assert e.value.status == isr.ISR_ERR_WORKSPACE
    isr.isr_set_workspace(m, 16)
    for kwargs in (dict(sigma=0), dict(sigma=1025), dict(n0=0), dict(n=0), dict(alpha=0.0), dict(alpha=1.0)):
        args = dict(sigma=32, n0=10, n=10, alpha=ALPHA)
        args.update(kwargs)
        with pytest.raises(isr.IsrError) as e:
            isr.isr_certify(m, x, args["sigma"], args["n0"], args["n"], args["alpha"])
        assert e.value.status == isr.ISR_ERR_ARG
    with pytest.raises(isr.IsrError):
        isr.isr_debug_noisy(m, x, 32, 0, 0, 0, 0, 17)   # more than the chunk
    with pytest.raises(isr.IsrError):
        isr.isr_load_model(blob[:-8])
    m.close()
