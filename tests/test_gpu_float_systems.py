"""GPU parity of the paper's two floating-point comparison systems (FloatRS-quant, FloatRS-fp) against
the CPU oracle on the same seeded inputs.  The binary32 noise, the rounded inputs and everything the
int8 network computes from them are bit-exact; the fp32 network is compared with the oracle's
binary64 evaluation of the same network within a tolerance derived from fp32 summation, and its
class decisions wherever the oracle's margin exceeds that tolerance."""
import ctypes

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

QUANT, FP = oracle.FLOATRS_QUANT, oracle.FLOATRS_FP
ALPHA = 0.001
# fp32 network against the binary64 oracle: every tensor element within REL of the tensor's largest
# magnitude.  A convolution sums K <= 4608 products in fp32 (relative error of a sum about sqrt(K) u
# typical, K u worst case, u = 2^-24 = 6e-8) and the nets are up to 110 layers deep with gains near 1:
# sqrt(110) * sqrt(4608) * u = 4e-5 if every layer erred in the same direction at its typical size.
# Measured on the workloads: 4e-7 (tiny, ResNet-20, ResNet-110) to 2.2e-6 (ResNet-50) of the largest logit.
REL = 1e-4


@pytest.fixture(scope="module")
def isr():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2108_09413_amd as lib
    return lib


def _load(isr, blob, chunk):
    m = isr.isr_load_model(blob)
    isr.isr_set_workspace(m, chunk, float_fp=True)
    return m


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("sigma", [0.0, 0.4, 31.875, 127.5, 255.0])
def test_continuous_noise_is_bit_exact_cifar_shape(isr, sigma):
    _say(f"float noise parity 32x32 sigma={sigma}")
    m = _load(isr, synth.build_model(0), 64)
    x = synth.make_image(0, 1)
    for seed, image, phase, begin, count in ((0, 0, 0, 0, 5), (0x0123456789ABCDEF, 7, 1, 99990, 9)):
        got_q = isr.isr_float_debug_noisy(m, x, sigma, seed, image, phase, begin, count, QUANT)
        got_f = isr.isr_float_debug_noisy(m, x, sigma, seed, image, phase, begin, count, FP)
        assert got_q.dtype == np.int8 and got_f.dtype == np.float32
        for s in range(count):
            want_f = oracle.noisy_float(x, sigma, seed, image, phase, begin + s)
            assert np.array_equal(got_f[s].view(np.uint32), want_f.view(np.uint32)), (sigma, seed, s)
            assert np.array_equal(got_q[s], oracle.noisy_quant(x, sigma, seed, image, phase, begin + s)), (sigma, seed, s)
    m.close()


def test_continuous_noise_is_bit_exact_224_shape_and_extreme_pixels(isr):
    _say("float noise parity 224x224")
    m = _load(isr, synth.build_model(3), 8)
    x = synth.make_image(3, 1)
    x[0, :8, :] = 0
    x[1, :8, :] = 255
    for sigma in (63.75, 255.0):
        got_q = isr.isr_float_debug_noisy(m, x, sigma, 5, 3, 1, 12345, 2, QUANT)
        got_f = isr.isr_float_debug_noisy(m, x, sigma, 5, 3, 1, 12345, 2, FP)
        for s in range(2):
            assert np.array_equal(got_f[s].view(np.uint32), oracle.noisy_float(x, sigma, 5, 3, 1, 12345 + s).view(np.uint32))
            assert np.array_equal(got_q[s], oracle.noisy_quant(x, sigma, 5, 3, 1, 12345 + s))
    m.close()


@pytest.mark.parametrize("cfg,size,chunk,count", [(0, None, 24, 70), (1, None, 64, 150), (3, 64, 16, 20)])
def test_floatrs_quant_logits_and_votes_are_bit_exact(isr, cfg, size, chunk, count):
    """Several chunks and a ragged last one; sample range not starting at 0."""
    _say(f"FloatRS-quant parity config {cfg}")
    blob = synth.build_model(cfg) if size is None else synth.build_model(cfg, size=size)
    m = _load(isr, blob, chunk)
    om = oracle.Model(blob)
    x = synth.make_image(cfg, 2) if size is None else synth.make_image(cfg, 2, shape=(3, size, size))
    for sigma, seed, image, phase, begin in ((63.75, 11, 2, 0, 0), (127.5, 0xABCDEF0123, 5, 1, 1000)):
        lg, am, cnt = isr.isr_float_debug_forward(m, x, sigma, seed, image, phase, begin, count, QUANT)
        wl, wa, wc = om.mc_float(x, sigma, seed, image, phase, begin, count, QUANT)
        assert np.array_equal(lg, wl) and np.array_equal(am, wa) and np.array_equal(cnt, wc)
    m.close()


def _check_fp_logits(got, want, got_argmax):
    """Logits within REL of the sample's largest magnitude; the class equals the oracle's wherever the
    oracle's top-two margin exceeds twice that tolerance, and is a near-tie of the oracle's otherwise."""
    ambiguous = 0
    for s in range(want.shape[0]):
        tol = REL * np.abs(want[s]).max()
        assert np.all(np.abs(got[s].astype(np.float64) - want[s]) <= tol), (s, np.abs(got[s] - want[s]).max(), tol)
        order = np.argsort(-want[s], kind="stable")
        margin = want[s][order[0]] - want[s][order[1]]
        if margin > 2 * tol:
            assert got_argmax[s] == order[0], s
        else:
            ambiguous += 1
            assert want[s][got_argmax[s]] >= want[s][order[0]] - 2 * tol, s
        assert got_argmax[s] == int(np.argmax(got[s])), s          # the vote kernel against the logits it read
    return ambiguous


@pytest.mark.parametrize("cfg,size,chunk,count", [(0, None, 64, 40), (1, None, 128, 70), (2, None, 32, 20), (3, 64, 32, 20)])
def test_floatrs_fp_logits_within_fp32_tolerance(isr, cfg, size, chunk, count):
    _say(f"FloatRS-fp parity config {cfg}")
    blob = synth.build_model(cfg) if size is None else synth.build_model(cfg, size=size)
    m = _load(isr, blob, chunk)
    assert 1 <= isr.isr_float_chunk(m, FP) <= chunk // 4 and count > 2 * isr.isr_float_chunk(m, FP)
    om = oracle.Model(blob)
    x = synth.make_image(cfg, 3) if size is None else synth.make_image(cfg, 3, shape=(3, size, size))
    worst = 0.0
    for sigma, seed, image, phase, begin in ((63.75, 11, 2, 0, 0), (127.5, 0xABCDEF0123, 5, 1, 1000)):
        lg, am, cnt = isr.isr_float_debug_forward(m, x, sigma, seed, image, phase, begin, count, FP)
        wl, wa, wc = om.mc_float(x, sigma, seed, image, phase, begin, count, FP)
        assert lg.dtype == np.float32
        amb = _check_fp_logits(lg, wl, am)
        assert np.array_equal(cnt, np.bincount(am, minlength=om.classes))
        assert np.abs(cnt.astype(np.int64) - wc.astype(np.int64)).sum() <= 2 * amb
        worst = max(worst, float((np.abs(lg - wl).max(axis=1) / np.abs(wl).max(axis=1)).max()))
    _say(f"  largest logit deviation / largest logit: {worst:.2e}")
    m.close()


@pytest.mark.parametrize("cfg,size", [(0, None), (1, None), (3, 64)])
def test_floatrs_fp_layer_tensors(isr, cfg, size):
    """Every tensor the fp32 kernels store, one noisy copy, against the oracle's float network."""
    _say(f"FloatRS-fp layer tensors config {cfg}")
    blob = synth.build_model(cfg) if size is None else synth.build_model(cfg, size=size)
    m = _load(isr, blob, 16)
    om = oracle.Model(blob)
    x = synth.make_image(cfg, 4) if size is None else synth.make_image(cfg, 4, shape=(3, size, size))
    sigma, seed, image, phase, sample = 63.75, 21, 1, 1, 77
    _, want = om.forward_float(oracle.noisy_float(x, sigma, seed, image, phase, sample))
    checked = skipped = 0
    for tid in range(om.n_tensors - 1):
        c, h, w, _ = om.tensor_shape(tid)
        try:
            got = isr.isr_float_debug_tensor(m, x, sigma, seed, image, phase, sample, tid, (c, h, w))
        except isr.IsrError as e:
            assert e.status == isr.ISR_ERR_UNSUPPORTED      # convolution output folded into the add after it
            skipped += 1
            continue
        tol = REL * max(np.abs(want[tid]).max(), 1e-30)
        assert np.all(np.abs(got.astype(np.float64) - want[tid]) <= tol), (tid, np.abs(got - want[tid]).max(), tol)
        checked += 1
    assert checked >= 3 and checked > skipped
    m.close()


def test_floatrs_fp_resnet50_full_size(isr):
    """224 x 224 inputs in the benchmarked chunk: a few scattered sample indices of a long run."""
    _say("FloatRS-fp ResNet-50 full size")
    blob = synth.build_model(3)
    m = _load(isr, blob, 668)
    om = oracle.Model(blob)
    x = synth.make_image(3, 1)
    sigma, seed, image, phase = 63.75, 9, 4, 1
    n = 2 * isr.isr_float_chunk(m, FP) + 37
    lg, am, cnt = isr.isr_float_debug_forward(m, x, sigma, seed, image, phase, 0, n, FP)
    idx = [0, 1, isr.isr_float_chunk(m, FP) - 1, isr.isr_float_chunk(m, FP), n - 2, n - 1]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=len(idx)) as ex:       # one host thread per index (the C oracle releases the GIL)
        wls = list(ex.map(lambda i: om.mc_float(x, sigma, seed, image, phase, i, 1, FP, threads=1)[0], idx))
    for i, wl in zip(idx, wls):
        _check_fp_logits(lg[i:i + 1], wl, am[i:i + 1])
    assert cnt.sum() == n
    m.close()


@pytest.mark.parametrize("system", [QUANT, FP])
def test_float_certify_against_the_oracle(isr, system):
    _say(f"float certify system {system}")
    blob = synth.build_model(1)
    m = _load(isr, blob, 256)
    om = oracle.Model(blob)
    x = synth.make_image(1, 5)
    sigma, n0, n, seed, image = 63.75, 40, 300, 3, 2
    res, c0, c1 = isr.isr_float_certify(m, x, sigma, n0, n, ALPHA, system, seed, image)
    cls, rad, p_l, k, w0, w1 = oracle.certify_float(om, x, sigma, n0, n, ALPHA, system, seed, image)
    assert c0.sum() == n0 and c1.sum() == n and res.radius_int == 0 and res.radius_sq_int == 0
    if system == QUANT:
        assert np.array_equal(c0, w0) and np.array_equal(c1, w1)
    else:
        # a class decision may differ only for samples whose two best logits are within the fp32 tolerance
        for phase, cnt, total, got in ((0, w0, n0, c0), (1, w1, n, c1)):
            wl, _, _ = om.mc_float(x, sigma, seed, image, phase, 0, total, FP)
            top2 = -np.sort(-wl, axis=1)[:, :2]
            amb = int(np.count_nonzero(top2[:, 0] - top2[:, 1] <= 2 * REL * np.abs(wl).max(axis=1)))
            assert np.abs(got.astype(np.int64) - cnt.astype(np.int64)).sum() <= 2 * amb
    # the decision is the host's function of the tallies the device produced (Alg. 1)
    want = oracle.stats.certify_decision(c0, c1, sigma, n, ALPHA)
    assert res.cls == want[0] and res.n_top == want[3]
    assert res.p_lower == pytest.approx(want[2], rel=1e-9) and res.radius == pytest.approx(want[1], rel=1e-9, abs=1e-12)
    if system == QUANT or np.array_equal(c0, w0) and np.array_equal(c1, w1):
        assert res.cls == cls and res.radius == pytest.approx(rad, rel=1e-9, abs=1e-12)
    m.close()


def test_float_entry_points_reject_bad_arguments(isr):
    import torch
    blob = synth.build_model(0)
    m = isr.isr_load_model(blob)
    x = torch.from_numpy(synth.make_image(0, 1)).cuda()
    L = isr.lib()
    res = isr.Result()
    args = lambda sigma, system: (m.handle, ctypes.c_void_p(x.data_ptr()), ctypes.c_float(sigma), 4, 8, 0.01,
                                  ctypes.c_uint64(0), 0, system, ctypes.byref(res), None, None)
    assert L.isr_float_certify(*args(10.0, QUANT)) == isr.ISR_ERR_WORKSPACE       # no workspace yet
    isr.isr_set_workspace(m, 2)                                                    # too small for one fp32 copy
    assert L.isr_float_certify(*args(10.0, FP)) == isr.ISR_ERR_WORKSPACE
    assert L.isr_float_certify(*args(10.0, QUANT)) == isr.ISR_OK
    isr.isr_set_workspace(m, 16, float_fp=True)
    assert L.isr_float_certify(*args(10.0, FP)) == isr.ISR_OK
    for sigma, system in ((-1.0, QUANT), (float("nan"), FP), (5000.0, FP), (10.0, 0), (10.0, 3)):
        assert L.isr_float_certify(*args(sigma, system)) == isr.ISR_ERR_ARG
    assert L.isr_float_chunk(m.handle, FP) == 4 and L.isr_float_chunk(m.handle, QUANT) == 16 and L.isr_float_chunk(m.handle, 7) == 0
    m.close()
