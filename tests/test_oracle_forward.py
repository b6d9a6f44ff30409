"""Pins for the oracle's integer forward pass: every op against a second,
independently written formulation (numpy int64 on explicitly padded arrays),
hand-computed rounding cases, and degenerate networks with known outputs."""
import numpy as np
import pytest

import oracle
from synth.models import NetBuilder


def _rha_ref(v, s):
    """Round half away from zero of v / 2^s on Python ints (exact rationals)."""
    v = int(v)
    if s == 0:
        return v
    q, r = divmod(abs(v), 1 << s)
    if 2 * r >= (1 << s):
        q += 1
    return q if v >= 0 else -q


def test_rha_hand_cases():
    for s in (1, 5, 31, 40, 61):   # products stay below 2^62 in the network, so v + half fits 64 bits
        h = 1 << (s - 1)
        assert oracle.rha(h, s) == 1 and oracle.rha(-h, s) == -1
        assert oracle.rha(h - 1, s) == 0 and oracle.rha(-(h - 1), s) == 0
        assert oracle.rha(3 * h, s) == 2 and oracle.rha(-3 * h, s) == -2
        assert oracle.rha(3 * h - 1, s) == 1 and oracle.rha(-(3 * h - 1), s) == -1
    rng = np.random.default_rng(0)
    for _ in range(2000):
        v = int(rng.integers(-2 ** 61, 2 ** 61))
        s = int(rng.integers(0, 62))
        assert oracle.rha(v, s) == _rha_ref(v, s)
    assert oracle.rha(7, 0) == 7 and oracle.rha(-7, 0) == -7


def _np_conv(x, zp_in, w, bias, m0, sh, stride, pad, relu, zp_out):
    """Third formulation: pad (q - z) with zeros, gather windows, einsum in int64."""
    cin, H, W = x.shape
    cout, _, k, _ = w.shape
    xp = np.zeros((cin, H + 2 * pad, W + 2 * pad), dtype=np.int64)
    xp[:, pad:pad + H, pad:pad + W] = x.astype(np.int64) - zp_in
    ho = (H + 2 * pad - k) // stride + 1
    wo = (W + 2 * pad - k) // stride + 1
    win = np.zeros((ho, wo, cin, k, k), dtype=np.int64)
    for oy in range(ho):
        for ox in range(wo):
            win[oy, ox] = xp[:, oy * stride:oy * stride + k, ox * stride:ox * stride + k]
    acc = np.einsum("yxikl,oikl->oyx", win, w.astype(np.int64)) + bias.astype(np.int64)[:, None, None]
    out = np.zeros((cout, ho, wo), dtype=np.int64)
    for oc in range(cout):
        for oy in range(ho):
            for ox in range(wo):
                out[oc, oy, ox] = zp_out + _rha_ref(int(acc[oc, oy, ox]) * int(m0[oc]), 31 + int(sh[oc]))
    lo = zp_out if relu else -128
    return np.clip(out, lo, 127).astype(np.int8), acc


CONV_CASES = [
    # cin, H, W, cout, k, stride, pad, relu, zp_in
    (3, 9, 7, 5, 3, 1, 1, True, 0),
    (4, 8, 8, 6, 3, 2, 1, False, -128),
    (2, 11, 10, 3, 7, 2, 3, True, 0),
    (8, 5, 6, 4, 1, 1, 0, False, -128),
    (8, 6, 6, 4, 1, 2, 0, False, 5),
    (1, 4, 4, 2, 3, 1, 0, True, -7),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_against_numpy_formulation(case):
    cin, H, W, cout, k, stride, pad, relu, zp_in = case
    rng = np.random.default_rng(hash(case) % 2 ** 32)
    b = NetBuilder(rng=np.random.default_rng(1), in_shape=(cin, H, W), num_classes=3)
    tin = b.tensor(cin, H, W, zp_in, 50.0)
    w = rng.integers(-127, 128, size=(cout, cin, k, k)).astype(np.int8)
    bias = rng.integers(-5000, 5000, size=cout).astype(np.int32)
    m0 = rng.integers(1 << 30, 1 << 31, size=cout, dtype=np.int64).astype(np.int32)
    sh = rng.integers(0, 9, size=cout).astype(np.int32)
    zp_out = -128 if relu else int(rng.integers(-20, 20))
    t = b.conv(tin, cout, k, stride, pad, relu, w=w, bias=bias, m0=m0, sh=sh, zp_out=zp_out)
    g = b.gap(t)
    b.fc(g, 3)
    m = oracle.Model(b.blob())
    x = rng.integers(-128, 128, size=(cin, H, W)).astype(np.int8)
    _, tensors = m.forward(x)
    want, _ = _np_conv(x, zp_in, w, bias, m0, sh, stride, pad, relu, zp_out)
    assert np.array_equal(tensors[t], want)


def test_conv_zero_weights_gives_bias_only():
    cin, H, W, cout = 3, 6, 6, 4
    b = NetBuilder(rng=np.random.default_rng(1), in_shape=(cin, H, W), num_classes=2)
    tin = b.tensor(cin, H, W, 0, 50.0)
    bias = np.array([1000, -1000, 12345, -99999], dtype=np.int32)
    m0 = np.array([1 << 30, (1 << 31) - 1, 1 << 30, 3 << 29], dtype=np.int32)
    sh = np.array([3, 4, 0, 9], dtype=np.int32)
    t = b.conv(tin, cout, 3, 1, 1, False, w=np.zeros((cout, cin, 3, 3)), bias=bias, m0=m0, sh=sh, zp_out=3)
    b.fc(b.gap(t), 2)
    m = oracle.Model(b.blob())
    x = np.random.default_rng(2).integers(-128, 128, size=(cin, H, W)).astype(np.int8)
    _, tensors = m.forward(x)
    for oc in range(cout):
        want = min(127, max(-128, 3 + _rha_ref(int(bias[oc]) * int(m0[oc]), 31 + int(sh[oc]))))
        assert np.all(tensors[t][oc] == want)


def test_identity_conv_halves_with_ties_away():
    """1x1 identity weights, M0 = 2^30, shift 0: out = RHA(q / 2) (ties away from zero)."""
    c = 4
    b = NetBuilder(rng=np.random.default_rng(1), in_shape=(c, 8, 8), num_classes=2)
    tin = b.tensor(c, 8, 8, 0, 50.0)
    w = np.eye(c, dtype=np.int8).reshape(c, c, 1, 1)
    t = b.conv(tin, c, 1, 1, 0, False, w=w, bias=np.zeros(c), m0=1 << 30, sh=0, zp_out=0)
    b.fc(b.gap(t), 2)
    m = oracle.Model(b.blob())
    x = np.arange(-128, 128, dtype=np.int16).astype(np.int8).reshape(c, 8, 8)
    _, tensors = m.forward(x)
    q = x.astype(np.int64)
    want = np.sign(q) * ((np.abs(q) + 1) // 2)
    assert np.array_equal(tensors[t].astype(np.int64), want)
    assert tensors[t][0, 0, 0] == -64 and int(x.reshape(-1)[1]) == -127 and tensors[t].reshape(-1)[1] == -64


def test_padding_contributes_zero_whatever_the_zero_point():
    """Out-of-bounds taps contribute 0: with input == zero-point everywhere the
    accumulator is the bias alone, also at the borders."""
    cin, H, W, cout = 2, 5, 5, 3
    for zp_in in (-128, 0, 17):
        b = NetBuilder(rng=np.random.default_rng(3), in_shape=(cin, H, W), num_classes=2)
        tin = b.tensor(cin, H, W, zp_in, 50.0)
        bias = np.array([256, -512, 1024], dtype=np.int32)
        t = b.conv(tin, cout, 3, 1, 1, False, bias=bias, m0=1 << 30, sh=0, zp_out=0)
        b.fc(b.gap(t), 2)
        m = oracle.Model(b.blob())
        x = np.full((cin, H, W), zp_in, dtype=np.int8)
        _, tensors = m.forward(x)
        for oc in range(cout):
            assert np.all(tensors[t][oc] == np.clip(_rha_ref(int(bias[oc]) << 30, 31), -128, 127))


def test_add_maxpool_gap_fc_against_numpy():
    rng = np.random.default_rng(7)
    C, H, W = 6, 9, 9
    b = NetBuilder(rng=np.random.default_rng(4), in_shape=(C, H, W), num_classes=5)
    tin = b.tensor(C, H, W, -128, 50.0)
    ta = b.conv(tin, C, 3, 1, 1, False)          # zp 0
    ma, mb, sh = 777777, 901234, 20
    tadd = b.add(tin, ta, True, ma=ma, mb=mb, sh=sh)
    tadd2 = b.add(ta, tadd, False, ma=-123456, mb=654321, sh=19, zp_out=4)
    tp = b.maxpool(tadd, 3, 2, 1)
    m0g, shg = 1402438301, 5
    tg = b.gap(tp, m0=m0g, sh=shg)
    wfc = rng.integers(-127, 128, size=(5, C)).astype(np.int8)
    bfc = rng.integers(-512, 513, size=5).astype(np.int32)
    b.fc(tg, 5, w=wfc, bias=bfc)
    m = oracle.Model(b.blob())
    x = rng.integers(-128, 128, size=(C, H, W)).astype(np.int8)
    logits, T = m.forward(x)
    # ADD
    A = x.astype(np.int64) + 128
    B = T[ta].astype(np.int64)
    want = np.vectorize(lambda v: _rha_ref(v, sh))(A * ma + B * mb) - 128
    assert np.array_equal(T[tadd], np.clip(want, -128, 127).astype(np.int8))
    want2 = np.vectorize(lambda v: _rha_ref(v, 19))(B * -123456 + (T[tadd].astype(np.int64) + 128) * 654321) + 4
    assert np.array_equal(T[tadd2], np.clip(want2, -128, 127).astype(np.int8))
    # MAXPOOL 3x3/s2/p1 via padding with -inf
    P = np.full((C, H + 2, W + 2), -1000, dtype=np.int64)
    P[:, 1:-1, 1:-1] = T[tadd]
    ho = (H + 2 - 3) // 2 + 1
    wantp = np.stack([[[P[c, 2 * y:2 * y + 3, 2 * xx:2 * xx + 3].max() for xx in range(ho)] for y in range(ho)]
                      for c in range(C)])
    assert np.array_equal(T[tp].astype(np.int64), wantp)
    # GAP
    S = (T[tp].astype(np.int64) + 128).reshape(C, -1).sum(axis=1)
    wantg = np.array([min(127, max(-128, -128 + _rha_ref(int(s) * m0g, 31 + shg))) for s in S])
    assert np.array_equal(T[tg].reshape(-1).astype(np.int64), wantg)
    # FC: int32 logits, no requantisation
    wantl = wfc.astype(np.int64) @ (T[tg].reshape(-1).astype(np.int64) + 128) + bfc
    assert np.array_equal(logits.astype(np.int64), wantl)


def test_argmax_lowest_index_and_vote_tally():
    """A network whose FC ignores its input gives the bias as logits: the vote
    goes to the lowest index among equal maxima, for every noisy copy."""
    b = NetBuilder(rng=np.random.default_rng(5), in_shape=(3, 8, 8), num_classes=6)
    tin = b.tensor(3, 8, 8, 0, 50.0)
    t = b.conv(tin, 4, 3, 1, 1, True)
    g = b.gap(t)
    b.fc(g, 6, w=np.zeros((6, 4)), bias=np.array([5, 9, -3, 9, 9, 0]))
    m = oracle.Model(b.blob())
    x = np.random.default_rng(1).integers(0, 256, size=(3, 8, 8)).astype(np.uint8)
    logits, am, counts = m.mc(x, 32, 0, 0, 0, 0, 50, threads=2)
    assert np.all(logits == np.array([5, 9, -3, 9, 9, 0]))
    assert np.all(am == 1) and counts.tolist() == [0, 50, 0, 0, 0, 0]


def test_mc_is_additive_over_ranges_and_thread_invariant():
    import synth
    m = oracle.Model(synth.build_model(0))
    x = synth.make_image(0, 1)
    la, aa, ca = m.mc(x, 32, 3, 1, 1, 0, 40, threads=1)
    lb, ab, cb = m.mc(x, 32, 3, 1, 1, 0, 25, threads=3)
    lc, ac, cc = m.mc(x, 32, 3, 1, 1, 25, 15, threads=2)
    assert np.array_equal(la, np.concatenate([lb, lc])) and np.array_equal(aa, np.concatenate([ab, ac]))
    assert np.array_equal(ca, cb + cc) and ca.sum() == 40
    # per-sample path == single forward on the noisy copy
    a0 = oracle.noisy(x, 32, 3, 1, 1, 7)
    lg, _ = m.forward(a0)
    assert np.array_equal(lg, la[7])
    assert aa[7] == int(np.flatnonzero(lg == lg.max())[0])


# ---- the drivers that assemble Alg. 1 and Alg. 2 from the loop above ----

def _golden_ratio(golden_dir, n, k):
    """R / sigma of the golden file (50-digit values, independent of scipy and of the oracle)."""
    import os
    for line in open(os.path.join(golden_dir, "cp_radius_values.txt")):
        f = line.split()
        if len(f) == 4 and f[0] == str(n) and f[1] == str(k):
            return float(f[3])
    raise KeyError((n, k))


def _vote_splitting_net():
    """Five classes on a 3x2x2 input with no pooling of the noise away: the votes of noisy copies of a
    grey image spread over all classes, so tallies tell streams, ranges and seeds apart."""
    b = NetBuilder(rng=np.random.default_rng(8), in_shape=(3, 2, 2), num_classes=5)
    tin = b.tensor(3, 2, 2, 0, 74.0)
    t = b.conv(tin, 8, 1, 1, 0, False, bias=np.zeros(8), sh=5)
    b.fc(b.gap(t), 5, bias=np.zeros(5))
    return oracle.Model(b.blob()), np.full((3, 2, 2), 128, dtype=np.uint8)


def test_certify_runs_selection_on_phase_0_and_estimation_on_phase_1():
    """Alg. 1: n0 selection samples and n estimation samples on two disjoint streams; the class
    comes from the first tally, the count that enters the bound from the second."""
    m, x = _vote_splitting_net()
    n0, n, sigma, seed, image = 60, 240, 64, 11, 5
    cls, rad, p_l, k, c0, c1 = oracle.certify(m, x, sigma, n0, n, 0.001, seed=seed, image=image, threads=2)
    _, _, want0 = m.mc(x, sigma, seed, image, 0, 0, n0, threads=1)
    _, _, want1 = m.mc(x, sigma, seed, image, 1, 0, n, threads=1)
    assert np.array_equal(c0, want0) and np.array_equal(c1, want1)
    assert int(c0.sum()) == n0 and int(c1.sum()) == n and np.count_nonzero(c0) == 5
    # the tallies a driver would get from one stream for both loops, from swapped streams or from
    # swapped sample counts are all different from these
    _, _, p1_n0 = m.mc(x, sigma, seed, image, 1, 0, n0, threads=1)
    _, _, p0_n = m.mc(x, sigma, seed, image, 0, 0, n, threads=1)
    assert not np.array_equal(c0, p1_n0) and not np.array_equal(c1, p0_n)
    assert not np.array_equal(oracle.noisy(x, sigma, seed, image, 0, 0), oracle.noisy(x, sigma, seed, image, 1, 0))
    # class from the selection tally (here it differs from the top class of the same number of
    # estimation samples), count of that class read from the estimation tally
    c_a = int(np.flatnonzero(c0 == c0.max())[0])
    assert c_a != int(np.argmax(p1_n0))
    assert k == int(c1[c_a])
    assert (cls, rad, p_l, k) == oracle.stats.certify_decision(c0, c1, float(sigma), n, 0.001)
    assert cls == oracle.stats.ABSTAIN and rad == 0.0    # 94 of 240 votes: the bound is far below 1/2
    # seed and image id reach both streams
    for kw in (dict(seed=seed + 1, image=image), dict(seed=seed, image=image + 1)):
        _, _, _, _, d0, d1 = oracle.certify(m, x, sigma, n0, n, 0.001, threads=2, **kw)
        _, _, e0 = m.mc(x, sigma, kw["seed"], kw["image"], 0, 0, n0, threads=1)
        _, _, e1 = m.mc(x, sigma, kw["seed"], kw["image"], 1, 0, n, threads=1)
        assert np.array_equal(d0, e0) and np.array_equal(d1, e1) and not np.array_equal(d1, c1)


def test_certify_on_the_small_workload_matches_its_two_loops():
    import synth
    m = oracle.Model(synth.build_model(0))
    x = synth.make_image(0, 1)
    cls, rad, p_l, k, c0, c1 = oracle.certify(m, x, 32, 100, 300, 0.001, seed=0, image=0, threads=4)
    assert np.array_equal(c0, m.mc(x, 32, 0, 0, 0, 0, 100, threads=2)[2])
    assert np.array_equal(c1, m.mc(x, 32, 0, 0, 1, 0, 300, threads=2)[2])
    assert (cls, rad, p_l, k) == oracle.stats.certify_decision(c0, c1, 32.0, 300, 0.001)


def _constant_net():
    """FC ignores its input: logits = bias, maxima at classes 1, 3, 4 (lowest index wins)."""
    b = NetBuilder(rng=np.random.default_rng(5), in_shape=(3, 8, 8), num_classes=6)
    tin = b.tensor(3, 8, 8, 0, 50.0)
    t = b.conv(tin, 4, 3, 1, 1, True)
    b.fc(b.gap(t), 6, w=np.zeros((6, 4)), bias=np.array([5, 9, -3, 9, 9, 0]))
    return oracle.Model(b.blob())


def test_certify_constant_classifier_reaches_the_largest_radius(golden_dir):
    """All n estimation votes on one class: p_A = alpha^(1/n), the largest radius the procedure
    can return (section on certified accuracy: every sample classified as the same class)."""
    m = _constant_net()
    x = np.random.default_rng(1).integers(0, 256, size=(3, 8, 8)).astype(np.uint8)
    for n0, n in ((7, 1000), (100, 100)):
        for sigma in (32, 64):
            cls, rad, p_l, k, c0, c1 = oracle.certify(m, x, sigma, n0, n, 0.001, seed=3, image=2, threads=2)
            assert cls == 1 and k == n
            assert c0.tolist() == [0, n0, 0, 0, 0, 0] and c1.tolist() == [0, n, 0, 0, 0, 0]
            want = sigma * _golden_ratio(golden_dir, n, n)
            assert abs(rad - want) <= 1e-12 * want
            assert abs(p_l - 0.001 ** (1.0 / n)) <= 1e-15


def test_predict_constant_classifier_needs_eleven_samples():
    """Alg. 2 with all n votes on one class: two-sided p-value 2 * 2^-n; at alpha = 0.001 ten
    samples abstain (1.95e-3) and eleven return the class (9.77e-4)."""
    m = _constant_net()
    x = np.random.default_rng(1).integers(0, 256, size=(3, 8, 8)).astype(np.uint8)
    cls, pv, n_a, n_b, counts = oracle.predict(m, x, 32, 10, 0.001, seed=0, image=0, threads=1)
    assert cls == oracle.stats.ABSTAIN and (n_a, n_b) == (10, 0) and pv == 2.0 ** -9 and counts.tolist() == [0, 10, 0, 0, 0, 0]
    cls, pv, n_a, n_b, counts = oracle.predict(m, x, 32, 11, 0.001, seed=0, image=0, threads=1)
    assert cls == 1 and (n_a, n_b) == (11, 0) and pv == 2.0 ** -10 and counts.tolist() == [0, 11, 0, 0, 0, 0]


def test_predict_runs_one_loop_on_phase_0():
    m, x = _vote_splitting_net()
    cls, pv, n_a, n_b, counts = oracle.predict(m, x, 64, 240, 0.001, seed=11, image=5, threads=2)
    _, _, want = m.mc(x, 64, 11, 5, 0, 0, 240, threads=1)
    assert np.array_equal(counts, want) and int(counts.sum()) == 240
    assert not np.array_equal(counts, m.mc(x, 64, 11, 5, 1, 0, 240, threads=1)[2])
    top = sorted(counts.tolist(), reverse=True)
    assert (n_a, n_b) == (top[0], top[1]) and n_b > 0
    assert (cls, pv, n_a, n_b) == oracle.stats.predict_decision(counts, 0.001)
