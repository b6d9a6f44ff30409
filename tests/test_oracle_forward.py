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
