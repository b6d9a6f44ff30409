"""CPU oracle for integer randomized smoothing -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path never does.  `isr_oracle.c` holds the integer
Monte-Carlo loop (noise, forward, votes) and the two floating-point comparison
systems of the paper's evaluation (continuous Gaussian noise; quantized or float
network), `stats.py` the float64 decisions.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

from . import stats  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "isr_oracle.c")
_LIB = os.path.join(_HERE, "libisr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP only splits the sample loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        # binary32 steps of the float sampler must stay single operations: no contraction into fused multiply-adds
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.isr_oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.isr_oracle_noise_table.argtypes = [C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.isr_oracle_noise_table.restype = C.c_int
        L.isr_oracle_delta.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64]
        L.isr_oracle_delta.restype = C.c_int32
        L.isr_oracle_uniform64.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.isr_oracle_uniform64.restype = C.c_uint64
        L.isr_oracle_noisy.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_uint64,
                                       C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.isr_oracle_noisy.restype = None
        L.isr_oracle_noise_bank.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                            C.c_uint32, C.c_void_p]
        L.isr_oracle_noise_bank.restype = None
        L.isr_oracle_load.argtypes = [C.c_void_p, C.c_size_t]
        L.isr_oracle_load.restype = C.c_void_p
        L.isr_oracle_free.argtypes = [C.c_void_p]
        L.isr_oracle_free.restype = None
        L.isr_oracle_info.argtypes = [C.c_void_p] + [C.c_void_p] * 5
        L.isr_oracle_info.restype = None
        L.isr_oracle_tensor_shape.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 4
        L.isr_oracle_tensor_shape.restype = None
        L.isr_oracle_tensor_offset.argtypes = [C.c_void_p, C.c_int32]
        L.isr_oracle_tensor_offset.restype = C.c_size_t
        L.isr_oracle_rha.argtypes = [C.c_int64, C.c_int32]
        L.isr_oracle_rha.restype = C.c_int64
        L.isr_oracle_forward.argtypes = [C.c_void_p] * 4
        L.isr_oracle_forward.restype = C.c_int
        L.isr_oracle_argmax.argtypes = [C.c_void_p, C.c_int32]
        L.isr_oracle_argmax.restype = C.c_int32
        L.isr_oracle_mc.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32,
                                    C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        L.isr_oracle_mc.restype = C.c_int
        L.isr_oracle_neg_log_u24.argtypes = [C.c_uint32]
        L.isr_oracle_neg_log_u24.restype = C.c_float
        L.isr_oracle_cos_sin_turn24.argtypes = [C.c_uint32, C.c_void_p, C.c_void_p]
        L.isr_oracle_cos_sin_turn24.restype = None
        L.isr_oracle_box_muller.argtypes = [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.isr_oracle_box_muller.restype = None
        L.isr_oracle_gauss4.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.isr_oracle_gauss4.restype = None
        L.isr_oracle_noisy_float.argtypes = [C.c_void_p, C.c_uint32, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                             C.c_uint32, C.c_void_p]
        L.isr_oracle_noisy_float.restype = None
        L.isr_oracle_noisy_quant.argtypes = L.isr_oracle_noisy_float.argtypes
        L.isr_oracle_noisy_quant.restype = None
        L.isr_oracle_forward_float.argtypes = [C.c_void_p] * 4
        L.isr_oracle_forward_float.restype = C.c_int
        L.isr_oracle_mc_float.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                          C.c_uint32, C.c_uint32, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_int]
        L.isr_oracle_mc_float.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().isr_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def noise_table(sigma: int):
    """(T, R): the 2R inverse-CDF thresholds of N_Z(0, sigma^2) and the support radius."""
    T = np.zeros(2 * 16384, dtype=np.uint64)
    R = C.c_uint32(0)
    rc = lib().isr_oracle_noise_table(int(sigma), _ptr(T), T.size, C.byref(R))
    if rc != 0:
        raise ValueError(f"noise table failed for sigma={sigma}: {rc}")
    return T[: 2 * R.value].copy(), R.value


def delta(T, R, u: int) -> int:
    return int(lib().isr_oracle_delta(_ptr(T), int(R), C.c_uint64(int(u))))


def uniform64(seed, image, phase, sample, p) -> int:
    return int(lib().isr_oracle_uniform64(C.c_uint64(seed), image, phase, sample, p))


def noisy(x: np.ndarray, sigma: int, seed: int, image: int, phase: int, sample: int) -> np.ndarray:
    """int8 [C][H][W]: clamp(x + delta, 0, 255) - 128 for one noisy copy."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    T, R = noise_table(sigma)
    out = np.zeros(x.shape, dtype=np.int8)
    lib().isr_oracle_noisy(_ptr(x), x.size, _ptr(T), R, C.c_uint64(seed), image, phase, sample, _ptr(out))
    return out


def noise_bank(sigma: int, seed: int, bank: int, first: int, count: int, d: int) -> np.ndarray:
    """int16 [count][d]: stored training noise, draws of N_Z(0, sigma^2) on the phase-2 stream."""
    T, R = noise_table(sigma)
    out = np.zeros((count, d), dtype=np.int16)
    lib().isr_oracle_noise_bank(_ptr(T), R, C.c_uint64(seed), bank, first, count, d, _ptr(out))
    return out


FLOATRS_QUANT, FLOATRS_FP = 1, 2   # the paper's two floating-point comparison systems


def neg_log_u24(n: int) -> float:
    """-ln(n / 2^24), n in [1, 2^24], by the sampler's binary32 steps."""
    return float(lib().isr_oracle_neg_log_u24(int(n)))


def cos_sin_turn24(t: int):
    """(cos, sin) of 2 pi t / 2^24, t in [0, 2^24), by the sampler's binary32 steps."""
    c, s = C.c_float(0), C.c_float(0)
    lib().isr_oracle_cos_sin_turn24(int(t), C.byref(c), C.byref(s))
    return c.value, s.value


def box_muller(wa: int, wb: int):
    a, b = C.c_float(0), C.c_float(0)
    lib().isr_oracle_box_muller(int(wa), int(wb), C.byref(a), C.byref(b))
    return a.value, b.value


def gauss4(seed, image, phase, sample, group) -> np.ndarray:
    """float32[4]: the standard-normal draws of elements 4*group .. 4*group+3 of one noisy copy."""
    z = np.zeros(4, dtype=np.float32)
    lib().isr_oracle_gauss4(C.c_uint64(seed), image, phase, sample, group, _ptr(z))
    return z


def noisy_float(x: np.ndarray, sigma: float, seed: int, image: int, phase: int, sample: int) -> np.ndarray:
    """float32 [C][H][W]: x + sigma z, z ~ N(0, I), for one noisy copy (FloatRS-fp input before recentring)."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    out = np.zeros(x.shape, dtype=np.float32)
    lib().isr_oracle_noisy_float(_ptr(x), x.size, C.c_float(sigma), C.c_uint64(seed), image, phase, sample, _ptr(out))
    return out


def noisy_quant(x: np.ndarray, sigma: float, seed: int, image: int, phase: int, sample: int) -> np.ndarray:
    """int8 [C][H][W]: clamp(round(x + sigma z), 0, 255) - 128 for one noisy copy (FloatRS-quant input)."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    out = np.zeros(x.shape, dtype=np.int8)
    lib().isr_oracle_noisy_quant(_ptr(x), x.size, C.c_float(sigma), C.c_uint64(seed), image, phase, sample, _ptr(out))
    return out


def rha(v: int, s: int) -> int:
    return int(lib().isr_oracle_rha(C.c_int64(v), s))


class Model:
    """Parsed quantized network (wraps the C oracle's model handle)."""

    def __init__(self, blob: bytes):
        self._buf = (C.c_char * len(blob)).from_buffer_copy(blob)
        self._h = lib().isr_oracle_load(self._buf, len(blob))
        if not self._h:
            raise ValueError("oracle: bad model blob")
        v = [C.c_int32(0) for _ in range(5)]
        lib().isr_oracle_info(self._h, *[C.byref(t) for t in v])
        self.C, self.H, self.W, self.classes, self.n_tensors = [t.value for t in v]

    def __del__(self):
        if getattr(self, "_h", None):
            lib().isr_oracle_free(self._h)
            self._h = None

    def tensor_shape(self, tid: int):
        v = [C.c_int32(0) for _ in range(4)]
        lib().isr_oracle_tensor_shape(self._h, tid, *[C.byref(t) for t in v])
        return tuple(t.value for t in v)  # C, H, W, zp

    def forward(self, a0: np.ndarray):
        """(logits int32[classes], {tensor id: int8 [C][H][W]}) for one int8 input."""
        a0 = np.ascontiguousarray(a0, dtype=np.int8)
        total = lib().isr_oracle_tensor_offset(self._h, self.n_tensors)
        acts = np.zeros(total, dtype=np.int8)
        logits = np.zeros(self.classes, dtype=np.int32)
        lib().isr_oracle_forward(self._h, _ptr(a0), _ptr(acts), _ptr(logits))
        tensors = {}
        for tid in range(self.n_tensors - 1):
            c, h, w, _ = self.tensor_shape(tid)
            off = lib().isr_oracle_tensor_offset(self._h, tid)
            tensors[tid] = acts[off: off + c * h * w].reshape(c, h, w)
        return logits, tensors

    def forward_float(self, v: np.ndarray):
        """(logits float64[classes], {tensor id: float64 [C][H][W]}) of the float network for the
        noisy pixel values v (float32 [C][H][W])."""
        v = np.ascontiguousarray(v, dtype=np.float32)
        total = lib().isr_oracle_tensor_offset(self._h, self.n_tensors)
        acts = np.zeros(total, dtype=np.float64)
        logits = np.zeros(self.classes, dtype=np.float64)
        lib().isr_oracle_forward_float(self._h, _ptr(v), _ptr(acts), _ptr(logits))
        tensors = {}
        for tid in range(self.n_tensors - 1):
            c, h, w, _ = self.tensor_shape(tid)
            off = lib().isr_oracle_tensor_offset(self._h, tid)
            tensors[tid] = acts[off: off + c * h * w].reshape(c, h, w)
        return logits, tensors

    def mc_float(self, x, sigma, seed, image, phase, begin, count, variant, threads=None, want_logits=True):
        """Monte-Carlo loop of a comparison system: (logits [count][classes] -- int32 for
        FLOATRS_QUANT, float64 for FLOATRS_FP -- or None, argmax [count], counts [classes])."""
        x = np.ascontiguousarray(x, dtype=np.uint8)
        li = np.zeros((count, self.classes), dtype=np.int32) if want_logits and variant == FLOATRS_QUANT else None
        ld = np.zeros((count, self.classes), dtype=np.float64) if want_logits and variant == FLOATRS_FP else None
        argmax = np.zeros(count, dtype=np.int32)
        counts = np.zeros(self.classes, dtype=np.uint32)
        threads = threads or min(os.cpu_count() or 1, 16)
        rc = lib().isr_oracle_mc_float(self._h, _ptr(x), C.c_float(sigma), C.c_uint64(seed), image, phase, begin, count,
                                       int(variant), _ptr(li), _ptr(ld), _ptr(argmax), _ptr(counts), threads)
        if rc != 0:
            raise RuntimeError(f"oracle mc_float failed: {rc}")
        return (li if variant == FLOATRS_QUANT else ld), argmax, counts

    def mc(self, x, sigma, seed, image, phase, begin, count, threads=None, want_logits=True):
        """Monte-Carlo loop over sample indices [begin, begin+count):
        returns (logits [count][classes] or None, argmax [count], counts [classes])."""
        x = np.ascontiguousarray(x, dtype=np.uint8)
        logits = np.zeros((count, self.classes), dtype=np.int32) if want_logits else None
        argmax = np.zeros(count, dtype=np.int32)
        counts = np.zeros(self.classes, dtype=np.uint32)
        threads = threads or min(os.cpu_count() or 1, 16)
        rc = lib().isr_oracle_mc(self._h, _ptr(x), int(sigma), C.c_uint64(seed), image, phase, begin, count,
                                 _ptr(logits), _ptr(argmax), _ptr(counts), threads)
        if rc != 0:
            raise RuntimeError(f"oracle mc failed: {rc}")
        return logits, argmax, counts


def certify(model: Model, x, sigma, n0, n, alpha, seed=0, image=0, threads=None):
    """Alg. 1: selection loop (phase 0, n0 samples), estimation loop (phase 1,
    n samples), then the decision.  Returns (class, radius, p_lower, n_top,
    counts0, counts1); class is stats.ABSTAIN on abstention."""
    _, _, counts0 = model.mc(x, sigma, seed, image, 0, 0, n0, threads, want_logits=False)
    _, _, counts1 = model.mc(x, sigma, seed, image, 1, 0, n, threads, want_logits=False)
    cls, rad, p_l, k = stats.certify_decision(counts0, counts1, float(sigma), n, alpha)
    return cls, rad, p_l, k, counts0, counts1


def certify_float(model: Model, x, sigma, n0, n, alpha, variant, seed=0, image=0, threads=None):
    """Alg. 1 run by a comparison system: the same two loops and the same decision with the
    continuous-Gaussian sampler (and the float network for FLOATRS_FP) in the loop."""
    _, _, counts0 = model.mc_float(x, sigma, seed, image, 0, 0, n0, variant, threads, want_logits=False)
    _, _, counts1 = model.mc_float(x, sigma, seed, image, 1, 0, n, variant, threads, want_logits=False)
    cls, rad, p_l, k = stats.certify_decision(counts0, counts1, float(sigma), n, alpha)
    return cls, rad, p_l, k, counts0, counts1


def predict(model: Model, x, sigma, n, alpha, seed=0, image=0, threads=None):
    """Alg. 2: one loop of n samples (phase 0), then the binomial test.
    Returns (class, p_value, n_A, n_B, counts)."""
    _, _, counts = model.mc(x, sigma, seed, image, 0, 0, n, threads, want_logits=False)
    cls, pv, n_a, n_b = stats.predict_decision(counts, alpha)
    return cls, pv, n_a, n_b, counts


def certify_batch(model: Model, xs, items, n0, n, alpha, seed=0, threads=None):
    """Alg. 1 for a list of (image index, sigma, image id) pairs: by definition the
    single-pair procedure applied to each pair in turn.  Returns a list of certify() tuples."""
    return [certify(model, xs[i], sigma, n0, n, alpha, seed, image_id, threads) for i, sigma, image_id in items]


def predict_batch(model: Model, xs, items, n, alpha, seed=0, threads=None):
    """Alg. 2 for a list of (image index, sigma, image id) pairs, one pair after the other."""
    return [predict(model, xs[i], sigma, n, alpha, seed, image_id, threads) for i, sigma, image_id in items]
