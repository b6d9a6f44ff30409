"""Python binding of the integer-randomized-smoothing HIP library (libisr.so).

Argument marshalling only: every step of the Monte-Carlo loop runs in the HIP
kernels behind the C ABI declared in include/isr.h.  torch is used for device
memory (workspace, images) and the stream.  There is no CPU fallback: if the
library cannot be loaded the import of a compute entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libisr.so")

ISR_OK, ISR_ERR_ARG, ISR_ERR_FORMAT, ISR_ERR_UNSUPPORTED, ISR_ERR_WORKSPACE, ISR_ERR_DEVICE = range(6)
ABSTAIN = -1

EXPORTS = [
    "isr_load_model", "isr_free_model", "isr_validate_model", "isr_model_info", "isr_workspace_bytes",
    "isr_set_workspace", "isr_certify", "isr_predict", "isr_debug_noisy", "isr_debug_forward",
    "isr_debug_tensor", "isr_debug_tensor_source", "isr_noise_table", "isr_cp_lower", "isr_normal_quantile", "isr_binom_pvalue",
    "isr_decide_certify", "isr_decide_predict", "isr_discrete_quantile", "isr_set_fusion", "isr_set_conv_tile", "isr_profile", "isr_profile_read", "isr_strerror",
    "isr_last_device_error", "isr_certify_batch", "isr_predict_batch", "isr_certified_metrics", "isr_noise_bank",
    "isr_noise_bank_static", "isr_noise_bank_static_capacity",
    "isr_float_workspace_bytes", "isr_float_chunk", "isr_float_certify", "isr_float_debug_noisy",
    "isr_float_debug_forward", "isr_float_debug_tensor",
]

FLOATRS_QUANT, FLOATRS_FP = 1, 2   # the paper's two floating-point comparison systems


class IsrError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = lib().isr_strerror(status).decode()
        if status == ISR_ERR_DEVICE:
            msg += f" (hipError {lib().isr_last_device_error()})"
        super().__init__(f"{what}: {msg}")


class Result(C.Structure):
    _fields_ = [("cls", C.c_int32), ("radius", C.c_double), ("p_lower", C.c_double),
                ("n_top", C.c_uint32), ("n_second", C.c_uint32),
                ("radius_int", C.c_int32), ("radius_sq_int", C.c_uint64)]

    def __repr__(self):
        return (f"Result(cls={self.cls}, radius={self.radius!r}, p_lower={self.p_lower!r}, "
                f"n_top={self.n_top}, n_second={self.n_second}, radius_int={self.radius_int}, "
                f"radius_sq_int={self.radius_sq_int})")


class Item(C.Structure):
    _fields_ = [("image", C.c_uint32), ("sigma", C.c_uint32), ("image_id", C.c_uint32)]


class KernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 80), ("is_conv", C.c_int32), ("launches", C.c_uint64), ("total_ms", C.c_double),
                ("alg_ops", C.c_double), ("alg_bytes", C.c_double)]


_lib = None


def lib():
    """The loaded C-ABI library; builds it in-tree first if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from .build import build_library
            build_library()
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i32, dbl, sz = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32, C.c_double, C.c_size_t
        L.isr_load_model.argtypes = [vp, sz, C.POINTER(vp)]
        L.isr_free_model.argtypes = [vp]
        L.isr_validate_model.argtypes = [vp, sz]
        L.isr_model_info.argtypes = [vp] + [C.POINTER(C.c_int)] * 4
        L.isr_workspace_bytes.argtypes = [vp, u32]
        L.isr_workspace_bytes.restype = sz
        L.isr_set_workspace.argtypes = [vp, vp, sz, u32, vp]
        L.isr_certify.argtypes = [vp, vp, u32, u32, u32, dbl, u64, u32, C.POINTER(Result), vp, vp]
        L.isr_predict.argtypes = [vp, vp, u32, u32, dbl, u64, u32, C.POINTER(Result), vp]
        L.isr_debug_noisy.argtypes = [vp, vp, u32, u64, u32, u32, u32, u32, vp]
        L.isr_debug_forward.argtypes = [vp, vp, u32, u64, u32, u32, u32, u32, vp, vp, vp]
        L.isr_debug_tensor.argtypes = [vp, vp, u32, u64, u32, u32, u32, i32, vp]
        L.isr_debug_tensor_source.argtypes = [vp, i32, C.POINTER(C.c_int)]
        L.isr_noise_table.argtypes = [u32, vp, sz, C.POINTER(u32)]
        L.isr_cp_lower.argtypes = [u32, u32, dbl, C.POINTER(dbl)]
        L.isr_normal_quantile.argtypes = [dbl, C.POINTER(dbl)]
        L.isr_binom_pvalue.argtypes = [u32, u32, C.POINTER(dbl)]
        L.isr_discrete_quantile.argtypes = [u32, dbl, C.POINTER(i32), C.POINTER(u64)]
        L.isr_decide_certify.argtypes = [vp, vp, u32, dbl, u32, dbl, C.POINTER(Result)]
        L.isr_decide_predict.argtypes = [vp, u32, dbl, C.POINTER(Result)]
        L.isr_certify_batch.argtypes = [vp, vp, u32, C.POINTER(Item), u32, u32, u32, dbl, u64, C.POINTER(Result), vp, vp]
        L.isr_predict_batch.argtypes = [vp, vp, u32, C.POINTER(Item), u32, u32, dbl, u64, C.POINTER(Result), vp]
        L.isr_certified_metrics.argtypes = [C.POINTER(Result), vp, u32, vp, u32, C.POINTER(dbl), vp]
        L.isr_noise_bank.argtypes = [u32, u64, u32, u32, u32, u32, vp, vp]
        L.isr_noise_bank_static.argtypes = [u32, u64, u32, u32, u32, u32, vp, vp]
        L.isr_noise_bank_static_capacity.argtypes = []
        L.isr_noise_bank_static_capacity.restype = sz
        flt = C.c_float
        L.isr_float_workspace_bytes.argtypes = [vp, u32, C.c_int]
        L.isr_float_workspace_bytes.restype = sz
        L.isr_float_chunk.argtypes = [vp, C.c_int]
        L.isr_float_chunk.restype = u32
        L.isr_float_certify.argtypes = [vp, vp, flt, u32, u32, dbl, u64, u32, C.c_int, C.POINTER(Result), vp, vp]
        L.isr_float_debug_noisy.argtypes = [vp, vp, flt, u64, u32, u32, u32, u32, C.c_int, vp]
        L.isr_float_debug_forward.argtypes = [vp, vp, flt, u64, u32, u32, u32, u32, C.c_int, vp, vp, vp]
        L.isr_float_debug_tensor.argtypes = [vp, vp, flt, u64, u32, u32, u32, i32, vp]
        L.isr_set_fusion.argtypes = [vp, C.c_int]
        L.isr_set_conv_tile.argtypes = [vp, C.c_int]
        L.isr_profile.argtypes = [vp, u32]
        L.isr_profile_read.argtypes = [vp, C.POINTER(KernelStat), u32, C.POINTER(u32)]
        L.isr_strerror.argtypes = [C.c_int]
        L.isr_strerror.restype = C.c_char_p
        L.isr_last_device_error.argtypes = []
        for name in EXPORTS:
            if name not in ("isr_workspace_bytes", "isr_strerror", "isr_noise_bank_static_capacity",
                            "isr_float_workspace_bytes", "isr_float_chunk"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(status: int, what: str):
    if status != ISR_OK:
        raise IsrError(status, what)


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


# ---- host-only entry points -------------------------------------------------

def isr_validate_model(blob: bytes) -> int:
    buf = (C.c_char * len(blob)).from_buffer_copy(blob)
    return lib().isr_validate_model(buf, len(blob))


def isr_noise_table(sigma: int):
    R = C.c_uint32(0)
    _check(lib().isr_noise_table(sigma, None, 0, C.byref(R)), "isr_noise_table")
    T = np.zeros(2 * R.value, dtype=np.uint64)
    _check(lib().isr_noise_table(sigma, _np_ptr(T), T.size, C.byref(R)), "isr_noise_table")
    return T, R.value


def isr_cp_lower(k: int, n: int, alpha: float) -> float:
    out = C.c_double(0)
    _check(lib().isr_cp_lower(k, n, alpha, C.byref(out)), "isr_cp_lower")
    return out.value


def isr_normal_quantile(p: float) -> float:
    out = C.c_double(0)
    _check(lib().isr_normal_quantile(p, C.byref(out)), "isr_normal_quantile")
    return out.value


def isr_discrete_quantile(sigma: int, p_lower: float):
    """(t, t*t or 0): discrete-Gaussian quantile in grid units and the squared radius."""
    t, r2 = C.c_int32(0), C.c_uint64(0)
    _check(lib().isr_discrete_quantile(sigma, p_lower, C.byref(t), C.byref(r2)), "isr_discrete_quantile")
    return t.value, r2.value


def isr_binom_pvalue(n_a: int, n_b: int) -> float:
    out = C.c_double(0)
    _check(lib().isr_binom_pvalue(n_a, n_b, C.byref(out)), "isr_binom_pvalue")
    return out.value


def isr_decide_certify(counts0, counts1, sigma: float, n: int, alpha: float) -> Result:
    c0 = np.ascontiguousarray(counts0, dtype=np.uint32)
    c1 = np.ascontiguousarray(counts1, dtype=np.uint32)
    res = Result()
    _check(lib().isr_decide_certify(_np_ptr(c0), _np_ptr(c1), c0.size, sigma, n, alpha, C.byref(res)),
           "isr_decide_certify")
    return res


def isr_decide_predict(counts, alpha: float) -> Result:
    c = np.ascontiguousarray(counts, dtype=np.uint32)
    res = Result()
    _check(lib().isr_decide_predict(_np_ptr(c), c.size, alpha, C.byref(res)), "isr_decide_predict")
    return res


def isr_certified_metrics(results, labels, radii):
    """(CP, CA at each radius) of a list of Result against ground-truth labels."""
    arr = (Result * len(results))(*results)
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    rad = np.ascontiguousarray(radii, dtype=np.float64)
    assert lab.size == len(results)
    cp = C.c_double(0)
    ca = np.zeros(rad.size, dtype=np.float64)
    _check(lib().isr_certified_metrics(arr, _np_ptr(lab), len(results), _np_ptr(rad), rad.size, C.byref(cp), _np_ptr(ca)),
           "isr_certified_metrics")
    return cp.value, ca


# ---- device entry points ----------------------------------------------------

class Model:
    """Handle returned by isr_load_model plus the torch-owned workspace."""

    def __init__(self, handle, blob_len):
        self.handle = handle
        self.workspace = None
        self.chunk = 0
        info = [C.c_int(0) for _ in range(4)]
        _check(lib().isr_model_info(handle, *[C.byref(v) for v in info]), "isr_model_info")
        self.C, self.H, self.W, self.classes = [v.value for v in info]
        self.blob_len = blob_len

    def close(self):
        if self.handle:
            lib().isr_free_model(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def isr_load_model(blob: bytes) -> Model:
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("isr_load_model needs a HIP device")
    buf = (C.c_char * len(blob)).from_buffer_copy(blob)
    h = C.c_void_p(None)
    _check(lib().isr_load_model(buf, len(blob), C.byref(h)), "isr_load_model")
    return Model(h, len(blob))


def isr_workspace_bytes(model: Model, chunk_samples: int) -> int:
    return int(lib().isr_workspace_bytes(model.handle, chunk_samples))


def isr_set_workspace(model: Model, chunk_samples: int, stream=None, float_fp: bool = False):
    """Allocates the device scratch as a torch uint8 tensor and hands it over
    together with the current (or given) torch stream.  float_fp: also large enough for the
    fp32 network of the FloatRS-fp comparison system."""
    import torch
    need = isr_workspace_bytes(model, chunk_samples)
    if float_fp:
        need = max(need, int(lib().isr_float_workspace_bytes(model.handle, chunk_samples, FLOATRS_FP)))
    if need == 0:
        raise IsrError(ISR_ERR_ARG, "isr_workspace_bytes")
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    ptr = (ws.data_ptr() + 255) // 256 * 256
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(lib().isr_set_workspace(model.handle, C.c_void_p(ptr), need, chunk_samples, C.c_void_p(st.cuda_stream)),
           "isr_set_workspace")
    model.workspace, model.chunk, model.stream = ws, chunk_samples, st


def _dev_image(model, x):
    """uint8 [C][H][W] image on the device (torch tensor); numpy input is uploaded with a blocking
    copy, so it is resident whatever stream the library works on.  A tensor the caller produced on
    another stream than the model's must be ordered before the call by the caller."""
    import torch
    if isinstance(x, np.ndarray):
        x = torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint8)).cuda()
    assert x.dtype == torch.uint8 and x.is_cuda and x.is_contiguous()
    # the kernels read exactly C*H*W bytes from this pointer
    if x.numel() != model.C * model.H * model.W:
        raise IsrError(ISR_ERR_ARG, f"image of {x.numel()} bytes for a {model.C}x{model.H}x{model.W} model")
    return x


def isr_certify(model: Model, x, sigma: int, n0: int, n: int, alpha: float, seed: int = 0, image_id: int = 0,
                want_counts: bool = True):
    x = _dev_image(model, x)
    res = Result()
    c0 = np.zeros(model.classes, dtype=np.uint32) if want_counts else None
    c1 = np.zeros(model.classes, dtype=np.uint32) if want_counts else None
    _check(lib().isr_certify(model.handle, C.c_void_p(x.data_ptr()), sigma, n0, n, alpha, C.c_uint64(seed), image_id,
                             C.byref(res), _np_ptr(c0), _np_ptr(c1)), "isr_certify")
    return res, c0, c1


def isr_predict(model: Model, x, sigma: int, n: int, alpha: float, seed: int = 0, image_id: int = 0):
    x = _dev_image(model, x)
    res = Result()
    c = np.zeros(model.classes, dtype=np.uint32)
    _check(lib().isr_predict(model.handle, C.c_void_p(x.data_ptr()), sigma, n, alpha, C.c_uint64(seed), image_id,
                             C.byref(res), _np_ptr(c)), "isr_predict")
    return res, c


def isr_noise_bank(sigma: int, seed: int, bank_id: int, first: int, count: int, d: int, out=None):
    """int16 [count][d] torch tensor (device) of discrete-Gaussian draws for stored training noise."""
    import torch
    if out is None:
        out = torch.empty((count, d), dtype=torch.int16, device="cuda")
    assert out.dtype == torch.int16 and out.is_cuda and out.is_contiguous() and out.numel() == count * d
    st = torch.cuda.current_stream()
    _check(lib().isr_noise_bank(sigma, C.c_uint64(seed), bank_id, first, count, d, C.c_void_p(out.data_ptr()),
                                C.c_void_p(st.cuda_stream)), "isr_noise_bank")
    return out


def isr_noise_bank_static(sigma: int, seed: int, bank_id: int, first: int, count: int, d: int, out):
    """isr_noise_bank into a caller-provided int16 [count][d] device tensor with no device allocation
    inside the library (the table goes into the library's fixed device array)."""
    import torch
    assert out.dtype == torch.int16 and out.is_cuda and out.is_contiguous() and out.numel() == count * d
    st = torch.cuda.current_stream()
    _check(lib().isr_noise_bank_static(sigma, C.c_uint64(seed), bank_id, first, count, d, C.c_void_p(out.data_ptr()),
                                       C.c_void_p(st.cuda_stream)), "isr_noise_bank_static")
    return out


def _dev_images(model, xs):
    """uint8 [n][C][H][W] image array on the device."""
    import torch
    if isinstance(xs, np.ndarray):
        xs = torch.from_numpy(np.ascontiguousarray(xs, dtype=np.uint8)).cuda()
    assert xs.dtype == torch.uint8 and xs.is_cuda and xs.is_contiguous() and xs.dim() == 4
    if tuple(xs.shape[1:]) != (model.C, model.H, model.W):
        raise IsrError(ISR_ERR_ARG, f"images of shape {tuple(xs.shape[1:])} for a {model.C}x{model.H}x{model.W} model")
    return xs


def _items(items):
    return (Item * len(items))(*[Item(int(i), int(s), int(d)) for i, s, d in items])


def isr_certify_batch(model: Model, xs, items, n0: int, n: int, alpha: float, seed: int = 0):
    """items: list of (image index, sigma, image_id).  Returns (results, counts0, counts1)."""
    xs = _dev_images(model, xs)
    res = (Result * len(items))()
    c0 = np.zeros((len(items), model.classes), dtype=np.uint32)
    c1 = np.zeros((len(items), model.classes), dtype=np.uint32)
    _check(lib().isr_certify_batch(model.handle, C.c_void_p(xs.data_ptr()), xs.shape[0], _items(items), len(items), n0, n,
                                   alpha, C.c_uint64(seed), res, _np_ptr(c0), _np_ptr(c1)), "isr_certify_batch")
    return list(res), c0, c1


def isr_predict_batch(model: Model, xs, items, n: int, alpha: float, seed: int = 0):
    xs = _dev_images(model, xs)
    res = (Result * len(items))()
    c = np.zeros((len(items), model.classes), dtype=np.uint32)
    _check(lib().isr_predict_batch(model.handle, C.c_void_p(xs.data_ptr()), xs.shape[0], _items(items), len(items), n,
                                   alpha, C.c_uint64(seed), res, _np_ptr(c)), "isr_predict_batch")
    return list(res), c


def isr_debug_noisy(model: Model, x, sigma: int, seed: int, image_id: int, phase: int, sample_begin: int, count: int):
    x = _dev_image(model, x)
    out = np.zeros((count, model.C, model.H, model.W), dtype=np.int8)
    _check(lib().isr_debug_noisy(model.handle, C.c_void_p(x.data_ptr()), sigma, C.c_uint64(seed), image_id, phase,
                                 sample_begin, count, _np_ptr(out)), "isr_debug_noisy")
    return out


def isr_debug_forward(model: Model, x, sigma: int, seed: int, image_id: int, phase: int, sample_begin: int,
                      count: int, want_logits: bool = True):
    x = _dev_image(model, x)
    logits = np.zeros((count, model.classes), dtype=np.int32) if want_logits else None
    argmax = np.zeros(count, dtype=np.int32)
    counts = np.zeros(model.classes, dtype=np.uint32)
    _check(lib().isr_debug_forward(model.handle, C.c_void_p(x.data_ptr()), sigma, C.c_uint64(seed), image_id, phase,
                                   sample_begin, count, _np_ptr(logits), _np_ptr(argmax), _np_ptr(counts)),
           "isr_debug_forward")
    return logits, argmax, counts


def isr_debug_tensor(model: Model, x, sigma: int, seed: int, image_id: int, phase: int, sample: int,
                     tensor_id: int, shape):
    x = _dev_image(model, x)
    out = np.zeros(shape, dtype=np.int8)
    _check(lib().isr_debug_tensor(model.handle, C.c_void_p(x.data_ptr()), sigma, C.c_uint64(seed), image_id, phase,
                                  sample, tensor_id, _np_ptr(out)), "isr_debug_tensor")
    return out


def isr_float_chunk(model: Model, system: int) -> int:
    return int(lib().isr_float_chunk(model.handle, system))


def isr_float_certify(model: Model, x, sigma: float, n0: int, n: int, alpha: float, system: int, seed: int = 0,
                      image_id: int = 0):
    """Alg. 1 run by a comparison system (FLOATRS_QUANT / FLOATRS_FP).  Returns (result, counts0, counts1)."""
    x = _dev_image(model, x)
    res = Result()
    c0 = np.zeros(model.classes, dtype=np.uint32)
    c1 = np.zeros(model.classes, dtype=np.uint32)
    _check(lib().isr_float_certify(model.handle, C.c_void_p(x.data_ptr()), C.c_float(sigma), n0, n, alpha, C.c_uint64(seed),
                                   image_id, system, C.byref(res), _np_ptr(c0), _np_ptr(c1)), "isr_float_certify")
    return res, c0, c1


def isr_float_debug_noisy(model: Model, x, sigma: float, seed: int, image_id: int, phase: int, sample_begin: int,
                          count: int, system: int):
    x = _dev_image(model, x)
    out = np.zeros((count, model.C, model.H, model.W), dtype=np.int8 if system == FLOATRS_QUANT else np.float32)
    _check(lib().isr_float_debug_noisy(model.handle, C.c_void_p(x.data_ptr()), C.c_float(sigma), C.c_uint64(seed), image_id,
                                       phase, sample_begin, count, system, _np_ptr(out)), "isr_float_debug_noisy")
    return out


def isr_float_debug_forward(model: Model, x, sigma: float, seed: int, image_id: int, phase: int, sample_begin: int,
                            count: int, system: int, want_logits: bool = True):
    x = _dev_image(model, x)
    logits = None
    if want_logits:
        logits = np.zeros((count, model.classes), dtype=np.int32 if system == FLOATRS_QUANT else np.float32)
    argmax = np.zeros(count, dtype=np.int32)
    counts = np.zeros(model.classes, dtype=np.uint32)
    _check(lib().isr_float_debug_forward(model.handle, C.c_void_p(x.data_ptr()), C.c_float(sigma), C.c_uint64(seed), image_id,
                                         phase, sample_begin, count, system, _np_ptr(logits), _np_ptr(argmax),
                                         _np_ptr(counts)), "isr_float_debug_forward")
    return logits, argmax, counts


def isr_float_debug_tensor(model: Model, x, sigma: float, seed: int, image_id: int, phase: int, sample: int,
                           tensor_id: int, shape):
    x = _dev_image(model, x)
    out = np.zeros(shape, dtype=np.float32)
    _check(lib().isr_float_debug_tensor(model.handle, C.c_void_p(x.data_ptr()), C.c_float(sigma), C.c_uint64(seed), image_id,
                                        phase, sample, tensor_id, _np_ptr(out)), "isr_float_debug_tensor")
    return out


def isr_debug_tensor_source(model: Model, tensor_id: int) -> bool:
    """True when isr_debug_tensor returns the fused kernels' own output for this tensor."""
    out = C.c_int(0)
    _check(lib().isr_debug_tensor_source(model.handle, tensor_id, C.byref(out)), "isr_debug_tensor_source")
    return bool(out.value)


def isr_set_fusion(model: Model, enable):
    """False / 0: one kernel per op; True / 1: the default fusions; 2: every fusion the kernels cover."""
    _check(lib().isr_set_fusion(model.handle, int(enable)), "isr_set_fusion")


def isr_set_conv_tile(model: Model, tile: int):
    _check(lib().isr_set_conv_tile(model.handle, tile), "isr_set_conv_tile")


def isr_profile(model: Model, every_chunks: int):
    _check(lib().isr_profile(model.handle, every_chunks), "isr_profile")


def isr_profile_read(model: Model):
    """List of dicts: name, is_conv, launches, total_ms, alg_ops, alg_bytes per kernel instance."""
    arr = (KernelStat * 64)()
    n = C.c_uint32(0)
    _check(lib().isr_profile_read(model.handle, arr, 64, C.byref(n)), "isr_profile_read")
    return [dict(name=arr[i].name.decode(), is_conv=bool(arr[i].is_conv), launches=int(arr[i].launches),
                 total_ms=arr[i].total_ms, alg_ops=arr[i].alg_ops, alg_bytes=arr[i].alg_bytes)
            for i in range(min(n.value, 64))]
