"""ctypes binding of include/lqsgd.h.  Argument marshalling only: every step of
the compressor runs in the HIP library.  torch is used for device memory and
the stream handle, nothing else."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LQSGD_LIB points at another build of the same library (kernel experiments)
LIB_PATH = os.environ.get("LQSGD_LIB") or os.path.join(_HERE, "liblqsgd.so")

OK, EINVAL, ESHAPE, EUNSUPPORTED, ENOMEM, EHIP, ESTATE = 0, -1, -2, -3, -4, -5, -6
LAYER_MATRIX, LAYER_VECTOR = 0, 1
FLAG_NONE, FLAG_EAGER_RESIDUAL, FLAG_AGGREGATE_FIRST, FLAG_BF16_GRADIENTS, FLAG_NO_COOPERATIVE_LAUNCH = 0, 1, 2, 4, 8
PHASE_P, PHASE_Q = 0, 1
FACTOR_P_PRE, FACTOR_P_ORTH, FACTOR_P_BAR, FACTOR_Q_W, FACTOR_Q_BAR, FACTOR_VMEAN, FACTOR_P_MEAN = range(7)
(KERNEL_ADD_PROJECT, KERNEL_ORTH, KERNEL_EXCHANGE_P, KERNEL_BACK_PROJECT, KERNEL_REDUCE_Q,
 KERNEL_EXCHANGE_Q, KERNEL_RESIDUAL, KERNEL_REDUCE_P) = range(8)
KERNEL_COUNT = 8
MAX_RANK, MAX_WORKERS = 64, 64

# every symbol the header declares
SYMBOLS = [
    "lqsgd_create", "lqsgd_destroy", "lqsgd_synchronize", "lqsgd_last_error", "lqsgd_set_q",
    "lqsgd_get_state", "lqsgd_set_state", "lqsgd_compress", "lqsgd_decompress", "lqsgd_step", "lqsgd_step_update",
    "lqsgd_get_packet", "lqsgd_set_packet", "lqsgd_get_packet_raw", "lqsgd_packet_device", "lqsgd_get_factor",
    "lqsgd_set_factor", "lqsgd_wire_bytes", "lqsgd_plan_query", "lqsgd_plan_tiles",
    "lqsgd_timing_enable", "lqsgd_timing_read", "lqsgd_kernel_name", "lqsgd_launched_kernel", "lqsgd_step_static",
]


class LqsgdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("lqsgd error %d: %s" % (code, msg))
        self.code = code


class Layer(C.Structure):
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("flags", C.c_uint32)]


class Config(C.Structure):
    _fields_ = [("rank", C.c_int32), ("bits_p", C.c_int32), ("bits_q", C.c_int32),
                ("workers", C.c_int32), ("alpha", C.c_float), ("flags", C.c_uint32)]


class PlanInfo(C.Structure):
    _fields_ = [("device_bytes", C.c_int64), ("wire_bytes", C.c_int64), ("matrix_elements", C.c_int64),
                ("n_matrix", C.c_int32), ("n_vector", C.c_int32), ("rank_pad", C.c_int32),
                ("tiles", C.c_int32 * 3), ("reserved", C.c_int32),
                ("residual_stride", C.c_int64), ("warm_q_floats", C.c_int64)]


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built: there is no
    fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2506_17974_amd.build` "
                           "(there is no CPU or PyTorch fallback)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    fp = C.POINTER(C.c_float)
    u8p = C.POINTER(C.c_uint8)
    L.lqsgd_create.argtypes = [C.POINTER(Config), C.POINTER(Layer), i32, vp, C.POINTER(vp)]
    L.lqsgd_destroy.argtypes = [vp]
    L.lqsgd_synchronize.argtypes = [vp]
    L.lqsgd_last_error.argtypes = [vp]
    L.lqsgd_last_error.restype = C.c_char_p
    L.lqsgd_set_q.argtypes = [vp, i32, fp]
    L.lqsgd_get_state.argtypes = [vp, i32, i32, fp, fp]
    L.lqsgd_set_state.argtypes = [vp, i32, i32, fp, fp]
    L.lqsgd_compress.argtypes = [vp, i32, C.POINTER(vp)]
    L.lqsgd_decompress.argtypes = [vp, i32]
    L.lqsgd_step.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    L.lqsgd_step_update.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.c_float]
    L.lqsgd_step_static.argtypes = [C.POINTER(Config), C.POINTER(Layer), i32, vp, C.POINTER(vp), vp, vp, C.POINTER(vp)]
    L.lqsgd_get_packet.argtypes = [vp, i32, i32, i32, u8p, u8p, fp]
    L.lqsgd_set_packet.argtypes = [vp, i32, i32, i32, u8p, u8p, C.c_float]
    L.lqsgd_get_packet_raw.argtypes = [vp, i32, i32, i32, u8p, C.POINTER(i64), u8p, C.POINTER(i64)]
    L.lqsgd_packet_device.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_void_p), C.POINTER(i64), C.POINTER(C.c_void_p),
                                      C.POINTER(i64), C.POINTER(C.c_void_p)]
    L.lqsgd_get_factor.argtypes = [vp, i32, i32, i32, fp]
    L.lqsgd_set_factor.argtypes = [vp, i32, i32, fp]
    L.lqsgd_wire_bytes.argtypes = [vp]
    L.lqsgd_wire_bytes.restype = i64
    L.lqsgd_plan_query.argtypes = [C.POINTER(Config), C.POINTER(Layer), i32, C.POINTER(PlanInfo)]
    L.lqsgd_plan_tiles.argtypes = [C.POINTER(Config), C.POINTER(Layer), i32, i32, C.POINTER(i32), i64]
    L.lqsgd_plan_tiles.restype = i64
    L.lqsgd_timing_enable.argtypes = [vp, i32]
    L.lqsgd_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    L.lqsgd_kernel_name.argtypes = [i32]
    L.lqsgd_kernel_name.restype = C.c_char_p
    L.lqsgd_launched_kernel.argtypes = [vp, i32]
    L.lqsgd_launched_kernel.restype = C.c_char_p
    _lib = L
    return L


def _layers_array(layers: Sequence):
    arr = (Layer * len(layers))()
    for i, l in enumerate(layers):
        rows, cols = int(l[0]), int(l[1])
        flags = int(l[2]) if len(l) > 2 else LAYER_MATRIX
        arr[i] = Layer(rows, cols, flags)
    return arr


def layer_list(matrices, vectors=()):
    """[(rows, cols, flags)] with the matrices first, then the 1-D tensors."""
    return [(r, c, LAYER_MATRIX) for r, c in matrices] + [(n, 1, LAYER_VECTOR) for n in vectors]


def _f32p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _u8p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def plan_query(layers, rank, bits_p, bits_q, workers, alpha=255.0, flags=0) -> PlanInfo:
    cfg = Config(rank, bits_p, bits_q, workers, alpha, flags)
    info = PlanInfo()
    rc = lib().lqsgd_plan_query(C.byref(cfg), _layers_array(layers), len(layers), C.byref(info))
    if rc:
        raise LqsgdError(rc, lib().lqsgd_last_error(None).decode())
    return info


def plan_tiles(layers, rank, bits_p, bits_q, workers, sweep, alpha=255.0) -> np.ndarray:
    cfg = Config(rank, bits_p, bits_q, workers, alpha, 0)
    arr = _layers_array(layers)
    n = lib().lqsgd_plan_tiles(C.byref(cfg), arr, len(layers), sweep, None, 0)
    if n < 0:
        raise LqsgdError(int(n), lib().lqsgd_last_error(None).decode())
    out = np.zeros((int(n), 6), np.int32)
    lib().lqsgd_plan_tiles(C.byref(cfg), arr, len(layers), sweep,
                           out.ctypes.data_as(C.POINTER(C.c_int32)), int(n))
    return out


class Compressor:
    """One lqsgd_ctx.  Gradients are torch CUDA tensors (or anything with
    .data_ptr()); the context's kernels run on torch's current stream at
    construction time."""

    def __init__(self, layers, rank, bits_p=8, bits_q=None, workers=1, alpha=255.0, flags=0, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the LQ-SGD compressor has no CPU path")
        self.layers = [tuple(l) if len(l) > 2 else (l[0], l[1], LAYER_MATRIX) for l in layers]
        self.rank, self.workers = rank, workers
        self.bits_p = bits_p
        self.bits_q = bits_p if bits_q is None else bits_q
        self.alpha = alpha
        self._cfg = Config(rank, self.bits_p, self.bits_q, workers, alpha, flags)
        self._h = C.c_void_p()
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.stream_handle = int(stream)
        rc = lib().lqsgd_create(C.byref(self._cfg), _layers_array(self.layers), len(self.layers),
                                C.c_void_p(self.stream_handle), C.byref(self._h))
        if rc:
            self._h = C.c_void_p()
            raise LqsgdError(rc, lib().lqsgd_last_error(None).decode())
        self._keep = None

    # -- helpers ---------------------------------------------------------
    def _check(self, rc):
        if rc:
            raise LqsgdError(rc, lib().lqsgd_last_error(self._h).decode())

    def layer_rank(self, l):
        rows, cols, _ = self.layers[l]
        return min(self.rank, rows, cols)

    def _ptr_table(self, grads):
        """grads[w][l] tensors -> (c_void_p * (W*L))"""
        n = len(self.layers)
        tab = (C.c_void_p * (self.workers * n))()
        for w in range(self.workers):
            for l in range(n):
                tab[w * n + l] = grads[w][l].data_ptr()
        return tab

    def close(self):
        if self._h:
            lib().lqsgd_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- state -----------------------------------------------------------
    def set_q(self, layer, q: np.ndarray):
        q = np.ascontiguousarray(q, np.float32)
        rows, cols, _ = self.layers[layer]
        assert q.shape == (cols, self.layer_rank(layer)), q.shape
        self._check(lib().lqsgd_set_q(self._h, layer, _f32p(q)))

    def get_state(self, layer, worker, want_e=True, want_q=True):
        if not (0 <= layer < len(self.layers)):      # let the library report it
            self._check(lib().lqsgd_get_state(self._h, layer, worker, None, None))
        rows, cols, _ = self.layers[layer]
        e = np.empty((rows, cols), np.float32) if want_e else None
        q = np.empty((cols, self.layer_rank(layer)), np.float32) if want_q else None
        self._check(lib().lqsgd_get_state(self._h, layer, worker, _f32p(e) if want_e else None,
                                          _f32p(q) if want_q else None))
        return e, q

    def set_state(self, layer, worker, e: Optional[np.ndarray] = None, q: Optional[np.ndarray] = None):
        if e is not None:
            e = np.ascontiguousarray(e, np.float32)
        if q is not None:
            q = np.ascontiguousarray(q, np.float32)
        self._check(lib().lqsgd_set_state(self._h, layer, worker, _f32p(e) if e is not None else None,
                                          _f32p(q) if q is not None else None))

    # -- the compressor --------------------------------------------------
    def compress(self, phase, grads=None):
        tab = self._ptr_table(grads) if grads is not None else None
        self._keep = grads if grads is not None else self._keep
        self._check(lib().lqsgd_compress(self._h, phase, tab))

    def decompress(self, phase):
        self._check(lib().lqsgd_decompress(self._h, phase))

    def step(self, grads, ghat=None):
        tab = self._ptr_table(grads)
        gt = None
        if ghat is not None:
            gt = (C.c_void_p * len(self.layers))()
            for l, t in enumerate(ghat):
                gt[l] = t.data_ptr() if t is not None else None
        self._keep = (grads, ghat)
        self._check(lib().lqsgd_step(self._h, tab, gt))

    def step_update(self, grads, params, eta):
        """lqsgd_step_update: the iteration plus w <- w - eta G-hat on `params`
        (a list over layers of device tensors or None), in place."""
        tab = self._ptr_table(grads)
        pt = (C.c_void_p * len(self.layers))()
        for l, t in enumerate(params):
            pt[l] = t.data_ptr() if t is not None else None
        self._keep = (grads, params)
        self._check(lib().lqsgd_step_update(self._h, tab, pt, float(eta)))

    def step_raw(self, tab, gt=None):
        """lqsgd_step with a pointer table made earlier by pointer_table()."""
        self._check(lib().lqsgd_step(self._h, tab, gt))

    def pointer_table(self, grads):
        self._keep = grads
        return self._ptr_table(grads)

    def synchronize(self):
        self._check(lib().lqsgd_synchronize(self._h))

    # -- taps ------------------------------------------------------------
    def _factor_len(self, phase, layer):
        rows, cols, _ = self.layers[layer]
        return (cols if phase == PHASE_Q else rows) * self.layer_rank(layer)

    def get_packet(self, phase, layer, worker):
        n = self._factor_len(phase, layer)
        k = np.empty(n, np.uint8)
        s = np.empty(n, np.uint8)
        sc = C.c_float()
        self._check(lib().lqsgd_get_packet(self._h, phase, layer, worker, _u8p(k), _u8p(s), C.byref(sc)))
        shape = (n // self.layer_rank(layer), self.layer_rank(layer))
        return k.reshape(shape), s.reshape(shape), np.float32(sc.value)

    def set_packet(self, phase, layer, worker, k, s, scale):
        k = np.ascontiguousarray(k, np.uint8).ravel()
        s = np.ascontiguousarray(s, np.uint8).ravel()
        assert k.size == self._factor_len(phase, layer) == s.size
        self._check(lib().lqsgd_set_packet(self._h, phase, layer, worker, _u8p(k), _u8p(s), float(scale)))

    def packet_device(self, phase, layer, worker):
        """(mag_ptr, mag_len, sign_ptr, sign_len, scale_ptr): device addresses of one packet."""
        mp, sp, cp = C.c_void_p(), C.c_void_p(), C.c_void_p()
        ml, sl = C.c_int64(), C.c_int64()
        self._check(lib().lqsgd_packet_device(self._h, phase, layer, worker, C.byref(mp), C.byref(ml), C.byref(sp),
                                              C.byref(sl), C.byref(cp)))
        return mp.value, ml.value, sp.value, sl.value, cp.value

    def get_packet_raw(self, phase, layer, worker):
        ml, sl = C.c_int64(), C.c_int64()
        self._check(lib().lqsgd_get_packet_raw(self._h, phase, layer, worker, None, C.byref(ml), None, C.byref(sl)))
        mag = np.empty(ml.value, np.uint8)
        sgn = np.empty(sl.value, np.uint8)
        self._check(lib().lqsgd_get_packet_raw(self._h, phase, layer, worker, _u8p(mag), C.byref(ml),
                                               _u8p(sgn), C.byref(sl)))
        return mag, sgn

    def get_factor(self, which, layer, worker=0):
        rows, cols, flags = self.layers[layer]
        if which == FACTOR_VMEAN:
            out = np.empty(rows, np.float32)
        elif which in (FACTOR_Q_W, FACTOR_Q_BAR):
            out = np.empty((cols, self.layer_rank(layer)), np.float32)
        else:
            out = np.empty((rows, self.layer_rank(layer)), np.float32)
        self._check(lib().lqsgd_get_factor(self._h, which, layer, worker, _f32p(out)))
        return out

    def set_factor(self, which, layer, value):
        value = np.ascontiguousarray(value, np.float32)
        self._check(lib().lqsgd_set_factor(self._h, which, layer, _f32p(value)))

    def wire_bytes(self) -> int:
        return int(lib().lqsgd_wire_bytes(self._h))

    # -- timing ----------------------------------------------------------
    def timing_enable(self, on=True):
        self._check(lib().lqsgd_timing_enable(self._h, 1 if on else 0))

    def launched_kernel(self, k: int) -> str:
        """Device function last launched for timing slot k (template arguments included)."""
        return lib().lqsgd_launched_kernel(self._h, k).decode()

    def timing_read(self):
        ms = (C.c_double * KERNEL_COUNT)()
        n = (C.c_int64 * KERNEL_COUNT)()
        self._check(lib().lqsgd_timing_read(self._h, ms, n))
        return [float(x) for x in ms], [int(x) for x in n]


def step_static(layers, rank, bits_p, bits_q, workers, alpha, flags, grads, residual, warm_q, ghat=None, stream=None):
    """lqsgd_step_static: one iteration on caller-held state, no device allocation.
    grads[w][l]: device tensors; residual, warm_q: device tensors laid out as the header says
    (None when there is no matrix layer); ghat: list over layers of device tensors / None."""
    import torch
    cfg = Config(rank, bits_p, bits_q, workers, alpha, flags)
    n = len(layers)
    tab = (C.c_void_p * (workers * n))()
    for w in range(workers):
        for l in range(n):
            tab[w * n + l] = grads[w][l].data_ptr()
    gt = None
    if ghat is not None:
        gt = (C.c_void_p * n)()
        for l, t in enumerate(ghat):
            gt[l] = t.data_ptr() if t is not None else None
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    rc = lib().lqsgd_step_static(C.byref(cfg), _layers_array(layers), n, C.c_void_p(int(stream)), tab,
                                 C.c_void_p(residual.data_ptr() if residual is not None else None),
                                 C.c_void_p(warm_q.data_ptr() if warm_q is not None else None), gt)
    if rc:
        raise LqsgdError(rc, lib().lqsgd_last_error(None).decode())


def kernel_name(k: int) -> str:
    return lib().lqsgd_kernel_name(k).decode()
