"""ctypes face of the C oracle (oracle/cdsgd_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
benchmark's cpu-baseline leg may import this.  It does argument marshalling
only; every number is computed by the scalar C code.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_f32p = ctypes.POINTER(ctypes.c_float)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_u8p = ctypes.POINTER(ctypes.c_uint8)

_lib = None


def lib():
    global _lib
    if _lib is None:
        # CDSGD_ORACLE_LIB lets the mutation test load a deliberately broken build
        path = os.environ.get("CDSGD_ORACLE_LIB") or _build.LIB
        if path == _build.LIB and (not os.path.exists(path)
                                   or os.path.getmtime(path) < os.path.getmtime(_build.SRC)):
            _build.build(force=True)
        L = ctypes.CDLL(path)
        L.oracle_dequant.restype = ctypes.c_float
        L.oracle_dequant.argtypes = [ctypes.c_uint8, ctypes.c_float]
        L.oracle_quantize.restype = None
        L.oracle_quantize.argtypes = [_f32p, _f32p, _u8p, ctypes.c_size_t, ctypes.c_float]
        L.oracle_pack.restype = None
        L.oracle_pack.argtypes = [_u8p, ctypes.c_size_t, _u32p]
        L.oracle_unpack.restype = None
        L.oracle_unpack.argtypes = [_u32p, ctypes.c_size_t, _u8p]
        L.oracle_decode_sum.restype = None
        L.oracle_decode_sum.argtypes = [ctypes.POINTER(_u32p), ctypes.c_int, _f32p, ctypes.c_size_t,
                                        ctypes.c_float]
        L.oracle_full_sum.restype = None
        L.oracle_full_sum.argtypes = [ctypes.POINTER(_f32p), ctypes.c_int, _f32p, ctypes.c_size_t]
        L.oracle_update.restype = None
        L.oracle_update.argtypes = [_f32p, _f32p, _f32p, _f32p, ctypes.c_size_t, ctypes.c_float,
                                    ctypes.c_float, ctypes.c_int]
        L.oracle_step.restype = ctypes.c_int
        L.oracle_step.argtypes = [_f32p, _f32p, ctypes.POINTER(_f32p), ctypes.POINTER(_f32p),
                                  ctypes.POINTER(_u32p), _f32p, _u8p, ctypes.c_size_t, ctypes.c_int,
                                  ctypes.c_int, ctypes.c_long, ctypes.c_int, ctypes.c_float,
                                  ctypes.c_float, ctypes.c_float]
        L.oracle_trainer_step.restype = ctypes.c_int
        L.oracle_trainer_step.argtypes = [_f32p, _f32p, ctypes.POINTER(_f32p), ctypes.POINTER(_f32p),
                                          ctypes.POINTER(_u32p), _f32p, _u8p, ctypes.c_size_t, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_long, ctypes.c_long, ctypes.c_int,
                                          ctypes.c_float, ctypes.c_float, ctypes.c_float]
        L.oracle_sparse_encode.restype = None
        L.oracle_sparse_encode.argtypes = [_u32p, ctypes.c_size_t, _u32p, _u32p]
        L.oracle_sparse_decode.restype = None
        L.oracle_sparse_decode.argtypes = [_u32p, ctypes.c_size_t, _u32p]
        L.oracle_cost_model.restype = None
        L.oracle_cost_model.argtypes = [ctypes.c_double] * 4 + [ctypes.c_int, ctypes.c_long,
                                                                ctypes.POINTER(ctypes.c_double)]
        _lib = L
    return _lib


def packed_words(n: int) -> int:
    return (int(n) + 15) // 16


def _chk(a, dtype, n=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.ndim == 1 and a.flags.c_contiguous, \
        "need a contiguous 1-D %s array" % np.dtype(dtype).name
    if n is not None:
        assert a.size == n, "size %d != %d" % (a.size, n)
    return a


def _p(a, ptype):
    return a.ctypes.data_as(ptype) if a is not None else ptype()


def _ptr_array(arrays, ptype):
    arr = (ptype * len(arrays))()
    for i, a in enumerate(arrays):
        arr[i] = a.ctypes.data_as(ptype)
    return arr


def dequant(code: int, t: float) -> float:
    return float(lib().oracle_dequant(int(code), float(t)))


def quantize(grad, residual, t):
    """residual is updated in place; returns the per-element codes (uint8)."""
    n = grad.size
    _chk(grad, np.float32)
    _chk(residual, np.float32, n)
    code = np.empty(n, np.uint8)
    lib().oracle_quantize(_p(grad, _f32p), _p(residual, _f32p), _p(code, _u8p), n, float(t))
    return code


def pack(code):
    _chk(code, np.uint8)
    word = np.empty(packed_words(code.size), np.uint32)
    lib().oracle_pack(_p(code, _u8p), code.size, _p(word, _u32p))
    return word


def unpack(word, n):
    _chk(word, np.uint32, packed_words(n))
    code = np.empty(n, np.uint8)
    lib().oracle_unpack(_p(word, _u32p), n, _p(code, _u8p))
    return code


def quantize_pack(grad, residual, t):
    return pack(quantize(grad, residual, t))


def decode_sum(words, n, t):
    for w in words:
        _chk(w, np.uint32, packed_words(n))
    agg = np.empty(n, np.float32)
    lib().oracle_decode_sum(_ptr_array(words, _u32p), len(words), _p(agg, _f32p), n, float(t))
    return agg


def full_sum(grads):
    n = grads[0].size
    for g in grads:
        _chk(g, np.float32, n)
    agg = np.empty(n, np.float32)
    lib().oracle_full_sum(_ptr_array(grads, _f32p), len(grads), _p(agg, _f32p), n)
    return agg


def update(w_global, w_local, grad_local, agg, lr_local, lr_global, num_workers):
    """In place on w_global (if agg is given) and w_local (if given with grad_local)."""
    n = w_global.size
    _chk(w_global, np.float32)
    for a in (w_local, grad_local, agg):
        if a is not None:
            _chk(a, np.float32, n)
    lib().oracle_update(_p(w_global, _f32p), _p(w_local, _f32p), _p(grad_local, _f32p), _p(agg, _f32p),
                        n, float(lr_local), float(lr_global), int(num_workers))


def sparse_segments(n: int) -> int:
    return (packed_words(n) + 255) // 256


def sparse_words(n: int) -> int:
    """Capacity of a sparse buffer for n elements: 264 words per segment of 256 packed words."""
    return 264 * sparse_segments(n)


def sparse_encode(word, n, fill=0):
    """(sparse buffer, words per segment on the wire).  Slots the format leaves alone keep `fill`."""
    _chk(word, np.uint32, packed_words(n))
    sparse = np.full(sparse_words(n), fill, np.uint32)
    seg = np.zeros(sparse_segments(n), np.uint32)
    lib().oracle_sparse_encode(_p(word, _u32p), n, _p(sparse, _u32p), _p(seg, _u32p))
    return sparse, seg


def sparse_decode(sparse, n):
    _chk(sparse, np.uint32, sparse_words(n))
    word = np.empty(packed_words(n), np.uint32)
    lib().oracle_sparse_decode(_p(sparse, _u32p), n, _p(word, _u32p))
    return word


def cost_model(tau, phi, psi, delta, k, i):
    """dict of the iteration times of eq. 2, 4, 5, 6, 7 and the two savings as differences."""
    out = (ctypes.c_double * 7)()
    lib().oracle_cost_model(float(tau), float(phi), float(psi), float(delta), int(k), int(i), out)
    names = ("t_ssgd", "t_loc", "t_bit", "phi_cd", "t_cd", "save_vs_loc", "save_vs_bit")
    return dict(zip(names, list(out)))


class Simulation:
    """State of Alg. 1's FormalTraining loop for N simulated workers on one tensor.

    w_global is shared, every worker has its own residual (zero at start), and
    the observed worker `self_rank` has the local weights.  step(grads) runs
    one pass and returns (compressed, agg, words) -- words is the list of the N
    packed streams of that pass (None on a correction pass).
    """

    def __init__(self, w0, num_workers, k, t, lr_local, lr_global, self_rank=0, w_local0=None):
        self.n = w0.size
        self.N = int(num_workers)
        self.k = int(k)
        self.t = float(t)
        self.lr_local = float(lr_local)
        self.lr_global = float(lr_global)
        self.self_rank = int(self_rank)
        self.count = 0
        self.w_global = np.array(w0, dtype=np.float32, copy=True)
        # the local buffer's initial content: a copy of w0 unless the caller gives its own
        # (a sentinel, say: Alg. 1 writes the buffer before it ever reads it)
        self.w_local = np.array(w0 if w_local0 is None else w_local0, dtype=np.float32, copy=True)
        assert self.w_local.size == self.n
        self.residual = [np.zeros(self.n, np.float32) for _ in range(self.N)]
        self.word = [np.zeros(packed_words(self.n), np.uint32) for _ in range(self.N)]
        self.agg = np.zeros(self.n, np.float32)
        self._code = np.zeros(self.n, np.uint8)

    def step(self, grads):
        assert len(grads) == self.N
        for g in grads:
            _chk(g, np.float32, self.n)
        c = lib().oracle_step(_p(self.w_global, _f32p), _p(self.w_local, _f32p),
                              _ptr_array(self.residual, _f32p), _ptr_array(grads, _f32p),
                              _ptr_array(self.word, _u32p), _p(self.agg, _f32p), _p(self._code, _u8p),
                              self.n, self.N, self.self_rank, self.count, self.k, self.t,
                              self.lr_local, self.lr_global)
        self.count += 1
        words = [w.copy() for w in self.word] if c else None
        return bool(c), self.agg.copy(), words


class TrainerSimulation(Simulation):
    """Alg. 1 end to end on one tensor: WARMUP passes for iterations 0..warmup_n, then
    FormalTraining.  step(grads) returns (mode, agg, words) with mode 0 = warm-up,
    1 = compressed, 2 = correction."""

    def __init__(self, w0, num_workers, warmup_n, k, t, lr_local, lr_global, self_rank=0, w_local0=None):
        super().__init__(w0, num_workers, k, t, lr_local, lr_global, self_rank, w_local0)
        self.warmup_n = int(warmup_n)
        self.iteration = 0

    def step(self, grads):
        assert len(grads) == self.N
        for g in grads:
            _chk(g, np.float32, self.n)
        mode = lib().oracle_trainer_step(_p(self.w_global, _f32p), _p(self.w_local, _f32p),
                                         _ptr_array(self.residual, _f32p), _ptr_array(grads, _f32p),
                                         _ptr_array(self.word, _u32p), _p(self.agg, _f32p),
                                         _p(self._code, _u8p), self.n, self.N, self.self_rank,
                                         self.iteration, self.warmup_n, self.k, self.t, self.lr_local,
                                         self.lr_global)
        self.iteration += 1
        words = [w.copy() for w in self.word] if mode == 1 else None
        return int(mode), self.agg.copy(), words
