"""ctypes binding of libcdsgd.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (include/cdsgd.h).
PyTorch is used for device memory and the current stream, nothing else.  There
is no fallback: a missing library is an error.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcdsgd.so")

MAX_WORKERS = 64
STATIC_MAX_TENSORS, STATIC_MAX_CHUNKS, STATIC_CHUNK_ELEMS = 1024, 524288, 4096   # cdsgd_step_fused_static
PASS_WARMUP, PASS_COMPRESSED, PASS_CORRECTION = 0, 1, 2
GRAD_DTYPES = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}   # cdsgd_grad_dtype
OK, ERR_NULL, ERR_SIZE, ERR_PARAM, ERR_ALIGN, ERR_WORKERS, ERR_DEVICE, ERR_ALIAS = range(8)


class CdsgdError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        msg = lib().cdsgd_status_string(int(status)).decode()
        super().__init__("%s: status %d (%s)" % (where, self.status, msg))


class cdsgd_tensor(ctypes.Structure):
    _fields_ = [("w_global", ctypes.c_void_p), ("w_local", ctypes.c_void_p),
                ("residual", ctypes.c_void_p), ("grad", ctypes.c_void_p),
                ("packed_self", ctypes.c_void_p), ("agg_full", ctypes.c_void_p),
                ("n", ctypes.c_size_t)]


class cdsgd_cost_params(ctypes.Structure):
    _fields_ = [("tau", ctypes.c_double), ("phi", ctypes.c_double), ("psi", ctypes.c_double),
                ("delta", ctypes.c_double), ("k", ctypes.c_int)]


class cdsgd_cost(ctypes.Structure):
    _fields_ = [("t_ssgd", ctypes.c_double), ("t_loc", ctypes.c_double), ("t_bit", ctypes.c_double),
                ("phi_cd", ctypes.c_double), ("t_cd", ctypes.c_double), ("save_vs_bit", ctypes.c_double),
                ("save_vs_loc", ctypes.c_double), ("case_bit", ctypes.c_int), ("case_loc", ctypes.c_int),
                ("eq9_assumption_holds", ctypes.c_int)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libcdsgd.so is not built (run: python -m paper_2106_10796_amd.build); "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, f, i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_int
        L.cdsgd_packed_words.restype = sz
        L.cdsgd_packed_words.argtypes = [sz]
        L.cdsgd_status_string.restype = ctypes.c_char_p
        L.cdsgd_status_string.argtypes = [i]
        L.cdsgd_build_id.restype = ctypes.c_char_p
        L.cdsgd_build_id.argtypes = []
        L.cdsgd_quantize_pack.restype = i
        L.cdsgd_quantize_pack.argtypes = [vp, vp, vp, sz, f, vp]
        L.cdsgd_decode_sum.restype = i
        L.cdsgd_decode_sum.argtypes = [ctypes.POINTER(vp), i, vp, sz, f, vp]
        L.cdsgd_update.restype = i
        L.cdsgd_update.argtypes = [vp, vp, vp, vp, sz, f, f, i, vp]
        L.cdsgd_plan_create.restype = i
        L.cdsgd_plan_create.argtypes = [ctypes.POINTER(cdsgd_tensor), i, ctypes.POINTER(ctypes.POINTER(vp)),
                                        i, i, ctypes.POINTER(vp)]
        L.cdsgd_plan_destroy.restype = i
        L.cdsgd_plan_destroy.argtypes = [vp]
        L.cdsgd_step_fused.restype = i
        L.cdsgd_step_fused.argtypes = [vp, ctypes.c_long, i, f, f, f, vp]
        L.cdsgd_plan_create_typed.restype = i
        L.cdsgd_plan_create_typed.argtypes = [ctypes.POINTER(cdsgd_tensor), i, ctypes.POINTER(ctypes.POINTER(vp)),
                                              i, i, i, ctypes.POINTER(vp)]
        L.cdsgd_plan_set_thresholds.restype = i
        L.cdsgd_plan_set_thresholds.argtypes = [vp, ctypes.POINTER(f)]
        L.cdsgd_sparse_segments.restype = sz
        L.cdsgd_sparse_segments.argtypes = [sz]
        L.cdsgd_sparse_words.restype = sz
        L.cdsgd_sparse_words.argtypes = [sz]
        L.cdsgd_sparse_encode.restype = i
        L.cdsgd_sparse_encode.argtypes = [vp, sz, vp, vp, vp]
        L.cdsgd_decode_sum_sparse.restype = i
        L.cdsgd_decode_sum_sparse.argtypes = [ctypes.POINTER(vp), i, vp, sz, f, vp]
        L.cdsgd_plan_set_peer_format.restype = i
        L.cdsgd_plan_set_peer_format.argtypes = [vp, i]
        L.cdsgd_probe_streams.restype = i
        L.cdsgd_probe_streams.argtypes = [ctypes.POINTER(vp), i, ctypes.POINTER(vp), i, sz, vp, ctypes.c_uint, vp]
        L.cdsgd_plan_set_max_workgroups.restype = i
        L.cdsgd_plan_set_max_workgroups.argtypes = [vp, i]
        L.cdsgd_step_local.restype = i
        L.cdsgd_step_local.argtypes = [vp, f, vp]
        L.cdsgd_step_global.restype = i
        L.cdsgd_step_global.argtypes = [vp, ctypes.c_long, i, f, f, vp]
        L.cdsgd_step_fused_range.restype = i
        L.cdsgd_step_fused_range.argtypes = [vp, i, i, ctypes.c_long, i, f, f, f, vp]
        L.cdsgd_step_local_range.restype = i
        L.cdsgd_step_local_range.argtypes = [vp, i, i, f, vp]
        L.cdsgd_step_global_range.restype = i
        L.cdsgd_step_global_range.argtypes = [vp, i, i, ctypes.c_long, i, f, f, vp]
        L.cdsgd_plan_bind_full_grads.restype = i
        L.cdsgd_plan_bind_full_grads.argtypes = [vp, ctypes.POINTER(ctypes.POINTER(vp))]
        L.cdsgd_step_warmup.restype = i
        L.cdsgd_step_warmup.argtypes = [vp, ctypes.c_long, ctypes.c_long, f, f, vp]
        L.cdsgd_trainer_create.restype = i
        L.cdsgd_trainer_create.argtypes = [vp, ctypes.c_long, i, f, f, f, ctypes.POINTER(vp)]
        L.cdsgd_trainer_step.restype = i
        L.cdsgd_trainer_step.argtypes = [vp, vp, ctypes.POINTER(i)]
        L.cdsgd_trainer_iteration.restype = ctypes.c_long
        L.cdsgd_trainer_iteration.argtypes = [vp]
        L.cdsgd_trainer_destroy.restype = i
        L.cdsgd_trainer_destroy.argtypes = [vp]
        L.cdsgd_step_fused_static.restype = i
        L.cdsgd_step_fused_static.argtypes = [ctypes.POINTER(cdsgd_tensor), i, ctypes.POINTER(ctypes.POINTER(vp)),
                                              i, i, i, ctypes.c_long, i, f, f, f, vp]
        L.cdsgd_cost_iteration.restype = i
        L.cdsgd_cost_iteration.argtypes = [ctypes.POINTER(cdsgd_cost_params), ctypes.c_long,
                                           ctypes.POINTER(cdsgd_cost)]
        L.cdsgd_cost_period_mean.restype = i
        L.cdsgd_cost_period_mean.argtypes = [ctypes.POINTER(cdsgd_cost_params), ctypes.POINTER(cdsgd_cost)]
        _lib = L
    return _lib


def packed_words(n: int) -> int:
    return int(lib().cdsgd_packed_words(int(n)))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, n=None, name="tensor"):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))
    if n is not None and t.numel() != n:
        raise ValueError("%s has %d elements, expected %d" % (name, t.numel(), n))
    return ctypes.c_void_p(t.data_ptr())


# packed streams are stored in int32 tensors (torch has no full uint32 support); the bits are what matter
PACKED_DTYPE = torch.int32


def new_packed(n: int, device="cuda") -> torch.Tensor:
    return torch.empty(packed_words(n), dtype=PACKED_DTYPE, device=device)


def _check(status, where):
    if status != OK:
        raise CdsgdError(status, where)


def cdsgd_quantize_pack(grad, residual, packed, threshold):
    n = grad.numel()
    st = lib().cdsgd_quantize_pack(_dev(grad, torch.float32, None, "grad"),
                                   _dev(residual, torch.float32, n, "residual"),
                                   _dev(packed, PACKED_DTYPE, packed_words(n), "packed"),
                                   n, float(threshold), _stream())
    _check(st, "cdsgd_quantize_pack")


def cdsgd_decode_sum(packed_list, agg, threshold):
    n = agg.numel()
    N = len(packed_list)
    arr = (ctypes.c_void_p * max(N, 1))()
    for j, p in enumerate(packed_list):
        arr[j] = _dev(p, PACKED_DTYPE, packed_words(n), "packed[%d]" % j)
    st = lib().cdsgd_decode_sum(arr, N, _dev(agg, torch.float32, None, "agg"), n, float(threshold), _stream())
    _check(st, "cdsgd_decode_sum")


PEERS_PACKED, PEERS_SPARSE = 0, 1   # cdsgd_peer_format


def sparse_segments(n: int) -> int:
    return int(lib().cdsgd_sparse_segments(int(n)))


def sparse_words(n: int) -> int:
    return int(lib().cdsgd_sparse_words(int(n)))


def new_sparse(n: int, device="cuda") -> torch.Tensor:
    return torch.empty(sparse_words(n), dtype=PACKED_DTYPE, device=device)


def cdsgd_sparse_encode(packed, n, sparse, segment_words=None):
    st = lib().cdsgd_sparse_encode(_dev(packed, PACKED_DTYPE, packed_words(n), "packed"), int(n),
                                   _dev(sparse, PACKED_DTYPE, sparse_words(n), "sparse"),
                                   _dev(segment_words, PACKED_DTYPE, sparse_segments(n), "segment_words"), _stream())
    _check(st, "cdsgd_sparse_encode")


def cdsgd_decode_sum_sparse(sparse_list, agg, threshold):
    n = agg.numel()
    N = len(sparse_list)
    arr = (ctypes.c_void_p * max(N, 1))()
    for j, p in enumerate(sparse_list):
        arr[j] = _dev(p, PACKED_DTYPE, sparse_words(n), "sparse[%d]" % j)
    st = lib().cdsgd_decode_sum_sparse(arr, N, _dev(agg, torch.float32, None, "agg"), n, float(threshold), _stream())
    _check(st, "cdsgd_decode_sum_sparse")


def cdsgd_probe_streams(reads, writes, sink=None, lds_bytes=0):
    """Bare streaming of len(reads) read and len(writes) write streams (cdsgd_probe_streams)."""
    n = (reads + writes)[0].numel()
    ra = (ctypes.c_void_p * max(len(reads), 1))(*[_dev(t, torch.float32, n, "reads").value for t in reads])
    wa = (ctypes.c_void_p * max(len(writes), 1))(*[_dev(t, torch.float32, n, "writes").value for t in writes])
    st = lib().cdsgd_probe_streams(ra, len(reads), wa, len(writes), n,
                                   _dev(sink, torch.float32, None, "sink"), int(lds_bytes), _stream())
    _check(st, "cdsgd_probe_streams")


def cdsgd_update(w_global, w_local, grad_local, agg, lr_local, lr_global, num_workers):
    n = w_global.numel()
    st = lib().cdsgd_update(_dev(w_global, torch.float32, None, "w_global"),
                            _dev(w_local, torch.float32, n, "w_local"),
                            _dev(grad_local, torch.float32, n, "grad_local"),
                            _dev(agg, torch.float32, n, "agg"),
                            n, float(lr_local), float(lr_global), int(num_workers), _stream())
    _check(st, "cdsgd_update")


def cdsgd_cost_iteration(tau, phi, psi, delta, k, i) -> dict:
    p = cdsgd_cost_params(float(tau), float(phi), float(psi), float(delta), int(k))
    out = cdsgd_cost()
    _check(lib().cdsgd_cost_iteration(ctypes.byref(p), int(i), ctypes.byref(out)), "cdsgd_cost_iteration")
    return out.as_dict()


def cdsgd_cost_period_mean(tau, phi, psi, delta, k) -> dict:
    p = cdsgd_cost_params(float(tau), float(phi), float(psi), float(delta), int(k))
    out = cdsgd_cost()
    _check(lib().cdsgd_cost_period_mean(ctypes.byref(p), ctypes.byref(out)), "cdsgd_cost_period_mean")
    return out.as_dict()


def _marshal_layer_list(tensors, peers, num_workers, grad_dtype, peers_sparse=False):
    """The C arrays of a layer list: (cdsgd_tensor[T], peers' row table or None, keep-alive list)."""
    peer_words = sparse_words if peers_sparse else packed_words
    T = len(tensors)
    if grad_dtype not in GRAD_DTYPES:
        raise TypeError("gradients must be float32, bfloat16 or float16")
    arr = (cdsgd_tensor * max(T, 1))()
    for i, t in enumerate(tensors):
        n = t["w_global"].numel()
        arr[i].w_global = _dev(t["w_global"], torch.float32, None, "w_global").value
        arr[i].w_local = _dev(t["w_local"], torch.float32, n, "w_local").value
        arr[i].residual = _dev(t["residual"], torch.float32, n, "residual").value
        arr[i].grad = _dev(t["grad"], grad_dtype, n, "grad").value
        arr[i].packed_self = _dev(t["packed_self"], PACKED_DTYPE, packed_words(n), "packed_self").value
        af = t.get("agg_full")
        arr[i].agg_full = _dev(af, torch.float32, n, "agg_full").value if af is not None else None
        arr[i].n = n
    if peers is None:
        return arr, None, []
    rows = (ctypes.POINTER(ctypes.c_void_p) * max(num_workers, 1))()
    keep = []
    for j in range(num_workers):
        if peers[j] is None:
            rows[j] = ctypes.POINTER(ctypes.c_void_p)()
            continue
        row = (ctypes.c_void_p * max(T, 1))()
        for i in range(T):
            n = tensors[i]["w_global"].numel()
            row[i] = _dev(peers[j][i], PACKED_DTYPE, peer_words(n), "peers[%d][%d]" % (j, i)).value
        keep.append(row)
        rows[j] = ctypes.cast(row, ctypes.POINTER(ctypes.c_void_p))
    return arr, rows, keep


def cdsgd_step_fused_static(tensors, peers, num_workers, self_rank, step, k, threshold, lr_local, lr_global,
                            grad_dtype=torch.float32):
    """One fused pass over a layer list without a plan and without any allocation in the library
    (cdsgd_step_fused_static); tensors and peers as for Plan."""
    arr, rows, _keep = _marshal_layer_list(tensors, peers, num_workers, grad_dtype)
    st = lib().cdsgd_step_fused_static(arr, len(tensors), rows, int(num_workers), int(self_rank),
                                       GRAD_DTYPES[grad_dtype], int(step), int(k), float(threshold),
                                       float(lr_local), float(lr_global), _stream())
    _check(st, "cdsgd_step_fused_static")


class StaticLayerList:
    """A layer list marshalled once for cdsgd_step_fused_static: the host arrays the call reads are built
    here, so that step() costs what the C entry point costs (the tensors are kept alive by this object)."""

    def __init__(self, tensors, peers, num_workers, grad_dtype=torch.float32):
        self._keep = (tensors, peers)
        self._n = len(tensors)
        self._num_workers = int(num_workers)
        self._grad = GRAD_DTYPES[grad_dtype]
        self._arr, self._rows, self._rows_keep = _marshal_layer_list(tensors, peers, num_workers, grad_dtype)

    def step(self, self_rank, step, k, threshold, lr_local, lr_global):
        st = lib().cdsgd_step_fused_static(self._arr, self._n, self._rows, self._num_workers, int(self_rank),
                                           self._grad, int(step), int(k), float(threshold), float(lr_local),
                                           float(lr_global), _stream())
        _check(st, "cdsgd_step_fused_static")


class Plan:
    """A fused-step plan over a layer list (cdsgd_plan_create / cdsgd_step_fused / cdsgd_plan_destroy).

    tensors: list of dicts with keys w_global, w_local, residual, grad, packed_self and
    optionally agg_full (torch CUDA tensors).  peers: list over workers of lists over
    tensors of packed tensors (sparse buffers with peers_sparse=True); the entry for `self_rank`
    may be None.  The plan keeps
    references to every tensor so that the borrowed pointers stay valid.
    """

    def __init__(self, tensors, peers, num_workers, self_rank, grad_dtype=torch.float32, peers_sparse=False):
        T = len(tensors)
        self._grad_dtype = grad_dtype
        self._keep = (tensors, peers)
        arr, rows, self._rows = _marshal_layer_list(tensors, peers, num_workers, grad_dtype, peers_sparse)
        self._sizes = [t["w_global"].numel() for t in tensors]
        handle = ctypes.c_void_p()
        if grad_dtype == torch.float32:
            st = lib().cdsgd_plan_create(arr, T, rows, int(num_workers), int(self_rank), ctypes.byref(handle))
        else:
            st = lib().cdsgd_plan_create_typed(arr, T, rows, int(num_workers), int(self_rank),
                                               GRAD_DTYPES[grad_dtype], ctypes.byref(handle))
        _check(st, "cdsgd_plan_create")
        self._handle = handle
        self.num_workers = int(num_workers)
        if peers_sparse:
            self.set_peer_format(PEERS_SPARSE)

    def step(self, step, k, threshold, lr_local, lr_global):
        st = lib().cdsgd_step_fused(self._handle, int(step), int(k), float(threshold), float(lr_local),
                                    float(lr_global), _stream())
        _check(st, "cdsgd_step_fused")

    def set_thresholds(self, thresholds):
        """One threshold per tensor (list of floats), or None to go back to the call's threshold."""
        if thresholds is None:
            st = lib().cdsgd_plan_set_thresholds(self._handle, None)
        else:
            if len(thresholds) != len(self._sizes):
                raise ValueError("need one threshold per tensor")
            arr = (ctypes.c_float * len(thresholds))(*[float(x) for x in thresholds])
            st = lib().cdsgd_plan_set_thresholds(self._handle, arr)
        _check(st, "cdsgd_plan_set_thresholds")

    def set_peer_format(self, fmt):
        """PEERS_PACKED or PEERS_SPARSE: how compressed passes read the peers' streams (cdsgd_plan_set_peer_format)."""
        _check(lib().cdsgd_plan_set_peer_format(self._handle, int(fmt)), "cdsgd_plan_set_peer_format")

    def set_max_workgroups(self, max_workgroups):
        """At most this many workgroups per pass (0: one per chunk); cdsgd_plan_set_max_workgroups."""
        _check(lib().cdsgd_plan_set_max_workgroups(self._handle, int(max_workgroups)),
               "cdsgd_plan_set_max_workgroups")

    def step_local(self, lr_local):
        st = lib().cdsgd_step_local(self._handle, float(lr_local), _stream())
        _check(st, "cdsgd_step_local")

    def step_global(self, step, k, threshold, lr_global):
        st = lib().cdsgd_step_global(self._handle, int(step), int(k), float(threshold), float(lr_global), _stream())
        _check(st, "cdsgd_step_global")

    def step_range(self, first_tensor, num_tensors, step, k, threshold, lr_local, lr_global):
        """The fused pass over tensors [first_tensor, first_tensor + num_tensors) only (cdsgd_step_fused_range)."""
        st = lib().cdsgd_step_fused_range(self._handle, int(first_tensor), int(num_tensors), int(step), int(k),
                                          float(threshold), float(lr_local), float(lr_global), _stream())
        _check(st, "cdsgd_step_fused_range")

    def step_local_range(self, first_tensor, num_tensors, lr_local):
        st = lib().cdsgd_step_local_range(self._handle, int(first_tensor), int(num_tensors), float(lr_local), _stream())
        _check(st, "cdsgd_step_local_range")

    def step_global_range(self, first_tensor, num_tensors, step, k, threshold, lr_global):
        st = lib().cdsgd_step_global_range(self._handle, int(first_tensor), int(num_tensors), int(step), int(k),
                                           float(threshold), float(lr_global), _stream())
        _check(st, "cdsgd_step_global_range")

    def bind_full_grads(self, peer_grads):
        """peer_grads[j][i]: worker j's fp32 gradient of tensor i; entry self_rank may be None
        (cdsgd_plan_bind_full_grads).  Correction and warm-up passes then sum in the kernel."""
        T = len(self._sizes)
        rows = (ctypes.POINTER(ctypes.c_void_p) * max(self.num_workers, 1))()
        keep = []
        for j in range(self.num_workers):
            if peer_grads[j] is None:
                rows[j] = ctypes.POINTER(ctypes.c_void_p)()
                continue
            row = (ctypes.c_void_p * max(T, 1))()
            for i in range(T):
                row[i] = _dev(peer_grads[j][i], self._grad_dtype, self._sizes[i], "peer_grads[%d][%d]" % (j, i)).value
            keep.append(row)
            rows[j] = ctypes.cast(row, ctypes.POINTER(ctypes.c_void_p))
        st = lib().cdsgd_plan_bind_full_grads(self._handle, rows)
        _check(st, "cdsgd_plan_bind_full_grads")
        self._keep_full = peer_grads

    def step_warmup(self, i, warmup_steps, lr_local, lr_global):
        st = lib().cdsgd_step_warmup(self._handle, int(i), int(warmup_steps), float(lr_local), float(lr_global),
                                     _stream())
        _check(st, "cdsgd_step_warmup")

    def destroy(self):
        if self._handle is not None and self._handle.value:
            lib().cdsgd_plan_destroy(self._handle)
        self._handle = None
        self._keep = None
        self._keep_full = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Trainer:
    """Alg. 1 end to end as a counter around a plan (cdsgd_trainer_*)."""

    def __init__(self, plan: Plan, warmup_steps, k, threshold, lr_local, lr_global):
        self._plan = plan
        handle = ctypes.c_void_p()
        st = lib().cdsgd_trainer_create(plan._handle, int(warmup_steps), int(k), float(threshold),
                                        float(lr_local), float(lr_global), ctypes.byref(handle))
        _check(st, "cdsgd_trainer_create")
        self._handle = handle

    def step(self) -> int:
        """Enqueue the next iteration; returns PASS_WARMUP / PASS_COMPRESSED / PASS_CORRECTION."""
        kind = ctypes.c_int(-1)
        st = lib().cdsgd_trainer_step(self._handle, _stream(), ctypes.byref(kind))
        _check(st, "cdsgd_trainer_step")
        return kind.value

    @property
    def iteration(self) -> int:
        return int(lib().cdsgd_trainer_iteration(self._handle))

    def destroy(self):
        if self._handle is not None and self._handle.value:
            lib().cdsgd_trainer_destroy(self._handle)
        self._handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
