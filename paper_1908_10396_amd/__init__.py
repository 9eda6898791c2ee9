"""Python binding of libavq (include/avq.h): argument marshalling only.

Every step of the query path, training and encoding runs in the HIP kernels of
libavq.so; this module loads the library with ctypes, passes torch tensors'
device pointers through, and turns error codes into exceptions. There is no
CPU fallback: if the library is missing, importing `lib()` raises.
Function names follow the C ABI (avq_create -> Index(...), avq_search ->
Index.search, ...).
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libavq.so")

AVQ_OK, AVQ_EINVAL, AVQ_ESTATE, AVQ_ENOMEM, AVQ_EHIP = 0, -1, -2, -3, -4
LUT_F32, LUT_U8 = 0, 1
ETA_LIMIT, ETA_EXACT, ETA_EXPLICIT = 0, 1, 2
MAX_SELECT = 512
STAGES = ("leaf_select", "lut", "scan", "merge", "finalize", "rescan", "sample")

# every symbol include/avq.h declares
SYMBOLS = [
    "avq_create", "avq_destroy", "avq_train", "avq_encode", "avq_update_codebooks", "avq_update_leaf_centers", "avq_search", "avq_search_noalloc", "avq_brute_force",
    "avq_set_codebooks", "avq_get_codebooks", "avq_set_leaf_centers", "avq_get_leaf_centers",
    "avq_set_database", "avq_get_codes", "avq_get_leaf_assign", "avq_size", "avq_debug_lut",
    "avq_debug_adc_scores", "avq_debug_leaf_select", "avq_debug_stream_codes", "avq_debug_scan_parts", "avq_debug_unverified_queries", "avq_eta", "avq_set_tuning",
    "avq_profile_enable", "avq_profile_read", "avq_last_error", "avq_version",
]


class AvqConfig(C.Structure):
    _fields_ = [
        ("d", C.c_int32), ("M", C.c_int32), ("bits", C.c_int32), ("T", C.c_float),
        ("eta_mode", C.c_int32), ("eta_explicit", C.c_float), ("kmeans_iters", C.c_int32),
        ("encode_passes", C.c_int32), ("n_leaves", C.c_int32), ("leaf_kmeans_iters", C.c_int32),
        ("borrow_x", C.c_int32), ("seed", C.c_uint64), ("leaf_aniso_iters", C.c_int32),
    ]


class AvqError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("avq error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    """The loaded libavq.so. Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_1908_10396_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.avq_create.argtypes = [C.POINTER(AvqConfig), C.POINTER(vp)]
        L.avq_destroy.argtypes = [vp]
        L.avq_destroy.restype = None
        L.avq_train.argtypes = [vp, vp, i64, vp]
        L.avq_encode.argtypes = [vp, vp, i64, vp]
        L.avq_update_codebooks.argtypes = [vp, vp, i64, i32, C.c_double, C.POINTER(i32), C.POINTER(C.c_double), vp]
        L.avq_update_leaf_centers.argtypes = [vp, vp, i64, i32, C.c_double, C.POINTER(i32), C.POINTER(C.c_double), vp]
        L.avq_search.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.avq_search_noalloc.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
        L.avq_brute_force.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.avq_set_codebooks.argtypes = [vp, vp]
        L.avq_get_codebooks.argtypes = [vp, vp]
        L.avq_set_leaf_centers.argtypes = [vp, vp]
        L.avq_get_leaf_centers.argtypes = [vp, vp]
        L.avq_set_database.argtypes = [vp, vp, vp, vp, i64, vp]
        L.avq_get_codes.argtypes = [vp, vp]
        L.avq_get_leaf_assign.argtypes = [vp, vp]
        L.avq_size.argtypes = [vp]
        L.avq_size.restype = i64
        L.avq_debug_lut.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp]
        L.avq_debug_adc_scores.argtypes = [vp, vp, i32, i32, vp, vp]
        L.avq_debug_leaf_select.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.avq_debug_stream_codes.argtypes = [vp, vp, C.POINTER(i64), vp]
        L.avq_debug_scan_parts.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.avq_debug_unverified_queries.argtypes = [vp, C.POINTER(i32)]
        L.avq_eta.argtypes = [i32, C.c_double, C.c_double, i32]
        L.avq_eta.restype = C.c_double
        L.avq_set_tuning.argtypes = [vp, C.c_char_p, i32]
        L.avq_profile_enable.argtypes = [vp, i32]
        L.avq_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
        L.avq_last_error.restype = C.c_char_p
        L.avq_version.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != AVQ_OK:
        raise AvqError(rc, lib().avq_last_error().decode())


def eta(d, T, norm=1.0, eta_mode=ETA_LIMIT):
    """avq_eta: eta of Section 3.2 of the paper for one norm (host computation)."""
    return float(lib().avq_eta(int(d), float(T), float(norm), int(eta_mode)))


def _torch():
    import torch
    return torch


def _stream_ptr(stream):
    if stream is None:
        return _torch().cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t, dtype, what, shape=None):
    """Device pointer of a contiguous CUDA tensor. shape: expected shape, None entries free. The C ABI sees
    pointers only, so a wrong shape would make a kernel read or write out of bounds: it is refused here."""
    torch = _torch()
    if not isinstance(t, torch.Tensor) or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (what, dtype))
    if shape is not None:
        if t.dim() != len(shape) or any(e is not None and int(s) != int(e) for s, e in zip(t.shape, shape)):
            raise ValueError("%s: shape %s, expected %s" % (what, tuple(t.shape), tuple("*" if e is None else e for e in shape)))
    if not t.is_cuda:
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (what, dtype))
    return t.data_ptr()


def _check_shape(t, shape, what):
    """Shape check alone (all of a call's shapes are checked before any of its device checks)."""
    if hasattr(t, "shape") and (len(t.shape) != len(shape) or
                                any(e is not None and int(s) != int(e) for s, e in zip(t.shape, shape))):
        raise ValueError("%s: shape %s, expected %s" % (what, tuple(t.shape), tuple("*" if e is None else e for e in shape)))


def _check_rows(a, cols, what):
    """A host array or tensor of `cols` columns (any number of rows)."""
    if a.ndim != 2 or int(a.shape[1]) != int(cols):
        raise ValueError("%s: shape %s, expected (*, %d)" % (what, tuple(a.shape), cols))


def _any_ptr(a, np_dtype, torch_dtype, what):
    """Host numpy array or torch tensor (host or device): (pointer, keepalive)."""
    import numpy as np
    torch = _torch()
    if isinstance(a, torch.Tensor):
        if a.dtype != torch_dtype or not a.is_contiguous():
            raise TypeError("%s: wrong dtype or not contiguous" % what)
        return a.data_ptr(), a
    a = np.ascontiguousarray(a, dtype=np_dtype)
    return a.ctypes.data, a


class Index:
    """Owns one avq_index. Tensors passed in must live on the index's GPU."""

    def __init__(self, d, M, bits, T=0.2, eta_mode=ETA_LIMIT, eta_explicit=1.0, kmeans_iters=20,
                 encode_passes=10, n_leaves=0, leaf_kmeans_iters=10, borrow_x=True, seed=0, leaf_aniso_iters=0):
        self.cfg = AvqConfig(d, M, bits, T, eta_mode, eta_explicit, kmeans_iters, encode_passes,
                             n_leaves, leaf_kmeans_iters, 1 if borrow_x else 0, seed, leaf_aniso_iters)
        self.d, self.M, self.bits, self.n_leaves = d, M, bits, n_leaves
        self.kc = 1 << bits
        self.ds = d // M if M > 0 and d % M == 0 else 0
        self.nb = (M * bits + 7) // 8
        self._h = C.c_void_p()
        self._keep = []
        _check(lib().avq_create(C.byref(self.cfg), C.byref(self._h)))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().avq_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except TypeError:       # interpreter shutdown: module globals are already gone
            pass

    @property
    def n(self):
        return int(lib().avq_size(self._h))

    def set_tuning(self, name, value):
        _check(lib().avq_set_tuning(self._h, name.encode(), int(value)))

    def profile_enable(self, on=True):
        _check(lib().avq_profile_enable(self._h, 1 if on else 0))

    def profile_read(self, reset=True):
        """{stage: (milliseconds, launches)} since the last reset."""
        ms = (C.c_double * len(STAGES))()
        cnt = (C.c_int64 * len(STAGES))()
        _check(lib().avq_profile_read(self._h, ms, cnt, 1 if reset else 0))
        return {name: (ms[i], cnt[i]) for i, name in enumerate(STAGES)}

    # -- build ---------------------------------------------------------------------
    def train(self, x, stream=None):
        torch = _torch()
        p = _dev(x, torch.float32, "x", (None, self.d))
        _check(lib().avq_train(self._h, p, x.shape[0], _stream_ptr(stream)))

    def encode(self, x, stream=None):
        torch = _torch()
        p = _dev(x, torch.float32, "x", (None, self.d))
        if self.cfg.borrow_x:
            self._keep = [x]
        _check(lib().avq_encode(self._h, p, x.shape[0], _stream_ptr(stream)))

    def update_codebooks(self, x, max_iters=1000, tol=1e-10, stream=None):
        """Returns (iterations, relative residual)."""
        torch = _torch()
        p = _dev(x, torch.float32, "x", (None, self.d))
        it, rel = C.c_int32(0), C.c_double(0.0)
        _check(lib().avq_update_codebooks(self._h, p, x.shape[0], max_iters, tol, C.byref(it), C.byref(rel),
                                          _stream_ptr(stream)))
        return it.value, rel.value

    def update_leaf_centers(self, x, max_iters=1000, tol=1e-10, stream=None):
        """avq_update_leaf_centers. Returns (iterations, relative residual)."""
        torch = _torch()
        p = _dev(x, torch.float32, "x", (None, self.d))
        it, rel = C.c_int32(0), C.c_double(0.0)
        _check(lib().avq_update_leaf_centers(self._h, p, x.shape[0], max_iters, tol, C.byref(it), C.byref(rel),
                                             _stream_ptr(stream)))
        return it.value, rel.value

    def set_codebooks(self, codebooks):
        import numpy as np
        p, keep = _any_ptr(codebooks, np.float32, _torch().float32, "codebooks")
        if tuple(keep.shape) != (self.M, self.kc, self.ds):
            raise ValueError("codebooks: shape %s, expected %s" % (tuple(keep.shape), (self.M, self.kc, self.ds)))
        _check(lib().avq_set_codebooks(self._h, p))

    def get_codebooks(self):
        import numpy as np
        out = np.empty((self.M, self.kc, self.ds), np.float32)
        _check(lib().avq_get_codebooks(self._h, out.ctypes.data))
        return out

    def set_leaf_centers(self, centers):
        import numpy as np
        p, keep = _any_ptr(centers, np.float32, _torch().float32, "centers")
        if tuple(keep.shape) != (self.n_leaves, self.d):
            raise ValueError("centers: shape %s, expected %s" % (tuple(keep.shape), (self.n_leaves, self.d)))
        _check(lib().avq_set_leaf_centers(self._h, p))

    def get_leaf_centers(self):
        import numpy as np
        out = np.empty((self.n_leaves, self.d), np.float32)
        _check(lib().avq_get_leaf_centers(self._h, out.ctypes.data))
        return out

    def set_database(self, x, packed, leaf_assign=None, stream=None):
        import numpy as np
        torch = _torch()
        pp, k1 = _any_ptr(packed, np.uint8, torch.uint8, "packed")
        _check_rows(k1, self.nb, "packed")
        n = k1.shape[0]
        if x is not None:
            _check_shape(x, (n, self.d), "x")
        if leaf_assign is not None:
            _check_shape(leaf_assign, (n,), "leaf_assign")
        xp = None if x is None else _dev(x, torch.float32, "x", (n, self.d))
        ap, k2 = (None, None) if leaf_assign is None else _any_ptr(leaf_assign, np.int32, torch.int32,
                                                                   "leaf_assign")
        if k2 is not None and tuple(k2.shape) != (n,):
            raise ValueError("leaf_assign: shape %s, expected (%d,)" % (tuple(k2.shape), n))
        if self.cfg.borrow_x:
            self._keep = [x]
        _check(lib().avq_set_database(self._h, xp, pp, ap, n, _stream_ptr(stream)))

    def get_codes(self):
        import numpy as np
        out = np.empty((self.n, self.nb), np.uint8)
        _check(lib().avq_get_codes(self._h, out.ctypes.data))
        return out

    def get_leaf_assign(self):
        import numpy as np
        out = np.empty(self.n, np.int32)
        _check(lib().avq_get_leaf_assign(self._h, out.ctypes.data))
        return out

    # -- query ---------------------------------------------------------------------
    def search(self, queries, k, reorder_k, lut_mode=LUT_F32, leaves_to_search=0, out=None,
               stream=None):
        """avq_search. Returns (ids int32 [nq][k], scores fp32 [nq][k]) on the GPU."""
        torch = _torch()
        _check_shape(queries, (None, self.d), "queries")
        if out is not None:
            _check_shape(out[0], (queries.shape[0], k), "ids")
            _check_shape(out[1], (queries.shape[0], k), "scores")
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        nq = queries.shape[0]
        if out is None:
            ids = torch.empty((nq, k), dtype=torch.int32, device=queries.device)
            sc = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        else:
            ids, sc = out
        _check(lib().avq_search(self._h, qp, nq, k, reorder_k, lut_mode, leaves_to_search,
                                _dev(ids, torch.int32, "ids", (nq, k)), _dev(sc, torch.float32, "scores", (nq, k)),
                                _stream_ptr(stream)))
        return ids, sc

    def search_noalloc(self, queries, k, reorder_k, lut_mode=LUT_F32, out=None, stream=None):
        """avq_search_noalloc: the caller supplies `out` = (ids, scores) so that nothing is allocated."""
        torch = _torch()
        _check_shape(queries, (None, self.d), "queries")
        _check_shape(out[0], (queries.shape[0], k), "ids")
        _check_shape(out[1], (queries.shape[0], k), "scores")
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        ids, sc = out
        nq = queries.shape[0]
        _check(lib().avq_search_noalloc(self._h, qp, nq, k, reorder_k, lut_mode,
                                        _dev(ids, torch.int32, "ids", (nq, k)), _dev(sc, torch.float32, "scores", (nq, k)),
                                        _stream_ptr(stream)))
        return ids, sc

    def brute_force(self, queries, k, stream=None):
        torch = _torch()
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        nq = queries.shape[0]
        ids = torch.empty((nq, k), dtype=torch.int32, device=queries.device)
        sc = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        _check(lib().avq_brute_force(self._h, qp, nq, k, ids.data_ptr(), sc.data_ptr(),
                                     _stream_ptr(stream)))
        return ids, sc

    def debug_lut(self, queries, lut_mode, stream=None):
        torch = _torch()
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        nq = queries.shape[0]
        if lut_mode == LUT_F32:
            lut = torch.empty((nq, self.M, self.kc), dtype=torch.float32, device=queries.device)
            _check(lib().avq_debug_lut(self._h, qp, nq, lut_mode, lut.data_ptr(), None, None,
                                       _stream_ptr(stream)))
            return lut
        lut = torch.empty((nq, self.M, self.kc), dtype=torch.uint8, device=queries.device)
        scale = torch.empty(nq, dtype=torch.float32, device=queries.device)
        bias = torch.empty(nq, dtype=torch.float32, device=queries.device)
        _check(lib().avq_debug_lut(self._h, qp, nq, lut_mode, lut.data_ptr(), scale.data_ptr(),
                                   bias.data_ptr(), _stream_ptr(stream)))
        return lut, scale, bias

    def debug_adc_scores(self, queries, lut_mode, stream=None):
        torch = _torch()
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        nq = queries.shape[0]
        dt = torch.float32 if lut_mode == LUT_F32 else torch.int32
        out = torch.empty((nq, self.n), dtype=dt, device=queries.device)
        _check(lib().avq_debug_adc_scores(self._h, qp, nq, lut_mode, out.data_ptr(),
                                          _stream_ptr(stream)))
        return out

    def debug_unverified_queries(self, reasons=False):
        """Queries of the last fp32 batch that were scanned again; reasons=True: the four counts of avq.h."""
        c = (C.c_int32 * 4)()
        _check(lib().avq_debug_unverified_queries(self._h, c))
        return list(c) if reasons else c[0]

    def debug_stream_codes(self, out=None, stream=None):
        """xor of every block's code words, uint32 [n_blocks] on the device (see avq.h)."""
        torch = _torch()
        nb = C.c_int64(0)
        _check(lib().avq_debug_stream_codes(self._h, None, C.byref(nb), None))
        if out is None:
            out = torch.empty(nb.value, dtype=torch.int32, device="cuda")
        if out.numel() < nb.value or out.dtype != torch.int32 or not out.is_cuda:
            raise ValueError("out: int32 cuda tensor of at least %d elements" % nb.value)
        _check(lib().avq_debug_stream_codes(self._h, out.data_ptr(), None, _stream_ptr(stream)))
        return out[:nb.value]

    def debug_scan_parts(self, queries, lut_mode, part, reps, stream=None):
        """avq_debug_scan_parts: `reps` back-to-back launches of one part of the small-batch scan."""
        torch = _torch()
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        _check(lib().avq_debug_scan_parts(self._h, qp, queries.shape[0], lut_mode, part, reps, _stream_ptr(stream)))

    def debug_leaf_select(self, queries, L, stream=None):
        torch = _torch()
        qp = _dev(queries, torch.float32, "queries", (None, self.d))
        nq = queries.shape[0]
        ids = torch.empty((nq, L), dtype=torch.int32, device=queries.device)
        ip = torch.empty((nq, L), dtype=torch.float32, device=queries.device)
        _check(lib().avq_debug_leaf_select(self._h, qp, nq, L, ids.data_ptr(), ip.data_ptr(),
                                           _stream_ptr(stream)))
        return ids, ip
