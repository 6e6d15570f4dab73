"""ctypes binding of libivftq.so: same names as include/ivftq.h, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing else);
every step of the hot path runs inside the library's HIP kernels.  There is no CPU fallback: if
the shared library is missing or a symbol cannot be found, importing or calling fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("IVFTQ_LIB") or os.path.join(_HERE, "libivftq.so")   # IVFTQ_LIB: load another build

OK, INVALID_ARG, BAD_STATE, OOM, HIP_ERROR, ZERO_NORM, UNSUPPORTED = range(7)
METRIC_COSINE, METRIC_IP, METRIC_L2 = range(3)
STATUS_NAMES = ["OK", "INVALID_ARG", "BAD_STATE", "OOM", "HIP_ERROR", "ZERO_NORM", "UNSUPPORTED"]

# every symbol include/ivftq.h declares, with its ctypes signature
_SIGNATURES = {
    "ivftq_build_codebook": (C.c_int, [C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "ivftq_quantiser_grid": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_float),
                                       C.POINTER(C.c_float), C.c_void_p, C.c_void_p]),
    "ivftq_haar_rotation": (C.c_int, [C.c_int, C.c_uint64, C.c_void_p]),
    "ivftq_haar_from_gaussian": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p]),
    "ivftq_create": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                               C.POINTER(C.c_void_p)]),
    "ivftq_create_refined": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.POINTER(C.c_void_p)]),
    "ivftq_build_refined_codebook": (C.c_int, [C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "ivftq_destroy": (C.c_int, [C.c_void_p]),
    "ivftq_reset": (C.c_int, [C.c_void_p]),
    "ivftq_train_coarse": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_uint64,
                                     C.POINTER(C.c_double), C.c_void_p]),
    "ivftq_set_coarse": (C.c_int, [C.c_void_p, C.c_void_p]),
    "ivftq_get_coarse": (C.c_int, [C.c_void_p, C.c_void_p]),
    "ivftq_set_rotation": (C.c_int, [C.c_void_p, C.c_void_p]),
    "ivftq_get_rotation": (C.c_int, [C.c_void_p, C.c_void_p]),
    "ivftq_get_codebook": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_encode_add": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]),
    "ivftq_add_encoded": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p]),
    "ivftq_encode_only": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p]),
    "ivftq_encode_only_noalloc": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p]),
    "ivftq_rerank": (C.c_int, [C.c_int, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int,
                               C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_reconstruct": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_reencode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_refresh_coarse": (C.c_int, [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_uint64, C.POINTER(C.c_double),
                                       C.c_void_p]),
    "ivftq_search": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                               C.c_void_p]),
    "ivftq_coarse_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p,
                                     C.c_void_p]),
    "ivftq_ntotal": (C.c_int64, [C.c_void_p]),
    "ivftq_list_size": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int64)]),
    "ivftq_export_list": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_index_bytes": (C.c_int64, [C.c_void_p]),
    "ivftq_set_workspace_limit": (C.c_int, [C.c_void_p, C.c_int64]),
    "ivftq_set_search_mode": (C.c_int, [C.c_void_p, C.c_int]),
    "ivftq_set_metric": (C.c_int, [C.c_void_p, C.c_int]),
    "ivftq_set_cascade_plane": (C.c_int, [C.c_void_p, C.c_int]),
    "ivftq_export_cascade_plane": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "ivftq_add_encoded_raw": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]),
    "ivftq_export_norms": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "ivftq_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "ivftq_profile_read": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_profile_kernel_count": (C.c_int, []),
    "ivftq_profile_kernel_name": (C.c_char_p, [C.c_int]),
    "ivftq_search_cascade": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                       C.c_void_p, C.c_void_p, C.c_void_p]),
    "ivftq_build_coarsened_codebook": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float)]),
    "ivftq_assign_undecided": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.c_void_p]),
    "ivftq_scan_stats": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                   C.POINTER(C.c_double), C.c_void_p]),
    "ivftq_measure_mfma_rate": (C.c_int, [C.c_int, C.POINTER(C.c_double)]),
    "ivftq_last_error": (C.c_char_p, []),
    "ivftq_version": (C.c_char_p, []),
}

_lib = None

# ivftq_alloc_fn / ivftq_free_fn
ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class IvftqError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status


def load_library(path: str | None = None) -> C.CDLL:
    """Load libivftq.so and bind every declared symbol; raises if anything is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2605_17415_amd.build`")
    lib = C.CDLL(path)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the export is missing
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def declared_symbols():
    return list(_SIGNATURES)


def _check(status: int):
    if status != OK:
        raise IvftqError(status, load_library().ivftq_last_error().decode())


def _np_ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _dev_ptr(t, dtype=None, name="tensor"):
    """Raw device pointer of a contiguous torch tensor on the GPU (None -> NULL)."""
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a torch tensor in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


# ---- host-only calls -----------------------------------------------------------------------------


def ivftq_build_codebook(b: int, d: int):
    """(centroids [2^b] f32, boundaries [2^b - 1] f32)"""
    lib = load_library()
    K = 1 << max(0, min(b, 16))
    c = np.empty(K, np.float32)
    t = np.empty(max(K - 1, 1), np.float32)
    _check(lib.ivftq_build_codebook(b, d, _np_ptr(c), _np_ptr(t)))
    return c, t[:K - 1]


def ivftq_build_refined_codebook(b: int, d: int):
    """(levels [2^(b+1)] f32, boundaries [2^(b+1) - 1] f32) of Stage 1 at b bits + sign bit"""
    lib = load_library()
    K2 = 2 << max(0, min(b, 15))
    lv = np.empty(K2, np.float32)
    bd = np.empty(K2 - 1, np.float32)
    _check(lib.ivftq_build_refined_codebook(b, d, _np_ptr(lv), _np_ptr(bd)))
    return lv, bd


def ivftq_build_coarsened_codebook(b: int, d: int, beta: int, sign_bit: bool = False):
    """[2^beta] f32: values of the Stage-1 codebook cut down to its top beta bits (cascade pass 1)"""
    out = np.empty(1 << max(0, min(beta, 15)), np.float32)
    _check(load_library().ivftq_build_coarsened_codebook(b, 1 if sign_bit else 0, d, beta,
                                                         out.ctypes.data_as(C.POINTER(C.c_float))))
    return out


def ivftq_quantiser_grid(b: int, d: int, sign_bit: bool = False):
    """(cells, scale, offset, boundary [cells] f32, index [cells] i32)"""
    sb = 1 if sign_bit else 0
    lib = load_library()
    cells, scale, offset = C.c_int(0), C.c_float(0), C.c_float(0)
    _check(lib.ivftq_quantiser_grid(b, sb, d, 0, C.byref(cells), C.byref(scale), C.byref(offset), None, None))
    boundary = np.empty(cells.value, np.float32)
    index = np.empty(cells.value, np.int32)
    _check(lib.ivftq_quantiser_grid(b, sb, d, cells.value, C.byref(cells), C.byref(scale), C.byref(offset),
                                    _np_ptr(boundary), _np_ptr(index)))
    return cells.value, np.float32(scale.value), np.float32(offset.value), boundary, index


def ivftq_haar_rotation(d: int, seed: int) -> np.ndarray:
    lib = load_library()
    pi = np.empty((d, d), np.float32)
    _check(lib.ivftq_haar_rotation(d, seed, _np_ptr(pi)))
    return pi


def ivftq_haar_from_gaussian(g: np.ndarray) -> np.ndarray:
    lib = load_library()
    g = np.ascontiguousarray(g, dtype=np.float64)
    d = g.shape[0]
    pi = np.empty((d, d), np.float32)
    _check(lib.ivftq_haar_from_gaussian(d, _np_ptr(g), _np_ptr(pi)))
    return pi


def ivftq_measure_mfma_rate(random_operands: bool = True) -> float:
    """TFLOP/s of a pure v_mfma_f32_32x32x16_f16 loop on the current device."""
    out = C.c_double(0)
    _check(load_library().ivftq_measure_mfma_rate(1 if random_operands else 0, C.byref(out)))
    return out.value


def ivftq_rerank(q, x, cand_ids, k: int, stream=None):
    """Exact re-ranking of candidate labels against raw rows x (all torch tensors on the device)."""
    import torch
    nq, d = q.shape
    r = cand_ids.shape[1]
    scores = torch.empty((nq, k), dtype=torch.float32, device=q.device)
    ids = torch.empty((nq, k), dtype=torch.int64, device=q.device)
    _check(load_library().ivftq_rerank(d, _dev_ptr(q, torch.float32, "q"), nq, _dev_ptr(x, torch.float32, "x"), x.shape[0],
                                       _dev_ptr(cand_ids, torch.int64, "cand_ids"), r, k, _dev_ptr(scores), _dev_ptr(ids),
                                       _stream_ptr(stream)))
    return scores, ids


def ivftq_version() -> str:
    return load_library().ivftq_version().decode()


# ---- index ---------------------------------------------------------------------------------------


def _torch_alloc(nbytes, ctx):
    """ivftq_alloc_fn on PyTorch's caching allocator (current device, current stream); NULL when it is out of memory."""
    try:
        import torch
        return torch.cuda.caching_allocator_alloc(int(nbytes))
    except Exception:
        return None


def _torch_free(ptr, ctx):
    try:
        import torch
        torch.cuda.caching_allocator_delete(ptr)
    except Exception:            # interpreter shutting down: the process is about to return the memory anyway
        pass


# the callback objects must outlive every index that holds their addresses
TORCH_ALLOC = ALLOC_FN(_torch_alloc)
TORCH_FREE = FREE_FN(_torch_free)


class Index:
    """Owner of one ivftq_index handle.  Methods carry the C names minus the prefix.

    allocator: "torch" (default) = the index takes all its device memory from PyTorch's caching allocator;
    "hip" = hipMalloc / hipFree inside the library; or a pair (ALLOC_FN, FREE_FN) of ctypes callbacks."""

    def __init__(self, d: int, b: int, nlist: int, rotation_seed: int = 0, sign_bit: bool = False, allocator="torch"):
        self._lib = load_library()
        self._h = C.c_void_p()
        if allocator == "torch":
            self._alloc = (TORCH_ALLOC, TORCH_FREE)
        elif allocator == "hip":
            self._alloc = (None, None)
        else:
            self._alloc = tuple(allocator)           # kept alive as long as the index
        af, ff = (C.cast(f, C.c_void_p) if f is not None else None for f in self._alloc)
        if sign_bit:
            _check(self._lib.ivftq_create_refined(d, b, 1, nlist, rotation_seed, af, ff, None, C.byref(self._h)))
        else:
            _check(self._lib.ivftq_create(d, b, nlist, rotation_seed, af, ff, None, C.byref(self._h)))
        self.d, self.nlist = d, nlist
        self.b = b + (1 if sign_bit else 0)      # bits stored per coordinate

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.ivftq_destroy(self._h)
            self._h = C.c_void_p()

    def reset(self):
        _check(self._lib.ivftq_reset(self._h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # constants
    def set_coarse(self, centroids: np.ndarray):
        c = np.ascontiguousarray(centroids, dtype=np.float32)
        if c.shape != (self.nlist, self.d):
            raise ValueError("centroids must be nlist x d")
        _check(self._lib.ivftq_set_coarse(self._h, _np_ptr(c)))

    def get_coarse(self) -> np.ndarray:
        c = np.empty((self.nlist, self.d), np.float32)
        _check(self._lib.ivftq_get_coarse(self._h, _np_ptr(c)))
        return c

    def set_rotation(self, pi: np.ndarray):
        p = np.ascontiguousarray(pi, dtype=np.float32)
        if p.shape != (self.d, self.d):
            raise ValueError("rotation must be d x d")
        _check(self._lib.ivftq_set_rotation(self._h, _np_ptr(p)))

    def get_rotation(self) -> np.ndarray:
        p = np.empty((self.d, self.d), np.float32)
        _check(self._lib.ivftq_get_rotation(self._h, _np_ptr(p)))
        return p

    def get_codebook(self):
        K = 1 << self.b
        c = np.empty(K, np.float32)
        t = np.empty(max(K - 1, 1), np.float32)
        _check(self._lib.ivftq_get_codebook(self._h, _np_ptr(c), _np_ptr(t)))
        return c, t[:K - 1]

    def set_search_mode(self, mode: int):
        _check(self._lib.ivftq_set_search_mode(self._h, mode))

    def set_metric(self, metric: int):
        _check(self._lib.ivftq_set_metric(self._h, metric))

    def set_cascade_plane(self, beta: int):
        _check(self._lib.ivftq_set_cascade_plane(self._h, beta))

    def export_cascade_plane(self, l: int) -> np.ndarray:
        """uint8 [n, d]: the top-bit plane of list l in stored order."""
        out = np.empty((self.list_size(l), self.d), np.uint8)
        if len(out):
            _check(self._lib.ivftq_export_cascade_plane(self._h, l, _np_ptr(out)))
        return out

    def set_workspace_limit(self, nbytes: int):
        _check(self._lib.ivftq_set_workspace_limit(self._h, nbytes))

    # coarse training
    def train_coarse(self, x, niter: int, init_rows: np.ndarray | None = None, seed: int = 0, stream=None) -> float:
        import torch
        n = x.shape[0]
        init = None
        if init_rows is not None:
            init = np.ascontiguousarray(init_rows, dtype=np.int64)
            if init.shape != (self.nlist,):
                raise ValueError("init_rows must hold nlist row numbers")
        inertia = C.c_double()
        _check(self._lib.ivftq_train_coarse(self._h, _dev_ptr(x, torch.float32, "x"), n, niter,
                                            _np_ptr(init) if init is not None else None, seed,
                                            C.byref(inertia), _stream_ptr(stream)))
        return inertia.value

    # encode
    def encode_add(self, x, ids=None, stream=None):
        import torch
        _check(self._lib.ivftq_encode_add(self._h, _dev_ptr(x, torch.float32, "x"), x.shape[0],
                                          _dev_ptr(ids, torch.int64, "ids"), _stream_ptr(stream)))

    def add_encoded(self, assign, codes, gamma, ids=None, stream=None):
        import torch
        n = assign.shape[0]
        if codes.shape != (n, self.d) or gamma.shape != (n,):
            raise ValueError("codes must be n x d and gamma n")
        _check(self._lib.ivftq_add_encoded(self._h, n, _dev_ptr(assign, torch.int32, "assign"),
                                           _dev_ptr(codes, torch.uint8, "codes"),
                                           _dev_ptr(gamma, torch.float16, "gamma"),
                                           _dev_ptr(ids, torch.int64, "ids"), _stream_ptr(stream)))

    def add_encoded_raw(self, assign, codes, gamma, xnorm, ids=None, stream=None):
        import torch
        n = assign.shape[0]
        if codes.shape != (n, self.d) or gamma.shape != (n,) or xnorm.shape != (n,):
            raise ValueError("codes must be n x d, gamma and xnorm n")
        _check(self._lib.ivftq_add_encoded_raw(self._h, n, _dev_ptr(assign, torch.int32, "assign"),
                                               _dev_ptr(codes, torch.uint8, "codes"),
                                               _dev_ptr(gamma, torch.float16, "gamma"),
                                               _dev_ptr(xnorm, torch.float32, "xnorm"),
                                               _dev_ptr(ids, torch.int64, "ids"), _stream_ptr(stream)))

    def encode_only(self, x, want_codes: bool = True, stream=None):
        """(assign int32 [n], codes uint8 [n, d] or None, gamma float16 [n]) as device tensors."""
        import torch
        n = x.shape[0]
        assign = torch.empty(n, dtype=torch.int32, device=x.device)
        codes = torch.empty((n, self.d), dtype=torch.uint8, device=x.device) if want_codes else None
        gamma = torch.empty(n, dtype=torch.float16, device=x.device)
        _check(self._lib.ivftq_encode_only(self._h, _dev_ptr(x, torch.float32, "x"), n, _dev_ptr(assign),
                                           _dev_ptr(codes), _dev_ptr(gamma), _stream_ptr(stream)))
        return assign, codes, gamma

    def encode_only_noalloc(self, x, assign, codes, gamma, stream=None):
        """ivftq_encode_only into caller-provided device tensors (any may be None), nothing allocated."""
        import torch
        _check(self._lib.ivftq_encode_only_noalloc(self._h, _dev_ptr(x, torch.float32, "x"), x.shape[0],
                                                   _dev_ptr(assign, torch.int32, "assign"), _dev_ptr(codes, torch.uint8, "codes"),
                                                   _dev_ptr(gamma, torch.float16, "gamma"), _stream_ptr(stream)))

    # search
    def reconstruct(self, stream=None):
        """(x^ [ntotal, d] f32, labels [ntotal] i64) on the device, list order"""
        import torch
        n = self.ntotal()
        dev = torch.device("cuda", torch.cuda.current_device())
        x = torch.empty((n, self.d), dtype=torch.float32, device=dev)
        ids = torch.empty((n,), dtype=torch.int64, device=dev)
        _check(self._lib.ivftq_reconstruct(self._h, _dev_ptr(x), _dev_ptr(ids), _stream_ptr(stream)))
        return x, ids

    def reencode(self, centroids: np.ndarray, stream=None):
        c = np.ascontiguousarray(centroids, dtype=np.float32)
        assert c.shape == (self.nlist, self.d)
        _check(self._lib.ivftq_reencode(self._h, _np_ptr(c), _stream_ptr(stream)))

    def refresh_coarse(self, sample_n: int, niter: int, init_rows: np.ndarray | None = None, seed: int = 0,
                       stream=None) -> float:
        inertia = C.c_double(0)
        rows = None
        if init_rows is not None:
            rows = np.ascontiguousarray(init_rows, dtype=np.int64)
            assert rows.shape == (self.nlist,)
        _check(self._lib.ivftq_refresh_coarse(self._h, sample_n, niter, _np_ptr(rows) if rows is not None else None,
                                              seed, C.byref(inertia), _stream_ptr(stream)))
        return inertia.value

    def search(self, q, nprobe: int, k: int, out_scores=None, out_ids=None, stream=None):
        import torch
        nq = q.shape[0]
        scores = out_scores if out_scores is not None else torch.empty((nq, k), dtype=torch.float32, device=q.device)
        ids = out_ids if out_ids is not None else torch.empty((nq, k), dtype=torch.int64, device=q.device)
        _check(self._lib.ivftq_search(self._h, _dev_ptr(q, torch.float32, "q"), nq, nprobe, k,
                                      _dev_ptr(scores, torch.float32, "scores"), _dev_ptr(ids, torch.int64, "ids"),
                                      _stream_ptr(stream)))
        return scores, ids

    def search_cascade(self, q, nprobe: int, k: int, beta: int, n_keep: int, stream=None):
        """Two-pass search: top-beta-bit scores keep n_keep candidates, full codes rank them."""
        import torch
        nq = q.shape[0]
        scores = torch.empty((nq, k), dtype=torch.float32, device=q.device)
        ids = torch.empty((nq, k), dtype=torch.int64, device=q.device)
        _check(self._lib.ivftq_search_cascade(self._h, _dev_ptr(q, torch.float32, "q"), nq, nprobe, k, beta, n_keep,
                                              _dev_ptr(scores, torch.float32, "scores"), _dev_ptr(ids, torch.int64, "ids"),
                                              _stream_ptr(stream)))
        return scores, ids

    def coarse_probe(self, q, nprobe: int, stream=None):
        import torch
        nq = q.shape[0]
        probe = torch.empty((nq, nprobe), dtype=torch.int32, device=q.device)
        coarse = torch.empty((nq, nprobe), dtype=torch.float32, device=q.device)
        _check(self._lib.ivftq_coarse_probe(self._h, _dev_ptr(q, torch.float32, "q"), nq, nprobe,
                                            _dev_ptr(probe), _dev_ptr(coarse), _stream_ptr(stream)))
        return probe, coarse

    # per-kernel timing
    def profile_enable(self, on: bool = True):
        _check(self._lib.ivftq_profile_enable(self._h, 1 if on else 0))

    def profile_read(self) -> dict:
        """{kernel class: (total ms, launches)} since the last read."""
        cnt = self._lib.ivftq_profile_kernel_count()
        ms = np.zeros(cnt, np.float64)
        launches = np.zeros(cnt, np.int64)
        _check(self._lib.ivftq_profile_read(self._h, _np_ptr(ms), _np_ptr(launches)))
        return {self._lib.ivftq_profile_kernel_name(i).decode(): (float(ms[i]), int(launches[i]))
                for i in range(cnt) if launches[i] > 0}

    def assign_undecided(self, stream=None) -> int:
        """Rows of the last encode call that the screening pass handed to the full-precision pass."""
        out = C.c_int64(0)
        _check(self._lib.ivftq_assign_undecided(self._h, C.byref(out), _stream_ptr(stream)))
        return out.value

    def scan_stats(self, stream=None) -> dict:
        """Candidates per query and queries redone exactly in the last pass of the most recent batched search."""
        nq, redone, mx, mean = C.c_int64(0), C.c_int64(0), C.c_int64(0), C.c_double(0)
        _check(self._lib.ivftq_scan_stats(self._h, C.byref(nq), C.byref(redone), C.byref(mx), C.byref(mean), _stream_ptr(stream)))
        return {"queries": nq.value, "redone_exactly": redone.value, "max_candidates": mx.value, "mean_candidates": mean.value}

    # inspection
    def ntotal(self) -> int:
        return int(self._lib.ivftq_ntotal(self._h))

    def index_bytes(self) -> int:
        return int(self._lib.ivftq_index_bytes(self._h))

    def list_size(self, l: int) -> int:
        n = C.c_int64()
        _check(self._lib.ivftq_list_size(self._h, l, C.byref(n)))
        return n.value

    def export_norms(self, l: int) -> np.ndarray:
        """float32 [n]: the stored |x| of list l in stored order (raw metrics only)."""
        norms = np.empty(self.list_size(l), np.float32)
        if len(norms):
            _check(self._lib.ivftq_export_norms(self._h, l, _np_ptr(norms)))
        return norms

    def export_list(self, l: int):
        """(ids int64 [n], codes uint8 [n, d], gamma float16 [n]) as numpy arrays in stored order."""
        n = self.list_size(l)
        ids = np.empty(n, np.int64)
        codes = np.empty((n, self.d), np.uint8)
        gamma = np.empty(n, np.float16)
        if n:
            _check(self._lib.ivftq_export_list(self._h, l, _np_ptr(ids), _np_ptr(codes), _np_ptr(gamma)))
        return ids, codes, gamma
