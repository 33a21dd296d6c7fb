"""Thin Python layer over ``libpqadc.so``: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers through the C ABI declared in ``include/pq_adc.h`` and returns
freshly allocated output tensors.  No step of the method is computed here.  The
library must be built (``python -m paper_1712_02912_amd.build`` or
``__graft_entry__.build()``); loading fails loudly otherwise -- there is no CPU
fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpqadc.so")

CODES_U8 = 0
CODES_U4_PACKED = 1
LUT_F32 = 0
LUT_U8 = 1

EXPORTS = ["pq_create", "pq_destroy", "pq_last_error", "pq_version", "pq_build_luts", "pq_quantize_luts",
           "pq_qmax_prescan", "pq_adc_scan_topk", "pq_rerank_f32", "ivf_adc_search", "pq_encode", "pq_rotate", "pq_derived_search", "pq_set_profiling",
           "pq_last_scan_kernel_ms", "pq_calibration_copy", "pq_set_option", "pq_unset_option", "pq_last_scan_info", "pq_adc_scan_topk_noalloc",
           "ivf_quick_adc_search"]

_lib = None


class IvfLists(ctypes.Structure):
    _fields_ = [("coarse_centroids", ctypes.c_void_p), ("list_offsets", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("ids", ctypes.c_void_p),
                ("nlist", ctypes.c_int), ("d", ctypes.c_int), ("ntotal", ctypes.c_int64)]


def load():
    """dlopen the library (built beforehand) and declare the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_1712_02912_amd.build); "
                           "there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.pq_create.argtypes = [ctypes.POINTER(vp), ci, vp]
    lib.pq_destroy.argtypes = [vp]
    lib.pq_last_error.argtypes = [vp]
    lib.pq_last_error.restype = ctypes.c_char_p
    lib.pq_version.restype = ctypes.c_char_p
    lib.pq_build_luts.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp]
    lib.pq_quantize_luts.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.pq_qmax_prescan.argtypes = [vp, vp, i64, ci, vp, ci, ci, ci, ci, ci, vp]
    lib.pq_adc_scan_topk.argtypes = [vp, vp, i64, ci, vp, ci, ci, ci, ci, ci, vp, vp]
    lib.pq_adc_scan_topk_noalloc.argtypes = lib.pq_adc_scan_topk.argtypes
    lib.pq_last_scan_info.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ci), ctypes.POINTER(ci),
                                      ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
    lib.pq_set_option.argtypes = [vp, ctypes.c_char_p, ci]
    lib.pq_unset_option.argtypes = [vp, ctypes.c_char_p]
    lib.pq_rerank_f32.argtypes = [vp, vp, i64, ci, vp, ci, ci, ci, vp, ci, ci, vp, vp]
    lib.ivf_adc_search.argtypes = [vp, ctypes.POINTER(IvfLists), vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp]
    lib.ivf_quick_adc_search.argtypes = [vp, ctypes.POINTER(IvfLists), vp, ci, ci, vp, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.pq_rotate.argtypes = [vp, vp, vp, i64, ci, vp]
    lib.pq_encode.argtypes = [vp, vp, vp, i64, ci, ci, ci, ci, vp]
    lib.pq_derived_search.argtypes = [vp, vp, i64, vp, vp, ci, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, i64]
    lib.pq_calibration_copy.argtypes = [vp, vp, vp, ctypes.c_size_t]
    lib.pq_set_profiling.argtypes = [vp, ci]
    lib.pq_last_scan_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    for name in EXPORTS:
        if name not in ("pq_last_error", "pq_version"):
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


class PqError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"libpqadc error {code}: {message}")
        self.code = code


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(t, dtype, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.contiguous()


class Context:
    """Owns a ``pq_ctx`` bound to a device and a HIP stream (default: torch's current stream)."""

    def __init__(self, device=0, stream=None):
        self.lib = load()
        self.device = torch.device("cuda", device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        handle = ctypes.c_void_p()
        rc = self.lib.pq_create(ctypes.byref(handle), device, ctypes.c_void_p(stream.cuda_stream))
        if rc != 0:
            raise PqError(rc, "pq_create failed")
        self.handle = handle

    def close(self):
        if getattr(self, "handle", None):
            self.lib.pq_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise PqError(rc, self.lib.pq_last_error(self.handle).decode())

    def pq_set_option(self, name, value):
        """Set a tuning/test switch (see include/pq_adc.h); value None returns it to its default."""
        if value is None:
            self._check(self.lib.pq_unset_option(self.handle, name.encode()))
        else:
            self._check(self.lib.pq_set_option(self.handle, name.encode(), int(value)))

    def pq_set_profiling(self, enable):
        self._check(self.lib.pq_set_profiling(self.handle, 1 if enable else 0))

    def pq_last_scan_kernel_ms(self):
        ms = ctypes.c_float()
        self._check(self.lib.pq_last_scan_kernel_ms(self.handle, ctypes.byref(ms)))
        return ms.value

    def pq_last_scan_info(self):
        name = ctypes.create_string_buffer(400)
        qpp, passes = ctypes.c_int(), ctypes.c_int()
        parked, inserted = ctypes.c_uint64(), ctypes.c_uint64()
        self._check(self.lib.pq_last_scan_info(self.handle, name, 400, ctypes.byref(qpp), ctypes.byref(passes),
                                               ctypes.byref(parked), ctypes.byref(inserted)))
        return {"kernel": name.value.decode(), "queries_per_pass": qpp.value, "passes": passes.value,
                "parked_lanes": parked.value, "inserted_keys": inserted.value}

    def pq_calibration_copy(self, src, dst):
        nbytes = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() == nbytes
        self._check(self.lib.pq_calibration_copy(self.handle, _ptr(src), _ptr(dst), nbytes))

    # -- Tables step -------------------------------------------------------------------------
    def pq_build_luts(self, queries, codebooks):
        queries = _dev(queries, torch.float32, "queries")
        codebooks = _dev(codebooks, torch.float32, "codebooks")
        nq, d = queries.shape
        m, k, _ = codebooks.shape
        luts = torch.empty((nq, m, k), dtype=torch.float32, device=queries.device)
        self._check(self.lib.pq_build_luts(self.handle, _ptr(queries), _ptr(codebooks), nq, d, m, k, _ptr(luts)))
        return luts

    def pq_quantize_luts(self, luts, qmax):
        luts = _dev(luts, torch.float32, "luts")
        qmax = _dev(qmax, torch.float32, "qmax")
        nq, m, k = luts.shape
        qluts = torch.empty((nq, m, k), dtype=torch.uint8, device=luts.device)
        qmin = torch.empty(nq, dtype=torch.float32, device=luts.device)
        scale = torch.empty(nq, dtype=torch.float32, device=luts.device)
        self._check(self.lib.pq_quantize_luts(self.handle, _ptr(luts), nq, m, k, _ptr(qmax), _ptr(qluts), _ptr(qmin),
                                              _ptr(scale)))
        return qluts, qmin, scale

    def pq_qmax_prescan(self, codes, code_fmt, luts, init, kq):
        codes = _dev(codes, torch.uint8, "codes")
        luts = _dev(luts, torch.float32, "luts")
        nq, m, k = luts.shape
        qmax = torch.empty(nq, dtype=torch.float32, device=luts.device)
        self._check(self.lib.pq_qmax_prescan(self.handle, _ptr(codes), codes.shape[0], code_fmt, _ptr(luts), nq, m, k,
                                             init, kq, _ptr(qmax)))
        return qmax

    # -- Scan step ---------------------------------------------------------------------------
    def pq_adc_scan_topk(self, codes, code_fmt, luts, topk, out=None, noalloc=False):
        """noalloc=True: the entry point that uses the library's fixed scratch (pass `out` so that this
        layer allocates nothing either)."""
        codes = _dev(codes, torch.uint8, "codes")
        if luts.dtype == torch.uint8:
            luts = _dev(luts, torch.uint8, "luts")
            lut_fmt, vdtype = LUT_U8, torch.int32
        else:
            luts = _dev(luts, torch.float32, "luts")
            lut_fmt, vdtype = LUT_F32, torch.float32
        nq, m, k = luts.shape
        if out is None:
            vals = torch.empty((nq, topk), dtype=vdtype, device=luts.device)
            ids = torch.empty((nq, topk), dtype=torch.int64, device=luts.device)
        else:
            vals, ids = out
        entry = self.lib.pq_adc_scan_topk_noalloc if noalloc else self.lib.pq_adc_scan_topk
        self._check(entry(self.handle, _ptr(codes), codes.shape[0], code_fmt, _ptr(luts), lut_fmt,
                          nq, m, k, topk, _ptr(vals), _ptr(ids)))
        return vals, ids

    def pq_rerank_f32(self, codes, code_fmt, luts, cand_ids, topk):
        codes = _dev(codes, torch.uint8, "codes")
        luts = _dev(luts, torch.float32, "luts")
        cand_ids = _dev(cand_ids, torch.int64, "cand_ids")
        nq, m, k = luts.shape
        ncand = cand_ids.shape[1]
        dist = torch.empty((nq, topk), dtype=torch.float32, device=luts.device)
        ids = torch.empty((nq, topk), dtype=torch.int64, device=luts.device)
        self._check(self.lib.pq_rerank_f32(self.handle, _ptr(codes), codes.shape[0], code_fmt, _ptr(luts), nq, m, k,
                                           _ptr(cand_ids), ncand, topk, _ptr(dist), _ptr(ids)))
        return dist, ids

    # -- OPQ rotation ------------------------------------------------------------------------
    def pq_rotate(self, vectors, rot):
        vectors = _dev(vectors, torch.float32, "vectors")
        rot = _dev(rot, torch.float32, "rot")
        n, d = vectors.shape
        if tuple(rot.shape) != (d, d):
            raise ValueError("rot must be [d][d]")
        out = torch.empty_like(vectors)
        self._check(self.lib.pq_rotate(self.handle, _ptr(vectors), _ptr(rot), n, d, _ptr(out)))
        return out

    # -- Encoder ----------------------------------------------------------------------------
    def pq_encode(self, vectors, codebooks, code_fmt=CODES_U8):
        vectors = _dev(vectors, torch.float32, "vectors")
        codebooks = _dev(codebooks, torch.float32, "codebooks")
        n, d = vectors.shape
        m, k, _ = codebooks.shape
        code_bytes = m // 2 if code_fmt == CODES_U4_PACKED else m
        codes = torch.empty((n, code_bytes), dtype=torch.uint8, device=vectors.device)
        self._check(self.lib.pq_encode(self.handle, _ptr(vectors), _ptr(codebooks), n, d, m, k, code_fmt, _ptr(codes)))
        return codes

    # -- Search with derived quantizers ---------------------------------------------------------
    def pq_derived_search(self, codes, derived_codebooks, codebooks, queries, r2, topk, cand_cap=0):
        """codes [n][4] int16/uint16 bit patterns (torch.int16), codebooks [4][k][d/4].
        Returns (dist, ids, bucket, ncand, cand_ids or None)."""
        if codes.dtype not in (torch.int16, torch.uint16):
            raise TypeError("codes must hold 16-bit indexes")
        if not codes.is_cuda or not codes.is_contiguous():
            raise ValueError("codes must be a contiguous device tensor")
        derived_codebooks = _dev(derived_codebooks, torch.float32, "derived_codebooks")
        codebooks = _dev(codebooks, torch.float32, "codebooks")
        queries = _dev(queries, torch.float32, "queries")
        n, m = codes.shape
        nq, d = queries.shape
        k = codebooks.shape[1]
        if tuple(derived_codebooks.shape) != (m, 256, d // m) or tuple(codebooks.shape) != (m, k, d // m):
            raise ValueError("codebook shapes do not match the codes and queries")
        dev = queries.device
        dist = torch.empty((nq, topk), dtype=torch.float32, device=dev)
        ids = torch.empty((nq, topk), dtype=torch.int64, device=dev)
        bucket = torch.empty((nq,), dtype=torch.int32, device=dev)
        ncand = torch.empty((nq,), dtype=torch.int64, device=dev)
        cand = torch.empty((nq, cand_cap), dtype=torch.int64, device=dev) if cand_cap > 0 else None
        self._check(self.lib.pq_derived_search(self.handle, _ptr(codes), n, _ptr(derived_codebooks), _ptr(codebooks), k,
                                               _ptr(queries), nq, d, m, r2, topk, _ptr(dist), _ptr(ids), _ptr(bucket),
                                               _ptr(ncand), _ptr(cand) if cand is not None else None, cand_cap))
        return dist, ids, bucket, ncand, cand

    # -- Index + Tables + Scan ---------------------------------------------------------------
    def ivf_adc_search(self, coarse_centroids, list_offsets, codes, ids, codebooks, code_fmt, queries, nprobe, topk,
                       return_probes=False):
        coarse_centroids = _dev(coarse_centroids, torch.float32, "coarse_centroids")
        list_offsets = _dev(list_offsets, torch.int64, "list_offsets")
        codes = _dev(codes, torch.uint8, "codes")
        if ids is not None:
            ids = _dev(ids, torch.int64, "ids")
        codebooks = _dev(codebooks, torch.float32, "codebooks")
        queries = _dev(queries, torch.float32, "queries")
        nlist, d = coarse_centroids.shape
        m, k, _ = codebooks.shape
        nq = queries.shape[0]
        lists = IvfLists(coarse_centroids.data_ptr(), list_offsets.data_ptr(), codes.data_ptr(),
                         ids.data_ptr() if ids is not None else None, nlist, d, codes.shape[0])
        dist = torch.empty((nq, topk), dtype=torch.float32, device=queries.device)
        out_ids = torch.empty((nq, topk), dtype=torch.int64, device=queries.device)
        probes = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device) if return_probes else None
        self._check(self.lib.ivf_adc_search(self.handle, ctypes.byref(lists), _ptr(codebooks), m, k, code_fmt,
                                            _ptr(queries), nq, nprobe, topk, _ptr(dist), _ptr(out_ids), _ptr(probes)))
        return (dist, out_ids, probes) if return_probes else (dist, out_ids)

    def ivf_quick_adc_search(self, coarse_centroids, list_offsets, codes, ids, codebooks, queries, nprobe, init, kprime,
                             topk, return_probes=False):
        coarse_centroids = _dev(coarse_centroids, torch.float32, "coarse_centroids")
        list_offsets = _dev(list_offsets, torch.int64, "list_offsets")
        codes = _dev(codes, torch.uint8, "codes")
        if ids is not None:
            ids = _dev(ids, torch.int64, "ids")
        codebooks = _dev(codebooks, torch.float32, "codebooks")
        queries = _dev(queries, torch.float32, "queries")
        nlist, d = coarse_centroids.shape
        m, k, _ = codebooks.shape
        nq = queries.shape[0]
        lists = IvfLists(coarse_centroids.data_ptr(), list_offsets.data_ptr(), codes.data_ptr(),
                         ids.data_ptr() if ids is not None else None, nlist, d, codes.shape[0])
        dist = torch.empty((nq, topk), dtype=torch.float32, device=queries.device)
        out_ids = torch.empty((nq, topk), dtype=torch.int64, device=queries.device)
        probes = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device) if return_probes else None
        self._check(self.lib.ivf_quick_adc_search(self.handle, ctypes.byref(lists), _ptr(codebooks), m, k, _ptr(queries),
                                                  nq, nprobe, init, kprime, topk, _ptr(dist), _ptr(out_ids),
                                                  _ptr(probes)))
        return (dist, out_ids, probes) if return_probes else (dist, out_ids)
