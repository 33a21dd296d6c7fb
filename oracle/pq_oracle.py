"""ctypes front-end of the CPU oracle (``pq_oracle.c``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import this module; the GPU library and its Python binding
never do.  Arguments and results are numpy arrays on the host.  Function names
follow the thesis: ``build_luts`` is Alg. 1 ``compute_tables`` (Eq. tables),
``adc_scan_topk_*`` is Alg. 1 ``scan`` / Alg. 3 ``quick_adc_scan``,
``quantize_luts`` is Alg. 5 ``quantize``, ``rerank_f32`` is Alg. 5 ``rerank``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pq_oracle.c")
_LIB = os.path.join(_HERE, "libpq_oracle.so")

CODES_U8 = 0
CODES_U4_PACKED = 1

_lib = None


def build(force=False):
    """Compile pq_oracle.c with gcc (no fast-math, no contraction).  PQ_ORACLE_SANITIZE=1 builds it with the address
    and undefined-behaviour sanitizers (CPU only; the interpreter then has to be started with libasan preloaded)."""
    sanitize = os.environ.get("PQ_ORACLE_SANITIZE", "") not in ("", "0")
    if force or sanitize or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        if sanitize:
            cmd[1:1] = ["-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-fno-sanitize-recover=undefined"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _i64(v):
    return ctypes.c_int64(int(v))


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def code_bytes(m, fmt):
    return m // 2 if fmt == CODES_U4_PACKED else m


def kmeans(x, k, iters, init_idx):
    x = _f32(x)
    n, dsub = x.shape
    init_idx = np.ascontiguousarray(init_idx, dtype=np.int64)
    cent = np.empty((k, dsub), np.float32)
    _check(lib().orc_kmeans(_p(x), _i64(n), dsub, _i64(dsub), k, iters, _p(init_idx), _p(cent)), "kmeans")
    return cent


def pq_train(x, m, k, iters, init_idx):
    x = _f32(x)
    n, d = x.shape
    init_idx = np.ascontiguousarray(init_idx, dtype=np.int64).reshape(m, k)
    cb = np.empty((m, k, d // m), np.float32)
    _check(lib().orc_pq_train(_p(x), _i64(n), d, m, k, iters, _p(init_idx), _p(cb)), "pq_train")
    return cb


def pq_encode(x, codebooks):
    x = _f32(x)
    codebooks = _f32(codebooks)
    n, d = x.shape
    m, k, _ = codebooks.shape
    codes = np.empty((n, m), np.uint8)
    _check(lib().orc_pq_encode(_p(x), _i64(n), d, m, k, _p(codebooks), _p(codes)), "pq_encode")
    return codes


def pack_u4(codes):
    codes = _u8(codes)
    n, m = codes.shape
    out = np.empty((n, m // 2), np.uint8)
    _check(lib().orc_pack_u4(_p(codes), _i64(n), m, _p(out)), "pack_u4")
    return out


def rotate(x, R):
    x = _f32(x)
    R = _f32(R)
    n, d = x.shape
    assert R.shape == (d, d)
    out = np.empty((n, d), np.float32)
    _check(lib().orc_rotate(_p(x), _i64(n), d, _p(R), _p(out)), "rotate")
    return out


def build_luts(queries, codebooks):
    queries = _f32(queries)
    codebooks = _f32(codebooks)
    nq, d = queries.shape
    m, k, _ = codebooks.shape
    luts = np.empty((nq, m, k), np.float32)
    _check(lib().orc_build_luts(_p(queries), nq, d, m, k, _p(codebooks), _p(luts)), "build_luts")
    return luts


def quantize_luts(luts, qmax):
    luts = _f32(luts)
    nq, m, k = luts.shape
    qmax = _f32(qmax).reshape(nq)
    q = np.empty((nq, m, k), np.uint8)
    qmin = np.empty(nq, np.float32)
    scale = np.empty(nq, np.float32)
    _check(lib().orc_quantize_luts(_p(luts), nq, m, k, _p(qmax), _p(q), _p(qmin), _p(scale)), "quantize_luts")
    return q, qmin, scale


def adc_all_f32(codes, fmt, lut):
    codes = _u8(codes)
    lut = _f32(lut)
    m, k = lut.shape
    n = codes.shape[0]
    assert codes.shape[1] == code_bytes(m, fmt)
    out = np.empty(n, np.float32)
    _check(lib().orc_adc_all_f32(_p(codes), _i64(n), fmt, _p(lut), m, k, _p(out)), "adc_all_f32")
    return out


def adc_all_u8(codes, fmt, qlut):
    codes = _u8(codes)
    qlut = _u8(qlut)
    m, k = qlut.shape
    n = codes.shape[0]
    assert codes.shape[1] == code_bytes(m, fmt)
    out = np.empty(n, np.uint32)
    _check(lib().orc_adc_all_u8(_p(codes), _i64(n), fmt, _p(qlut), m, k, _p(out)), "adc_all_u8")
    return out


def adc_scan_topk_f32(codes, fmt, luts, topk):
    codes = _u8(codes)
    luts = _f32(luts)
    nq, m, k = luts.shape
    n = codes.shape[0]
    assert codes.shape[1] == code_bytes(m, fmt)
    dist = np.empty((nq, topk), np.float32)
    ids = np.empty((nq, topk), np.int64)
    _check(lib().orc_adc_scan_topk_f32(_p(codes), _i64(n), fmt, _p(luts), nq, m, k, topk, _p(dist), _p(ids)),
           "adc_scan_topk_f32")
    return dist, ids


def adc_scan_topk_u8(codes, fmt, qluts, topk):
    codes = _u8(codes)
    qluts = _u8(qluts)
    nq, m, k = qluts.shape
    n = codes.shape[0]
    assert codes.shape[1] == code_bytes(m, fmt)
    sums = np.empty((nq, topk), np.uint32)
    ids = np.empty((nq, topk), np.int64)
    _check(lib().orc_adc_scan_topk_u8(_p(codes), _i64(n), fmt, _p(qluts), nq, m, k, topk, _p(sums), _p(ids)),
           "adc_scan_topk_u8")
    return sums, ids


def rerank_f32(codes, fmt, luts, cand_ids, topk):
    codes = _u8(codes)
    luts = _f32(luts)
    nq, m, k = luts.shape
    cand_ids = np.ascontiguousarray(cand_ids, dtype=np.int64)
    ncand = cand_ids.shape[1]
    dist = np.empty((nq, topk), np.float32)
    ids = np.empty((nq, topk), np.int64)
    _check(lib().orc_rerank_f32(_p(codes), fmt, _p(luts), nq, m, k, _p(cand_ids), ncand, topk, _p(dist), _p(ids)),
           "rerank_f32")
    return dist, ids


def qmax_prescan(codes, fmt, luts, init, kq):
    codes = _u8(codes)
    luts = _f32(luts)
    nq, m, k = luts.shape
    n = codes.shape[0]
    out = np.empty(nq, np.float32)
    _check(lib().orc_qmax_prescan(_p(codes), _i64(n), fmt, _p(luts), nq, m, k, _i64(init), kq, _p(out)),
           "qmax_prescan")
    return out


def ivf_probe(queries, coarse, nprobe):
    queries = _f32(queries)
    coarse = _f32(coarse)
    nq, d = queries.shape
    nlist = coarse.shape[0]
    probes = np.empty((nq, nprobe), np.int32)
    pd = np.empty((nq, nprobe), np.float32)
    _check(lib().orc_ivf_probe(_p(queries), nq, d, _p(coarse), nlist, nprobe, _p(probes), _p(pd)), "ivf_probe")
    return probes, pd


def ivf_scan(queries, coarse, list_offsets, codes, ids, codebooks, fmt, probes, topk):
    queries = _f32(queries)
    coarse = _f32(coarse)
    codebooks = _f32(codebooks)
    codes = _u8(codes)
    list_offsets = np.ascontiguousarray(list_offsets, dtype=np.int64)
    probes = np.ascontiguousarray(probes, dtype=np.int32)
    if ids is not None:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
    nq, d = queries.shape
    nlist = coarse.shape[0]
    m, k, _ = codebooks.shape
    nprobe = probes.shape[1]
    dist = np.empty((nq, topk), np.float32)
    out_ids = np.empty((nq, topk), np.int64)
    _check(lib().orc_ivf_scan(_p(queries), nq, d, _p(coarse), nlist, _p(list_offsets), _p(codes), _p(ids),
                              _p(codebooks), m, k, fmt, _p(probes), nprobe, topk, _p(dist), _p(out_ids)),
           "ivf_scan")
    return dist, out_ids


def ivf_search(queries, coarse, list_offsets, codes, ids, codebooks, fmt, nprobe, topk):
    probes, _ = ivf_probe(queries, coarse, nprobe)
    return ivf_scan(queries, coarse, list_offsets, codes, ids, codebooks, fmt, probes, topk)


def ivf_quick_scan(queries, coarse, list_offsets, codes, ids, codebooks, fmt, probes, init, kprime, topk):
    """IVFADC search with Quick ADC in the Scan step (orc_ivf_quick_scan)."""
    queries = _f32(queries)
    coarse = _f32(coarse)
    codebooks = _f32(codebooks)
    codes = _u8(codes)
    list_offsets = np.ascontiguousarray(list_offsets, dtype=np.int64)
    probes = np.ascontiguousarray(probes, dtype=np.int32)
    if ids is not None:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
    nq, d = queries.shape
    nlist = coarse.shape[0]
    m, k, _ = codebooks.shape
    nprobe = probes.shape[1]
    dist = np.empty((nq, topk), np.float32)
    out_ids = np.empty((nq, topk), np.int64)
    _check(lib().orc_ivf_quick_scan(_p(queries), nq, d, _p(coarse), nlist, _p(list_offsets), _p(codes), _p(ids),
                                    _p(codebooks), m, k, fmt, _p(probes), nprobe, _i64(init), kprime, topk,
                                    _p(dist), _p(out_ids)), "ivf_quick_scan")
    return dist, out_ids


def ivf_quick_search(queries, coarse, list_offsets, codes, ids, codebooks, fmt, nprobe, init, kprime, topk):
    probes, _ = ivf_probe(queries, coarse, nprobe)
    return ivf_quick_scan(queries, coarse, list_offsets, codes, ids, codebooks, fmt, probes, init, kprime, topk)


def set_threads(n):
    """Number of OpenMP threads the query-parallel loops use (0 = library default)."""
    omp = ctypes.CDLL("libgomp.so.1")
    if n > 0:
        omp.omp_set_num_threads(int(n))
    return omp.omp_get_max_threads()
