"""ctypes front end of the CPU oracle (oracle/avq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by the cpu_baseline leg of bench.py. The product package never imports this.
All arrays are host numpy arrays; nothing here touches a GPU.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "avq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc. -ffp-contract=off keeps the written fp32
    operation order (no fused multiply-adds other than the explicit fmaf)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_eta_limit.restype = C.c_double
        _lib.orc_eta_limit.argtypes = [C.c_int, C.c_double, C.c_double]
        _lib.orc_eta_exact.restype = C.c_double
        _lib.orc_eta_exact.argtypes = [C.c_int, C.c_double, C.c_double]
        _lib.orc_sin_power_integral.restype = C.c_double
        _lib.orc_sin_power_integral.argtypes = [C.c_int, C.c_double]
        _lib.orc_eta.restype = C.c_double
        _lib.orc_eta.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, C.c_double]
        _lib.orc_aniso_loss.restype = C.c_double
        _lib.orc_encode_exhaustive.restype = C.c_double
        _lib.orc_init_index.restype = C.c_int64
        _lib.orc_init_index.argtypes = [C.c_uint64, C.c_uint32, C.c_int, C.c_int, C.c_int64]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def num_threads():
    return int(lib().orc_num_threads())


def set_num_threads(t):
    lib().orc_set_num_threads(C.c_int(int(t)))


# ---- eta, decomposition, loss -------------------------------------------------

def eta_limit(d, T, norm=1.0):
    return float(lib().orc_eta_limit(int(d), float(T), float(norm)))


def eta_exact(d, T, norm=1.0):
    return float(lib().orc_eta_exact(int(d), float(T), float(norm)))


def sin_power_integral(d, alpha):
    return float(lib().orc_sin_power_integral(int(d), float(alpha)))


def eta(mode, d, T, norm=1.0, eta_explicit=1.0):
    return float(lib().orc_eta(int(mode), int(d), float(T), float(norm), float(eta_explicit)))


def residual_decompose(x, xt):
    x, xt = _f64(x), _f64(xt)
    rp, ro = np.empty_like(x), np.empty_like(x)
    lib().orc_residual_decompose(_p(x), _p(xt), C.c_int(x.size), _p(rp), _p(ro))
    return rp, ro


def aniso_loss(x, xt, eta_):
    x, xt = _f64(x), _f64(xt)
    return float(lib().orc_aniso_loss(_p(x), _p(xt), C.c_int(x.size), C.c_double(eta_)))


# ---- training / encoding ------------------------------------------------------

def init_index(seed, stream, j, k, n):
    return int(lib().orc_init_index(int(seed), int(stream), int(j), int(k), int(n)))


def kmeans(x, k, iters, seed, stream=0):
    """Lloyd on full rows of x; returns centers [k][d] fp32."""
    x = _f32(x)
    n, d = x.shape
    centers = np.empty((k, d), np.float32)
    rc = lib().orc_kmeans(_p(x), C.c_int64(n), C.c_int(d), C.c_int(0), C.c_int(d), C.c_int(k),
                          C.c_int(iters), C.c_uint64(seed), C.c_uint32(stream), None, None,
                          _p(centers))
    if rc:
        raise ValueError("orc_kmeans rc=%d" % rc)
    return centers


def assign_nearest(x, centers):
    x, centers = _f32(x), _f32(centers)
    out = np.empty(x.shape[0], np.int32)
    lib().orc_assign_nearest(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(centers),
                             C.c_int(centers.shape[0]), _p(out))
    return out


def train_pq(x, M, kc, iters, seed, leaf_centers=None, leaf_assign=None):
    """codebooks [M][kc][d/M] fp32 by per-subspace k-means (on residuals to
    the leaf centers when those are given)."""
    x = _f32(x)
    n, d = x.shape
    cb = np.empty((M, kc, d // M), np.float32)
    lc = None if leaf_centers is None else _f32(leaf_centers)
    la = _i32(leaf_assign)
    rc = lib().orc_train_pq(_p(x), C.c_int64(n), C.c_int(d), C.c_int(M), C.c_int(kc),
                            C.c_int(iters), C.c_uint64(seed), _p(lc), _p(la), _p(cb))
    if rc:
        raise ValueError("orc_train_pq rc=%d" % rc)
    return cb


def encode(x, codebooks, T, eta_mode=0, eta_explicit=1.0, passes=10, leaf_centers=None,
           leaf_assign=None):
    """codes [n][M] uint8, one byte per subspace."""
    x, cb = _f32(x), _f32(codebooks)
    n, d = x.shape
    M, kc, _ = cb.shape
    codes = np.empty((n, M), np.uint8)
    lc = None if leaf_centers is None else _f32(leaf_centers)
    la = _i32(leaf_assign)
    rc = lib().orc_encode(_p(x), C.c_int64(n), C.c_int(d), C.c_int(M), C.c_int(kc), _p(cb),
                          _p(lc), _p(la), C.c_int(eta_mode), C.c_double(T),
                          C.c_double(eta_explicit), C.c_int(passes), _p(codes))
    if rc:
        raise ValueError("orc_encode rc=%d" % rc)
    return codes


def encode_exhaustive(x, codebooks, eta_, center=None):
    x, cb = _f32(x), _f32(codebooks)
    M, kc, ds = cb.shape
    code = np.empty(M, np.uint8)
    ce = None if center is None else _f32(center)
    v = lib().orc_encode_exhaustive(_p(x), _p(ce), C.c_int(M * ds), C.c_int(M), C.c_int(kc),
                                    _p(cb), C.c_double(eta_), _p(code))
    return code, float(v)


def reconstruct(codes, codebooks, centers=None, assign=None):
    codes, cb = _u8(codes), _f32(codebooks)
    n, M = codes.shape
    _, kc, ds = cb.shape
    xt = np.empty((n, M * ds), np.float64)
    ce = None if centers is None else _f32(centers)
    lib().orc_reconstruct(_p(codes), C.c_int64(n), _p(cb), _p(ce), _p(_i32(assign)),
                          C.c_int(M * ds), C.c_int(M), C.c_int(kc), _p(xt))
    return xt


def pack_codes(codes, bits):
    codes = _u8(codes)
    n, M = codes.shape
    bpp = (M * bits + 7) // 8
    out = np.empty((n, bpp), np.uint8)
    lib().orc_pack_codes(_p(codes), C.c_int64(n), C.c_int(M), C.c_int(bits), _p(out))
    return out


def vq_update(x_members, h_par, h_perp):
    x = _f64(x_members)
    cnt, d = x.shape
    out = np.empty(d, np.float64)
    rc = lib().orc_vq_update(_p(x), C.c_int64(cnt), C.c_int(d), _p(_f64(h_par)),
                             _p(_f64(h_perp)), _p(out))
    if rc:
        raise ValueError("orc_vq_update rc=%d" % rc)
    return out


def pq_joint_update(x, codes, eta_per_point, codebooks, centers=None, assign=None):
    """Appendix 7.5's joint codeword update; with centers/assign, for residual PQ on a partitioned index."""
    x, codes = _f32(x), _u8(codes)
    cb = _f32(codebooks).copy()
    n, d = x.shape
    M, kc, _ = cb.shape
    if centers is None:
        rc = lib().orc_pq_joint_update(_p(x), C.c_int64(n), C.c_int(d), C.c_int(M), C.c_int(kc),
                                       _p(codes), _p(_f64(eta_per_point)), _p(cb))
    else:
        ce, la = _f32(centers), _i32(assign)
        rc = lib().orc_pq_joint_update_resid(_p(x), C.c_int64(n), C.c_int(d), C.c_int(M), C.c_int(kc),
                                             _p(codes), _p(_f64(eta_per_point)), _p(ce), _p(la), _p(cb))
    if rc:
        raise ValueError("orc_pq_joint_update rc=%d" % rc)
    return cb


def assign_aniso(x, centers, T, eta_mode=0, eta_explicit=1.0):
    """Every row to the center of smallest anisotropic loss (Definition 4.1's assignment step)."""
    x, centers = _f32(x), _f32(centers)
    out = np.empty(x.shape[0], np.int32)
    lib().orc_assign_aniso(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(centers),
                           C.c_int(centers.shape[0]), C.c_int(eta_mode), C.c_double(T),
                           C.c_double(eta_explicit), _p(out))
    return out


def vq_centers_update(x, assign, centers, T, eta_mode=0, eta_explicit=1.0):
    """Theorem 4.2 for every partition: the center that minimises the anisotropic loss of its members
    (h_perp = 1, h_par = eta_i); a partition without members keeps its center. Returns fp32 centers."""
    x = _f32(x)
    out = _f32(centers).copy()
    d = x.shape[1]
    for l in range(out.shape[0]):
        mem = np.nonzero(np.asarray(assign) == l)[0]
        if mem.size == 0:
            continue
        xm = x[mem].astype(np.float64)
        h_par = np.array([eta(eta_mode, d, T, float(np.sqrt((r * r).sum())), eta_explicit) for r in xm])
        out[l] = vq_update(xm, h_par, np.ones(mem.size)).astype(np.float32)
    return out


# ---- query path -----------------------------------------------------------------

def lut_f32(q, codebooks):
    q, cb = _f32(q), _f32(codebooks)
    M, kc, ds = cb.shape
    L = np.empty((M, kc), np.float32)
    lib().orc_lut_f32(_p(q), _p(cb), C.c_int(M * ds), C.c_int(M), C.c_int(kc), _p(L))
    return L


def lut_u8(L):
    L = _f32(L)
    M, kc = L.shape
    Q8 = np.empty((M, kc), np.uint8)
    scale, bias = C.c_float(), C.c_float()
    lib().orc_lut_u8(_p(L), C.c_int(M), C.c_int(kc), _p(Q8), C.byref(scale), C.byref(bias))
    return Q8, np.float32(scale.value), np.float32(bias.value)


def adc_f32(L, codes, bits):
    L, codes = _f32(L), _u8(codes)
    n, M = codes.shape
    out = np.empty(n, np.float32)
    lib().orc_adc_f32(_p(L), _p(codes), C.c_int64(n), C.c_int(M), C.c_int(L.shape[1]),
                      C.c_int(bits), _p(out))
    return out


def adc_u8(Q8, codes):
    Q8, codes = _u8(Q8), _u8(codes)
    n, M = codes.shape
    out = np.empty(n, np.uint32)
    lib().orc_adc_u8(_p(Q8), _p(codes), C.c_int64(n), C.c_int(M), C.c_int(Q8.shape[1]), _p(out))
    return out


def topk(scores, k, ids=None):
    scores = _f32(scores)
    ids_out = np.empty(k, np.int32)
    s_out = np.empty(k, np.float32)
    lib().orc_topk(_p(scores), _p(_i32(ids)), C.c_int64(scores.size), C.c_int(k), _p(ids_out),
                   _p(s_out))
    return ids_out, s_out


def exact_scores(x, q):
    x, q = _f32(x), _f32(q)
    out = np.empty(x.shape[0], np.float32)
    lib().orc_exact_scores(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(q), _p(out))
    return out


def brute_force(x, queries, k):
    x, queries = _f32(x), _f32(queries)
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.int32)
    sc = np.empty((nq, k), np.float32)
    lib().orc_brute_force(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(queries),
                          C.c_int(nq), C.c_int(k), _p(ids), _p(sc))
    return ids, sc


def leaf_select(centers, q, L):
    centers, q = _f32(centers), _f32(q)
    ids = np.empty(L, np.int32)
    ip = np.empty(L, np.float32)
    lib().orc_leaf_select(_p(centers), C.c_int(centers.shape[0]), C.c_int(centers.shape[1]),
                          _p(q), C.c_int(L), _p(ids), _p(ip))
    return ids, ip


def adc_keys_flat(q, codebooks, codes, bits, lut_mode):
    """All n ADC keys of one query on a flat index, plus (scale, bias)."""
    q, cb, codes = _f32(q), _f32(codebooks), _u8(codes)
    n, M = codes.shape
    keys = np.empty(n, np.float32)
    scale, bias = C.c_float(), C.c_float()
    lib().orc_adc_keys_flat(_p(q), C.c_int(q.size), C.c_int(M), C.c_int(bits), _p(cb),
                            _p(codes), C.c_int64(n), C.c_int(lut_mode), _p(keys),
                            C.byref(scale), C.byref(bias))
    return keys, np.float32(scale.value), np.float32(bias.value)


def search(x, codebooks, codes, bits, queries, k, reorder_k, lut_mode, centers=None,
           assign=None, leaves_to_search=0):
    """The whole query path; returns (ids [nq][k] int32, scores [nq][k] fp32)."""
    cb, codes, queries = _f32(codebooks), _u8(codes), _f32(queries)
    n, M = codes.shape
    nq, d = queries.shape
    xx = None if x is None else _f32(x)
    ce = None if centers is None else _f32(centers)
    n_leaves = 0 if ce is None else ce.shape[0]
    ids = np.empty((nq, k), np.int32)
    sc = np.empty((nq, k), np.float32)
    rc = lib().orc_search(_p(xx), C.c_int64(n), C.c_int(d), C.c_int(M), C.c_int(bits), _p(cb),
                          _p(codes), C.c_int(n_leaves), _p(ce), _p(_i32(assign)), _p(queries),
                          C.c_int(nq), C.c_int(k), C.c_int(reorder_k), C.c_int(lut_mode),
                          C.c_int(leaves_to_search), _p(ids), _p(sc))
    if rc:
        raise ValueError("orc_search rc=%d" % rc)
    return ids, sc


# ---- quality metrics of Section 5 ---------------------------------------------------------

def quality_metrics(x, queries, codebooks, codes, bits, top_n=(1, 2, 5, 10, 20, 50, 100)):
    """Section 5.2's retrieval metric and Section 5.1's estimation error for one encoding, from the definitions:

    hits[N] = number of queries whose true best datapoint (arg max <q, x_i>, exact search as in Section 1)
    is among the N datapoints with the largest quantized scores <q, x~_i> (ADC with fp32 tables, ordered by
    score descending then id ascending); Recall 1@N = hits[N] / number of queries.
    rel[i] = |<q_i, x~> - <q_i, x>| / |<q_i, x>| for query i and its true best datapoint x (Figure 2b).
    """
    x, queries = _f32(x), _f32(queries)
    nq, n = queries.shape[0], x.shape[0]
    gt_ids, gt_sc = brute_force(x, queries, 1)
    kmax = min(max(top_n), n)
    hits = {N: 0 for N in top_n if N <= kmax}
    rel = np.empty(nq, np.float64)
    for i in range(nq):
        keys, _, _ = adc_keys_flat(queries[i], codebooks, codes, bits, 0)
        best, _ = topk(keys, kmax)
        for N in hits:
            hits[N] += int(gt_ids[i, 0] in best[:N])
        rel[i] = abs(float(keys[gt_ids[i, 0]]) - float(gt_sc[i, 0])) / abs(float(gt_sc[i, 0]))
    return hits, rel
