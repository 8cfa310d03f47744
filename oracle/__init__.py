"""ctypes binding of the CPU oracle (oracle/hca_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  The product package never imports this module
and this module never imports the product package.

All arrays are numpy, host memory, canonical layouts:
  keys / values / queries   uint16 views of fp16 data
  codes  uint8  [R, cap, D*bits/8]   scale, zero  uint16 [R, cap, D/gs]
R = batch * kv_heads rows; query head r*G+g belongs to row r.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        # HCO_ORACLE_LIB: an already built variant of the same sources (the sanitizer test's)
        path = os.environ.get("HCO_ORACLE_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        L.hco_h2f.restype = C.c_float
        L.hco_h2f.argtypes = [C.c_uint16]
        L.hco_f2h.restype = C.c_uint16
        L.hco_f2h.argtypes = [C.c_float]
        L.hco_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def num_threads():
    return int(lib().hco_num_threads())


def h2f(bits):
    return float(lib().hco_h2f(int(bits)))


def f2h(x):
    return int(lib().hco_f2h(float(x)))


class Cache:
    """Canonical quantised key cache for R rows."""

    def __init__(self, R, cap, D=128, bits=4, gs=32):
        self.R, self.cap, self.D, self.bits, self.gs = R, cap, D, bits, gs
        self.NG, self.CB = D // gs, D * bits // 8
        self.codes = np.zeros((R, cap, self.CB), np.uint8)
        self.scale = np.zeros((R, cap, self.NG), np.uint16)
        self.zero = np.zeros((R, cap, self.NG), np.uint16)
        self.n = np.zeros(R, np.int64)

    def copy(self):
        o = Cache(self.R, self.cap, self.D, self.bits, self.gs)
        o.codes[...] = self.codes
        o.scale[...] = self.scale
        o.zero[...] = self.zero
        o.n[...] = self.n
        return o


def attention_exact(q, K, V, sm_scale):
    """Eq. 1 in fp64 for one head.  q [D], K [n,D], V [n,D] fp16."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    n, D = K.shape
    y = np.zeros(D, np.float64)
    _check(lib().hco_attention_exact(_p(q), _p(K), _p(V), C.c_int64(n), C.c_int(D),
                                     C.c_double(sm_scale), _p(y)), "attention_exact")
    return y


def quantize(cache, k_new):
    """Append k_new [R,T,D] fp16 to the cache at slots n..n+T-1."""
    k_new = _u16(k_new)
    R, T, D = k_new.shape
    assert R == cache.R and D == cache.D
    _check(lib().hco_quantize(_p(k_new), C.c_int64(R), C.c_int64(T), C.c_int(D),
                              C.c_int(cache.bits), C.c_int(cache.gs), C.c_int64(cache.cap),
                              _p(cache.n), _p(cache.codes), _p(cache.scale), _p(cache.zero)),
           "quantize")
    cache.n += T


def dequantize(cache):
    khat = np.zeros((cache.R, cache.cap, cache.D), np.float32)
    _check(lib().hco_dequantize(_p(cache.codes), _p(cache.scale), _p(cache.zero),
                                C.c_int64(cache.R), C.c_int(cache.D), C.c_int(cache.bits),
                                C.c_int(cache.gs), C.c_int64(cache.cap), _p(cache.n), _p(khat)),
           "dequantize")
    return khat


def query_fixed(q):
    """q [D] fp16 -> (qfx int32 [D], s)."""
    q = _u16(q)
    qfx = np.zeros(q.shape[0], np.int32)
    s = C.c_int32(0)
    _check(lib().hco_query_fixed(_p(q), C.c_int(q.shape[0]), _p(qfx), C.byref(s)), "query_fixed")
    return qfx, int(s.value)


def score(cache, q, want_z=True):
    """q [R*G, D] fp16 -> (sel [R,cap] fp32, z [R*G,cap] fp32 or None)."""
    q = _u16(q)
    G = q.shape[0] // cache.R
    sel = np.zeros((cache.R, cache.cap), np.float32)
    z = np.zeros((cache.R * G, cache.cap), np.float32) if want_z else None
    _check(lib().hco_score(_p(q), _p(cache.codes), _p(cache.scale), _p(cache.zero),
                           C.c_int64(cache.R), C.c_int(G), C.c_int(cache.D), C.c_int(cache.bits),
                           C.c_int(cache.gs), C.c_int64(cache.cap), _p(cache.n), _p(sel), _p(z)),
           "score")
    return sel, z


def topk(sel, n, k):
    """sel [R,cap] fp32, n [R] -> (idx int32 [R,k] ascending, -1 padded; count int32 [R])."""
    sel = np.ascontiguousarray(sel, np.float32)
    R, cap = sel.shape
    n = _i64(n)
    idx = np.zeros((R, max(k, 1)), np.int32)[:, :k].copy()
    idx = np.ascontiguousarray(idx)
    count = np.zeros(R, np.int32)
    _check(lib().hco_topk(_p(sel), C.c_int64(R), C.c_int64(cap), _p(n), C.c_int64(k),
                          _p(idx), _p(count)), "topk")
    return idx, count


def lse(z, R, n, sm_scale):
    """z [R*G, cap] fp32 -> log-sum-exp of z * sm_scale over the resident tokens, fp32 [R*G]."""
    z = np.ascontiguousarray(z, np.float32)
    G = z.shape[0] // R
    out = np.zeros(R * G, np.float32)
    _check(lib().hco_lse(_p(z), C.c_int64(R), C.c_int(G), C.c_int64(z.shape[1]), _p(_i64(n)), C.c_float(sm_scale),
                         _p(out)), "lse")
    return out


def attend(cache, q, idx, count, pos, V, sm_scale, acc=None, want_w=False, lse=None):
    """V [R, vrows, D] fp16; pos int32 [R,cap].  Returns (y [R*G,D] fp32, w or None).
    acc (fp32 [R,cap]) is updated in place when given.  lse (fp32 [R*G]): the paper's weights (Eq. 5),
    normalised over all resident tokens instead of over the selected set."""
    q, V = _u16(q), _u16(V)
    G = q.shape[0] // cache.R
    idx = np.ascontiguousarray(idx, np.int32)
    count = np.ascontiguousarray(count, np.int32)
    pos = np.ascontiguousarray(pos, np.int32)
    k = idx.shape[1]
    y = np.zeros((cache.R * G, cache.D), np.float32)
    w = np.zeros((cache.R * G, k), np.float32) if want_w else None
    if acc is not None:
        assert acc.dtype == np.float32 and acc.flags.c_contiguous
    _check(lib().hco_attend(_p(q), _p(cache.codes), _p(cache.scale), _p(cache.zero),
                            C.c_int64(cache.R), C.c_int(G), C.c_int(cache.D), C.c_int(cache.bits),
                            C.c_int(cache.gs), C.c_int64(cache.cap), _p(idx), _p(count),
                            C.c_int64(k), _p(pos), _p(V), C.c_int64(V.shape[1]),
                            C.c_float(sm_scale), _p(y), _p(w), _p(acc),
                            _p(None if lse is None else np.ascontiguousarray(lse, np.float32))), "attend")
    return y, w


def evict(cache, acc, pos, M, n_protect):
    """Compacts cache / acc / pos in place.  Returns kept int32 [R,M] (-1 padded)."""
    assert acc.dtype == np.float32 and acc.flags.c_contiguous
    assert pos.dtype == np.int32 and pos.flags.c_contiguous
    kept = np.zeros((cache.R, M), np.int32)
    n_new = np.zeros(cache.R, np.int64)
    _check(lib().hco_evict(_p(cache.codes), _p(cache.scale), _p(cache.zero), _p(acc), _p(pos),
                           C.c_int64(cache.R), C.c_int(cache.D), C.c_int(cache.bits),
                           C.c_int(cache.gs), C.c_int64(cache.cap), _p(cache.n), C.c_int64(M),
                           C.c_int64(n_protect), _p(kept), _p(n_new)), "evict")
    cache.n[...] = n_new
    return kept


# ---- codebook form of the key path (hca_vq_oracle.c) -------------------------------------

class VQCache:
    """Index matrix P for R rows: uint16 [R, cap, g]; codebook C fp32 [n_kv, g, c, D/g]."""

    def __init__(self, R, cap, codebook, D=128):
        codebook = np.ascontiguousarray(codebook, np.float32)
        self.n_kv, self.g, self.c, dbar = codebook.shape
        assert self.g * dbar == D
        self.R, self.cap, self.D, self.C = R, cap, D, codebook
        self.P = np.zeros((R, cap, self.g), np.uint16)
        self.n = np.zeros(R, np.int64)


def vq_train(kval, g, c, init, iters, shared=False):
    """kval [nval, D] fp16; init int32 [g, c] (or [c] when shared).  Returns (C fp32 [g,c,D/g],
    inertia fp64 [iters+1])."""
    kval = _u16(kval)
    nval, D = kval.shape
    init = np.ascontiguousarray(init, np.int32)
    assert init.shape == ((c,) if shared else (g, c))
    Cb = np.zeros((g, c, D // g), np.float32)
    inertia = np.zeros(iters + 1, np.float64)
    _check(lib().hco_vq_train(_p(kval), C.c_int64(nval), C.c_int(D), C.c_int(g), C.c_int(c), _p(init),
                              C.c_int(iters), C.c_int(1 if shared else 0), _p(Cb), _p(inertia)), "vq_train")
    return Cb, inertia


def vq_assign(cache, k_new):
    """Append k_new [R,T,D] fp16: nearest-centroid indices at slots n..n+T-1."""
    k_new = _u16(k_new)
    R, T, D = k_new.shape
    assert R == cache.R and D == cache.D
    _check(lib().hco_vq_assign(_p(k_new), C.c_int64(R), C.c_int64(T), C.c_int(D), C.c_int(cache.g),
                               C.c_int(cache.c), C.c_int(cache.n_kv), _p(cache.C), C.c_int64(cache.cap),
                               _p(cache.n), _p(cache.P)), "vq_assign")


def vq_dequant(cache):
    out = np.zeros((cache.R, cache.cap, cache.D), np.float32)
    _check(lib().hco_vq_dequant(_p(cache.P), C.c_int64(cache.R), C.c_int(cache.D), C.c_int(cache.g),
                                C.c_int(cache.c), C.c_int(cache.n_kv), _p(cache.C), C.c_int64(cache.cap),
                                _p(cache.n), _p(out)), "vq_dequant")
    return out


def vq_lut(cache, q):
    """q [R*G, D] fp16 -> T fp32 [R*G, g, c]."""
    q = _u16(q)
    G = q.shape[0] // cache.R
    T = np.zeros((cache.R * G, cache.g, cache.c), np.float32)
    _check(lib().hco_vq_lut(_p(q), C.c_int64(cache.R), C.c_int(G), C.c_int(cache.D), C.c_int(cache.g),
                            C.c_int(cache.c), C.c_int(cache.n_kv), _p(cache.C), _p(T)), "vq_lut")
    return T


def vq_lut_fx(T):
    """T [nq, g, c] fp32 -> (Tfx int32 [nq, g, c], sexp int32 [nq]): the tables on their power-of-two grids."""
    T = np.ascontiguousarray(T, np.float32)
    nq, g, c = T.shape
    Tfx = np.zeros((nq, g, c), np.int32)
    sexp = np.zeros(nq, np.int32)
    _check(lib().hco_vq_lut_fx(_p(T), C.c_int64(nq), C.c_int(g), C.c_int(c), _p(Tfx), _p(sexp)), "vq_lut_fx")
    return Tfx, sexp


def vq_score(cache, T, want_z=True):
    """T [R*G, g, c] -> (sel [R,cap] fp32, z [R*G,cap] fp32 or None)."""
    T = np.ascontiguousarray(T, np.float32)
    G = T.shape[0] // cache.R
    sel = np.zeros((cache.R, cache.cap), np.float32)
    z = np.zeros((cache.R * G, cache.cap), np.float32) if want_z else None
    _check(lib().hco_vq_score(_p(T), _p(cache.P), C.c_int64(cache.R), C.c_int(G), C.c_int(cache.g),
                              C.c_int(cache.c), C.c_int64(cache.cap), _p(cache.n), _p(sel), _p(z)), "vq_score")
    return sel, z


def vq_attend(cache, T, idx, count, pos, V, sm_scale, acc=None, want_w=False):
    """As attend(), with the logits of Eq. 3 taken from the table T."""
    T, V = np.ascontiguousarray(T, np.float32), _u16(V)
    G = T.shape[0] // cache.R
    idx = np.ascontiguousarray(idx, np.int32)
    count = np.ascontiguousarray(count, np.int32)
    pos = np.ascontiguousarray(pos, np.int32)
    k = idx.shape[1]
    y = np.zeros((cache.R * G, cache.D), np.float32)
    w = np.zeros((cache.R * G, k), np.float32) if want_w else None
    if acc is not None:
        assert acc.dtype == np.float32 and acc.flags.c_contiguous
    _check(lib().hco_vq_attend(_p(T), _p(cache.P), C.c_int64(cache.R), C.c_int(G), C.c_int(cache.D),
                               C.c_int(cache.g), C.c_int(cache.c), C.c_int64(cache.cap), _p(idx), _p(count),
                               C.c_int64(k), _p(pos), _p(V), C.c_int64(V.shape[1]), C.c_float(sm_scale),
                               _p(y), _p(w), _p(acc)), "vq_attend")
    return y, w


def vq_evict(cache, acc, pos, M, n_protect):
    """Compacts cache.P / acc / pos in place.  Returns kept int32 [R,M] (-1 padded)."""
    assert acc.dtype == np.float32 and acc.flags.c_contiguous
    assert pos.dtype == np.int32 and pos.flags.c_contiguous
    kept = np.zeros((cache.R, M), np.int32)
    n_new = np.zeros(cache.R, np.int64)
    _check(lib().hco_vq_evict(_p(cache.P), _p(acc), _p(pos), C.c_int64(cache.R), C.c_int(cache.g),
                              C.c_int64(cache.cap), _p(cache.n), C.c_int64(M), C.c_int64(n_protect),
                              _p(kept), _p(n_new)), "vq_evict")
    cache.n[...] = n_new
    return kept


# ---- the paper's selection rule, Eq. 4 (hca_topp_oracle.c) ---------------------------------------

def topp_weight(u):
    f = lib().hco_topp_weight
    f.restype = C.c_uint64
    f.argtypes = [C.c_float]
    return int(f(float(u)))


def topp(sel, n, sm_scale, tau, k_max):
    """sel [R,cap] fp32 -> (idx int32 [R,k_max] ascending, -1 padded; count int32 [R] = min(k*, k_max);
    kstar int64 [R]; mass uint64 [R,2] = (Theta, Z))."""
    sel = np.ascontiguousarray(sel, np.float32)
    R, cap = sel.shape
    n = _i64(n)
    idx = np.zeros((R, k_max), np.int32)
    count = np.zeros(R, np.int32)
    kstar = np.zeros(R, np.int64)
    mass = np.zeros((R, 2), np.uint64)
    _check(lib().hco_topp(_p(sel), C.c_int64(R), C.c_int64(cap), _p(n), C.c_float(sm_scale), C.c_double(tau),
                          C.c_int64(k_max), _p(idx), _p(count), _p(kstar), _p(mass)), "topp")
    return idx, count, kstar, mass


# ---- plain fp64 definitions (hca_plain_oracle.c): what the bit-reproducible forms above stand for ----------

def score_plain(cache, q):
    """Eq. 2's z~ = q . Q(K)^T with the query as it is, every term in fp64.  q [R*G, D] fp16 -> z [R*G, cap] fp64."""
    q = _u16(q)
    G = q.shape[0] // cache.R
    z = np.zeros((cache.R * G, cache.cap), np.float64)
    _check(lib().hco_score_plain(_p(q), _p(cache.codes), _p(cache.scale), _p(cache.zero), C.c_int64(cache.R),
                                 C.c_int(G), C.c_int(cache.D), C.c_int(cache.bits), C.c_int(cache.gs),
                                 C.c_int64(cache.cap), _p(cache.n), _p(z)), "score_plain")
    return z


def score_fp32(cache, q):
    """Eq. 2's z~ in plain fp32 with the query as it is (per-group ascending fused multiply-add chains, the pairwise
    group sum).  q [R*G, D] fp16 -> z [R*G, cap] fp32."""
    q = _u16(q)
    G = q.shape[0] // cache.R
    z = np.zeros((cache.R * G, cache.cap), np.float32)
    _check(lib().hco_score_fp32(_p(q), _p(cache.codes), _p(cache.scale), _p(cache.zero), C.c_int64(cache.R),
                                C.c_int(G), C.c_int(cache.D), C.c_int(cache.bits), C.c_int(cache.gs),
                                C.c_int64(cache.cap), _p(cache.n), _p(z)), "score_fp32")
    return z


def vq_score_plain(cache, T):
    """Eq. 3 as written: z[hq, j] = sum_i T[hq, i, P[j, i]] in fp64.  T [R*G, g, c] fp32 -> z [R*G, cap] fp64."""
    T = np.ascontiguousarray(T, np.float32)
    G = T.shape[0] // cache.R
    z = np.zeros((cache.R * G, cache.cap), np.float64)
    _check(lib().hco_vq_score_plain(_p(T), _p(cache.P), C.c_int64(cache.R), C.c_int(G), C.c_int(cache.g),
                                    C.c_int(cache.c), C.c_int64(cache.cap), _p(cache.n), _p(z)), "vq_score_plain")
    return z


def topp_plain(sel, n, sm_scale, tau, want_cum=True):
    """Eq. 4 as written, fp64 softmax over each row.  Returns (kstar int64 [R], order int32 [R,cap] or None,
    cum fp64 [R,cap] or None): order[r, t] is the slot at sorted position t (score descending, slot
    ascending), cum[r, t] the attention mass of the first t + 1 sorted slots."""
    sel = np.ascontiguousarray(sel, np.float32)
    R, cap = sel.shape
    n = _i64(n)
    kstar = np.zeros(R, np.int64)
    order = np.zeros((R, cap), np.int32) if want_cum else None
    cum = np.zeros((R, cap), np.float64) if want_cum else None
    _check(lib().hco_topp_plain(_p(sel), C.c_int64(R), C.c_int64(cap), _p(n), C.c_double(sm_scale),
                                C.c_double(tau), _p(kstar), _p(order), _p(cum)), "topp_plain")
    return kstar, order, cum


# ---- the paper's CPU-side weighted sum (Sec. 3.2 "CPU part", Sec. 3.3: 2 bytes per weight) ----------

def weighted_sum_f16(w, idx, count, pos, V):
    """y [R*G, D] (fp64) = sum_i fp16(w[hq, i]) * V[r, pos[r, idx[r, i]]]: the weights cross the link as
    2-byte values, the host sums.  w [R*G, k] fp32 (from attend(..., want_w=True)), V [R, vrows, D] fp16."""
    w16 = np.asarray(w, np.float32).astype(np.float16).astype(np.float64)
    R = idx.shape[0]
    G = w16.shape[0] // R
    V = np.asarray(V)
    y = np.zeros((R * G, V.shape[2]), np.float64)
    for r in range(R):
        c = int(count[r])
        rows = pos[r, idx[r, :c]]
        vr = V[r, rows].astype(np.float64)
        for h in range(G):
            y[r * G + h] = w16[r * G + h, :c] @ vr
    return y
