"""Thin ctypes binding of libhca.so: argument marshalling only.

Every function has the name and the argument order of its C entry point (include/hca.h).
Tensors are torch tensors whose data_ptr() is handed over; streams are torch.cuda.Stream
objects (or None for the current stream).  No step of the path runs in Python, and there is
no fallback: a missing library raises at import of the first call.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhca.so")

HCA_OK = 0
ERRORS = {-1: "HCA_ERR_BAD_ARG", -2: "HCA_ERR_UNSUPPORTED", -3: "HCA_ERR_CAPACITY", -4: "HCA_ERR_HIP"}


class HcaError(RuntimeError):
    def __init__(self, what, code, hip=0):
        self.code = code
        super().__init__(f"{what}: {ERRORS.get(code, code)}" + (f" (hipError {hip})" if code == -4 else ""))


class hca_shape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32),
                ("capacity", C.c_int64)]


class hca_layer(C.Structure):
    _fields_ = [("kcache", C.c_void_p), ("acc", C.c_void_p), ("pos", C.c_void_p), ("k_new", C.c_void_p),
                ("q", C.c_void_p), ("v_host", C.c_void_p), ("v_hbm", C.c_void_p), ("y", C.c_void_p),
                ("vq_centroids", C.c_void_p), ("vq_lut", C.c_void_p)]


PIPELINE_MAX_SEL = 64
PIPELINE_MAX_PIPE = 8


class hca_pipeline_desc(C.Structure):
    _fields_ = [("stream_scan", C.c_void_p), ("stream_topk", C.c_void_p), ("stream_gather", C.c_void_p),
                ("stream_attend", C.c_void_p), ("sel", C.c_void_p * PIPELINE_MAX_SEL), ("n_sel", C.c_int32),
                ("idx", C.c_void_p * PIPELINE_MAX_PIPE),
                ("count", C.c_void_p * PIPELINE_MAX_PIPE), ("ws_attend", C.c_void_p * PIPELINE_MAX_PIPE), ("ws_topk", C.c_void_p),
                ("ws_evict", C.c_void_p), ("spare_kcache", C.c_void_p), ("spare_acc", C.c_void_p),
                ("spare_pos", C.c_void_p), ("scan_stamps", C.c_void_p), ("scan_stamp_pairs", C.c_int64),
                ("timing_layer_stride", C.c_int32), ("vq_groups", C.c_int32), ("vq_codewords", C.c_int32),
                ("topp_tau", C.c_double), ("fused_select", C.c_int32),
                ("ws_select", C.c_void_p * PIPELINE_MAX_SEL), ("gather_stamps", C.c_void_p),
                ("host_chunks", C.c_int32), ("host_threads", C.c_int32), ("host_spin_limit", C.c_int32),
                ("gather_wgs", C.c_int32), ("gather_unroll", C.c_int32), ("score_bpw", C.c_int32),
                ("score_depth", C.c_int32), ("select_wg", C.c_int32), ("n_pipe", C.c_int32), ("dual_scan", C.c_int32),
                ("layer_idx", C.c_void_p), ("layer_count", C.c_void_p), ("layer_idx_stride", C.c_int64)]


class hca_vq_codebook(C.Structure):
    _fields_ = [("groups", C.c_int32), ("codewords", C.c_int32), ("centroids", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        sp = C.POINTER(hca_shape)
        L.hca_version.restype = C.c_char_p
        L.hca_last_hip_error.restype = i32
        L.hca_tune.restype = i32
        L.hca_tune.argtypes = [C.c_char_p, i32]
        L.hca_kcache_bytes.restype = C.c_size_t
        L.hca_kcache_bytes.argtypes = [sp]
        L.hca_workspace_bytes.restype = C.c_size_t
        L.hca_workspace_bytes.argtypes = [sp, i64, i64]
        L.hca_quantize_keys.restype = i32
        L.hca_quantize_keys.argtypes = [sp, vp, vp, i64, vp, vp, vp, vp, vp]
        L.hca_score_qkeys.restype = i32
        L.hca_score_qkeys.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
        L.hca_topk.restype = i32
        L.hca_topk.argtypes = [sp, vp, vp, i32, vp, vp, vp, vp]
        L.hca_topk_noalloc.restype = i32
        L.hca_topk_noalloc.argtypes = [sp, vp, vp, i32, vp, vp, vp]
        L.hca_score_topk.restype = i32
        L.hca_score_topk.argtypes = [sp, vp, vp, vp, i32, vp, vp, vp, vp]
        L.hca_score_topk_report.restype = i32
        L.hca_score_topk_report.argtypes = [sp, vp, vp, vp, vp, vp]
        L.hca_score_topk_monitor.restype = i32
        L.hca_score_topk_monitor.argtypes = [sp, vp, vp, i32, vp]
        L.hca_score_qkeys_lse.restype = i32
        L.hca_score_qkeys_lse.argtypes = [sp, vp, vp, vp, f32, vp, vp, vp, vp]
        L.hca_attend_gathered_global.restype = i32
        L.hca_attend_gathered_global.argtypes = [sp, vp, vp, vp, vp, i32, f32, vp, vp, vp, vp, vp]
        L.hca_attend_weights.restype = i32
        L.hca_attend_weights.argtypes = [sp, vp, vp, vp, vp, i32, vp, f32, vp, vp, vp, vp, vp, vp]
        L.hca_host_weighted_sum.restype = i32
        L.hca_host_weighted_sum.argtypes = [sp, vp, vp, i32, vp, vp, i64, vp, i32]
        L.hca_topp.restype = i32
        L.hca_topp.argtypes = [sp, vp, vp, f32, C.c_double, i32, vp, vp, vp, vp, vp]
        L.hca_sparse_attend.restype = i32
        L.hca_sparse_attend.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp, i64, i64, vp, i64, f32, vp, vp,
                                        vp, vp, vp]
        L.hca_gather_values.restype = i32
        L.hca_gather_values.argtypes = [sp, vp, vp, i32, vp, vp, i64, i64, vp, i64, vp, vp]
        L.hca_attend_gathered.restype = i32
        L.hca_attend_gathered.argtypes = [sp, vp, vp, vp, vp, i32, f32, vp, vp, vp, vp]
        L.hca_evict.restype = i32
        L.hca_evict.argtypes = [sp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp]
        L.hca_pipeline_create.restype = vp
        L.hca_pipeline_create.argtypes = [sp, i32, C.POINTER(hca_pipeline_desc), i32]
        L.hca_pipeline_destroy.restype = None
        L.hca_pipeline_destroy.argtypes = [vp]
        L.hca_pipeline_step.restype = i32
        L.hca_pipeline_step.argtypes = [vp, C.POINTER(hca_layer), C.POINTER(i64), i64, i32, i64, i64, i64, f32,
                                        C.POINTER(i64), i64, i32]
        L.hca_pipeline_host_status.restype = i32
        L.hca_pipeline_host_status.argtypes = [vp, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                               C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.hca_debug_host_chunk_sum.restype = i32
        L.hca_debug_host_chunk_sum.argtypes = [i32, vp, vp, vp, i64, vp]
        L.hca_host_prefault.restype = i32
        L.hca_host_prefault.argtypes = [vp, C.c_size_t, i32]
        L.hca_scan_stamp_pairs.restype = i64
        L.hca_scan_stamp_pairs.argtypes = [sp, i64]
        L.hca_wall_clock_khz.restype = i32
        L.hca_pipeline_scan_ms.restype = i32
        L.hca_pipeline_scan_ms.argtypes = [vp, i32, C.POINTER(f32)]
        L.hca_export_kcache.restype = i32
        L.hca_export_kcache.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        cbp = C.POINTER(hca_vq_codebook)
        L.hca_vq_pcache_bytes.restype = C.c_size_t
        L.hca_vq_pcache_bytes.argtypes = [sp, cbp]
        L.hca_vq_workspace_bytes.restype = C.c_size_t
        L.hca_vq_workspace_bytes.argtypes = [sp, cbp, i64, i64]
        L.hca_vq_lut_bytes.restype = C.c_size_t
        L.hca_vq_lut_bytes.argtypes = [sp, cbp]
        L.hca_vq_train.restype = i32
        L.hca_vq_train.argtypes = [vp, i64, i32, i32, i32, vp, i32, i32, vp, vp]
        L.hca_vq_assign.restype = i32
        L.hca_vq_assign.argtypes = [sp, cbp, vp, vp, i64, vp, vp, vp, vp, vp]
        L.hca_vq_score.restype = i32
        L.hca_vq_score.argtypes = [sp, cbp, vp, vp, vp, vp, vp, vp, vp]
        L.hca_vq_export_pcache.restype = i32
        L.hca_vq_export_pcache.argtypes = [sp, cbp, vp, vp, vp, vp]
        L.hca_vq_evict.restype = i32
        L.hca_vq_evict.argtypes = [sp, cbp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp]
        L.hca_vq_attend_gathered.restype = i32
        L.hca_vq_attend_gathered.argtypes = [sp, cbp, vp, vp, vp, vp, i32, f32, vp, vp, vp, vp]
        _lib = L
    return _lib


def make_shape(batch, n_q_heads, n_kv_heads, capacity, bits=4, group=32, head_dim=128):
    return hca_shape(batch, n_q_heads, n_kv_heads, head_dim, bits, group, capacity)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(s):
    if s is None:
        s = torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _nres(n_resident, batch):
    arr = (C.c_int64 * batch)(*[int(x) for x in n_resident])
    return arr


def _check(rc, what):
    if rc != HCA_OK:
        raise HcaError(what, rc, lib().hca_last_hip_error())


def hca_version():
    return lib().hca_version().decode()


def hca_tune(name, value):
    _check(lib().hca_tune(name.encode(), int(value)), "hca_tune")


def hca_kcache_bytes(shape):
    return int(lib().hca_kcache_bytes(C.byref(shape)))


def hca_workspace_bytes(shape, k_max, m_max):
    return int(lib().hca_workspace_bytes(C.byref(shape), int(k_max), int(m_max)))


def hca_quantize_keys(shape, kcache, k_new_f16, T, n_resident, acc_opt=None, pos_opt=None, value_row0=None,
                      stream=None):
    nr = _nres(n_resident, shape.batch)
    vr = None if value_row0 is None else _nres(value_row0, shape.batch)
    _check(lib().hca_quantize_keys(C.byref(shape), _ptr(kcache), _ptr(k_new_f16), int(T), nr, _ptr(acc_opt),
                                   _ptr(pos_opt), vr, _stream(stream)), "hca_quantize_keys")


def hca_score_qkeys(shape, kcache, q_f16, n_resident, sel, z_opt=None, workspace=None, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_score_qkeys(C.byref(shape), _ptr(kcache), _ptr(q_f16), nr, _ptr(sel), _ptr(z_opt),
                                 _ptr(workspace), _stream(stream)), "hca_score_qkeys")


def hca_score_topk(shape, kcache, q_f16, n_resident, k, idx, count, workspace, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_score_topk(C.byref(shape), _ptr(kcache), _ptr(q_f16), nr, int(k), _ptr(idx), _ptr(count),
                                _ptr(workspace), _stream(stream)), "hca_score_topk")


def hca_score_topk_report(shape, n_resident, workspace, candidates, rescanned, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_score_topk_report(C.byref(shape), nr, _ptr(workspace), _ptr(candidates), _ptr(rescanned),
                                       _stream(stream)), "hca_score_topk_report")


def hca_score_topk_monitor(shape, workspace, out=None, reset=False, stream=None):
    _check(lib().hca_score_topk_monitor(C.byref(shape), _ptr(workspace), _ptr(out) if out is not None else None,
                                        1 if reset else 0, _stream(stream)), "hca_score_topk_monitor")


def hca_topk(shape, sel, n_resident, k, idx, count, workspace, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_topk(C.byref(shape), _ptr(sel), nr, int(k), _ptr(idx), _ptr(count), _ptr(workspace),
                          _stream(stream)), "hca_topk")


def hca_topk_noalloc(shape, sel, n_resident, k, idx, count, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_topk_noalloc(C.byref(shape), _ptr(sel), nr, int(k), _ptr(idx), _ptr(count), _stream(stream)),
           "hca_topk_noalloc")


def hca_sparse_attend(shape, kcache, q_f16, idx, count, k, pos, v_host, host_stride, n_host_rows, v_hbm,
                      hbm_stride, sm_scale, y, acc_opt, workspace, gather_stream=None, stream=None):
    st = _stream(stream)
    gst = st if gather_stream is None else _stream(gather_stream)
    _check(lib().hca_sparse_attend(C.byref(shape), _ptr(kcache), _ptr(q_f16), _ptr(idx), _ptr(count), int(k),
                                   _ptr(pos), _ptr(v_host), int(host_stride), int(n_host_rows), _ptr(v_hbm),
                                   int(hbm_stride), float(sm_scale), _ptr(y), _ptr(acc_opt), _ptr(workspace),
                                   gst, st), "hca_sparse_attend")


def hca_gather_values(shape, idx, count, k, pos, v_host, host_stride, n_host_rows, v_hbm, hbm_stride, workspace,
                      stream=None):
    _check(lib().hca_gather_values(C.byref(shape), _ptr(idx), _ptr(count), int(k), _ptr(pos), _ptr(v_host),
                                   int(host_stride), int(n_host_rows), _ptr(v_hbm), int(hbm_stride),
                                   _ptr(workspace), _stream(stream)), "hca_gather_values")


def hca_attend_gathered(shape, kcache, q_f16, idx, count, k, sm_scale, y, acc_opt, workspace, stream=None):
    _check(lib().hca_attend_gathered(C.byref(shape), _ptr(kcache), _ptr(q_f16), _ptr(idx), _ptr(count), int(k),
                                     float(sm_scale), _ptr(y), _ptr(acc_opt), _ptr(workspace), _stream(stream)),
           "hca_attend_gathered")


def hca_evict(shape, kcache, acc, pos, n_resident, M, n_protect, kept_opt, workspace, kcache_dst=None, acc_dst=None,
              pos_dst=None, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_evict(C.byref(shape), _ptr(kcache), _ptr(acc), _ptr(pos), nr, int(M), int(n_protect),
                           _ptr(kept_opt), _ptr(workspace), _ptr(kcache_dst), _ptr(acc_dst), _ptr(pos_dst),
                           _stream(stream)), "hca_evict")


def hca_export_kcache(shape, kcache, n_resident, codes, scale_f16, zero_f16, stream=None):
    nr = _nres(n_resident, shape.batch)
    _check(lib().hca_export_kcache(C.byref(shape), _ptr(kcache), nr, _ptr(codes), _ptr(scale_f16),
                                   _ptr(zero_f16), _stream(stream)), "hca_export_kcache")


def hca_pipeline_create(shape, n_layers, desc, timing_slots=0):
    h = lib().hca_pipeline_create(C.byref(shape), int(n_layers), C.byref(desc), int(timing_slots))
    if not h:
        raise HcaError("hca_pipeline_create", -1)
    return h


def hca_pipeline_destroy(handle):
    lib().hca_pipeline_destroy(handle)


def hca_pipeline_step(handle, layers, n_resident, value_row0, k, host_stride, n_host_rows, hbm_stride, sm_scale,
                      evict_M=None, n_protect=0, timing_slot=-1):
    """layers: ctypes array of hca_layer; n_resident: ctypes int64 array [n_layers * batch] (both updated);
    evict_M: ctypes int64 array [n_layers] (0 = leave that layer alone) or None."""
    _check(lib().hca_pipeline_step(handle, layers, n_resident, int(value_row0), int(k), int(host_stride),
                                   int(n_host_rows), int(hbm_stride), float(sm_scale), evict_M, int(n_protect),
                                   int(timing_slot)), "hca_pipeline_step")


def hca_pipeline_scan_ms(handle, timing_slot, n_layers):
    out = (C.c_float * n_layers)()
    _check(lib().hca_pipeline_scan_ms(handle, int(timing_slot), out), "hca_pipeline_scan_ms")
    return list(out)


def hca_pipeline_host_status(handle):
    """(wait_timeouts, bad_rows) of the hybrid value side; both 0 in a correct run."""
    a, b = C.c_uint32(0), C.c_uint32(0)
    _check(lib().hca_pipeline_host_status(handle, C.byref(a), C.byref(b), None, None), "hca_pipeline_host_status")
    return int(a.value), int(b.value)


def hca_pipeline_host_times(handle):
    """(mean microseconds per layer, mean microseconds per chunk) of the hybrid value side's host threads."""
    ju, tu = C.c_double(0), C.c_double(0)
    _check(lib().hca_pipeline_host_status(handle, None, None, C.byref(ju), C.byref(tu)), "hca_pipeline_host_status")
    return float(ju.value), float(tu.value)


def hca_host_prefault(t, n_threads=16):
    """Walks a pinned tensor once on the CPU so that later random reads of it do not page-fault."""
    _check(lib().hca_host_prefault(_ptr(t), t.numel() * t.element_size(), int(n_threads)), "hca_host_prefault")


def hca_scan_stamp_pairs(shape, n_tokens):
    return int(lib().hca_scan_stamp_pairs(C.byref(shape), int(n_tokens)))


def hca_wall_clock_khz():
    return int(lib().hca_wall_clock_khz())


# ---- codebook form of the key path --------------------------------------------------------------

def make_codebook(groups, codewords, centroids=None):
    """centroids: device tensor fp32 [n_kv_heads, g, c, head_dim/g] (kept alive by the caller) or None."""
    return hca_vq_codebook(int(groups), int(codewords), None if centroids is None else centroids.data_ptr())


def hca_vq_pcache_bytes(shape, cb):
    return int(lib().hca_vq_pcache_bytes(C.byref(shape), C.byref(cb)))


def hca_vq_workspace_bytes(shape, cb, k_max, m_max=1):
    return int(lib().hca_vq_workspace_bytes(C.byref(shape), C.byref(cb), int(k_max), int(m_max)))


def hca_vq_lut_bytes(shape, cb):
    return int(lib().hca_vq_lut_bytes(C.byref(shape), C.byref(cb)))


def hca_vq_train(kval, groups, codewords, init, iters, shared=False):
    """kval: host fp16 array-like [n_val, head_dim] (numpy or CPU tensor); init: int32 [g, c] or [c].
    Returns (centroids fp32 numpy [g, c, head_dim/g], inertia float64 numpy [iters+1])."""
    import numpy as np
    kval = np.ascontiguousarray(kval.numpy() if hasattr(kval, "numpy") else kval)
    assert kval.dtype == np.float16 and kval.ndim == 2
    n_val, D = kval.shape
    init = np.ascontiguousarray(init, np.int32)
    assert init.shape == ((codewords,) if shared else (groups, codewords))
    cen = np.zeros((groups, codewords, D // groups), np.float32)
    inertia = np.zeros(iters + 1, np.float64)
    _check(lib().hca_vq_train(kval.ctypes.data_as(C.c_void_p), n_val, D, int(groups), int(codewords),
                              init.ctypes.data_as(C.c_void_p), int(iters), 1 if shared else 0,
                              cen.ctypes.data_as(C.c_void_p), inertia.ctypes.data_as(C.c_void_p)), "hca_vq_train")
    return cen, inertia


def hca_vq_assign(shape, cb, pcache, k_new, T, n_resident, acc=None, pos=None, value_row0=None, stream=None):
    _check(lib().hca_vq_assign(C.byref(shape), C.byref(cb), _ptr(pcache), _ptr(k_new), int(T),
                               _nres(n_resident, shape.batch), _ptr(acc), _ptr(pos),
                               None if value_row0 is None else _nres(value_row0, shape.batch), _stream(stream)),
           "hca_vq_assign")


def hca_vq_score(shape, cb, pcache, q, n_resident, lut, sel, z=None, stream=None):
    _check(lib().hca_vq_score(C.byref(shape), C.byref(cb), _ptr(pcache), _ptr(q), _nres(n_resident, shape.batch),
                              _ptr(lut), _ptr(sel), _ptr(z), _stream(stream)), "hca_vq_score")


def hca_vq_export_pcache(shape, cb, pcache, n_resident, indices, stream=None):
    _check(lib().hca_vq_export_pcache(C.byref(shape), C.byref(cb), _ptr(pcache), _nres(n_resident, shape.batch),
                                      _ptr(indices), _stream(stream)), "hca_vq_export_pcache")


def hca_vq_attend_gathered(shape, cb, pcache, lut, idx, count, k, sm_scale, y, acc, workspace, stream=None):
    _check(lib().hca_vq_attend_gathered(C.byref(shape), C.byref(cb), _ptr(pcache), _ptr(lut), _ptr(idx), _ptr(count),
                                        int(k), float(sm_scale), _ptr(y), _ptr(acc), _ptr(workspace), _stream(stream)),
           "hca_vq_attend_gathered")


def hca_vq_evict(shape, cb, pcache, acc, pos, n_resident, M, n_protect, kept, workspace, pcache_dst=None, acc_dst=None,
                 pos_dst=None, stream=None):
    _check(lib().hca_vq_evict(C.byref(shape), C.byref(cb), _ptr(pcache), _ptr(acc), _ptr(pos),
                              _nres(n_resident, shape.batch), int(M), int(n_protect), _ptr(kept), _ptr(workspace),
                              _ptr(pcache_dst), _ptr(acc_dst), _ptr(pos_dst), _stream(stream)), "hca_vq_evict")


def hca_topp(shape, sel, n_resident, sm_scale, tau, k_max, idx, count, mass=None, workspace=None, stream=None):
    _check(lib().hca_topp(C.byref(shape), _ptr(sel), _nres(n_resident, shape.batch), float(sm_scale), float(tau),
                          int(k_max), _ptr(idx), _ptr(count), _ptr(mass), _ptr(workspace), _stream(stream)), "hca_topp")


def hca_score_qkeys_lse(shape, kcache, q_f16, n_resident, sm_scale, sel, lse, workspace, stream=None):
    _check(lib().hca_score_qkeys_lse(C.byref(shape), _ptr(kcache), _ptr(q_f16), _nres(n_resident, shape.batch),
                                     float(sm_scale), _ptr(sel), _ptr(lse), _ptr(workspace), _stream(stream)),
           "hca_score_qkeys_lse")


def hca_attend_gathered_global(shape, kcache, q_f16, idx, count, k, sm_scale, lse, y, acc, workspace, stream=None):
    _check(lib().hca_attend_gathered_global(C.byref(shape), _ptr(kcache), _ptr(q_f16), _ptr(idx), _ptr(count), int(k),
                                            float(sm_scale), _ptr(lse), _ptr(y), _ptr(acc), _ptr(workspace),
                                            _stream(stream)), "hca_attend_gathered_global")


def hca_attend_weights(shape, kcache, q_f16, idx, count, k, pos, sm_scale, lse, w_f16, vrow, acc, workspace, stream=None):
    _check(lib().hca_attend_weights(C.byref(shape), _ptr(kcache), _ptr(q_f16), _ptr(idx), _ptr(count), int(k), _ptr(pos),
                                    float(sm_scale), _ptr(lse), _ptr(w_f16), _ptr(vrow), _ptr(acc), _ptr(workspace),
                                    _stream(stream)), "hca_attend_weights")


def hca_host_weighted_sum(shape, vrow, count, k, w_f16, v_host, host_stride, y, n_threads=16):
    """All tensors are CPU tensors (pinned or not); blocks until y is written."""
    _check(lib().hca_host_weighted_sum(C.byref(shape), _ptr(vrow), _ptr(count), int(k), _ptr(w_f16), _ptr(v_host),
                                       int(host_stride), _ptr(y), int(n_threads)), "hca_host_weighted_sum")
