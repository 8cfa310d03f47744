"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes follow the layout, and invalid arguments are rejected before any device work."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2507_19823_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    binding.lib()
    return binding


def test_every_declared_symbol_is_exported(B):
    hdr = open(os.path.join(ROOT, "include", "hca.h")).read()
    names = set(re.findall(r"\b(hca_[a-z_]+)\s*\(", hdr))
    assert {"hca_quantize_keys", "hca_score_qkeys", "hca_topk", "hca_sparse_attend", "hca_evict"} <= names
    for n in names:
        assert hasattr(B.lib(), n), n
    assert B.hca_version().startswith("hca")


def test_cache_bytes_follow_the_layout(B):
    # 4-bit / group 32: 64 B codes + 16 B scale/zero per token and KV head; blocks of 16 tokens
    s = B.make_shape(1, 32, 8, 1 << 20)
    assert B.hca_kcache_bytes(s) == 8 * (1 << 20) * 80
    # 2-bit / group 64: 32 + 8 B; blocks of 32 tokens; capacity rounded up to a block
    s = B.make_shape(2, 8, 2, 33, bits=2, group=64)
    assert B.hca_kcache_bytes(s) == 4 * 2 * (1024 + 256)
    assert B.hca_workspace_bytes(s, 8, 8) > 0


@pytest.mark.parametrize("kw", [dict(bits=3), dict(bits=8), dict(group=64), dict(head_dim=64),
                                dict(n_q_heads=64), dict(batch=65)])
def test_unsupported_shapes(B, kw):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, capacity=1024, bits=4, group=32, head_dim=128)
    base.update(kw)
    s = B.make_shape(**base)
    assert B.hca_kcache_bytes(s) == 0
    assert B.lib().hca_score_qkeys(C.byref(s), 1, 1, (C.c_int64 * 65)(), 1, None, None, None) == -2


def test_bad_arguments_are_rejected_on_the_host(B):
    L = B.lib()
    s = B.make_shape(1, 32, 8, 1024)
    n = (C.c_int64 * 1)(100)
    one = C.c_void_p(256)      # never dereferenced: validation fails first
    assert L.hca_quantize_keys(C.byref(s), None, one, 1, n, None, None, None, None) == -1
    assert L.hca_quantize_keys(C.byref(s), one, one, 925, n, None, None, None, None) == -3          # 100 + 925 > 1024
    assert L.hca_quantize_keys(C.byref(s), one, one, -1, n, None, None, None, None) == -1
    assert L.hca_quantize_keys(C.byref(s), one, one, 1, n, None, one, None, None) == -1   # pos without value_row0
    assert L.hca_score_qkeys(C.byref(s), one, one, None, one, None, None, None) == -1
    assert L.hca_topk(C.byref(s), one, n, 0, one, one, one, None) == -3
    assert L.hca_topk(C.byref(s), one, n, 1025, one, one, one, None) == -3
    assert L.hca_topk(C.byref(s), one, n, 8, one, one, None, None) == -1
    assert L.hca_score_topk(C.byref(s), one, one, n, 0, one, one, one, None) == -3
    assert L.hca_score_topk(C.byref(s), one, one, n, 1025, one, one, one, None) == -3
    assert L.hca_score_topk(C.byref(s), one, None, n, 8, one, one, one, None) == -1
    assert L.hca_score_topk(C.byref(s), one, one, n, 8, one, one, None, None) == -1
    big = B.make_shape(1, 32, 8, 9 << 20)                    # more than 8 Mi resident slots in a row: refused
    nb = (C.c_int64 * 1)(9 << 20)
    assert L.hca_score_topk(C.byref(big), one, one, nb, 8, one, one, one, None) == -3
    assert L.hca_evict(C.byref(s), one, one, one, n, 0, 0, None, one, None, None, None, None) == -3
    assert L.hca_evict(C.byref(s), one, one, one, n, 10, 11, None, one, None, None, None, None) == -3
    assert L.hca_evict(C.byref(s), one, one, one, n, 200, 0, None, one, None, None, None, None) == 0   # n <= M: nothing to do
    assert L.hca_evict(C.byref(s), one, one, one, n, 50, 0, None, one, one, None, None, None) == -1  # dst without acc/pos
    assert L.hca_evict(C.byref(s), one, one, one, n, 50, 0, None, one, one, one, one, None) == -1    # dst aliases src
    bad = (C.c_int64 * 1)(2000)
    assert L.hca_score_qkeys(C.byref(s), one, one, bad, one, None, None, None) == -3
    neg = (C.c_int64 * 1)(-1)
    assert L.hca_score_qkeys(C.byref(s), one, one, neg, one, None, None, None) == -1
    assert L.hca_sparse_attend(C.byref(s), one, one, one, one, 8, one, None, 0, 0, None, 0,
                               C.c_float(1.0), one, None, one, None, None) == -1
    s2 = B.make_shape(1, 32, 7, 1024)
    assert L.hca_score_qkeys(C.byref(s2), one, one, n, one, None, None, None) == -1   # 32 % 7 != 0
    assert L.hca_score_topk_monitor(C.byref(s), None, one, 1, None) == -1             # no workspace
    assert L.hca_score_topk_monitor(C.byref(s2), one, one, 1, None) == -1
    assert L.hca_score_topk_report(C.byref(s), n, None, one, one, None) == -1
    assert L.hca_topk_noalloc(C.byref(s), None, n, 8, one, one, None) == -1
    assert L.hca_topk_noalloc(C.byref(s), one, n, 0, one, one, None) == -3


# ---- codebook form of the key path: host-side checks and the host-side trainer -------------------

def test_vq_sizes_and_unsupported_shapes(B):
    s = B.make_shape(2, 32, 8, 1000, bits=7, group=5)          # bits / group are not looked at by hca_vq_*
    cb = B.make_codebook(32, 256)
    assert B.hca_vq_pcache_bytes(s, cb) == 2 * 8 * 1000 * 32
    assert B.hca_vq_lut_bytes(s, cb) == 2 * 8 * 32 * 256 * 4 * 4 + 2 * 8 * (32 + 1) * 4 * 4   # tables + per-group maxima + grid exponents
    assert B.hca_vq_pcache_bytes(s, B.make_codebook(64, 128)) == 2 * 8 * 1000 * 64
    for g, c in ((16, 256), (32, 8193), (48, 64), (32, 0)):
        assert B.hca_vq_pcache_bytes(s, B.make_codebook(g, c)) == 0
    # wide form (16-bit indices): more than 256 centroids, or a table beyond 128 KiB of LDS (64 x 256 x 4 heads)
    # stored in whole tiles of 16 Ki slots
    assert B.hca_vq_pcache_bytes(s, B.make_codebook(32, 257)) == 2 * 8 * 16384 * 32 * 2
    assert B.hca_vq_pcache_bytes(s, B.make_codebook(32, 8192)) == 2 * 8 * 16384 * 32 * 2
    assert B.hca_vq_pcache_bytes(s, B.make_codebook(64, 256)) == 2 * 8 * 16384 * 64 * 2
    assert B.hca_vq_pcache_bytes(B.make_shape(1, 32, 8, 16385), B.make_codebook(32, 1024)) == 8 * 2 * 16384 * 32 * 2
    assert B.hca_vq_lut_bytes(s, B.make_codebook(32, 8192)) == 2 * 8 * 32 * 8192 * 4 * 4 + 2 * 8 * (32 + 1) * 4 * 4
    s1 = B.make_shape(1, 8, 8, 1000)                            # one query head per KV head: 64 x 256 fits in LDS
    assert B.hca_vq_pcache_bytes(s1, B.make_codebook(64, 256)) == 8 * 1000 * 64
    # workspace of the hca_vq_* calls: that of the 4-bit uniform path, whatever the shape's bits / group say
    s4 = B.make_shape(2, 32, 8, 1000)
    assert B.hca_vq_workspace_bytes(s, cb, 64, 500) == B.hca_workspace_bytes(s4, 64, 500) > 0


def test_vq_bad_arguments_are_rejected_on_the_host(B):
    L = B.lib()
    s = B.make_shape(1, 32, 8, 1024)
    one = C.c_void_p(256)
    n = (C.c_int64 * 1)(1000)
    cb = B.hca_vq_codebook(32, 256, 256)
    nocb = B.hca_vq_codebook(32, 256, None)
    assert L.hca_vq_assign(C.byref(s), C.byref(nocb), one, one, 1, n, None, None, None, None) == -1
    assert L.hca_vq_assign(C.byref(s), C.byref(cb), None, one, 1, n, None, None, None, None) == -1
    assert L.hca_vq_assign(C.byref(s), C.byref(cb), one, one, 25, n, None, None, None, None) == -3
    assert L.hca_vq_score(C.byref(s), C.byref(cb), one, one, n, None, one, None, None) == -1
    assert L.hca_vq_score(C.byref(s), C.byref(B.hca_vq_codebook(48, 256, 256)), one, one, n, one, one, None, None) == -2
    assert L.hca_vq_attend_gathered(C.byref(s), C.byref(cb), one, one, one, one, 0, 1.0, one, None, one, None) == -3
    assert L.hca_vq_export_pcache(C.byref(s), C.byref(cb), one, n, None, None) == -1
    assert L.hca_vq_train(None, 10, 128, 32, 4, one, 1, 0, one, None) == -1
    assert L.hca_vq_train(one, 10, 128, 48, 4, one, 1, 0, one, None) == -1


@pytest.mark.parametrize("g,c,shared", [(32, 64, False), (64, 16, False), (32, 24, True)])
def test_vq_trainer_matches_the_oracle(B, g, c, shared):
    """The library's host-side k-means and the oracle's follow the same definition in the same order,
    so codebooks and objective values must be identical."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(g + c)
    nval = 1200
    kval = rng.standard_normal((nval, 128)).astype(np.float16)
    init = (rng.choice(nval * g, c, replace=False) if shared else
            np.stack([rng.choice(nval, c, replace=False) for _ in range(g)])).astype(np.int32)
    cen, iner = B.hca_vq_train(kval, g, c, init, 5, shared)
    ocen, oiner = oracle.vq_train(kval, g, c, init, 5, shared)
    assert np.array_equal(cen, ocen)
    assert np.allclose(iner, oiner, rtol=1e-12)
    bad = init.copy()
    bad.flat[0] = nval * g + 7
    with pytest.raises(B.HcaError):
        B.hca_vq_train(kval, g, c, bad, 1, shared)


def test_tune_accepts_known_knobs_only(B):
    for name in ("gather_wgs", "gather_unroll", "score_bpw", "score_depth"):
        B.hca_tune(name, 0)
    B.hca_tune("gather_unroll", 4)                 # back to the defaults
    assert B.lib().hca_tune(b"no_such_knob", 1) == -1
    assert B.lib().hca_tune(None, 1) == -1


def test_tune_refuses_values_the_kernels_buffers_are_not_sized_for(B):
    """Fewer than 4 code blocks per wave would give a scan launch more waves than the per-wave stamp and
    partial-sum buffers hold; every knob has a closed range."""
    L = B.lib()
    for name, bad in ((b"score_bpw", (1, 2, 3, 33, -1)), (b"score_depth", (1, 2, 3, 16, -4)),
                      (b"gather_wgs", (-1, 1025)), (b"gather_unroll", (-1, 5))):
        for v in bad:
            assert L.hca_tune(name, v) == -1, (name, v)
    for name, good in ((b"score_bpw", (4, 16, 32, 0)), (b"score_depth", (4, 8, 0)), (b"gather_wgs", (1, 1024, 0)),
                       (b"gather_unroll", (1, 2, 4))):
        for v in good:
            assert L.hca_tune(name, v) == 0, (name, v)


@pytest.mark.parametrize("bits,group,tpb", [(4, 32, 16), (2, 64, 32)])
def test_scan_stamp_pairs_cover_every_accepted_launch_shape(B, bits, group, tpb):
    """One (start, end) pair per wave: 4 waves per workgroup, ceil(blocks / (4 * blocks per wave)) workgroups per
    row, for every blocks-per-wave value hca_tune accepts."""
    for batch, n in ((1, 1), (1, 4097), (4, 131072 + 64), (1, (1 << 20) + 1), (2, 12345)):
        s = B.make_shape(batch, 32, 8, n, bits, group)
        pairs = B.lib().hca_scan_stamp_pairs(C.byref(s), n)
        nblocks = -(-n // tpb)
        for bpw in range(4, 33):
            waves = -(-nblocks // (4 * bpw)) * 4 * batch * 8
            assert waves <= pairs, (batch, n, bpw)


def test_topp_and_global_weight_arguments(B):
    L = B.lib()
    s = B.make_shape(1, 32, 8, 1024)
    n = (C.c_int64 * 1)(100)
    one = C.c_void_p(256)
    assert L.hca_topp(C.byref(s), one, n, 0.1, C.c_double(0.0), 8, one, one, None, one, None) == -1      # tau must be > 0
    assert L.hca_topp(C.byref(s), one, n, 0.0, C.c_double(0.5), 8, one, one, None, one, None) == -1      # sm_scale > 0
    assert L.hca_topp(C.byref(s), one, n, 0.1, C.c_double(0.5), 0, one, one, None, one, None) == -3
    assert L.hca_topp(C.byref(s), one, n, 0.1, C.c_double(0.5), 2000, one, one, None, one, None) == -3   # k_max > capacity
    assert L.hca_topp(C.byref(s), None, n, 0.1, C.c_double(0.5), 8, one, one, None, one, None) == -1
    assert L.hca_score_qkeys_lse(C.byref(s), one, one, n, 0.1, one, None, one, None) == -1
    assert L.hca_score_qkeys_lse(C.byref(s), one, one, n, 0.1, one, one, None, None) == -1               # needs a workspace
    assert L.hca_attend_gathered_global(C.byref(s), one, one, one, one, 8, 0.1, None, one, None, one, None) == -1


def test_host_weighted_sum_matches_numpy(B):
    """The host half of the paper's CPU-GPU split runs without a GPU: weights (fp16) times value rows."""
    import numpy as np
    import torch
    import oracle
    rng = np.random.default_rng(3)
    batch, hkv, G, k, vrows = 2, 3, 4, 300, 900
    R = batch * hkv
    shape = B.make_shape(batch, hkv * G, hkv, 1000)
    V = rng.standard_normal((R, vrows, 128)).astype(np.float16)
    count = rng.integers(0, k + 1, R).astype(np.int32)
    count[0], count[1] = 0, k
    idx = np.stack([np.sort(rng.choice(1000, k, replace=False)) for _ in range(R)]).astype(np.int32)
    pos = np.stack([rng.permutation(1000) % vrows for _ in range(R)]).astype(np.int32)
    w = rng.random((R * G, k)).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    vrow = np.full((R, k), -1, np.int32)
    w16 = np.zeros((R * G, k), np.float16)
    for r in range(R):
        vrow[r, :count[r]] = pos[r, idx[r, :count[r]]]
        w16[r * G:(r + 1) * G, :count[r]] = w[r * G:(r + 1) * G, :count[r]].astype(np.float16)
    ref = oracle.weighted_sum_f16(w, idx, count, pos, V)
    for nt in (1, 5, 16):
        y = torch.zeros(R * G, 128)
        B.hca_host_weighted_sum(shape, torch.from_numpy(vrow), torch.from_numpy(count), k, torch.from_numpy(w16),
                                torch.from_numpy(V), vrows, y, nt)
        assert np.allclose(y.numpy(), ref, rtol=1e-4, atol=1e-5)
    # the worker threads are kept between calls and serve one call at a time: callers on two threads,
    # with different thread counts, both get the full sum every time
    import threading
    wrong = []

    def caller(nt):
        yy = torch.zeros(R * G, 128)
        for _ in range(25):
            yy.zero_()
            B.hca_host_weighted_sum(shape, torch.from_numpy(vrow), torch.from_numpy(count), k,
                                    torch.from_numpy(w16), torch.from_numpy(V), vrows, yy, nt)
            if not np.allclose(yy.numpy(), ref, rtol=1e-4, atol=1e-5):
                wrong.append(nt)
    th = [threading.Thread(target=caller, args=(nt,)) for nt in (3, 8)]
    for t in th:
        t.start()
    for t in th:
        t.join()
    assert not wrong
    # a forked child has none of the parent's worker threads and must start its own
    # (every tensor is made before the fork: the child only calls the library and compares)
    yy = torch.zeros(R * G, 128)
    yy_np = yy.numpy()
    args = (shape, torch.from_numpy(vrow), torch.from_numpy(count), k, torch.from_numpy(w16), torch.from_numpy(V),
            vrows, yy, 4)
    pid = os.fork()
    if pid == 0:
        code = 1
        try:
            B.hca_host_weighted_sum(*args)
            code = 0 if np.allclose(yy_np, ref, rtol=1e-4, atol=1e-5) else 2
        finally:
            os._exit(code)
    import time
    t_end = time.time() + 30
    status = None
    while time.time() < t_end:
        done, st = os.waitpid(pid, os.WNOHANG)
        if done == pid:
            status = st
            break
        time.sleep(0.02)
    if status is None:
        os.kill(pid, 9)
        os.waitpid(pid, 0)
        pytest.fail("the forked child did not finish its host sum")
    assert os.WIFEXITED(status) and os.WEXITSTATUS(status) == 0
    bad = vrow.copy()
    bad[1, 0] = vrows
    with pytest.raises(B.HcaError):
        B.hca_host_weighted_sum(shape, torch.from_numpy(bad), torch.from_numpy(count), k, torch.from_numpy(w16),
                                torch.from_numpy(V), vrows, torch.zeros(R * G, 128), 2)


def _c_program(name):
    import importlib.util
    path = os.path.join(ROOT, "tests", "c", "bin", name)
    if not os.path.exists(path):
        spec = importlib.util.spec_from_file_location("c_boundary_build", os.path.join(ROOT, "tests", "c", "build.py"))
        cb = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(cb)
        cb.build()
    return path


def test_header_and_library_from_plain_c(B):
    """tests/c/abi_from_c.c: include/hca.h compiles as C11 with gcc -pedantic -Werror (no HIP, no C++), links
    against libhca.so, and the host-side checks and the host-side trainer run without a GPU."""
    import subprocess
    r = subprocess.run([_c_program("abi_from_c")], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi ok" in r.stdout


def test_host_prefault_walks_any_range(B):
    import numpy as np
    L = B.lib()
    a = np.ones(3 * 4096 + 17, np.uint8)
    for threads in (1, 3, 64, 1000):
        assert L.hca_host_prefault(C.c_void_p(a.ctypes.data), a.nbytes, threads) == 0
    assert L.hca_host_prefault(None, 0, 4) == 0
    assert L.hca_host_prefault(None, 10, 4) == -1


@pytest.mark.parametrize("isa", [0, 2])
@pytest.mark.parametrize("gqa", [1, 2, 4])
def test_host_chunk_sum_against_numpy(B, gqa, isa):
    """One chunk of the hybrid value side's host work against a float64 matrix product; entries marked -1 are left
    out, rows beyond the store are skipped and counted.  isa 0: the widest vector form this CPU has; 2: AVX2."""
    import numpy as np
    L = B.lib()
    B.hca_tune("host_isa", isa)
    rng = np.random.default_rng(gqa)
    n_rows = 5000
    V = rng.standard_normal((n_rows, 128)).astype(np.float16)
    p = np.zeros((4, 256), np.float32)
    p[:gqa] = rng.random((gqa, 256)).astype(np.float32) * np.exp2(rng.integers(-40, 1, (gqa, 256))).astype(np.float32)
    vrow = rng.integers(0, n_rows, 256).astype(np.int32)
    vrow[5::17] = -1
    vrow[200:] = -1                                   # a ragged chunk
    py = np.full((4, 128), 7.0, np.float32)
    assert L.hca_debug_host_chunk_sum(gqa, p.ctypes.data, vrow.ctypes.data, V.ctypes.data, n_rows, py.ctypes.data) == 0
    live = vrow >= 0
    ref = p[:, live].astype(np.float64) @ V[vrow[live]].astype(np.float64)
    assert np.allclose(py[:gqa], ref[:gqa], rtol=1e-5, atol=1e-6)
    assert np.all(py[gqa:] == 0)
    vrow[3] = n_rows + 5                              # outside the store: skipped, reported
    assert L.hca_debug_host_chunk_sum(gqa, p.ctypes.data, vrow.ctypes.data, V.ctypes.data, n_rows, py.ctypes.data) == 1
    live = (vrow >= 0) & (vrow < n_rows)
    ref = p[:, live].astype(np.float64) @ V[vrow[live]].astype(np.float64)
    assert np.allclose(py[:gqa], ref[:gqa], rtol=1e-5, atol=1e-6)
    assert L.hca_debug_host_chunk_sum(5, p.ctypes.data, vrow.ctypes.data, V.ctypes.data, n_rows, py.ctypes.data) == -1
    B.hca_tune("host_isa", 0)
