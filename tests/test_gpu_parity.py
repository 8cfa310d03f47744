"""GPU parity: every stage of the HIP path against the CPU oracle on the same seeded inputs.
Integer results (codes, scale/zero bits, scores as produced by exact integer dots, index sets,
eviction decisions) must match bit for bit; the attention output within 2e-3 max relative error."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as S

pytestmark = pytest.mark.gpu

TOL = 2e-3   # max_c |y_gpu - y_oracle| / max_c |y_oracle| per head (spec tolerance)


@pytest.fixture(scope="module")
def H():
    import paper_2507_19823_amd as H
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    H.lib()
    return H


def _state(H, w, cap=None, want_z=True, k_max=None, m_max=None):
    from paper_2507_19823_amd.session import LayerState
    cap = cap or w.n
    return LayerState(w.batch, w.n_q_heads, w.n_kv_heads, cap, w.bits, w.group, k_max=k_max or w.k,
                      m_max=m_max, want_z=want_z)


def _rows(t):
    """[B, H, ...] torch tensor -> numpy [B*H, ...]"""
    a = t.detach().cpu().numpy()
    return a.reshape(a.shape[0] * a.shape[1], *a.shape[2:])


def _ocache(oracle, w, cap):
    return oracle.Cache(w.batch * w.n_kv_heads, cap, 128, w.bits, w.group)


def _cmp_cache(st, oc):
    codes, scale, zero = st.export()
    torch.cuda.synchronize()
    for r in range(oc.R):
        n = int(oc.n[r])
        assert st.n[r // st.hkv] == n
        assert np.array_equal(_rows(codes)[r, :n], oc.codes[r, :n]), f"codes differ in row {r}"
        assert np.array_equal(_rows(scale).view(np.uint16)[r, :n], oc.scale[r, :n]), f"scales differ in row {r}"
        assert np.array_equal(_rows(zero).view(np.uint16)[r, :n], oc.zero[r, :n]), f"zeros differ in row {r}"


def _rel_err(y, ref):
    return float(np.max(np.abs(y - ref).max(-1) / np.maximum(np.abs(ref).max(-1), 1e-30)))


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64)])
def test_quantize_bit_exact_with_ragged_appends(H, oracle, bits, gs):
    w = S.Workload("q", 50 + bits, 2, 8, 2, 1200, bits, gs, 64)
    d = S.make_layer(w, want_values=False)
    keys = d["keys"]
    # special groups: constant, signed-zero minimum, huge range, subnormal step
    keys[0, 0, 3, :] = 0.75
    keys[0, 0, 4, :64] = 0.0
    keys[0, 0, 4, 0] = -0.0
    keys[0, 1, 5, 0] = 65504.0
    keys[0, 1, 5, 1] = -65504.0
    keys[1, 0, 6, :] = 0.0
    keys[1, 0, 6, 7] = 6e-8
    # tiny ranges: the fp16 scale is subnormal and badly rounded, so unclamped codes would exceed qmax
    rs = np.random.default_rng(9)
    for t in range(20, 60):
        step = rs.integers(1, 40)
        tiny = (rs.integers(0, step + 1, 128) * 2.0 ** -24 * rs.choice([1, 3, 7])).astype(np.float16)
        keys[1, 1, t] = torch.from_numpy(tiny * rs.choice([-1.0, 1.0]).astype(np.float16))
    for t in range(60, 80):                 # exact .5 ties before rounding: codes must round to even
        base = rs.standard_normal(128).astype(np.float16)
        keys[0, 1, t] = torch.from_numpy(np.round(base * 4) / 4)
    cap = 1210
    st = _state(H, w, cap=cap)
    oc = _ocache(oracle, w, cap)
    kd = keys.cuda()
    for a, b in ((0, 777), (777, 778), (778, 1000), (1000, 1200)):      # unaligned appends, T = 1 included
        st.quantize(kd[:, :, a:b].contiguous())
        oracle.quantize(oc, _rows(keys[:, :, a:b]))
    _cmp_cache(st, oc)
    with pytest.raises(H.HcaError) as e:
        st.quantize(kd[:, :, :11].contiguous())
    assert e.value.code == -3


@pytest.mark.parametrize("bits,gs,G", [(4, 32, 4), (2, 64, 4), (4, 32, 1), (4, 32, 2), (2, 64, 1)])
def test_scores_bit_exact(H, oracle, bits, gs, G):
    w = S.Workload("s", 60 + bits + G, 2, 2 * G, 2, 3000 + 7, bits, gs, 64)
    d = S.make_layer(w, want_values=False)
    st = _state(H, w)
    oc = _ocache(oracle, w, w.n)
    st.quantize(d["keys"].cuda())
    oracle.quantize(oc, _rows(d["keys"]))
    q = d["q"].clone()
    q[0, 0] = 0                       # an all-zero query head
    q[1, 1] = q[1, 1] * 1e-4          # tiny magnitudes (large fixed-point shift)
    st.score(q.cuda())
    torch.cuda.synchronize()
    sel, z = oracle.score(oc, q.numpy().reshape(-1, 128))
    zg = st.z.cpu().numpy().reshape(-1, w.n)
    assert np.array_equal(zg, z)
    assert np.array_equal(_rows(st.sel), sel)


def test_scores_different_lengths_per_sequence(H, oracle):
    w = S.Workload("s2", 71, 3, 12, 3, 900, 4, 32, 32)
    d = S.make_layer(w, want_values=False)
    st = _state(H, w)
    oc = _ocache(oracle, w, w.n)
    lens = [900, 0, 37]
    kd = d["keys"].cuda()
    # all sequences receive the same appends; n_resident then cuts each one to its own length
    st.quantize(kd)
    oracle.quantize(oc, _rows(d["keys"]))
    st.n = lens
    oc.n[...] = np.repeat(lens, 3)
    st.sel.fill_(-7.0)
    st.score(d["q"].cuda())
    st.topk(32)
    torch.cuda.synchronize()
    sel, _ = oracle.score(oc, d["q"].numpy().reshape(-1, 128), want_z=False)
    idx, count = oracle.topk(sel, oc.n, 32)
    sg = _rows(st.sel)
    for r in range(9):
        n = lens[r // 3]
        assert np.array_equal(sg[r, :n], sel[r, :n])
        assert np.all(sg[r, n:] == -7.0)                 # nothing written past n_resident
        c = int(_rows(st.count[..., None])[r, 0])
        assert c == count[r] == min(32, n)
        assert np.array_equal(_rows(st.idx)[r, :c], idx[r, :c])


@pytest.mark.parametrize("case", ["random", "all_equal", "two_valued", "signed_zero", "few_distinct", "sorted_desc"])
@pytest.mark.parametrize("n,k", [(5000, 1), (5000, 256), (5000, 4999), (5000, 5000), (70000, 2048), (1, 1), (300, 1000),
                                 ((1 << 20) + 7, 4096)])
def test_topk_bit_exact_including_ties(H, oracle, case, n, k):
    rng = np.random.default_rng(n * 7 + k)
    rows = 4
    if case == "random":
        v = rng.standard_normal((rows, n)).astype(np.float32) * 100
    elif case == "all_equal":
        v = np.full((rows, n), -3.25, np.float32)
    elif case == "two_valued":
        v = rng.integers(0, 2, (rows, n)).astype(np.float32)
    elif case == "signed_zero":
        v = np.zeros((rows, n), np.float32)
        v[:, ::3] = -0.0
        v[:, 1::7] = 1e-38
        v[:, 2::11] = -1e-38
    elif case == "few_distinct":
        v = rng.integers(-20, 20, (rows, n)).astype(np.float32) * 0.5
    else:
        v = -np.sort(-rng.standard_normal((rows, n)).astype(np.float32), axis=1)
    from paper_2507_19823_amd import binding as B
    cap = n + 5
    kk = min(k, cap)
    shape = B.make_shape(2, 8, 2, cap)
    sel = torch.full((4, cap), 1e30, dtype=torch.float32)
    sel[:, :n] = torch.from_numpy(v)
    sel = sel.cuda()
    idx = torch.full((4, kk), -9, dtype=torch.int32, device="cuda")
    count = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.hca_workspace_bytes(shape, kk, 1), dtype=torch.uint8, device="cuda")
    B.hca_topk(shape, sel, [n, n], kk, idx, count, ws)
    torch.cuda.synchronize()
    ridx, rcount = oracle.topk(sel.cpu().numpy(), np.full(4, n), kk)
    c = min(kk, n)
    assert np.all(count.cpu().numpy() == c) and np.all(rcount == c)
    assert np.array_equal(idx.cpu().numpy()[:, :c], ridx[:, :c])
    assert np.all(idx.cpu().numpy()[:, c:] == -9)          # entries past k' untouched


@pytest.mark.parametrize("cfg,host_rows", [(1, "all"), (1, "none"), (2, "half")])
def test_pipeline_configs_against_oracle(H, oracle, cfg, host_rows):
    """Workloads 1 and 2 end to end: quantise -> score -> top-k -> attend (-> evict)."""
    w = S.CONFIGS[cfg]
    d = S.make_layer(w)
    R, G, n = w.batch * w.n_kv_heads, w.gqa, w.n
    st = _state(H, w, want_z=False)
    oc = _ocache(oracle, w, n)
    st.quantize(d["keys"].cuda())
    oracle.quantize(oc, _rows(d["keys"]))
    _cmp_cache(st, oc)
    qd = d["q"].cuda()
    st.score(qd)
    st.topk(w.k)
    nh = {"all": n, "none": 0, "half": n // 2}[host_rows]
    v = d["values"]
    v_host = v[:, :, :nh].contiguous().pin_memory() if nh > 0 else None
    v_hbm = v[:, :, nh:].contiguous().cuda() if nh < n else None
    side = torch.cuda.Stream()
    st.attend(qd, v_host, nh, v_hbm, use_acc=True, gather_stream=side)
    torch.cuda.synchronize()

    q16 = d["q"].numpy().reshape(-1, 128)
    sel, _ = oracle.score(oc, q16, want_z=False)
    assert np.array_equal(_rows(st.sel), sel)
    idx, count = oracle.topk(sel, oc.n, w.k)
    assert np.array_equal(_rows(st.idx), idx)
    assert np.array_equal(st.count.cpu().numpy().reshape(-1), count)
    pos = np.tile(np.arange(n, dtype=np.int32), (R, 1))
    acc = np.zeros((R, n), np.float32)
    y, _ = oracle.attend(oc, q16, idx, count, pos, _rows(v), st.sm_scale, acc=acc)
    yg = st.y.cpu().numpy().reshape(-1, 128)
    assert _rel_err(yg, y) <= TOL
    accg = _rows(st.acc)
    assert np.allclose(accg, acc, rtol=1e-4, atol=1e-7)
    assert np.array_equal(accg > 0, acc > 0)

    if w.evict_keep:
        M = w.evict_keep
        kept = torch.full((w.batch, w.n_kv_heads, M), -1, dtype=torch.int32, device="cuda")
        # eviction decisions from the GPU's own accumulated scores vs the oracle's from its own:
        # after one step fewer than M slots were ever selected, so ties (acc == 0) decide the rest
        assert int((acc > 0).sum(1).max()) < M
        st.evict(M, 0, kept)
        torch.cuda.synchronize()
        posn = pos.copy()
        okept = oracle.evict(oc, acc, posn, M, 0)
        assert np.array_equal(_rows(kept), okept)
        _cmp_cache(st, oc)
        assert np.array_equal(_rows(st.pos)[:, :M], posn[:, :M])
        assert np.allclose(_rows(st.acc)[:, :M], acc[:, :M], rtol=1e-4, atol=1e-7)


@pytest.mark.parametrize("mode", ["inplace", "spare"])
@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64)])
@pytest.mark.parametrize("n,M,Rp", [(5000, 3000, 0), (5000, 3000, 100), (5000, 5000, 16), (4000, 5000, 16),
                                    (5000, 17, 17), (5000, 1, 0), (70001, 35000, 1)])
def test_evict_bit_exact_stagewise(H, oracle, bits, gs, n, M, Rp, mode):
    """Same accumulated scores on both sides (many ties): identical keep lists and compacted state."""
    w = S.Workload("e", 80 + bits, 2, 4, 2, n, bits, gs, 16)
    rng = np.random.default_rng(n + M + Rp)
    d = S.make_layer(w, want_values=False)
    cap = max(n, M) + 3
    st = _state(H, w, cap=cap, m_max=max(M, 1))
    oc = _ocache(oracle, w, cap)
    st.quantize(d["keys"].cuda())
    oracle.quantize(oc, _rows(d["keys"]))
    R = 4
    acc = np.zeros((R, cap), np.float32)
    acc[:, :n] = rng.integers(0, 5, (R, n)).astype(np.float32) * 0.125
    acc[1, :n] = rng.random(n).astype(np.float32)
    acc[2, :n] = 0.0
    pos = np.zeros((R, cap), np.int32)
    pos[:, :n] = rng.permutation(n).astype(np.int32)[None]
    st.acc.copy_(torch.from_numpy(acc.reshape(2, 2, cap)))
    st.pos.copy_(torch.from_numpy(pos.reshape(2, 2, cap)))
    kept = torch.full((2, 2, M), -5, dtype=torch.int32, device="cuda")
    if mode == "spare":
        spare = (torch.full_like(st.kcache, 0xAB), torch.full_like(st.acc, -1.0), torch.full_like(st.pos, -1))
        old = st.evict(M, Rp, kept, spare=spare)
        assert old is not None and st.kcache is spare[0]
    else:
        st.evict(M, Rp, kept)
    torch.cuda.synchronize()
    okept = oracle.evict(oc, acc, pos, M, Rp)
    m = min(n, M)
    if n > M:
        assert np.array_equal(_rows(kept), okept)
    else:
        assert np.all(_rows(kept) == -5)                   # rows left alone are not reported
    _cmp_cache(st, oc)
    assert np.array_equal(_rows(st.acc)[:, :m], acc[:, :m])
    assert np.array_equal(_rows(st.pos)[:, :m], pos[:, :m])


@pytest.mark.parametrize("with_list", [True, False])
@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64)])
@pytest.mark.parametrize("n,M,Rp", [(13000, 12000, 16), (13000, 12990, 16), (9000, 4100, 0),
                                    # first dropped slot on a chunk edge of the ordered pass (8192) and just before it
                                    (8300, 8208, 16), (8300, 8207, 16)])
def test_evict_when_the_threshold_is_zero(H, oracle, bits, gs, n, M, Rp, with_list):
    """Rows whose accumulated scores are mostly exact zeros, as in a long context, with the number of positive
    entries just below, at and just above the number of slots to keep from the unprotected part (the cases on
    both sides of the point where the M-th largest score becomes 0), a row with -0.0 among the zeros and negative
    entries, a row with too few non-negative entries, and the positive entries either spread out or packed at the
    front (so that whole chunks keep every slot): keep lists (when asked for) and compacted state against the
    oracle, in place, with and without a caller's keep list."""
    w = S.Workload("ez", 90 + bits, 2, 4, 2, n, bits, gs, 16)
    want = M - Rp
    nsel = n - Rp
    for variant in range(2):
        rng = np.random.default_rng(1000 * variant + n + M)
        d = S.make_layer(w, want_values=False)
        cap = n + 5
        st = _state(H, w, cap=cap, m_max=M)
        oc = _ocache(oracle, w, cap)
        st.quantize(d["keys"].cuda())
        oracle.quantize(oc, _rows(d["keys"]))
        R = 4
        acc = np.zeros((R, cap), np.float32)
        counts = [want - 1, want, want + 1, 7] if variant == 0 else [want - 1, 0, min(want + 300, nsel), want // 2]
        for r, c in enumerate(counts):
            c = max(0, min(c, nsel))
            where = rng.permutation(nsel)[:c] if (r + variant) % 2 == 0 else np.arange(c)
            acc[r, where] = (rng.integers(1, 4, c) * 0.25).astype(np.float32)
        if variant == 1:
            z = rng.permutation(nsel)[:nsel // 3]
            acc[3, z] = np.where(acc[3, z] == 0, np.float32(-0.0), acc[3, z])      # -0.0 among the zeros
            neg = rng.permutation(nsel)[:50]
            acc[3, neg] = -1.5                                                     # below every zero
            neg = rng.permutation(nsel)[:nsel - want + 40]
            acc[1, :nsel] = 0.0
            acc[1, neg] = -rng.random(neg.size).astype(np.float32) - 0.5           # fewer than `want` entries >= 0
        acc[:, nsel:n] = 0.125
        pos = np.zeros((R, cap), np.int32)
        pos[:, :n] = rng.permutation(n).astype(np.int32)[None]
        st.acc.copy_(torch.from_numpy(acc.reshape(2, 2, cap)))
        st.pos.copy_(torch.from_numpy(pos.reshape(2, 2, cap)))
        kept = torch.full((2, 2, M), -5, dtype=torch.int32, device="cuda") if with_list else None
        st.evict(M, Rp, kept)
        torch.cuda.synchronize()
        okept = oracle.evict(oc, acc, pos, M, Rp)
        if with_list:
            assert np.array_equal(_rows(kept), okept), f"variant {variant}"
        _cmp_cache(st, oc)
        assert np.array_equal(_rows(st.acc)[:, :M].view(np.uint32), acc[:, :M].view(np.uint32)), f"variant {variant}"
        assert np.array_equal(_rows(st.pos)[:, :M], pos[:, :M]), f"variant {variant}"


def test_decode_loop_with_appends_and_eviction(H, oracle):
    """Config-3-like loop at reduced length: append one token per step, attend, evict every 4 steps;
    the GPU state is compared with the oracle after every step (stage-wise on acc)."""
    w = S.Workload("loop", 3, 2, 8, 2, 2000, 4, 32, 128, evict_keep=2000, evict_every=4, steps=12)
    d = S.make_layer(w)
    R, n0 = w.batch * w.n_kv_heads, w.n
    cap = n0 + 8
    vcap = n0 + w.steps
    st = _state(H, w, cap=cap, want_z=False)
    oc = _ocache(oracle, w, cap)
    st.quantize(d["keys"].cuda())
    oracle.quantize(oc, _rows(d["keys"]))
    v_host = torch.zeros(w.batch, w.n_kv_heads, vcap, 128, dtype=torch.float16).pin_memory()
    v_host[:, :, :n0] = d["values"]
    pos = np.zeros((R, cap), np.int32)
    pos[:, :n0] = np.arange(n0)
    acc = np.zeros((R, cap), np.float32)
    for step in range(w.steps):
        k_new, v_new, q = S.make_step(w, 0, step)
        n = st.n[0]
        v_host[:, :, n0 + step] = v_new[:, :, 0]
        st.acc[:, :, n] = 123.0                      # stale value the fused append must clear
        pos[:, n] = n0 + step
        acc[:, n] = 0
        st.quantize(k_new.cuda(), value_row0=[n0 + step] * w.batch)
        oracle.quantize(oc, _rows(k_new))
        qd = q.cuda()
        st.score(qd)
        st.topk(w.k)
        st.attend(qd, v_host, vcap, None, use_acc=True)
        torch.cuda.synchronize()
        q16 = q.numpy().reshape(-1, 128)
        sel, _ = oracle.score(oc, q16, want_z=False)
        idx, count = oracle.topk(sel, oc.n, w.k)
        assert np.array_equal(_rows(st.idx), idx), f"step {step}"
        y, _ = oracle.attend(oc, q16, idx, count, pos, _rows(v_host), st.sm_scale, acc=acc)
        assert _rel_err(st.y.cpu().numpy().reshape(-1, 128), y) <= TOL
        assert np.allclose(_rows(st.acc), acc, rtol=1e-4, atol=1e-7)
        # stage-wise: continue from identical accumulated scores so that decisions stay comparable
        st.acc.copy_(torch.from_numpy(acc.reshape(w.batch, w.n_kv_heads, cap)))
        if (step + 1) % w.evict_every == 0:
            st.evict(w.evict_keep, w.evict_every)
            torch.cuda.synchronize()
            oracle.evict(oc, acc, pos, w.evict_keep, w.evict_every)
            assert st.n[0] == w.evict_keep == oc.n[0]
            _cmp_cache(st, oc)
            m = w.evict_keep
            assert np.array_equal(_rows(st.pos)[:, :m], pos[:, :m])
            assert np.array_equal(_rows(st.acc)[:, :m], acc[:, :m])


def test_empty_cache_and_tiny_k(H, oracle):
    w = S.Workload("z", 9, 1, 4, 1, 40, 4, 32, 8, planted=4)
    d = S.make_layer(w)
    st = _state(H, w, cap=64)
    qd = d["q"].cuda()
    vh = torch.zeros(1, 1, 64, 128, dtype=torch.float16).pin_memory()
    st.score(qd)                      # n = 0: nothing to do
    st.topk(8)
    st.attend(qd, vh, 64, None)
    torch.cuda.synchronize()
    assert int(st.count.sum()) == 0 and float(st.y.abs().sum()) == 0.0
    st.quantize(d["keys"][:, :, :3].cuda())     # n = 3 < k
    oc = _ocache(oracle, w, 64)
    oracle.quantize(oc, _rows(d["keys"][:, :, :3]))
    vh[:, :, :3] = d["values"][:, :, :3]
    st.score(qd)
    st.topk(8)
    st.attend(qd, vh, 64, None)
    torch.cuda.synchronize()
    assert st.count.cpu().tolist() == [[3]]
    assert st.idx.cpu().numpy().reshape(-1)[:3].tolist() == [0, 1, 2]
    q16 = d["q"].numpy().reshape(-1, 128)
    sel, _ = oracle.score(oc, q16, want_z=False)
    idx, count = oracle.topk(sel, oc.n, 8)
    y, _ = oracle.attend(oc, q16, idx, count, np.arange(64, dtype=np.int32)[None], _rows(vh), st.sm_scale)
    assert _rel_err(st.y.cpu().numpy().reshape(-1, 128), y) <= TOL


def test_kernels_are_deterministic(H):
    w = S.CONFIGS[1]
    d = S.make_layer(w)
    outs = []
    for _ in range(2):
        st = _state(H, w, want_z=True)
        st.quantize(d["keys"].cuda())
        st.score(d["q"].cuda())
        st.topk(w.k)
        st.attend(d["q"].cuda(), None, 0, d["values"].cuda())
        torch.cuda.synchronize()
        outs.append((st.kcache.cpu(), st.z.cpu(), st.idx.cpu().clone(), st.y.cpu()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("Lr,n_sel,spare,tau,fused,host", [
    (3, 3, True, 0.0, False, 0), (5, 3, True, 0.0, False, 0), (5, 5, True, 0.0, False, 0), (5, 5, False, 0.0, False, 0),
    (3, 3, False, 0.0, False, 0), (4, 4, False, 0.9, False, 0), (3, 3, True, 0.95, False, 0),
    (5, 3, True, 0.0, True, 0), (5, 5, False, 0.0, True, 0), (1, 3, False, 0.0, True, 0), (4, 4, True, 0.0, True, 0),
    # hybrid value side: the first `host` chunks of 256 selected tokens are summed by the driver's host threads
    (5, 5, False, 0.0, True, 1), (3, 3, True, 0.0, False, 2), (5, 3, False, 0.9, False, 1), (6, 6, False, 0.0, True, 3)])
def test_native_step_driver_matches_oracle(H, oracle, Lr, n_sel, spare, tau, fused, host):
    _step_driver_case(oracle, Lr, n_sel, spare, tau, fused, host, 4, 32)


@pytest.mark.parametrize("Lr,n_sel,spare,tau,fused,host", [
    (5, 5, False, 0.0, True, 1), (6, 6, False, 0.0, True, 3), (5, 3, True, 0.0, True, 0), (3, 3, True, 0.0, False, 2),
    (4, 4, False, 0.9, False, 0)])
def test_native_step_driver_with_two_bit_codes(H, oracle, Lr, n_sel, spare, tau, fused, host):
    """The same cases on 2-bit / group-64 codes (32-token blocks, two tiles per block): paired and single scan
    launches, the hybrid value side, both eviction forms."""
    _step_driver_case(oracle, Lr, n_sel, spare, tau, fused, host, 2, 64)


@pytest.mark.parametrize("Lr,n_sel,spare,fused,host,bits,gs", [
    (1, 3, False, True, 2, 4, 32), (1, 3, False, True, 1, 2, 64), (3, 3, True, False, 2, 4, 32), (2, 3, False, True, 0, 4, 32)])
def test_native_step_driver_on_one_stream(H, oracle, Lr, n_sel, spare, fused, host, bits, gs):
    """All four stages handed the same stream (the form the single-layer latency figures use): nothing
    overlaps, results as with four streams."""
    _step_driver_case(oracle, Lr, n_sel, spare, 0.0, fused, host, bits, gs, one_stream=True)


@pytest.mark.parametrize("Lr,n_sel,fused,host", [(5, 5, True, 2), (3, 3, True, 0), (4, 4, False, 0)])
def test_native_step_driver_with_timing_on(H, oracle, Lr, n_sel, fused, host):
    """The same steps with the driver's timing on - event brackets around the scan launches (in the paired form the
    launch's completion event is the bracket's end and what the selection waits for) and per-wave clock stamps:
    results unchanged, a positive duration for every timed launch, stamps in order."""
    _step_driver_case(oracle, Lr, n_sel, False, 0.0, fused, host, 4, 32, timing=True)


def _step_driver_case(oracle, Lr, n_sel, spare, tau, fused, host, bits, gs, one_stream=False, timing=False):
    """hca_pipeline_step over 1 to 5 layers (score buffers shared between layers or one each), 12 decode
    steps, staggered eviction every 4 steps (sliced into a spare buffer set, or in place), top-k (as scan +
    top-k or fused as in hca_score_topk) or the cumulative-weight selection of Eq. 4 (tau > 0): every layer's
    output, resident count and final cache state against the oracle run layer by layer."""
    import ctypes as C
    from paper_2507_19823_amd import binding as B
    steps, E = 12, 4
    # with a host share the selection spans several chunks (k = 600: three chunks, the last ragged), and the
    # appended tokens' value rows (HBM slice) fall into the host's chunks whenever they rank early
    w = S.Workload("drv", 7, 2, 8, 2, 1500, bits, gs, 600 if host else 96)
    R, n0 = w.batch * w.n_kv_heads, w.n
    cap, vnew = n0 + E + 16, steps + 4
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap, bits, gs)
    dev = "cuda"
    kb = B.hca_kcache_bytes(shape)
    data = [S.make_layer(w, l) for l in range(Lr)]
    kc = [torch.zeros(kb, dtype=torch.uint8, device=dev) for _ in range(Lr + 1)]
    acc = [torch.zeros(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device=dev) for _ in range(Lr + 1)]
    pos = [torch.arange(cap, dtype=torch.int32, device=dev).repeat(w.batch, w.n_kv_heads, 1).contiguous()
           for _ in range(Lr + 1)]
    vh = [d["values"].contiguous().pin_memory() for d in data]
    vd = [torch.zeros(w.batch, w.n_kv_heads, vnew, 128, dtype=torch.float16, device=dev) for _ in range(Lr)]
    y = torch.zeros(Lr, w.batch, w.n_q_heads, 128, dtype=torch.float32, device=dev)
    ocs, oacc, opos, oV = [], [], [], []
    for l in range(Lr):
        B.hca_quantize_keys(shape, kc[l], data[l]["keys"].cuda(), n0, [0] * w.batch)
        oc = oracle.Cache(R, cap, 128, bits, gs)
        oracle.quantize(oc, _rows(data[l]["keys"]))
        ocs.append(oc)
        oacc.append(np.zeros((R, cap), np.float32))
        p = np.zeros((R, cap), np.int32)
        p[:] = np.arange(cap)
        opos.append(p)
        V = np.zeros((R, n0 + vnew, 128), np.float16)
        V[:, :n0] = _rows(data[l]["values"])
        oV.append(V)
    streams = [torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()]
    if one_stream:
        streams = [streams[0]] * 4
    d = B.hca_pipeline_desc()
    d.stream_scan, d.stream_topk, d.stream_gather, d.stream_attend = (s.cuda_stream for s in streams)
    wsb = B.hca_workspace_bytes(shape, w.k, n0)
    keep = []
    for i in range(n_sel):
        if fused:
            t = torch.zeros(B.hca_workspace_bytes(shape, w.k, 1), dtype=torch.uint8, device=dev)
            d.ws_select[i] = t.data_ptr()
        else:
            t = torch.zeros(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device=dev)
            d.sel[i] = t.data_ptr()
        keep.append(t)
    d.n_sel = n_sel
    d.fused_select = int(fused)
    n_pipe = 4 + Lr % 5 if host else 4          # with the hybrid value side: 4 .. 8 sets of selection buffers
    d.n_pipe = n_pipe
    for i in range(n_pipe):
        a = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device=dev)
        b = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device=dev)
        c = torch.zeros(wsb, dtype=torch.uint8, device=dev)
        keep += [a, b, c]
        d.idx[i], d.count[i], d.ws_attend[i] = a.data_ptr(), b.data_ptr(), c.data_ptr()
    wt, we = torch.zeros(wsb, dtype=torch.uint8, device=dev), torch.zeros(wsb, dtype=torch.uint8, device=dev)
    d.ws_topk, d.ws_evict = wt.data_ptr(), we.data_ptr()
    if (Lr + host + int(spare) + int(fused) + bits // 2) % 2 == 0:
        # every other case: one selection result per layer instead of the sets' idx / count (a stride with slack)
        stride = R * w.k + 24
        lidx = torch.full((Lr * stride,), -5, dtype=torch.int32, device=dev)
        lcnt = torch.full((Lr, R), -5, dtype=torch.int32, device=dev)
        keep += [lidx, lcnt]
        d.layer_idx, d.layer_count, d.layer_idx_stride = lidx.data_ptr(), lcnt.data_ptr(), stride
    if spare:
        d.spare_kcache, d.spare_acc, d.spare_pos = kc[Lr].data_ptr(), acc[Lr].data_ptr(), pos[Lr].data_ptr()
    d.topp_tau = tau
    d.host_chunks, d.host_threads = host, 3
    # two scan streams, or one scan launch per two layers, wherever the mode allows it
    d.dual_scan = (2 if Lr in (5, 1) else 1) if (fused and n_sel >= Lr and Lr != 4) else 0
    n_slots = 3 if timing else 0
    if timing:
        pairs = B.hca_scan_stamp_pairs(shape, cap)
        stamps = torch.zeros(n_slots, Lr, pairs, 2, dtype=torch.int64, device=dev)
        d.scan_stamps, d.scan_stamp_pairs, d.timing_layer_stride = stamps.data_ptr(), pairs, 1
    pl = B.hca_pipeline_create(shape, Lr, d, n_slots)
    layers = (B.hca_layer * Lr)()
    for l in range(Lr):
        layers[l].kcache, layers[l].acc, layers[l].pos = kc[l].data_ptr(), acc[l].data_ptr(), pos[l].data_ptr()
        layers[l].v_host, layers[l].v_hbm, layers[l].y = vh[l].data_ptr(), vd[l].data_ptr(), y[l].data_ptr()
    nres = (C.c_int64 * (Lr * w.batch))(*([n0] * (Lr * w.batch)))
    sm = 1.0 / math.sqrt(128.0)
    for t in range(steps):
        ins = [S.make_step(w, l, t) for l in range(Lr)]
        kn = [x[0].cuda() for x in ins]
        qs = [x[2].cuda() for x in ins]
        for l in range(Lr):
            vd[l][:, :, t] = ins[l][1][:, :, 0].cuda()
            layers[l].k_new, layers[l].q = kn[l].data_ptr(), qs[l].data_ptr()
        due = [(t + 1 + l) % E == 0 for l in range(Lr)]
        ev = (C.c_int64 * Lr)(*[n0 if x else 0 for x in due])
        torch.cuda.synchronize()
        B.hca_pipeline_step(pl, layers, nres, n0 + t, w.k, n0, n0, vnew, sm, ev, E, t % n_slots if timing else -1)
        torch.cuda.synchronize()
        if timing:
            ms = B.hca_pipeline_scan_ms(pl, t % n_slots, Lr)
            paired = d.dual_scan == 2
            for l in range(Lr):
                if paired and l % 2 == 1:
                    assert ms[l] == -1.0, f"step {t}: the second layer of a pair reports no launch of its own"
                else:
                    assert 0.0 < ms[l] < 100.0, f"step {t} layer {l}: scan bracket {ms[l]} ms"
            st_ = stamps[t % n_slots].cpu().numpy()
            for l in range(Lr):
                used = st_[l][st_[l, :, 0] > 0]
                assert len(used) > 0 and np.all(used[:, 1] >= used[:, 0]), f"step {t} layer {l}: wave stamps"
            stamps[t % n_slots].zero_()
        for l in range(Lr):
            oc = ocs[l]
            n = int(oc.n[0])
            oV[l][:, n0 + t] = _rows(ins[l][1])[:, 0]
            opos[l][:, n] = n0 + t
            oacc[l][:, n] = 0
            oracle.quantize(oc, _rows(ins[l][0]))
            q16 = ins[l][2].numpy().reshape(-1, 128)
            sel, _ = oracle.score(oc, q16, want_z=False)
            if tau > 0:
                idx, count, _, _ = oracle.topp(sel, oc.n, np.float32(sm), tau, w.k)
            else:
                idx, count = oracle.topk(sel, oc.n, w.k)
            yo, _ = oracle.attend(oc, q16, idx, count, opos[l], oV[l], np.float32(sm), acc=oacc[l])
            assert _rel_err(y[l].cpu().numpy().reshape(-1, 128), yo) <= TOL, f"step {t} layer {l}"
            if due[l]:
                # stage-wise: the oracle evicts on its own accumulated scores; both sides must keep the same slots
                oracle.evict(oc, oacc[l], opos[l], n0, E)
            assert nres[l * w.batch] == int(oc.n[0]), f"step {t} layer {l}"
    # final cache state of every layer (pointers may have swapped with the spare set)
    bufs = {kc[i].data_ptr(): (kc[i], acc[i], pos[i]) for i in range(Lr + 1)}
    for l in range(Lr):
        k_t, a_t, p_t = bufs[layers[l].kcache]
        assert layers[l].acc == a_t.data_ptr() and layers[l].pos == p_t.data_ptr()
        n = int(ocs[l].n[0])
        cb = torch.zeros(w.batch, w.n_kv_heads, cap, 128 * bits // 8, dtype=torch.uint8, device=dev)
        sc = torch.zeros(w.batch, w.n_kv_heads, cap, 128 // gs, dtype=torch.float16, device=dev)
        zr = torch.zeros_like(sc)
        B.hca_export_kcache(shape, k_t, [n] * w.batch, cb, sc, zr)
        torch.cuda.synchronize()
        assert np.array_equal(_rows(cb)[:, :n], ocs[l].codes[:, :n])
        assert np.array_equal(_rows(sc).view(np.uint16)[:, :n], ocs[l].scale[:, :n])
        assert np.array_equal(_rows(p_t)[:, :n], opos[l][:, :n])
        assert np.allclose(_rows(a_t)[:, :n], oacc[l][:, :n], rtol=1e-3, atol=1e-6)
    assert B.hca_pipeline_host_status(pl) == (0, 0)
    B.hca_pipeline_destroy(pl)


def test_step_driver_merge_gives_up_on_a_silent_host(H):
    """Hybrid value side with no host threads started and a tiny poll limit: every merge's bounded wait runs out,
    the kernels end normally, and the driver reports the timeout."""
    import ctypes as C
    from paper_2507_19823_amd import binding as B
    w = S.Workload("drv", 8, 1, 8, 2, 900, 4, 32, 300)
    n0, cap = w.n, w.n + 8
    shape = B.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, cap)
    dev = "cuda"
    data = S.make_layer(w, 0)
    kc = torch.zeros(B.hca_kcache_bytes(shape), dtype=torch.uint8, device=dev)
    acc = torch.zeros(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device=dev)
    pos = torch.arange(cap, dtype=torch.int32, device=dev).repeat(w.batch, w.n_kv_heads, 1).contiguous()
    B.hca_quantize_keys(shape, kc, data["keys"].cuda(), n0, [0] * w.batch)
    vh = data["values"].contiguous().pin_memory()
    vd = torch.zeros(w.batch, w.n_kv_heads, 4, 128, dtype=torch.float16, device=dev)
    y = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device=dev)
    streams = [torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()]
    d = B.hca_pipeline_desc()
    d.stream_scan, d.stream_topk, d.stream_gather, d.stream_attend = (s.cuda_stream for s in streams)
    wsb = B.hca_workspace_bytes(shape, w.k, 1)
    keep = []
    for i in range(3):
        t = torch.zeros(w.batch, w.n_kv_heads, cap, dtype=torch.float32, device=dev)
        d.sel[i] = t.data_ptr()
        keep.append(t)
    d.n_sel = 3
    for i in range(4):
        a = torch.zeros(w.batch, w.n_kv_heads, w.k, dtype=torch.int32, device=dev)
        b = torch.zeros(w.batch, w.n_kv_heads, dtype=torch.int32, device=dev)
        c = torch.zeros(wsb, dtype=torch.uint8, device=dev)
        keep += [a, b, c]
        d.idx[i], d.count[i], d.ws_attend[i] = a.data_ptr(), b.data_ptr(), c.data_ptr()
    wt = torch.zeros(wsb, dtype=torch.uint8, device=dev)
    d.ws_topk = wt.data_ptr()
    d.host_chunks, d.host_threads, d.host_spin_limit = 1, 0, 20
    pl = B.hca_pipeline_create(shape, 1, d, 0)
    layers = (B.hca_layer * 1)()
    layers[0].kcache, layers[0].acc, layers[0].pos = kc.data_ptr(), acc.data_ptr(), pos.data_ptr()
    layers[0].v_host, layers[0].v_hbm, layers[0].y = vh.data_ptr(), vd.data_ptr(), y.data_ptr()
    k_new, _, q = S.make_step(w, 0, 0)
    kn, qd = k_new.cuda(), q.cuda()
    layers[0].k_new, layers[0].q = kn.data_ptr(), qd.data_ptr()
    nres = (C.c_int64 * 1)(n0)
    assert B.hca_pipeline_host_status(pl) == (0, 0)
    B.hca_pipeline_step(pl, layers, nres, n0, w.k, n0, n0, 4, 1.0 / math.sqrt(128.0), None, 0, -1)
    torch.cuda.synchronize()
    assert B.hca_pipeline_host_status(pl)[0] != 0
    assert nres[0] == n0 + 1
    B.hca_pipeline_destroy(pl)


@pytest.mark.parametrize("bits,gs,G,k,n", [(2, 64, 4, 512, 9000), (2, 64, 2, 100, 3001), (4, 32, 2, 16384, 20000),
                                           (4, 32, 1, 1, 100), (2, 64, 1, 777, 777)])
def test_small_pipelines_other_shapes(H, oracle, bits, gs, G, k, n):
    """2-bit codes, 1 / 2 / 4 query heads per KV head, k = 1, k = n and the largest supported k."""
    w = S.Workload("p", 200 + bits + G, 2, 2 * G, 2, n, bits, gs, k, planted=4)
    d = S.make_layer(w)
    R = w.batch * w.n_kv_heads
    st = _state(H, w, want_z=True)
    oc = _ocache(oracle, w, n)
    st.quantize(d["keys"].cuda())
    oracle.quantize(oc, _rows(d["keys"]))
    qd = d["q"].cuda()
    st.score(qd)
    st.topk(k)
    nh = n // 3
    vh = d["values"][:, :, :nh].contiguous().pin_memory()
    vd = d["values"][:, :, nh:].contiguous().cuda()
    st.attend(qd, vh, nh, vd, use_acc=True, gather_stream=torch.cuda.Stream())
    torch.cuda.synchronize()
    q16 = d["q"].numpy().reshape(-1, 128)
    sel, z = oracle.score(oc, q16)
    assert np.array_equal(st.z.cpu().numpy().reshape(-1, n), z)
    idx, count = oracle.topk(sel, oc.n, k)
    assert np.array_equal(_rows(st.idx), idx)
    pos = np.tile(np.arange(n, dtype=np.int32), (R, 1))
    acc = np.zeros((R, n), np.float32)
    y, _ = oracle.attend(oc, q16, idx, count, pos, _rows(d["values"]), st.sm_scale, acc=acc)
    assert _rel_err(st.y.cpu().numpy().reshape(-1, 128), y) <= TOL
    assert np.allclose(_rows(st.acc), acc, rtol=1e-4, atol=1e-7)


def test_clustered_heavy_hitters_in_one_chunk(H, oracle):
    """All the large scores sit in one 4096-slot chunk (what eviction produces when it packs the ever-selected
    tokens together): the chunk's candidate list is long, the result must not change."""
    from paper_2507_19823_amd import binding as B
    rng = np.random.default_rng(5)
    n, k = 40000, 3000
    v = rng.standard_normal((4, n)).astype(np.float32)
    v[:, 36000:40000] += 6.0                      # ~4000 of the top values in the last chunk
    v[1, 36000:39000] = 7.5                       # and a mass tie there
    shape = B.make_shape(2, 8, 2, n)
    sel = torch.from_numpy(v).cuda()
    idx = torch.full((4, k), -9, dtype=torch.int32, device="cuda")
    count = torch.zeros(4, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.hca_workspace_bytes(shape, k, 1), dtype=torch.uint8, device="cuda")
    B.hca_topk(shape, sel, [n, n], k, idx, count, ws)
    torch.cuda.synchronize()
    ridx, _ = oracle.topk(v, np.full(4, n), k)
    assert np.array_equal(idx.cpu().numpy(), ridx)


def test_decode_step_through_the_c_abi_without_torch(H):
    """tests/c/decode_step_no_torch.cpp: hipMalloc / hipHostMalloc memory, libhca.so and the oracle's shared
    object, no Python in the data path (the program is built by __graft_entry__.build())."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "c", "bin", "decode_step_no_torch")
    assert os.path.exists(exe), "run __graft_entry__.build() first"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ok" in r.stdout
