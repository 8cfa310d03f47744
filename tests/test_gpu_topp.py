"""GPU parity of hca_topp (the paper's cumulative-weight selection, Eq. 4) against the oracle, through the
C ABI: Theta, Z, k* and the selected slots bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2507_19823_amd import binding
    binding.lib()
    return binding


def _run(B, v, lens, hkv, sm, tau, k_max):
    batch = len(lens)
    R, cap = v.shape
    assert R == batch * hkv
    shape = B.make_shape(batch, hkv, hkv, cap)
    sel = torch.from_numpy(v).cuda()
    idx = torch.full((R, k_max), -9, dtype=torch.int32, device="cuda")
    count = torch.full((R,), -9, dtype=torch.int32, device="cuda")
    mass = torch.full((R, 2), 7, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.hca_workspace_bytes(shape, k_max, 1), dtype=torch.uint8, device="cuda")
    B.hca_topp(shape, sel, lens, sm, tau, k_max, idx, count, mass, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), count.cpu().numpy(), mass.cpu().numpy().view(np.uint64)


def _check(oracle, v, lens, hkv, sm, tau, k_max, got):
    idx, count, mass = got
    n = np.repeat(lens, hkv)
    oidx, ocount, okstar, omass = oracle.topp(v, n, sm, tau, k_max)
    assert np.array_equal(mass, omass), "Theta / Z differ"
    assert np.array_equal(count, ocount)
    for r in range(v.shape[0]):
        assert np.array_equal(idx[r, :count[r]], oidx[r, :count[r]])
    # validity against Eq. 4 as written (fp64 softmax, sort, shortest prefix with mass >= tau): the GPU's prefix
    # holds at least tau - eps of the plain mass and one slot less holds less than tau + eps, eps being the margin
    # derived for the integer weights (6e-5 relative plus n units out of Z); rows cut at k_max are top-k_max sets
    _, order, cum = oracle.topp_plain(v, n, sm, tau)
    for r in range(v.shape[0]):
        nr, c = int(n[r]), int(count[r])
        if nr == 0 or okstar[r] > k_max:
            continue
        eps = 6e-5 + nr / float(mass[r, 1])
        assert c == okstar[r]
        assert cum[r, c - 1] >= min(tau, 1.0) - eps, (r, c, cum[r, c - 1])
        assert c == 1 or cum[r, c - 2] < tau + eps, (r, c, cum[r, c - 2])
        assert np.array_equal(np.sort(order[r, :c]), idx[r, :c])      # the same sorted prefix, as a set
    return okstar


@pytest.mark.parametrize("case", ["normal", "ties", "dominant", "all_equal", "flat", "signed_zero"])
@pytest.mark.parametrize("n,k_max,tau,sm", [(5000, 5000, 0.9, 0.0884), (5000, 300, 0.99, 0.0884), (70000, 4096, 0.5, 0.3),
                                           (70000, 70000, 1.0, 0.0884), (300, 64, 0.2, 1.0), (1, 1, 0.7, 0.1)])
def test_topp_bit_exact(B, oracle, case, n, k_max, tau, sm):
    rng = np.random.default_rng(n + k_max + len(case))
    R, hkv = 4, 2
    cap = n + 3
    v = np.full((R, cap), 1e30, np.float32)
    if case == "normal":
        x = rng.standard_normal((R, n)) * 12
    elif case == "ties":
        x = np.round(rng.standard_normal((R, n)) * 6)
    elif case == "dominant":
        x = rng.standard_normal((R, n))
        x[:, rng.integers(0, n, 3)] += 150
    elif case == "all_equal":
        x = np.full((R, n), -2.5)
    elif case == "flat":
        x = rng.uniform(-0.01, 0.01, (R, n))
    else:
        x = np.zeros((R, n))
        x[:, ::3] = -0.0
        x[:, 1::5] = 1e-30
    v[:, :n] = x.astype(np.float32)
    got = _run(B, v, [n, n], hkv, sm, tau, k_max)
    _check(oracle, v, [n, n], hkv, sm, tau, k_max, got)


def test_topp_ragged_empty_and_clip(B, oracle):
    rng = np.random.default_rng(9)
    cap, hkv = 40000, 2
    lens = [40000, 0, 17, 25000]
    v = (rng.standard_normal((8, cap)) * 10).astype(np.float32)
    got = _run(B, v, lens, hkv, 0.0884, 0.95, 2000)
    ks = _check(oracle, v, lens, hkv, 0.0884, 0.95, 2000, got)
    assert got[1][2] == 0 and got[1][3] == 0 and np.all(got[2][2:4] == 0)      # the empty sequence
    assert ks[0] > 2000 and got[1][0] == 2000                                   # clipped rows keep the top-k_max set
    ridx, _ = oracle.topk(v, np.repeat(lens, hkv), 2000)
    assert np.array_equal(got[0][0], ridx[0])


def test_topp_at_one_million(B, oracle):
    """Planted-query-like score profile at the bench shape: 8 rows x 1 Mi slots."""
    rng = np.random.default_rng(10)
    n = (1 << 20) + 5
    v = (rng.standard_normal((8, n)) * 11).astype(np.float32)
    v[:, rng.integers(0, n, 64)] += 60
    for tau, k_max in ((0.9, 16384), (0.999, 16384), (0.5, 4096)):
        got = _run(B, v, [n], 8, 0.0884, tau, k_max)
        _check(oracle, v, [n], 8, 0.0884, tau, k_max, got)


def test_decode_step_with_cumulative_weight_selection(B, oracle):
    """scan -> hca_topp -> gather -> attend: the variable-length selection feeds the same attend calls."""
    import synth_inputs as S
    from paper_2507_19823_amd.session import LayerState
    w = S.Workload("tp", 31, 2, 8, 2, 6000, 4, 32, 2048, planted=8)
    d = S.make_layer(w)
    R, n, k_max = w.batch * w.n_kv_heads, w.n, 2048
    st = LayerState(w.batch, w.n_q_heads, w.n_kv_heads, n + 8, w.bits, w.group, k_max=k_max, m_max=1)
    st.quantize(d["keys"].cuda())
    qd = d["q"].cuda()
    st.score(qd)
    sm = st.sm_scale
    B.hca_topp(st.shape, st.sel, st.n, sm, 0.97, k_max, st.idx, st.count, None, st.ws)
    vh = d["values"].contiguous().pin_memory()
    B.hca_gather_values(st.shape, st.idx, st.count, k_max, st.pos, vh, n, n, None, 0, st.ws)
    B.hca_attend_gathered(st.shape, st.kcache, qd, st.idx, st.count, k_max, sm, st.y, st.acc, st.ws)
    torch.cuda.synchronize()
    oc = oracle.Cache(R, n + 8, 128, w.bits, w.group)
    oracle.quantize(oc, d["keys"].numpy().reshape(R, n, 128))
    q16 = d["q"].numpy().reshape(-1, 128)
    sel, _ = oracle.score(oc, q16, want_z=False)
    idx, count, kstar, _ = oracle.topp(sel, oc.n, sm, 0.97, k_max)
    cg = st.count.cpu().numpy().reshape(R)
    assert np.array_equal(cg, count) and 1 <= count.min() and len(set(count.tolist())) > 1   # really variable
    ig = st.idx.cpu().numpy().reshape(R, k_max)
    for r in range(R):
        assert np.array_equal(ig[r, :count[r]], idx[r, :count[r]])
    pos = np.tile(np.arange(n + 8, dtype=np.int32), (R, 1))
    acc = np.zeros((R, n + 8), np.float32)
    y, _ = oracle.attend(oc, q16, idx, count, pos, d["values"].numpy().reshape(R, n, 128), sm, acc=acc)
    yg = st.y.cpu().numpy().reshape(-1, 128)
    assert float(np.max(np.abs(yg - y).max(-1) / np.maximum(np.abs(y).max(-1), 1e-30))) <= 2e-3
    assert np.allclose(st.acc.cpu().numpy().reshape(R, -1), acc, rtol=1e-4, atol=1e-7)


@pytest.mark.parametrize("bits,gs,G,n,k", [(4, 32, 4, 9000, 512), (2, 64, 4, 5000, 100), (4, 32, 2, 3001, 3001), (4, 32, 1, 70, 5)])
def test_global_softmax_denominator_and_unrenormalised_weights(B, oracle, bits, gs, G, n, k):
    """hca_score_qkeys_lse: the same selection scores as hca_score_qkeys plus lse over all resident tokens;
    hca_attend_gathered_global: the paper's Eq. 5 weights.  Sequences of different length, one empty."""
    import synth_inputs as S
    rng = np.random.default_rng(n + k)
    batch, hkv = 3, 2
    R, cap = batch * hkv, n + 40
    lens = [n, 0, n // 3]
    shape = B.make_shape(batch, hkv * G, hkv, cap, bits, gs)
    keys = rng.standard_normal((batch, hkv, n, 128)).astype(np.float16)
    keys[..., 7] *= 8
    vals = rng.standard_normal((batch, hkv, n, 128)).astype(np.float16)
    q = (1.5 * rng.standard_normal((batch, hkv * G, 128))).astype(np.float16)
    kc = torch.zeros(B.hca_kcache_bytes(shape), dtype=torch.uint8, device="cuda")
    B.hca_quantize_keys(shape, kc, torch.from_numpy(keys).cuda(), n, [0] * batch)
    sel = torch.full((batch, hkv, cap), -7.0, device="cuda")
    sel2 = torch.full((batch, hkv, cap), -7.0, device="cuda")
    lse = torch.full((batch, hkv * G), 123.0, device="cuda")
    ws = torch.empty(B.hca_workspace_bytes(shape, k, 1), dtype=torch.uint8, device="cuda")
    qd = torch.from_numpy(q).cuda()
    sm = 1.0 / np.sqrt(128.0)
    B.hca_score_qkeys(shape, kc, qd, lens, sel2)
    B.hca_score_qkeys_lse(shape, kc, qd, lens, sm, sel, lse, ws)
    torch.cuda.synchronize()
    assert torch.equal(sel, sel2)
    oc = oracle.Cache(R, cap, 128, bits, gs)
    oracle.quantize(oc, keys.reshape(R, n, 128))
    oc.n[:] = np.repeat(lens, hkv)
    osel, oz = oracle.score(oc, q.reshape(R * G, 128))
    olse = oracle.lse(oz, R, oc.n, sm)
    lg = lse.cpu().numpy().reshape(R * G)
    live = np.repeat(np.array(lens) > 0, hkv * G)
    assert np.all(np.isneginf(lg[~live])) and np.all(np.isneginf(olse[~live]))
    assert np.allclose(lg[live], olse[live], rtol=2e-6, atol=2e-5)

    idx = torch.zeros(batch, hkv, k, dtype=torch.int32, device="cuda")
    count = torch.zeros(batch, hkv, dtype=torch.int32, device="cuda")
    pos = torch.arange(cap, dtype=torch.int32, device="cuda").repeat(batch, hkv, 1).contiguous()
    acc = torch.zeros(batch, hkv, cap, device="cuda")
    y = torch.zeros(batch, hkv * G, 128, device="cuda")
    B.hca_topk(shape, sel, lens, k, idx, count, ws)
    vh = torch.from_numpy(vals).contiguous().pin_memory()
    B.hca_gather_values(shape, idx, count, k, pos, vh, n, n, None, 0, ws)
    B.hca_attend_gathered_global(shape, kc, qd, idx, count, k, sm, lse, y, acc, ws)
    torch.cuda.synchronize()
    oidx, ocount = oracle.topk(osel, oc.n, k)
    opos = np.tile(np.arange(cap, dtype=np.int32), (R, 1))
    oacc = np.zeros((R, cap), np.float32)
    oy, ow = oracle.attend(oc, q.reshape(R * G, 128), oidx, ocount, opos, vals.reshape(R, n, 128), sm, acc=oacc,
                           want_w=True, lse=olse)
    yg = y.cpu().numpy().reshape(R * G, 128)
    assert np.all(yg[~live] == 0)
    err = np.abs(yg[live] - oy[live]).max(-1) / np.maximum(np.abs(oy[live]).max(-1), 1e-30)
    assert err.max() <= 2e-3
    if k < n // 3:
        assert ow[live].sum(1).max() < 0.999999        # the weights really are not renormalised
    assert np.allclose(acc.cpu().numpy().reshape(R, cap), oacc, rtol=2e-4, atol=1e-7)


@pytest.mark.parametrize("bits,gs,G,n,k,use_lse", [(4, 32, 4, 9000, 512, False), (2, 64, 4, 5000, 300, True), (4, 32, 1, 700, 700, False)])
def test_paper_split_weights_on_gpu_sum_on_host(B, oracle, bits, gs, G, n, k, use_lse):
    """hca_attend_weights leaves fp16 weights and value-row numbers in pinned host memory;
    hca_host_weighted_sum forms y from the host-resident values (the paper's CPU part)."""
    rng = np.random.default_rng(n + k + bits)
    batch, hkv = 2, 2
    R, cap = batch * hkv, n + 8
    shape = B.make_shape(batch, hkv * G, hkv, cap, bits, gs)
    keys = rng.standard_normal((batch, hkv, n, 128)).astype(np.float16)
    vals = rng.standard_normal((batch, hkv, n, 128)).astype(np.float16)
    q = (1.5 * rng.standard_normal((batch, hkv * G, 128))).astype(np.float16)
    kc = torch.zeros(B.hca_kcache_bytes(shape), dtype=torch.uint8, device="cuda")
    B.hca_quantize_keys(shape, kc, torch.from_numpy(keys).cuda(), n, [0] * batch)
    lens = [n, n - 123]
    sel = torch.zeros(batch, hkv, cap, device="cuda")
    lse = torch.zeros(batch, hkv * G, device="cuda")
    ws = torch.empty(B.hca_workspace_bytes(shape, k, 1), dtype=torch.uint8, device="cuda")
    qd = torch.from_numpy(q).cuda()
    sm = 1.0 / np.sqrt(128.0)
    B.hca_score_qkeys_lse(shape, kc, qd, lens, sm, sel, lse, ws)
    idx = torch.zeros(batch, hkv, k, dtype=torch.int32, device="cuda")
    count = torch.zeros(batch, hkv, dtype=torch.int32, device="cuda")
    permv = rng.permutation(cap).astype(np.int32) % n
    pos = torch.from_numpy(np.tile(permv, (R, 1)).reshape(batch, hkv, cap)).cuda()
    acc = torch.zeros(batch, hkv, cap, device="cuda")
    B.hca_topk(shape, sel, lens, k, idx, count, ws)
    w16 = torch.zeros(batch, hkv * G, k, dtype=torch.float16).pin_memory()
    vrow = torch.zeros(batch, hkv, k, dtype=torch.int32).pin_memory()
    B.hca_attend_weights(shape, kc, qd, idx, count, k, pos, sm, lse if use_lse else None, w16, vrow, acc, ws)
    torch.cuda.synchronize()
    vh = torch.from_numpy(vals)
    y = torch.zeros(batch, hkv * G, 128)
    B.hca_host_weighted_sum(shape, vrow, count.cpu(), k, w16, vh, n, y, 8)

    oc = oracle.Cache(R, cap, 128, bits, gs)
    oracle.quantize(oc, keys.reshape(R, n, 128))
    oc.n[:] = np.repeat(lens, hkv)
    osel, oz = oracle.score(oc, q.reshape(R * G, 128))
    olse = oracle.lse(oz, R, oc.n, sm) if use_lse else None
    oidx, ocount = oracle.topk(osel, oc.n, k)
    opos = np.tile(permv, (R, 1))
    oacc = np.zeros((R, cap), np.float32)
    oy, ow = oracle.attend(oc, q.reshape(R * G, 128), oidx, ocount, opos, vals.reshape(R, n, 128), sm, acc=oacc,
                           want_w=True, lse=olse)
    ig = idx.cpu().numpy().reshape(R, k)
    for r in range(R):
        assert np.array_equal(ig[r, :ocount[r]], oidx[r, :ocount[r]])
    vg = vrow.numpy().reshape(R, k)
    for r in range(R):
        assert np.array_equal(vg[r, :ocount[r]], opos[r, oidx[r, :ocount[r]]]) and np.all(vg[r, ocount[r]:] == -1)
    wg = w16.numpy().reshape(R * G, k).astype(np.float32)
    assert np.allclose(wg, ow.astype(np.float16).astype(np.float32), rtol=2e-3, atol=1e-7)      # within an fp16 ulp
    ref16 = oracle.weighted_sum_f16(ow, oidx, ocount, opos, vals.reshape(R, n, 128))
    yg = y.numpy().reshape(R * G, 128)
    scale = np.maximum(np.abs(oy).max(-1), 1e-30)
    assert (np.abs(yg - ref16).max(-1) / scale).max() <= 1e-3
    assert (np.abs(yg - oy).max(-1) / scale).max() <= 2e-3            # against the unrounded weights
    assert np.allclose(acc.cpu().numpy().reshape(R, cap), oacc, rtol=2e-4, atol=1e-7)
