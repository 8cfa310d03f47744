"""GPU parity of hca_score_topk (scan and top-k in one call, Sec. 3.2) against the oracle's score + top-k."""
import numpy as np
import pytest
import torch

import synth_inputs as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import paper_2507_19823_amd as H
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    H.lib()
    return H


@pytest.fixture(autouse=True, params=[0, 256], ids=["wg1024", "wg256"])
def select_wg(request, H):
    """Every case runs with both forms of the selection over the candidate lists: one 1024-thread workgroup per
    row with the pairs staged in LDS (the per-call default), and the four-wave form that reads them from L2 (what
    the step driver uses beside a running scan)."""
    H.hca_tune("select_wg", request.param)
    yield request.param
    H.hca_tune("select_wg", 0)


def _rows(t):
    a = t.detach().cpu().numpy()
    return a.reshape(a.shape[0] * a.shape[1], *a.shape[2:])


def _run(H, oracle, w, keys, q, lens, k):
    """Quantises `keys` on both sides, cuts the sequences to `lens`, selects k per row; compares index sets."""
    from paper_2507_19823_amd import binding as B
    from paper_2507_19823_amd.session import LayerState
    st = LayerState(w.batch, w.n_q_heads, w.n_kv_heads, w.n, w.bits, w.group, k_max=k, want_z=False)
    oc = oracle.Cache(w.batch * w.n_kv_heads, w.n, 128, w.bits, w.group)
    st.quantize(keys.cuda())
    oracle.quantize(oc, _rows(keys))
    st.n = list(lens)
    oc.n[...] = np.repeat(lens, w.n_kv_heads)
    R = w.batch * w.n_kv_heads
    idx = torch.full((R, k), -9, dtype=torch.int32, device="cuda")
    count = torch.full((R,), -9, dtype=torch.int32, device="cuda")
    B.hca_score_topk(st.shape, st.kcache, q.cuda(), st.n, k, idx, count, st.ws)
    torch.cuda.synchronize()
    sel, _ = oracle.score(oc, q.numpy().reshape(-1, 128), want_z=False)
    ridx, rcount = oracle.topk(sel, oc.n, k)
    gi, gc = idx.cpu().numpy(), count.cpu().numpy()
    for r in range(R):
        c = min(k, lens[r // w.n_kv_heads])
        assert gc[r] == c == rcount[r], f"row {r}: count {gc[r]} / {rcount[r]} / {c}"
        assert np.array_equal(gi[r, :c], ridx[r, :c]), f"row {r}: index sets differ"
        assert np.all(gi[r, c:] == -9)
    cand = torch.full((R,), -1, dtype=torch.int32, device="cuda")
    resc = torch.full((R,), -1, dtype=torch.int32, device="cuda")
    B.hca_score_topk_report(st.shape, st.n, st.ws, cand, resc)
    torch.cuda.synchronize()
    return cand.cpu().numpy(), resc.cpu().numpy()


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64)])
@pytest.mark.parametrize("n,k,lens", [
    (300, 64, [300, 17]), (5000, 256, [5000, 0]), (5000, 5000, [4999, 5000]), (70001, 2048, [70001, 33000]),
    (300000, 1024, [300000, 150001]),
])
def test_score_topk_matches_the_oracle(H, oracle, bits, gs, n, k, lens):
    w = S.Workload("st", 90 + bits, 2, 8, 2, n, bits, gs, k)
    d = S.make_layer(w, want_values=False)
    cand, resc = _run(H, oracle, w, d["keys"], d["q"], lens, k)
    for r in range(w.batch * w.n_kv_heads):
        nr_ = lens[r // w.n_kv_heads]
        if nr_ > 0:
            assert min(k, nr_) <= cand[r] <= nr_
            assert resc[r] == 0, "seeded random keys: the sampled threshold must hold"
    if n >= 70001:      # long rows: the threshold discards almost everything
        assert cand[0] < n // 8


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64)])
def test_the_largest_k(H, oracle, bits, gs):
    """k = 16384, the most the step driver accepts: more candidates than the LDS stage holds, one row barely
    longer than k."""
    n, k = 120000, 16384
    lens = [n, k + 5]
    w = S.Workload("stmax", 95 + bits, 2, 8, 2, n, bits, gs, k)
    d = S.make_layer(w, want_values=False)
    cand, resc = _run(H, oracle, w, d["keys"], d["q"], lens, k)
    assert int(cand.min()) >= k


@pytest.mark.parametrize("hq,hkv", [(4, 2), (2, 2), (6, 3)])
def test_fewer_query_heads_per_kv_head(H, oracle, hq, hkv):
    """Groups of two query heads and of one: the selection score is the maximum over the heads that exist."""
    w = S.Workload("gqa", 97 + hq, 2, hq, hkv, 40000, 4, 32, 512)
    d = S.make_layer(w, want_values=False)
    _run(H, oracle, w, d["keys"], d["q"], [40000, 12345], 512)


def test_ties_and_a_list_too_long_for_lds(H, oracle):
    """Every key the same: every slot passes any threshold (50 000 pairs, more than are staged in LDS) and the
    k lowest slots win."""
    w = S.Workload("tie", 95, 1, 4, 1, 50000, 4, 32, 777)
    d = S.make_layer(w, want_values=False)
    keys = d["keys"][:, :, :1].expand(-1, -1, w.n, -1).contiguous()
    cand, resc = _run(H, oracle, w, keys, d["q"], [w.n], w.k)
    assert cand[0] == w.n and resc[0] == 0        # one key value: every slot passes the threshold


@pytest.mark.parametrize("bits,gs,tpb", [(4, 32, 16), (2, 64, 32)])
def test_a_sample_that_misleads_still_gives_the_exact_set(H, oracle, bits, gs, tpb):
    """The sample reads block floor(s * nblocks / S), s < S = 8192 / (slots per block).  Those blocks get keys along
    the query (large scores), all others keys against it: the sampled threshold then admits far fewer than k
    slots and the row has to go through the second, unthresholded scan."""
    n, k = 200000, 1024
    w = S.Workload("mis", 96 + bits, 1, 4, 1, n, bits, gs, k)
    d = S.make_layer(w, want_values=False)
    q = d["q"].clone()
    q[0, 1:] = q[0, :1]                                       # four equal query heads
    g = torch.Generator().manual_seed(5)
    noise = 0.05 * torch.randn(n, 128, generator=g)
    nblocks = (n + tpb - 1) // tpb
    Sn = min(nblocks, 8192 // tpb)
    sampled = torch.zeros(nblocks, dtype=torch.bool)
    sampled[(torch.arange(Sn, dtype=torch.int64) * nblocks) // Sn] = True
    sign = torch.where(sampled.repeat_interleave(tpb)[:n], 1.0, -1.0)[:, None]
    keys = (sign * q[0, 0].float()[None, :] * (0.5 + torch.rand(n, 1, generator=g)) + noise).to(torch.float16)
    cand, resc = _run(H, oracle, w, keys[None, None], q, [n], k)
    assert resc[0] == 1 and k <= cand[0] <= n      # the row went through the second scan


def test_second_scan_with_the_deeper_threshold(H, oracle):
    """As above, but the slots outside the sampled blocks score only a little lower than those inside: the first
    threshold (inside the sampled blocks' range) lets too few through, the second one - the 8r-th largest sample,
    counted against during the first scan - lets enough through, and the second scan keeps far fewer than n."""
    n, k, tpb = 300000, 2048, 16
    w = S.Workload("mis2", 99, 1, 4, 1, n, 4, 32, k)
    d = S.make_layer(w, want_values=False)
    q = d["q"].clone()
    q[0, 1:] = q[0, :1]
    g = torch.Generator().manual_seed(7)
    nblocks = (n + tpb - 1) // tpb
    Sn = min(nblocks, 8192 // tpb)
    sampled = torch.zeros(nblocks, dtype=torch.bool)
    sampled[(torch.arange(Sn, dtype=torch.int64) * nblocks) // Sn] = True
    inside = sampled.repeat_interleave(tpb)[:n]
    # projection on the query (x 40 = score): inside the sampled blocks uniform in [1.0, 2.0], so the first
    # threshold (123rd largest sample) sits near 1.985 and the second (984th, rounded down to its 12-bit bin:
    # scores 72..80) at 1.8; outside, 3 % of the slots uniform in [1.85, 1.95] - below the first, above the
    # second, some 8700 of them -, the rest negative
    u = torch.rand(n, generator=g)
    mid = torch.rand(n, generator=g) < 0.03
    proj = torch.where(inside, 1.0 + u, torch.where(mid, 1.85 + 0.1 * u, -1.0 - u))
    keys = (proj[:, None] * q[0, 0].float()[None, :] / q[0, 0].float().norm() ** 2 * 40.0
            + 0.02 * torch.randn(n, 128, generator=g)).to(torch.float16)
    cand, resc = _run(H, oracle, w, keys[None, None], q, [n], k)
    assert resc[0] == 1 and k <= cand[0] < n // 4


def test_running_monitor_over_several_calls(H):
    """hca_score_topk_monitor: calls counted, fewest / most pairs of a first scan and second scans per row, over
    three selections at different lengths (compared with the per-call report after each)."""
    from paper_2507_19823_amd import binding as B
    from paper_2507_19823_amd.session import LayerState
    w = S.Workload("mon", 93, 2, 8, 2, 60000, 4, 32, 512)
    d = S.make_layer(w, want_values=False)
    st = LayerState(w.batch, w.n_q_heads, w.n_kv_heads, w.n, w.bits, w.group, k_max=w.k, want_z=False)
    st.quantize(d["keys"].cuda())
    R = w.batch * w.n_kv_heads
    idx = torch.zeros(R, w.k, dtype=torch.int32, device="cuda")
    count = torch.zeros(R, dtype=torch.int32, device="cuda")
    cand = torch.zeros(R, dtype=torch.int32, device="cuda")
    resc = torch.zeros(R, dtype=torch.int32, device="cuda")
    mon = torch.full((R, 4), -7, dtype=torch.int32, device="cuda")
    B.hca_score_topk_monitor(st.shape, st.ws, None, True)
    seen = []
    for lens in ([60000, 700], [31000, 31000], [45000, 60000]):
        st.n = list(lens)
        B.hca_score_topk(st.shape, st.kcache, d["q"].cuda(), st.n, w.k, idx, count, st.ws)
        B.hca_score_topk_report(st.shape, st.n, st.ws, cand, resc)
        torch.cuda.synchronize()
        assert int(resc.sum()) == 0
        seen.append(cand.cpu().numpy().copy())
    B.hca_score_topk_monitor(st.shape, st.ws, mon, True)
    torch.cuda.synchronize()
    m, seen = mon.cpu().numpy(), np.stack(seen)
    assert np.all(m[:, 0] == 3) and np.all(m[:, 3] == 0)
    assert np.array_equal(m[:, 1], seen.min(0)) and np.array_equal(m[:, 2], seen.max(0))
    B.hca_score_topk_monitor(st.shape, st.ws, mon, False)       # after the reset above
    torch.cuda.synchronize()
    m = mon.cpu().numpy()
    assert np.all(m[:, 0] == 0) and np.all(m[:, 1] == 2**31 - 1) and np.all(m[:, 2] == 0) and np.all(m[:, 3] == 0)


@pytest.mark.parametrize("own_idx", [False, True])
def test_step_driver_pair_with_a_row_that_needs_the_second_scan(H, oracle, own_idx):
    """Two layers through hca_pipeline_step with paired scan launches: layer 0's keys mislead the sample (as in
    test_a_sample_that_misleads_still_gives_the_exact_set), layer 1's do not.  The paired fall-back launches
    (second scan of the failed row, second selection) must leave the oracle's index sets for both layers; the
    running monitor counts one second scan on layer 0's workspace and none on layer 1's."""
    import ctypes as C
    from paper_2507_19823_amd import binding as B
    n, k, tpb = 200000, 1024, 16
    w = S.Workload("mispair", 98, 1, 4, 1, n, 4, 32, k)
    R, cap, Lr = 1, n + 8, 2
    d = S.make_layer(w, want_values=False)
    q = d["q"].clone()
    q[0, 1:] = q[0, :1]
    g = torch.Generator().manual_seed(5)
    nblocks = (n + tpb - 1) // tpb
    Sn = min(nblocks, 8192 // tpb)
    sampled = torch.zeros(nblocks, dtype=torch.bool)
    sampled[(torch.arange(Sn, dtype=torch.int64) * nblocks) // Sn] = True
    sign = torch.where(sampled.repeat_interleave(tpb)[:n], 1.0, -1.0)[:, None]
    k0 = (sign * q[0, 0].float()[None, :] * (0.5 + torch.rand(n, 1, generator=g))
          + 0.05 * torch.randn(n, 128, generator=g)).to(torch.float16)[None, None]
    keys = [k0, d["keys"]]
    shape = B.make_shape(1, 4, 1, cap)
    dev = "cuda"
    kc = [torch.zeros(B.hca_kcache_bytes(shape), dtype=torch.uint8, device=dev) for _ in range(Lr)]
    acc = [torch.zeros(1, 1, cap, dtype=torch.float32, device=dev) for _ in range(Lr)]
    pos = [torch.arange(cap, dtype=torch.int32, device=dev).view(1, 1, cap).contiguous() for _ in range(Lr)]
    vals = torch.zeros(1, 1, 64, 128, dtype=torch.float16).pin_memory()          # every value row reads row < 64
    vd = torch.zeros(1, 1, 8, 128, dtype=torch.float16, device=dev)
    y = torch.zeros(Lr, 1, 4, 128, dtype=torch.float32, device=dev)
    ocs = []
    for l in range(Lr):
        B.hca_quantize_keys(shape, kc[l], keys[l].cuda(), n, [0])
        pos[l].zero_()                                                         # all slots share value row 0
        oc = oracle.Cache(R, cap, 128, 4, 32)
        oracle.quantize(oc, keys[l].numpy().reshape(R, n, 128))
        ocs.append(oc)
    streams = [torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()]
    dsc = B.hca_pipeline_desc()
    dsc.stream_scan, dsc.stream_topk, dsc.stream_gather, dsc.stream_attend = (s_.cuda_stream for s_ in streams)
    wsb = B.hca_workspace_bytes(shape, k, 1)
    keep = []
    wsel = [torch.zeros(wsb, dtype=torch.uint8, device=dev) for _ in range(3)]
    for i in range(3):
        dsc.ws_select[i] = wsel[i].data_ptr()
    dsc.n_sel, dsc.fused_select, dsc.n_pipe, dsc.dual_scan = 3, 1, 4, 2
    sets = []
    for i in range(4):
        a = torch.full((1, 1, k), -3, dtype=torch.int32, device=dev)
        b_ = torch.zeros(1, 1, dtype=torch.int32, device=dev)
        c_ = torch.zeros(wsb, dtype=torch.uint8, device=dev)
        sets.append((a, b_, c_))
        dsc.idx[i], dsc.count[i], dsc.ws_attend[i] = a.data_ptr(), b_.data_ptr(), c_.data_ptr()
    wt = torch.zeros(wsb, dtype=torch.uint8, device=dev)
    dsc.ws_topk = wt.data_ptr()
    lidx = torch.full((Lr, k), -3, dtype=torch.int32, device=dev)
    lcnt = torch.zeros(Lr, 1, dtype=torch.int32, device=dev)
    if own_idx:
        dsc.layer_idx, dsc.layer_count, dsc.layer_idx_stride = lidx.data_ptr(), lcnt.data_ptr(), k
    pl = B.hca_pipeline_create(shape, Lr, dsc, 0)
    for i in range(2):
        B.hca_score_topk_monitor(shape, wsel[i], None, True)
    layers = (B.hca_layer * Lr)()
    k_new = torch.zeros(1, 1, 1, 128, dtype=torch.float16, device=dev)         # the appended token: a zero key
    qd = q.cuda()
    for l in range(Lr):
        layers[l].kcache, layers[l].acc, layers[l].pos = kc[l].data_ptr(), acc[l].data_ptr(), pos[l].data_ptr()
        layers[l].v_host, layers[l].v_hbm, layers[l].y = vals.data_ptr(), vd.data_ptr(), y[l].data_ptr()
        layers[l].k_new, layers[l].q = k_new.data_ptr(), qd.data_ptr()
    nres = (C.c_int64 * Lr)(n, n)
    torch.cuda.synchronize()
    B.hca_pipeline_step(pl, layers, nres, 0, k, 64, 64, 8, 0.0884, None, 0, -1)
    torch.cuda.synchronize()
    mon = torch.zeros(2, R, 4, dtype=torch.int32, device=dev)
    for i in range(2):
        B.hca_score_topk_monitor(shape, wsel[i], mon[i], False)
    torch.cuda.synchronize()
    for l in range(Lr):
        oracle.quantize(ocs[l], np.zeros((R, 1, 128), np.float16))
        sel, _ = oracle.score(ocs[l], q.numpy().reshape(-1, 128), want_z=False)
        oidx, ocount = oracle.topk(sel, ocs[l].n, k)
        gi = (lidx[l] if own_idx else sets[l][0].view(-1)).cpu().numpy()
        assert np.array_equal(gi, oidx[0]), f"layer {l}: index sets differ"
    m = mon.cpu().numpy()
    assert m[0, 0, 0] == 1 and m[0, 0, 3] == 1, "layer 0 should have needed the second scan"
    assert m[1, 0, 0] == 1 and m[1, 0, 3] == 0
    B.hca_pipeline_destroy(pl)
