"""Full-size GPU parity in the launch configuration bench.py times: one layer of BASELINE config 4
(1 Mi tokens, 4-bit / group 32, top-k 4096) and one layer of config 5 (4 Mi tokens, 2-bit / group 64,
top-k 8192, eviction to 2 Mi), every output compared with the oracle run on the same inputs."""
import numpy as np
import pytest
import torch

import synth_inputs as S

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _rows(t):
    a = t.detach().cpu().numpy()
    return a.reshape(a.shape[0] * a.shape[1], *a.shape[2:])


def _rel_err(y, ref):
    return float(np.max(np.abs(y - ref).max(-1) / np.maximum(np.abs(ref).max(-1), 1e-30)))


def _decode_step(B, st, q, v_host, n_host, v_hbm, side):
    """score -> top-k -> gather on the side stream -> attend, as bench.py issues them."""
    main = torch.cuda.current_stream()
    st.score(q)
    st.topk(st.k_max)
    done = torch.cuda.Event()
    done.record(main)
    side.wait_event(done)
    hs = v_host.shape[2]
    B.hca_gather_values(st.shape, st.idx, st.count, st.k, st.pos, v_host, hs, n_host, v_hbm,
                        0 if v_hbm is None else v_hbm.shape[2], st.ws, side)
    g = torch.cuda.Event()
    g.record(side)
    main.wait_event(g)
    B.hca_attend_gathered(st.shape, st.kcache, q, st.idx, st.count, st.k, st.sm_scale, st.y, st.acc, st.ws)


@pytest.mark.parametrize("cfg", [4, 5])
def test_one_layer_at_full_size(oracle, cfg):
    from paper_2507_19823_amd import binding as B
    from paper_2507_19823_amd.session import LayerState
    w = S.CONFIGS[cfg]
    R, n = w.batch * w.n_kv_heads, w.n
    d = S.make_layer(w, 0, device="cuda")
    cap = n + 32
    M = w.evict_keep if cfg == 5 else 0
    st = LayerState(w.batch, w.n_q_heads, w.n_kv_heads, cap, w.bits, w.group, k_max=w.k, m_max=max(M, 1))
    # bulk quantise in chunks, as a prefill would hand the keys over
    step = 1 << 20
    for a in range(0, n, step):
        st.quantize(d["keys"][:, :, a:a + step].contiguous())
    v_host = torch.empty(w.batch, w.n_kv_heads, n, 128, dtype=torch.float16, pin_memory=True)
    v_host.copy_(d["values"])
    q = d["q"]
    side = torch.cuda.Stream()
    _decode_step(B, st, q, v_host, n, None, side)
    torch.cuda.synchronize()

    keys = d["keys"].cpu()
    oc = oracle.Cache(R, cap, 128, w.bits, w.group)
    oracle.quantize(oc, _rows(keys))
    del keys
    q16 = q.cpu().numpy().reshape(-1, 128)
    sel, _ = oracle.score(oc, q16, want_z=False)
    assert np.array_equal(_rows(st.sel)[:, :n], sel[:, :n]), "selection scores differ"
    idx, count = oracle.topk(sel, oc.n, w.k)
    assert np.array_equal(_rows(st.idx), idx), "top-k index sets differ"
    assert np.array_equal(st.count.cpu().numpy().reshape(-1), count)
    pos = np.tile(np.arange(cap, dtype=np.int32), (R, 1))
    acc = np.zeros((R, cap), np.float32)
    V = v_host.numpy().reshape(R, n, 128)
    y, _ = oracle.attend(oc, q16, idx, count, pos, V, st.sm_scale, acc=acc)
    assert _rel_err(st.y.cpu().numpy().reshape(-1, 128), y) <= TOL
    assert np.array_equal(_rows(st.acc) > 0, acc > 0)
    assert np.allclose(_rows(st.acc), acc, rtol=1e-4, atol=1e-7)

    if M:
        # fewer than M slots have a non-zero accumulated score, so ties decide most of the keep-set
        assert int((acc > 0).sum(1).max()) < M
        kept = torch.full((w.batch, w.n_kv_heads, M), -1, dtype=torch.int32, device="cuda")
        st.evict(M, 0, kept)
        torch.cuda.synchronize()
        okept = oracle.evict(oc, acc, pos, M, 0)
        assert np.array_equal(_rows(kept), okept), "eviction keep-sets differ"
        assert np.array_equal(_rows(st.pos)[:, :M], pos[:, :M])
        # a second decode step on the compacted cache (codes moved by the GPU, by the oracle on its side)
        _, _, q2 = S.make_step(w, 0, 0)
        _decode_step(B, st, q2.cuda(), v_host, n, None, side)
        torch.cuda.synchronize()
        q16 = q2.numpy().reshape(-1, 128)
        sel, _ = oracle.score(oc, q16, want_z=False)
        assert np.array_equal(_rows(st.sel)[:, :M], sel[:, :M])
        idx, count = oracle.topk(sel, oc.n, w.k)
        assert np.array_equal(_rows(st.idx), idx)
        y, _ = oracle.attend(oc, q16, idx, count, pos, V, st.sm_scale)
        assert _rel_err(st.y.cpu().numpy().reshape(-1, 128), y) <= TOL
