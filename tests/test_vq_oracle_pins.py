"""Pins for the codebook half of the CPU oracle (oracle/hca_vq_oracle.c): every check compares it with
something other than itself - numpy brute force in fp64, Eq. 1 evaluated exactly, planted clusters,
the k-means objective's monotone decrease, the paper's printed footprint ratios.  CPU only."""
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
D = 128


def _golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_closed_forms.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def _codebook(rng, n_kv, g, c):
    return rng.standard_normal((n_kv, g, c, D // g)).astype(np.float32)


def _keys(rng, R, T):
    return rng.standard_normal((R, T, D)).astype(np.float16)


# ---------------------------------------------------------------- assign ---

@pytest.mark.parametrize("g,c", [(32, 256), (64, 128), (32, 17), (16, 300)])
def test_assign_is_the_nearest_centroid(oracle, g, c):
    """Sec. 3.2: each sub-vector is represented by its nearest centroid.  Brute force in fp64."""
    rng = np.random.default_rng(g * 1000 + c)
    R, T, n_kv = 4, 50, 2
    Cb = _codebook(rng, n_kv, g, c)
    K = _keys(rng, R, T)
    vc = oracle.VQCache(R, T + 3, Cb)
    oracle.vq_assign(vc, K)
    assert np.array_equal(vc.n, [T] * R)
    x = K.astype(np.float64).reshape(R, T, g, 1, D // g)
    agree = 0
    for r in range(R):
        d = ((x[r] - Cb[r % n_kv].astype(np.float64)[None]) ** 2).sum(-1)       # [T, g, c]
        best = d.argmin(-1)
        got = vc.P[r, :T].astype(np.int64)
        agree += (best == got).sum()
        # where fp32 and fp64 disagree the two distances must be equal to fp32 rounding
        dg = np.take_along_axis(d, got[..., None], -1)[..., 0]
        assert np.all(dg <= d.min(-1) * (1 + 1e-5) + 1e-12)
    assert agree >= 0.999 * R * T * g
    assert np.all(vc.P[:, T:] == 0)                                              # nothing past n


def test_assign_uses_each_rows_own_codebook_and_breaks_ties_low(oracle):
    rng = np.random.default_rng(3)
    g, c, n_kv = 32, 8, 2
    Cb = _codebook(rng, n_kv, g, c)
    Cb[0, :, 5] = Cb[0, :, 2]                       # duplicate centroid: index 2 must win over 5
    Cb = Cb.astype(np.float16).astype(np.float32)   # centroids representable in fp16: distance exactly 0
    # row r's key is exactly centroid 2 (KV head 0) or centroid 6 (KV head 1) of every group
    K = np.stack([Cb[r % n_kv, :, 2 if r % n_kv == 0 else 6].reshape(1, -1) for r in range(4)]).astype(np.float16)
    vc = oracle.VQCache(4, 2, Cb)
    oracle.vq_assign(vc, K)
    assert np.all(vc.P[0, 0] == 2) and np.all(vc.P[2, 0] == 2)
    assert np.all(vc.P[1, 0] == 6) and np.all(vc.P[3, 0] == 6)


def test_append_continues_at_n(oracle):
    rng = np.random.default_rng(4)
    Cb = _codebook(rng, 1, 32, 16)
    K = _keys(rng, 2, 9)
    a = oracle.VQCache(2, 12, Cb)
    oracle.vq_assign(a, K)
    b = oracle.VQCache(2, 12, Cb)
    oracle.vq_assign(b, K[:, :4])
    oracle.vq_assign(b, K[:, 4:])
    assert np.array_equal(a.P, b.P) and np.array_equal(b.n, [9, 9])


# ------------------------------------------------------- table and scores ---

@pytest.mark.parametrize("g,c,G", [(32, 256, 4), (64, 128, 4), (32, 40, 1), (8, 5, 2)])
def test_table_and_eq3_equal_q_dot_quantised_keys(oracle, g, c, G):
    """T = qbar . C and z~_j = sum_i T[i, P_ji] (Eq. 3) must equal q . Q(K)_j computed directly in fp64
    from the centroids the indices stand for; the selection score is the max over the row's heads."""
    rng = np.random.default_rng(g + c + G)
    R, n, n_kv = 4, 70, 2
    Cb = _codebook(rng, n_kv, g, c)
    vc = oracle.VQCache(R, n + 2, Cb)
    oracle.vq_assign(vc, _keys(rng, R, n))
    q = rng.standard_normal((R * G, D)).astype(np.float16)
    T = oracle.vq_lut(vc, q)
    q64 = q.astype(np.float64)
    for hq in range(R * G):
        ref = np.einsum("id,icd->ic", q64[hq].reshape(g, D // g), Cb[(hq // G) % n_kv].astype(np.float64))
        assert np.allclose(T[hq], ref, rtol=1e-5, atol=1e-5)
    khat = oracle.vq_dequant(vc).astype(np.float64)                  # independent of T
    for r in range(R):                                               # dequant itself against numpy indexing
        ref = Cb[r % n_kv][np.arange(g)[None, :], vc.P[r, :n].astype(np.int64)].reshape(n, D)
        assert np.array_equal(khat[r, :n], ref)
    sel, z = oracle.vq_score(vc, T)
    for hq in range(R * G):
        ref = khat[hq // G, :n] @ q64[hq]
        assert np.allclose(z[hq, :n], ref, rtol=1e-4, atol=2e-4)
    assert np.array_equal(sel[:, :n], z.reshape(R, G, -1).max(1)[:, :n])
    assert np.all(sel[:, n:] == 0)


def test_eq3_sum_is_exact_on_the_tables_grid(oracle):
    """Eq. 3 as the oracle evaluates it: the sum over the groups is exact on a power-of-two grid that keeps 24 bits
    of the table's largest entry.  Pins: (a) a table of small integers is summed without any rounding (plain
    integer arithmetic is the reference); (b) the order of the groups does not matter, bit for bit; (c) against
    the fp64 sum of the fp32 table the error stays within the grid's half steps plus one final rounding;
    (d) an all-zero table scores 0 and a table with an infinity or a NaN is refused."""
    rng = np.random.default_rng(5)
    R, G, g, c, n = 2, 4, 32, 64, 300
    vc = oracle.VQCache(R, n, np.zeros((1, g, c, D // g), np.float32))
    vc.P[:, :n] = rng.integers(0, c, size=(R, n, g)).astype(np.uint16)
    vc.n[:] = n
    # (a) integers up to 2^20 in magnitude: 32 of them sum below 2^25, every partial result is an integer
    Ti = rng.integers(-(1 << 20), 1 << 20, size=(R * G, g, c)).astype(np.float32)
    _, z = oracle.vq_score(vc, Ti)
    for hq in range(R * G):
        ref = Ti[hq].astype(np.int64)[np.arange(g)[None, :], vc.P[hq // G, :n].astype(np.int64)].sum(1)
        assert np.array_equal(z[hq, :n].astype(np.float64), ref.astype(np.float32).astype(np.float64))
    # (b) + (c) Gaussian tables with entries over many binades
    T = (rng.standard_normal((R * G, g, c)) * np.exp2(rng.integers(-12, 3, size=(R * G, g, c)))).astype(np.float32)
    sel, z = oracle.vq_score(vc, T)
    perm = rng.permutation(g)
    vp = oracle.VQCache(R, n, np.zeros((1, g, c, D // g), np.float32))
    vp.P[:, :n] = vc.P[:, :n][:, :, perm]
    vp.n[:] = n
    sel_p, z_p = oracle.vq_score(vp, np.ascontiguousarray(T[:, perm]))
    assert np.array_equal(z.view(np.uint32), z_p.view(np.uint32))
    assert np.array_equal(sel.view(np.uint32), sel_p.view(np.uint32))
    Tfx, sexp = oracle.vq_lut_fx(T)
    for hq in range(R * G):
        amax = float(np.abs(T[hq]).max())
        assert 2.0 ** 23 <= amax * 2.0 ** int(sexp[hq]) < 2.0 ** 24          # 24 bits for the largest entry
        assert np.abs(Tfx[hq].astype(np.float64) - T[hq].astype(np.float64) * 2.0 ** int(sexp[hq])).max() <= 0.5
        ref = T[hq].astype(np.float64)[np.arange(g)[None, :], vc.P[hq // G, :n].astype(np.int64)].sum(1)
        bound = g * 0.5 * 2.0 ** -int(sexp[hq]) + np.abs(ref) * 2.0 ** -23
        assert np.all(np.abs(z[hq, :n].astype(np.float64) - ref) <= bound)
    # the grid follows the largest magnitude, whatever its sign: negating the table negates every score exactly
    Ta = np.abs(T)
    _, za = oracle.vq_score(vc, Ta)
    _, zn = oracle.vq_score(vc, -Ta)
    assert np.array_equal(zn.view(np.uint32), (-za).view(np.uint32))
    assert np.array_equal(oracle.vq_lut_fx(-Ta)[1], oracle.vq_lut_fx(Ta)[1])
    # a table far below the normal range of the sums still resolves its entries
    Tt = (T * np.float32(2.0 ** -100)).astype(np.float32)
    _, zt = oracle.vq_score(vc, Tt)
    assert np.array_equal(zt.astype(np.float64), z.astype(np.float64) * 2.0 ** -100)
    # (d)
    sel0, z0 = oracle.vq_score(vc, np.zeros_like(T))
    assert np.all(z0 == 0) and np.all(sel0 == 0)
    for bad in (np.inf, -np.inf, np.nan):
        Tb = T.copy()
        Tb[3, 5, 7] = bad
        with pytest.raises(Exception):
            oracle.vq_score(vc, Tb)


def test_plain_eq3_against_numpy_and_the_grid_form_against_it(oracle):
    """hco_vq_score_plain is Eq. 3 as written (fp64 sum of the fp32 table entries a token's indices select):
    checked against numpy indexing.  The grid form (hco_vq_score) stays within g half steps of the grid plus one
    final fp32 rounding of it, for Gaussian tables and for tables spread over many binades."""
    rng = np.random.default_rng(17)
    R, G, g, c, n = 3, 2, 32, 300, 200
    vc = oracle.VQCache(R, n + 4, np.zeros((1, g, c, D // g), np.float32))
    vc.P[:, :n] = rng.integers(0, c, size=(R, n, g)).astype(np.uint16)
    vc.n[:] = [n, n - 7, 0]
    for spread in (0, 10):
        T = (rng.standard_normal((R * G, g, c)) * np.exp2(rng.integers(-spread, 1, size=(R * G, g, c)))).astype(np.float32)
        zp = oracle.vq_score_plain(vc, T)
        _, z = oracle.vq_score(vc, T)
        _, sexp = oracle.vq_lut_fx(T)
        for hq in range(R * G):
            nr = int(vc.n[hq // G])
            ref = T[hq].astype(np.float64)[np.arange(g)[None, :], vc.P[hq // G, :nr].astype(np.int64)].sum(1)
            assert np.allclose(zp[hq, :nr], ref, rtol=1e-13, atol=1e-13)
            assert np.all(zp[hq, nr:] == 0)
            bound = g * 0.5 * 2.0 ** -int(sexp[hq]) + np.abs(ref) * 2.0 ** -23
            assert np.all(np.abs(z[hq, :nr].astype(np.float64) - zp[hq, :nr]) <= bound)
    with pytest.raises(Exception):                                   # an index beyond the codebook is refused
        vc.P[0, 0, 0] = c
        oracle.vq_score_plain(vc, T)


def test_codebook_holding_every_subvector_reproduces_eq1(oracle):
    """With one centroid per distinct sub-vector the compressor is the identity, so the scores are the
    exact q . K and selecting every token gives standard attention (Eq. 1)."""
    rng = np.random.default_rng(11)
    n, g = 48, 32
    K = _keys(rng, 1, n)
    V = rng.standard_normal((1, n, D)).astype(np.float16)
    q = rng.standard_normal((1, D)).astype(np.float16)
    Cb = K[0].astype(np.float32).reshape(n, g, D // g).transpose(1, 0, 2)[None].copy()   # [1, g, n, dbar]
    vc = oracle.VQCache(1, n, Cb)
    oracle.vq_assign(vc, K)
    assert np.array_equal(oracle.vq_dequant(vc)[0], K[0].astype(np.float32))
    T = oracle.vq_lut(vc, q)
    sel, z = oracle.vq_score(vc, T)
    exact = K[0].astype(np.float64) @ q[0].astype(np.float64)
    assert np.allclose(z[0], exact, rtol=1e-5, atol=1e-4)
    idx, count = oracle.topk(sel, vc.n, n)
    pos = np.arange(n, dtype=np.int32)[None].copy()
    sm = 1.0 / np.sqrt(D)
    y, _ = oracle.vq_attend(vc, T, idx, count, pos, V, sm)
    ref = oracle.attention_exact(q[0], K[0], V[0], sm)
    assert np.allclose(y[0], ref, rtol=1e-4, atol=1e-5)


def test_attend_is_softmax_over_the_selected_set(oracle):
    rng = np.random.default_rng(12)
    R, G, g, c, n, k = 2, 4, 32, 64, 200, 37
    Cb = _codebook(rng, 2, g, c)
    vc = oracle.VQCache(R, n + 4, Cb)
    oracle.vq_assign(vc, _keys(rng, R, n))
    q = (3 * rng.standard_normal((R * G, D))).astype(np.float16)
    V = rng.standard_normal((R, n + 4, D)).astype(np.float16)
    T = oracle.vq_lut(vc, q)
    sel, z = oracle.vq_score(vc, T)
    idx, count = oracle.topk(sel, vc.n, k)
    pos = np.tile(rng.permutation(n + 4).astype(np.int32), (R, 1))
    acc = np.full((R, n + 4), 0.5, np.float32)
    sm = 0.25
    y, w = oracle.vq_attend(vc, T, idx, count, pos, V, sm, acc=acc, want_w=True)
    acc_ref = np.full((R, n + 4), 0.5, np.float64)
    for hq in range(R * G):
        r = hq // G
        l = z[hq, idx[r]].astype(np.float64) * sm
        p = np.exp(l - l.max())
        p /= p.sum()
        assert abs(w[hq].sum() - 1) < 1e-5 and np.allclose(w[hq], p, rtol=1e-5, atol=1e-9)
        ref = p @ V[r, pos[r, idx[r]]].astype(np.float64)
        assert np.allclose(y[hq], ref, rtol=1e-5, atol=1e-6)
        acc_ref[r, idx[r]] += np.maximum(p.astype(np.float32), np.float32(1e-30))
    assert np.allclose(acc, acc_ref, rtol=1e-5)
    # k = 1: the output is the value row of the best token
    idx1, count1 = oracle.topk(sel, vc.n, 1)
    y1, _ = oracle.vq_attend(vc, T, idx1, count1, pos, V, sm)
    for hq in range(R * G):
        r = hq // G
        assert np.array_equal(y1[hq], V[r, pos[r, idx1[r, 0]]].astype(np.float32))


def test_attend_survives_huge_logits_and_floors_the_accumulated_weight(oracle):
    """Logits far beyond exp's range: the softmax must subtract the maximum, and a selected token whose
    weight underflows still leaves a positive mark (1e-30 per head) in the accumulated scores."""
    rng = np.random.default_rng(13)
    R, G, g, c, n, k = 1, 2, 32, 32, 60, 60
    Cb = (20 * _codebook(rng, 1, g, c)).astype(np.float32)
    vc = oracle.VQCache(R, n, Cb)
    oracle.vq_assign(vc, (20 * rng.standard_normal((R, n, D))).astype(np.float16))
    q = (30 * rng.standard_normal((R * G, D))).astype(np.float16)
    V = rng.standard_normal((R, n, D)).astype(np.float16)
    T = oracle.vq_lut(vc, q)
    sel, z = oracle.vq_score(vc, T)
    assert np.abs(z).max() > 2000                                  # exp(z) alone would overflow
    idx, count = oracle.topk(sel, vc.n, k)
    pos = np.arange(n, dtype=np.int32)[None].copy()
    acc = np.zeros((R, n), np.float32)
    y, w = oracle.vq_attend(vc, T, idx, count, pos, V, 1.0, acc=acc, want_w=True)
    assert np.all(np.isfinite(y))
    for hq in range(G):
        l = z[hq, idx[0]].astype(np.float64)
        p = np.exp(l - l.max())
        p /= p.sum()
        assert np.allclose(y[hq], p @ V[0, idx[0]].astype(np.float64), rtol=1e-5, atol=1e-6)
    assert (w == 0).sum() > 0                                      # some weights did underflow
    assert np.all(acc[0, idx[0]] > 0)
    dead = (w == 0).all(0)                                         # underflowed for both heads
    assert dead.any() and np.allclose(acc[0, idx[0]][dead], 2e-30, rtol=1e-6)


# --------------------------------------------------------------- trainer ---

def test_trainer_recovers_planted_clusters_and_objective_decreases(oracle):
    """Sec. 3.1: per group, k-means over the validation sub-vectors.  Well separated planted clusters,
    one seed per cluster: the centroids must land on the cluster means."""
    rng = np.random.default_rng(21)
    g, c, per = 32, 12, 40
    dbar = D // g
    centres = (4 * rng.standard_normal((g, c, dbar))).astype(np.float32)
    label = np.stack([rng.permutation(np.repeat(np.arange(c), per)) for _ in range(g)])      # [g, nval]
    nval = c * per
    X = centres[np.arange(g)[:, None], label] + 0.01 * rng.standard_normal((g, nval, dbar))
    kval = X.transpose(1, 0, 2).reshape(nval, D).astype(np.float16)
    init = np.stack([[int(np.flatnonzero(label[i] == cc)[0]) for cc in range(c)] for i in range(g)]).astype(np.int32)
    Cb, iner = oracle.vq_train(kval, g, c, init, 5)
    x16 = kval.astype(np.float64).reshape(nval, g, dbar)
    for i in range(g):
        for cc in range(c):
            mean = x16[label[i] == cc, i].mean(0)
            assert np.allclose(Cb[i, cc], mean, atol=1e-5)
    assert np.all(np.diff(iner) <= 1e-9 * iner[0])
    # objective of the final codebook, recomputed by brute force
    d = ((x16[:, :, None, :] - Cb.astype(np.float64)[None]) ** 2).sum(-1).min(-1).sum()
    assert abs(iner[-1] - d) <= 1e-4 * d


def test_trainer_objective_is_monotone_on_gaussian_keys(oracle):
    rng = np.random.default_rng(22)
    nval, g, c = 1500, 64, 32
    kval = rng.standard_normal((nval, D)).astype(np.float16)
    init = np.stack([rng.choice(nval, c, replace=False) for _ in range(g)]).astype(np.int32)
    Cb0, i0 = oracle.vq_train(kval, g, c, init, 0)
    assert np.array_equal(Cb0, kval.astype(np.float32).reshape(nval, g, -1)[init, np.arange(g)[:, None]])
    Cb, iner = oracle.vq_train(kval, g, c, init, 8)
    assert iner[0] == i0[0] and np.all(np.diff(iner) <= 0) and iner[-1] < 0.8 * iner[0]
    # every centroid with members is the mean of its members under the final assignment's predecessor:
    # one more Lloyd step done in numpy from Cb must not raise the objective either
    x = kval.astype(np.float64).reshape(nval, g, 1, -1)
    d = ((x - Cb.astype(np.float64)[None]) ** 2).sum(-1)
    assert abs(d.min(-1).sum() - iner[-1]) <= 1e-5 * iner[-1]


def test_trainer_empty_cluster_keeps_its_centroid(oracle):
    """Only two distinct validation vectors, three centroids, two of them seeded on the same vector: the
    later twin never wins a tie, has no members in any round and must keep its seed (not 0/0)."""
    rng = np.random.default_rng(23)
    g, c = 32, 3
    A, B = rng.standard_normal((2, D)).astype(np.float16)
    kval = np.stack([A] * 30 + [B] * 34)
    init = np.tile(np.array([0, 5, 40], np.int32), (g, 1))
    Cb, iner = oracle.vq_train(kval, g, c, init, 3)
    assert np.array_equal(Cb[:, 0], A.astype(np.float32).reshape(g, -1))
    assert np.array_equal(Cb[:, 1], A.astype(np.float32).reshape(g, -1))
    assert np.array_equal(Cb[:, 2], B.astype(np.float32).reshape(g, -1))
    assert np.all(iner == 0)


def test_shared_codebook_is_trained_on_the_pooled_subvectors(oracle):
    """The variant in which the groups share one codebook (Table 4b's unstarred rows)."""
    rng = np.random.default_rng(24)
    nval, g, c = 300, 32, 16
    dbar = D // g
    kval = rng.standard_normal((nval, D)).astype(np.float16)
    init = rng.choice(nval * g, c, replace=False).astype(np.int32)
    Cb, iner = oracle.vq_train(kval, g, c, init, 4, shared=True)
    assert all(np.array_equal(Cb[0], Cb[i]) for i in range(g))
    # the same thing as a single-group problem on the pooled vectors, padded to one group of width dbar:
    # the pooled problem by brute-force Lloyd in numpy
    x = kval.reshape(nval * g, dbar).astype(np.float32)
    cen = x[init].copy()
    for _ in range(4):
        d = ((x[:, None, :].astype(np.float64) - cen[None].astype(np.float64)) ** 2).sum(-1)
        a = d.argmin(1)
        for cc in range(c):
            if np.any(a == cc):
                cen[cc] = x[a == cc].astype(np.float64).mean(0).astype(np.float32)
    assert np.allclose(Cb[0], cen, atol=1e-5)
    assert np.all(np.diff(iner) <= 0)


# ------------------------------------------------------------- footprint ---

def test_index_matrix_footprint_matches_the_papers_ratios(oracle):
    """Sec. 3.3 / Table 1a: with 16-bit indices P takes g/d of the fp16 key matrix: 1/2 at g = 64, 1/4 at g = 32."""
    gold = _golden()
    for g, key in ((64, "k_budget_g64"), (32, "k_budget_g32")):
        vc = oracle.VQCache(3, 1000, np.zeros((1, g, 4, D // g), np.float32))
        assert vc.P.itemsize * 8 == gold["index_bits"]
        assert vc.P.nbytes / (3 * 1000 * gold["head_dim"] * 2) == gold[key]


# ----------------------------------------------------------------- evict ---

def _brute_evict(acc, n, M, Rp):
    """Keep-set by a full stable sort: newest Rp slots plus the M - Rp highest acc among the others
    (ties to the lower slot), in ascending slot order."""
    if n <= M:
        return list(range(n))
    free = n - Rp
    order = sorted(range(free), key=lambda j: (-float(acc[j]), j))[:M - Rp]
    return sorted(order) + list(range(free, n))


@pytest.mark.parametrize("n,M,Rp", [(64, 48, 0), (64, 48, 8), (50, 64, 4), (64, 1, 1), (33, 32, 32), (64, 17, 3)])
def test_vq_evict_brute_force(oracle, n, M, Rp):
    rng = np.random.default_rng(n * 100 + M + Rp)
    R, g, cap = 3, 32, 70
    vc = oracle.VQCache(R, cap, _codebook(rng, 1, g, 16))
    oracle.vq_assign(vc, _keys(rng, R, n))
    P0 = vc.P.copy()
    acc = np.zeros((R, cap), np.float32)
    acc[:, :n] = rng.integers(0, 6, (R, n)).astype(np.float32) * 0.25      # many ties
    acc[2, :n] = rng.standard_normal(n).astype(np.float32) ** 2
    pos = np.zeros((R, cap), np.int32)
    pos[:, :n] = rng.permutation(1000)[:n].astype(np.int32)
    acc0, pos0 = acc.copy(), pos.copy()
    kept = oracle.vq_evict(vc, acc, pos, M, Rp)
    for r in range(R):
        ref = _brute_evict(acc0[r], n, M, Rp)
        m = len(ref)
        assert vc.n[r] == m == min(n, M)
        assert list(kept[r, :m]) == ref and np.all(kept[r, m:] == -1)
        assert np.array_equal(vc.P[r, :m], P0[r, ref])
        assert np.array_equal(acc[r, :m], acc0[r, ref]) and np.array_equal(pos[r, :m], pos0[r, ref])
    snap = vc.P.copy()
    oracle.vq_evict(vc, acc, pos, M, Rp)                                    # idempotent once n <= M
    assert np.array_equal(vc.P, snap)
