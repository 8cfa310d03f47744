"""GPU parity of the codebook form of the key path (hca_vq_*) against the oracle, through the C ABI:
indices, tables, scores and top-k sets bit for bit, attention output within 2e-3."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
TOL = 2e-3
D = 128


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2507_19823_amd import binding
    binding.lib()
    return binding


def _rel_err(y, ref):
    return float(np.max(np.abs(y - ref).max(-1) / np.maximum(np.abs(ref).max(-1), 1e-30)))


def _codebook(oracle, rng, keys, n_kv, g, c, iters=3):
    """One trained codebook per KV head (oracle-side trainer; the GPU path only consumes the result).  Beyond 256
    centroids the codebook is drawn instead (training that many centroids in the plain oracle takes minutes and
    adds nothing to a parity check)."""
    if c > 256:
        return (rng.standard_normal((n_kv, g, c, D // g)) * 1.5).astype(np.float32)
    out = []
    for h in range(n_kv):
        kval = keys[0, h, :min(keys.shape[2], 2000)]
        init = np.stack([rng.choice(kval.shape[0], c, replace=kval.shape[0] < c) for _ in range(g)]).astype(np.int32)
        out.append(oracle.vq_train(kval, g, c, init, iters)[0])
    return np.stack(out)


class _State:
    def __init__(self, B, batch, hq, hkv, cap, g, c, cen, k):
        self.B, self.batch, self.hq, self.hkv, self.cap, self.g, self.c, self.k = B, batch, hq, hkv, cap, g, c, k
        self.shape = B.make_shape(batch, hq, hkv, cap)
        self.cen = torch.from_numpy(cen).cuda()
        self.cb = B.make_codebook(g, c, self.cen)
        self.wide = c > 256 or g * c * (hq // hkv) > 32768          # 16-bit indices, table read through L2
        self.P = torch.full((B.hca_vq_pcache_bytes(self.shape, self.cb),), 0xEE, dtype=torch.uint8, device="cuda")
        tiled = -(-cap // 16384) * 16384                              # the wide form stores whole tiles of 16 Ki slots
        assert self.P.numel() == batch * hkv * (tiled * g * 2 if self.wide else cap * g)
        self.lut = torch.zeros(B.hca_vq_lut_bytes(self.shape, self.cb) // 4, dtype=torch.float32, device="cuda")
        self.sel = torch.full((batch, hkv, cap), -7.0, dtype=torch.float32, device="cuda")
        self.z = torch.full((batch, hq, cap), -7.0, dtype=torch.float32, device="cuda")
        self.acc = torch.full((batch, hkv, cap), 9.0, dtype=torch.float32, device="cuda")
        self.pos = torch.full((batch, hkv, cap), -1, dtype=torch.int32, device="cuda")
        self.idx = torch.full((batch, hkv, k), -9, dtype=torch.int32, device="cuda")
        self.count = torch.zeros(batch, hkv, dtype=torch.int32, device="cuda")
        self.ws = torch.empty(B.hca_vq_workspace_bytes(self.shape, self.cb, k, 1), dtype=torch.uint8, device="cuda")
        self.y = torch.zeros(batch, hq, D, dtype=torch.float32, device="cuda")
        self.n = [0] * batch

    def assign(self, k_new, row0=None):
        T = k_new.shape[2]
        self.B.hca_vq_assign(self.shape, self.cb, self.P, k_new.contiguous().cuda(), T, self.n, self.acc, self.pos,
                             self.n if row0 is None else row0)
        self.n = [x + T for x in self.n]

    def P_rows(self, P=None, n=None):
        """Index rows in canonical order [R, cap, g] (the library stores a slot's byte indices rotated by its slot
        number); slots at or beyond n read 0xEE (0xEEEE in the wide form)."""
        out = torch.full((self.batch * self.hkv, self.cap, self.g * (2 if self.wide else 1)), 0xEE, dtype=torch.uint8,
                         device="cuda")
        self.B.hca_vq_export_pcache(self.shape, self.cb, self.P if P is None else P, self.n if n is None else n, out)
        a = out.cpu().numpy()
        return a.view(np.uint16) if self.wide else a

    def fill(self):
        return 0xEEEE if self.wide else 0xEE

    def idx_dtype(self):
        return np.uint16 if self.wide else np.uint8

    def table(self):
        """(T fp32 [R*G, g, c], exponents int32 [R*G]) from the library's lut buffer."""
        R, G = self.batch * self.hkv, self.hq // self.hkv
        flat = self.lut.cpu().numpy()
        if self.wide:                                                 # [R, g, c, G]
            T = flat[:R * self.c * self.g * G].reshape(R, self.g, self.c, G).transpose(0, 3, 1, 2).reshape(R * G, self.g, self.c)
        else:                                                         # [R, c, g, G]
            T = flat[:R * self.c * self.g * G].reshape(R, self.c, self.g, G).transpose(0, 3, 2, 1).reshape(R * G, self.g, self.c)
        sexp = flat[R * self.g * (self.c * G + 4):].view(np.int32).reshape(R, 4)[:, :G].reshape(R * G)
        return np.ascontiguousarray(T), sexp


@pytest.mark.parametrize("g,c,G,hkv,batch", [(32, 256, 4, 2, 2), (64, 128, 4, 2, 1), (32, 17, 2, 3, 1), (64, 256, 1, 2, 2),
                                             (32, 1, 4, 1, 1), (32, 1024, 4, 2, 1), (32, 8192, 4, 1, 1), (64, 256, 4, 2, 1),
                                             (64, 2048, 2, 1, 2), (32, 300, 1, 2, 1)])
def test_assign_table_scores_bit_exact(B, oracle, g, c, G, hkv, batch):
    rng = np.random.default_rng(g * 7 + c + G)
    n, cap = 2500, 2600
    keys = rng.standard_normal((batch, hkv, n, D)).astype(np.float16)
    keys[:, :, :, 5] *= 8
    cen = _codebook(oracle, rng, keys, hkv, g, c)
    R = batch * hkv
    st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, 64)
    # bulk, then ragged appends: 37 tokens at once, then single tokens
    kt = torch.from_numpy(keys)
    st.assign(kt[:, :, :2400])
    st.assign(kt[:, :, 2400:2437])
    for t in range(2437, 2440):
        st.assign(kt[:, :, t:t + 1])
    torch.cuda.synchronize()
    n_used = 2440
    oc = oracle.VQCache(R, cap, cen)
    oracle.vq_assign(oc, keys.reshape(R, n, D)[:, :n_used])
    Pg = st.P_rows()
    assert np.array_equal(Pg[:, :n_used], oc.P[:, :n_used].astype(st.idx_dtype()))
    assert np.all(Pg[:, n_used:] == st.fill())
    if st.wide:                                                           # [R, tiles, g, 16384] uint16
        raw = st.P.cpu().numpy().view(np.uint16).reshape(R, -1, g, 16384).transpose(0, 1, 3, 2).reshape(R, -1, g)
        assert np.all(raw[:, n_used:] == 0xEEEE)
    else:
        assert np.all(st.P.cpu().numpy().reshape(R, cap, -1)[:, n_used:] == 0xEE)  # nothing written past n
    assert np.array_equal(st.pos.cpu().numpy().reshape(R, cap)[:, :n_used], np.tile(np.arange(n_used), (R, 1)))
    assert np.all(st.acc.cpu().numpy().reshape(R, cap)[:, :n_used] == 0) and np.all(st.acc.cpu().numpy().reshape(R, cap)[:, n_used:] == 9)

    q = (2 * rng.standard_normal((batch, hkv * G, D))).astype(np.float16)
    B.hca_vq_score(st.shape, st.cb, st.P, torch.from_numpy(q).cuda(), st.n, st.lut, st.sel, st.z)
    torch.cuda.synchronize()
    T = oracle.vq_lut(oc, q.reshape(R * G, D))
    Tg, sg_exp = st.table()
    assert np.array_equal(Tg.view(np.uint32), T.view(np.uint32))
    assert np.array_equal(sg_exp, oracle.vq_lut_fx(T)[1])
    sel, z = oracle.vq_score(oc, T)
    zg = st.z.cpu().numpy().reshape(R * G, cap)
    sg = st.sel.cpu().numpy().reshape(R, cap)
    assert np.array_equal(zg[:, :n_used].view(np.uint32), z[:, :n_used].view(np.uint32))
    assert np.array_equal(sg[:, :n_used].view(np.uint32), sel[:, :n_used].view(np.uint32))
    assert np.all(sg[:, n_used:] == -7.0) and np.all(zg[:, n_used:] == -7.0)
    # validity against Eq. 3 as written (fp64 sum of the table entries the indices select): the GPU's scores lie
    # within g half steps of the head's grid plus one fp32 rounding of it
    zp = oracle.vq_score_plain(oc, Tg)
    for hq in range(R * G):
        bound = g * 0.5 * 2.0 ** -int(sg_exp[hq]) + np.abs(zp[hq, :n_used]) * 2.0 ** -23
        assert np.all(np.abs(zg[hq, :n_used].astype(np.float64) - zp[hq, :n_used]) <= bound)


@pytest.mark.parametrize("g,c,big", [(32, 600, False), (64, 1030, False), (32, 520, True)])
def test_bulk_assign_with_awkward_keys_and_centroids(B, oracle, g, c, big):
    """The bulk form of the assignment (matrix-core shortlist, exact chain on the shortlist) on what could trip
    it: a codebook size that is no multiple of the tile, duplicate centroids and centroids one fp32 step apart
    (ties and near-ties: the lowest index, the exact chain's verdict), centroids of very different norms, keys that
    are zero, fp16-subnormal, infinite or so large that the shortlist bound does not apply, keys that sit exactly
    on a centroid; with `big` some centroids are large enough that no token can use the shortlist."""
    rng = np.random.default_rng(3 * g + c)
    batch, hkv, G, n = 1, 2, 2, 4200
    dbar = D // g
    cap = n + 8
    keys = rng.standard_normal((batch, hkv, n, D)).astype(np.float16)
    cen = (rng.standard_normal((hkv, g, c, dbar)) * 1.2).astype(np.float32)
    cen[:, :, 7] = cen[:, :, 3]                                        # exact duplicates
    cen[:, :, 40] = np.nextafter(cen[:, :, 41], np.float32(np.inf))      # one step apart
    cen[:, :, 90] = np.nextafter(cen[:, :, 91], np.float32(-np.inf))
    cen[:, :, 100:110] *= 9.0                                          # large norms
    cen[:, :, 110:120] *= 1e-3                                         # tiny norms
    cen[:, :, c - 1] = cen[:, :, c - 2]                                # a duplicate in the last, ragged tile
    if big:
        cen[:, :, 200:203] *= 400.0
    kf = keys.reshape(hkv, n, g, dbar)
    kf[:, 10] = 0.0
    kf[:, 11] = np.float16(6e-8)                                       # subnormal
    kf[:, 12, :, 0] = np.float16(np.inf)
    kf[:, 13, :, 0] = np.float16(-np.inf)
    kf[:, 14] = np.float16(300.0)                                      # beyond the shortlist's range
    kf[:, 15, ::2] = np.float16(-250.0)
    for t in range(20, 60):                                            # keys exactly on a centroid (as far as fp16 allows)
        kf[:, t] = cen[:, :, (t * 13) % c].astype(np.float16)
    kf[:, 60] = cen[:, :, 3].astype(np.float16)                        # on the duplicated centroid
    kf[:, 61] = cen[:, :, 41].astype(np.float16)
    keys = kf.reshape(batch, hkv, n, D)
    R = batch * hkv
    st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, 64)
    st.assign(torch.from_numpy(keys))
    torch.cuda.synchronize()
    oc = oracle.VQCache(R, cap, cen)
    oracle.vq_assign(oc, keys.reshape(R, n, D))
    Pg = st.P_rows()
    bad = np.argwhere(Pg[:, :n] != oc.P[:, :n].astype(st.idx_dtype()))
    assert len(bad) == 0, f"{len(bad)} indices differ, first (row, token, group): {bad[:5].tolist()}"


@pytest.mark.parametrize("g,c", [(32, 256), (32, 8192), (64, 1024)])
def test_blockwise_bulk_assign_equals_one_shot(B, oracle, g, c):
    """Block-wise prefill hands the keys over a block at a time (App. B): appending 40 000 tokens per row in blocks
    of 16 384 + 16 384 + 7 232 (the wide form's tile size, so the second block ends on a tile edge) and in uneven
    blocks of 10 001 + 1 + 29 998 leaves the same index cache as one call with all of them, and the indices around
    every block edge are the oracle's (brute force on those tokens only: the full set would take minutes at
    c = 8192)."""
    rng = np.random.default_rng(5 * g + c)
    batch, hkv, G, n = 1, 2, 4, 40000
    cap = n + 100
    keys = rng.standard_normal((batch, hkv, n, D)).astype(np.float16)
    keys[:, :, :, 9] *= 8
    cen = _codebook(oracle, rng, keys, hkv, g, c)
    kt = torch.from_numpy(keys)
    R = batch * hkv
    ref = _State(B, batch, hkv * G, hkv, cap, g, c, cen, 64)
    ref.assign(kt)
    torch.cuda.synchronize()
    Pref = ref.P_rows()
    for cuts in ([16384, 32768], [10001, 10002]):
        st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, 64)
        edges = [0] + cuts + [n]
        for a, b in zip(edges[:-1], edges[1:]):
            st.assign(kt[:, :, a:b])
        torch.cuda.synchronize()
        assert st.n == [n] * batch
        assert np.array_equal(st.P_rows(), Pref), f"blocks cut at {cuts}: index cache differs from the one-shot one"
        assert np.array_equal(st.pos.cpu().numpy(), ref.pos.cpu().numpy())
    sample = np.unique(np.concatenate([np.arange(max(0, e - 40), min(n, e + 40)) for e in (0, 10001, 10002, 16384, 32768, n)]))
    oc = oracle.VQCache(R, len(sample), cen)
    oracle.vq_assign(oc, keys.reshape(R, n, D)[:, sample])
    assert np.array_equal(Pref[:, sample], oc.P[:, :len(sample)].astype(ref.idx_dtype()))


@pytest.mark.parametrize("g,c,G,n,k", [(32, 256, 4, 9000, 512), (64, 128, 4, 3001, 100), (32, 64, 2, 5000, 5000),
                                       (32, 256, 1, 700, 1), (32, 1024, 4, 6000, 300), (64, 512, 2, 2500, 2500),
                                       (32, 512, 4, 20000, 700)])     # the last: two index tiles, the second ragged
def test_vq_decode_path_matches_oracle(B, oracle, g, c, G, n, k):
    """assign -> table + scores -> top-k -> gather (host + HBM rows) -> attend with accumulated scores."""
    rng = np.random.default_rng(n + k)
    batch, hkv = 2, 2
    R, cap = batch * hkv, n + 9
    keys = rng.standard_normal((batch, hkv, n, D)).astype(np.float16)
    values = rng.standard_normal((batch, hkv, n, D)).astype(np.float16)
    cen = _codebook(oracle, rng, keys, hkv, g, c)
    st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, k)
    st.assign(torch.from_numpy(keys))
    q = np.zeros((batch, hkv * G, D), np.float16)
    for b in range(batch):
        for h in range(hkv * G):                       # the query looks like a few of the keys
            q[b, h] = (keys[b, h // G, rng.integers(0, n, 3)].astype(np.float32).sum(0) + 0.3 * rng.standard_normal(D)).astype(np.float16)
    qd = torch.from_numpy(q).cuda()
    B.hca_vq_score(st.shape, st.cb, st.P, qd, st.n, st.lut, st.sel, None)
    B.hca_topk(st.shape, st.sel, st.n, k, st.idx, st.count, st.ws)
    nh = n // 3
    vh = torch.from_numpy(values[:, :, :nh]).contiguous().pin_memory()
    vd = torch.from_numpy(values[:, :, nh:]).contiguous().cuda()
    B.hca_gather_values(st.shape, st.idx, st.count, k, st.pos, vh, nh, nh, vd, n - nh, st.ws)
    sm = 1.0 / np.sqrt(D)
    B.hca_vq_attend_gathered(st.shape, st.cb, st.P, st.lut, st.idx, st.count, k, sm, st.y, st.acc, st.ws)
    torch.cuda.synchronize()

    oc = oracle.VQCache(R, cap, cen)
    oracle.vq_assign(oc, keys.reshape(R, n, D))
    T = oracle.vq_lut(oc, q.reshape(R * G, D))
    sel, _ = oracle.vq_score(oc, T, want_z=False)
    idx, count = oracle.topk(sel, oc.n, k)
    assert np.array_equal(st.idx.cpu().numpy().reshape(R, k), idx)
    assert np.array_equal(st.count.cpu().numpy().reshape(R), count)
    pos = np.tile(np.arange(cap, dtype=np.int32), (R, 1))
    acc = np.zeros((R, cap), np.float32)
    y, _ = oracle.vq_attend(oc, T, idx, count, pos, values.reshape(R, n, D), sm, acc=acc)
    assert _rel_err(st.y.cpu().numpy().reshape(R * G, D), y) <= TOL
    ag = st.acc.cpu().numpy().reshape(R, cap)[:, :n]
    assert np.array_equal(ag > 0, acc[:, :n] > 0)
    assert np.allclose(ag, acc[:, :n], rtol=1e-4, atol=1e-7)


def test_vq_ragged_lengths_and_empty_rows(B, oracle):
    rng = np.random.default_rng(77)
    batch, hkv, G, g, c, cap, k = 3, 2, 4, 32, 128, 1500, 40
    R = batch * hkv
    lens = [0, 1300, 17]
    keys = rng.standard_normal((batch, hkv, cap, D)).astype(np.float16)
    cen = _codebook(oracle, rng, keys, hkv, g, c)
    st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, k)
    # every sequence gets 1300 tokens; the calls below then see different resident lengths
    st.assign(torch.from_numpy(keys[:, :, :1300]))
    torch.cuda.synchronize()
    oc = oracle.VQCache(R, cap, cen)
    oracle.vq_assign(oc, keys.reshape(R, cap, D)[:, :1300])
    oc.n[:] = np.repeat(lens, hkv)
    q = rng.standard_normal((batch, hkv * G, D)).astype(np.float16)
    B.hca_vq_score(st.shape, st.cb, st.P, torch.from_numpy(q).cuda(), lens, st.lut, st.sel, st.z)
    B.hca_topk(st.shape, st.sel, lens, k, st.idx, st.count, st.ws)
    torch.cuda.synchronize()
    T = oracle.vq_lut(oc, q.reshape(R * G, D))
    sel, z = oracle.vq_score(oc, T)
    sg = st.sel.cpu().numpy().reshape(R, cap)
    for r in range(R):
        L = lens[r // hkv]
        assert np.array_equal(sg[r, :L], sel[r, :L]) and np.all(sg[r, L:] == -7.0)
    idx, count = oracle.topk(sel, oc.n, k)
    cg = st.count.cpu().numpy().reshape(R)
    assert np.array_equal(cg, count) and list(cg[:2]) == [0, 0]
    ig = st.idx.cpu().numpy().reshape(R, k)
    for r in range(R):
        assert np.array_equal(ig[r, :count[r]], idx[r, :count[r]])


@pytest.mark.parametrize("mode", ["inplace", "spare"])
@pytest.mark.parametrize("g,c,n,M,Rp", [(32, 64, 5000, 3000, 16), (64, 64, 1200, 700, 0), (32, 64, 900, 900, 4),
                                        (32, 64, 3000, 1, 1), (32, 300, 4000, 2500, 8), (64, 300, 2600, 1700, 3)])
def test_vq_evict_matches_oracle(B, oracle, mode, g, c, n, M, Rp):
    """Keep-set, compacted index rows, acc and pos against the oracle; one sequence is short enough to be
    left alone (n <= M) and must come through unchanged, also into the spare buffers.  c = 300: 16-bit indices,
    rows of 64 and 128 bytes (the latter pass through the staging area in two halves)."""
    rng = np.random.default_rng(n + M + Rp + g)
    batch, hkv, G = 2, 2, 4
    R, cap = batch * hkv, n + 5
    lens = [n, min(n, M) - (1 if M > 1 else 0)]
    keys = rng.standard_normal((batch, hkv, n, D)).astype(np.float16)
    cen = _codebook(oracle, rng, keys, hkv, g, c, iters=1)
    st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, 8)
    st.assign(torch.from_numpy(keys))
    oc = oracle.VQCache(R, cap, cen)
    oracle.vq_assign(oc, keys.reshape(R, n, D))
    oc.n[:] = np.repeat(lens, hkv)
    acc = np.zeros((R, cap), np.float32)
    acc[:, :n] = rng.integers(0, 5, (R, n)).astype(np.float32) * 0.5              # many ties
    acc[1, :n] = rng.standard_normal(n).astype(np.float32) ** 2
    pos = np.tile(rng.permutation(cap).astype(np.int32), (R, 1))
    accd = torch.from_numpy(acc.reshape(batch, hkv, cap)).cuda()
    posd = torch.from_numpy(pos.reshape(batch, hkv, cap)).cuda()
    kept = torch.full((batch, hkv, M), -5, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.hca_vq_workspace_bytes(st.shape, st.cb, 8, M), dtype=torch.uint8, device="cuda")
    if mode == "spare":
        P2 = torch.full_like(st.P, 0xAB)
        acc2, pos2 = torch.full_like(accd, -1.0), torch.full_like(posd, -1)
        B.hca_vq_evict(st.shape, st.cb, st.P, accd, posd, lens, M, Rp, kept, ws, P2, acc2, pos2)
        Pout, aout, pout = P2, acc2, pos2
    else:
        B.hca_vq_evict(st.shape, st.cb, st.P, accd, posd, lens, M, Rp, kept, ws)
        Pout, aout, pout = st.P, accd, posd
    torch.cuda.synchronize()
    okept = oracle.vq_evict(oc, acc, pos, M, Rp)
    Pg = st.P_rows(Pout, [min(x, M) for x in lens])
    ag, pg = aout.cpu().numpy().reshape(R, cap), pout.cpu().numpy().reshape(R, cap)
    kg = kept.cpu().numpy().reshape(R, M)
    for r in range(R):
        m = int(oc.n[r])
        assert m == min(lens[r // hkv], M)
        if lens[r // hkv] > M:
            assert np.array_equal(kg[r], okept[r])
        else:
            assert np.all(kg[r] == -5)                       # rows left alone report nothing
        assert np.array_equal(Pg[r, :m], oc.P[r, :m].astype(st.idx_dtype()))
        assert np.array_equal(ag[r, :m], acc[r, :m]) and np.array_equal(pg[r, :m], pos[r, :m])


def test_vq_decode_loop_with_appends_topp_and_eviction(B, oracle):
    """The paper-faithful step on a codebook cache, twelve times over: append one token, table + scores,
    cumulative-weight selection (Eq. 4), gather, attend with accumulated scores, eviction every 4 steps.
    The GPU state is compared with the oracle after every step (stage-wise on acc)."""
    import synth_inputs as S
    w = S.Workload("vqloop", 5, 2, 8, 2, 2000, 4, 32, 160, evict_keep=2000, evict_every=4, steps=12)
    d = S.make_layer(w)
    rng = np.random.default_rng(55)
    batch, hkv, G, g, c, k_max = w.batch, w.n_kv_heads, w.gqa, 32, 128, w.k
    R, n0 = batch * hkv, w.n
    cap, vcap = n0 + 8, n0 + w.steps
    keys = d["keys"].numpy()
    cen = _codebook(oracle, rng, keys, hkv, g, c)
    st = _State(B, batch, hkv * G, hkv, cap, g, c, cen, k_max)
    st.assign(d["keys"])
    oc = oracle.VQCache(R, cap, cen)
    oracle.vq_assign(oc, keys.reshape(R, n0, D))
    v_host = torch.zeros(batch, hkv, vcap, D, dtype=torch.float16).pin_memory()
    v_host[:, :, :n0] = d["values"]
    pos = np.zeros((R, cap), np.int32)
    pos[:, :n0] = np.arange(n0)
    acc = np.zeros((R, cap), np.float32)
    sm = 1.0 / np.sqrt(D)
    ws_e = torch.empty(B.hca_vq_workspace_bytes(st.shape, st.cb, k_max, w.evict_keep), dtype=torch.uint8, device="cuda")
    counts_seen = set()
    for step in range(w.steps):
        k_new, v_new, q = S.make_step(w, 0, step)
        n = st.n[0]
        v_host[:, :, n0 + step] = v_new[:, :, 0]
        pos[:, n] = n0 + step
        acc[:, n] = 0
        st.assign(k_new, row0=[n0 + step] * batch)
        oracle.vq_assign(oc, k_new.numpy().reshape(R, 1, D))
        qd = q.cuda()
        B.hca_vq_score(st.shape, st.cb, st.P, qd, st.n, st.lut, st.sel, None)
        B.hca_topp(st.shape, st.sel, st.n, sm, 0.9, k_max, st.idx, st.count, None, st.ws)
        B.hca_gather_values(st.shape, st.idx, st.count, k_max, st.pos, v_host, vcap, vcap, None, 0, st.ws)
        B.hca_vq_attend_gathered(st.shape, st.cb, st.P, st.lut, st.idx, st.count, k_max, sm, st.y, st.acc, st.ws)
        torch.cuda.synchronize()
        T = oracle.vq_lut(oc, q.numpy().reshape(R * G, D))
        sel, _ = oracle.vq_score(oc, T, want_z=False)
        idx, count, _, _ = oracle.topp(sel, oc.n, sm, 0.9, k_max)
        cg = st.count.cpu().numpy().reshape(R)
        assert np.array_equal(cg, count), f"step {step}"
        counts_seen |= set(count.tolist())
        ig = st.idx.cpu().numpy().reshape(R, k_max)
        for r in range(R):
            assert np.array_equal(ig[r, :count[r]], idx[r, :count[r]]), f"step {step} row {r}"
        y, _ = oracle.vq_attend(oc, T, idx, count, pos, v_host.numpy().reshape(R, vcap, D), sm, acc=acc)
        assert _rel_err(st.y.cpu().numpy().reshape(R * G, D), y) <= TOL
        nn = st.n[0]
        assert np.allclose(st.acc.cpu().numpy().reshape(R, cap)[:, :nn], acc[:, :nn], rtol=1e-4, atol=1e-7)
        st.acc.copy_(torch.from_numpy(acc.reshape(batch, hkv, cap)))            # stage-wise from here on
        if (step + 1) % w.evict_every == 0:
            B.hca_vq_evict(st.shape, st.cb, st.P, st.acc, st.pos, st.n, w.evict_keep, w.evict_every, None, ws_e)
            st.n = [min(x, w.evict_keep) for x in st.n]
            torch.cuda.synchronize()
            oracle.vq_evict(oc, acc, pos, w.evict_keep, w.evict_every)
            m = w.evict_keep
            assert st.n[0] == m == oc.n[0]
            assert np.array_equal(st.P_rows()[:, :m], oc.P[:, :m].astype(st.idx_dtype()))
            assert np.array_equal(st.pos.cpu().numpy().reshape(R, cap)[:, :m], pos[:, :m])
            assert np.array_equal(st.acc.cpu().numpy().reshape(R, cap)[:, :m], acc[:, :m])
    assert len(counts_seen) > 1


@pytest.mark.parametrize("tau,Lr,n_sel,c", [(0.0, 3, 3, 64), (0.9, 3, 3, 64), (0.9, 5, 3, 64), (0.97, 4, 4, 64), (0.9, 3, 3, 512)])
def test_native_step_driver_in_the_papers_form(B, oracle, tau, Lr, n_sel, c):
    """hca_pipeline_step with a codebook cache per layer (and Eq. 4 selection when tau > 0) over 3 to 5 layers,
    12 decode steps, staggered in-place eviction every 4 steps: every layer's output, resident count and final
    index rows / pos / acc against the oracle run layer by layer."""
    import ctypes as C
    import math
    import synth_inputs as S
    steps, E = 12, 4
    w = S.Workload("vqdrv", 9, 2, 8, 2, 1500, 4, 32, 96)
    batch, hkv, G, g = w.batch, w.n_kv_heads, w.gqa, 32
    wide = c > 256
    R, n0 = batch * hkv, w.n
    cap, vnew = n0 + E + 16, steps + 4
    shape = B.make_shape(batch, w.n_q_heads, hkv, cap)
    rng = np.random.default_rng(77)
    data = [S.make_layer(w, l) for l in range(Lr)]
    cens = [_codebook(oracle, rng, data[l]["keys"].numpy(), hkv, g, c, iters=1) for l in range(Lr)]
    cend = [torch.from_numpy(x).cuda() for x in cens]
    cbs = [B.make_codebook(g, c, x) for x in cend]
    P = [torch.zeros(B.hca_vq_pcache_bytes(shape, cbs[0]), dtype=torch.uint8, device="cuda") for _ in range(Lr)]
    lut = [torch.zeros(B.hca_vq_lut_bytes(shape, cbs[0]) // 4, dtype=torch.float32, device="cuda") for _ in range(Lr)]
    acc = [torch.zeros(batch, hkv, cap, dtype=torch.float32, device="cuda") for _ in range(Lr)]
    pos = [torch.arange(cap, dtype=torch.int32, device="cuda").repeat(batch, hkv, 1).contiguous() for _ in range(Lr)]
    vh = [d["values"].contiguous().pin_memory() for d in data]
    vd = [torch.zeros(batch, hkv, vnew, D, dtype=torch.float16, device="cuda") for _ in range(Lr)]
    y = torch.zeros(Lr, batch, w.n_q_heads, D, dtype=torch.float32, device="cuda")
    ocs, oacc, opos, oV = [], [], [], []
    for l in range(Lr):
        B.hca_vq_assign(shape, cbs[l], P[l], data[l]["keys"].cuda(), n0, [0] * batch)
        oc = oracle.VQCache(R, cap, cens[l])
        oracle.vq_assign(oc, data[l]["keys"].numpy().reshape(R, n0, D))
        ocs.append(oc)
        oacc.append(np.zeros((R, cap), np.float32))
        p = np.zeros((R, cap), np.int32)
        p[:] = np.arange(cap)
        opos.append(p)
        V = np.zeros((R, n0 + vnew, D), np.float16)
        V[:, :n0] = data[l]["values"].numpy().reshape(R, n0, D)
        oV.append(V)
    streams = [torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()]
    d = B.hca_pipeline_desc()
    d.stream_scan, d.stream_topk, d.stream_gather, d.stream_attend = (s.cuda_stream for s in streams)
    wsb = B.hca_vq_workspace_bytes(shape, cbs[0], w.k, n0)
    keep = []
    for i in range(n_sel):
        t = torch.zeros(batch, hkv, cap, dtype=torch.float32, device="cuda")
        keep.append(t)
        d.sel[i] = t.data_ptr()
    d.n_sel = n_sel
    for i in range(4):
        a = torch.zeros(batch, hkv, w.k, dtype=torch.int32, device="cuda")
        b = torch.zeros(batch, hkv, dtype=torch.int32, device="cuda")
        cws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
        keep += [a, b, cws]
        d.idx[i], d.count[i], d.ws_attend[i] = a.data_ptr(), b.data_ptr(), cws.data_ptr()
    wt, we = torch.zeros(wsb, dtype=torch.uint8, device="cuda"), torch.zeros(wsb, dtype=torch.uint8, device="cuda")
    d.ws_topk, d.ws_evict = wt.data_ptr(), we.data_ptr()
    d.vq_groups, d.vq_codewords, d.topp_tau = g, c, tau
    pl = B.hca_pipeline_create(shape, Lr, d, 0)
    layers = (B.hca_layer * Lr)()
    for l in range(Lr):
        layers[l].kcache, layers[l].acc, layers[l].pos = P[l].data_ptr(), acc[l].data_ptr(), pos[l].data_ptr()
        layers[l].v_host, layers[l].v_hbm, layers[l].y = vh[l].data_ptr(), vd[l].data_ptr(), y[l].data_ptr()
        layers[l].vq_centroids, layers[l].vq_lut = cend[l].data_ptr(), lut[l].data_ptr()
    nres = (C.c_int64 * (Lr * batch))(*([n0] * (Lr * batch)))
    sm = 1.0 / math.sqrt(float(D))
    counts_seen = set()
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
        B.hca_pipeline_step(pl, layers, nres, n0 + t, w.k, n0, n0, vnew, sm, ev, E, -1)
        torch.cuda.synchronize()
        for l in range(Lr):
            oc = ocs[l]
            n = int(oc.n[0])
            oV[l][:, n0 + t] = ins[l][1].numpy().reshape(R, 1, D)[:, 0]
            opos[l][:, n] = n0 + t
            oacc[l][:, n] = 0
            oracle.vq_assign(oc, ins[l][0].numpy().reshape(R, 1, D))
            q16 = ins[l][2].numpy().reshape(R * G, D)
            T = oracle.vq_lut(oc, q16)
            sel, _ = oracle.vq_score(oc, T, want_z=False)
            if tau > 0:
                idx, count, _, _ = oracle.topp(sel, oc.n, sm, tau, w.k)
            else:
                idx, count = oracle.topk(sel, oc.n, w.k)
            counts_seen |= set(count.tolist())
            yo, _ = oracle.vq_attend(oc, T, idx, count, opos[l], oV[l], sm, acc=oacc[l])
            assert _rel_err(y[l].cpu().numpy().reshape(R * G, D), yo) <= TOL, f"step {t} layer {l}"
            if due[l]:
                oracle.vq_evict(oc, oacc[l], opos[l], n0, E)
            assert nres[l * batch] == int(oc.n[0]), f"step {t} layer {l}"
    if tau > 0:
        assert len(counts_seen) > 1
    for l in range(Lr):
        n = int(ocs[l].n[0])
        out = torch.zeros(R, cap, g * (2 if wide else 1), dtype=torch.uint8, device="cuda")
        B.hca_vq_export_pcache(shape, cbs[l], P[l], [n] * batch, out)
        torch.cuda.synchronize()
        og = out.cpu().numpy().view(np.uint16) if wide else out.cpu().numpy()
        assert np.array_equal(og[:, :n], ocs[l].P[:, :n].astype(og.dtype))
        assert np.array_equal(pos[l].cpu().numpy().reshape(R, cap)[:, :n], opos[l][:, :n])
        assert np.allclose(acc[l].cpu().numpy().reshape(R, cap)[:, :n], oacc[l][:, :n], rtol=1e-3, atol=1e-6)
    B.hca_pipeline_destroy(pl)
