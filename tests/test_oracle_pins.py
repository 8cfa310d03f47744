"""Pins for the CPU oracle: every check compares it with something other than itself
(numpy / torch library routines, closed forms, brute force, invariants, the paper's
printed closed-form figures).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_closed_forms.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def _keys(rng, R, T, D=128, outliers=True):
    x = rng.standard_normal((R, T, D)).astype(np.float32)
    if outliers:
        for r in range(R):
            x[r][:, rng.choice(D, 4, replace=False)] *= 8.0
    return x.astype(np.float16)


def _unpack(codes, bits):
    """Independent decode of the canonical packing via numpy bit unpacking."""
    b = np.unpackbits(codes, axis=-1, bitorder="little")
    b = b.reshape(*codes.shape[:-1], -1, bits)
    w = (1 << np.arange(bits)).astype(np.int64)
    return (b * w).sum(-1)


# ------------------------------------------------------------------ fp16 ---

def test_h2f_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.h2f(int(b)) for b in bits], np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_f2h_matches_numpy_rne(oracle):
    rng = np.random.default_rng(0)
    xs = [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
          2.0 ** -14, np.nextafter(np.float32(2.0 ** -14), np.float32(0)), 1.0, 1.00048828125,
          1.0009765625 + 2.0 ** -12, 0.333333]
    xs += list(rng.standard_normal(4000) * 10.0 ** rng.integers(-8, 5, 4000))
    # every midpoint between consecutive halfs in a few binades (ties-to-even cases)
    h = np.arange(0x0001, 0x0c00, dtype=np.uint16).view(np.float16).astype(np.float64)
    xs += list((h[:-1] + h[1:]) / 2)
    h = np.arange(0x3c00, 0x4400, dtype=np.uint16).view(np.float16).astype(np.float64)
    xs += list((h[:-1] + h[1:]) / 2)
    xs = np.array(xs, np.float32)
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f2h(float(x)) for x in xs], np.uint16)
    assert np.array_equal(got, ref)


# -------------------------------------------------------------- quantise ---

@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64), (8, 32), (2, 32), (4, 64), (8, 64)])
def test_quantize_invariants(oracle, bits, gs):
    rng = np.random.default_rng(bits * 100 + gs)
    R, T, D = 3, 200, 128
    k = _keys(rng, R, T)
    k[0, 0, :] = np.float16(0.75)              # constant token
    k[0, 1, :gs] = np.float16(-2.5)            # constant group
    k[0, 2, :gs] = 0.0
    k[0, 2, 0] = np.float16(-0.0)              # first-seen minimum is a negative zero
    c = oracle.Cache(R, T + 5, D, bits, gs)
    oracle.quantize(c, k)
    assert np.all(c.n == T)
    qmax = (1 << bits) - 1
    code = _unpack(c.codes[:, :T], bits)                       # [R,T,D]
    x = k.astype(np.float32).reshape(R, T, D // gs, gs)
    cg = code.reshape(R, T, D // gs, gs)
    scale = c.scale[:, :T].view(np.float16).astype(np.float32)
    zero = c.zero[:, :T].view(np.float16).astype(np.float32)
    mn, mx = x.min(-1), x.max(-1)
    # zero point is the group minimum, exactly
    assert np.array_equal(zero, mn)
    assert not np.any(np.signbit(zero) & (zero == 0))
    # codes in range, min -> 0, max -> qmax (non-constant groups)
    assert cg.min() >= 0 and cg.max() <= qmax
    nonconst = mx > mn
    arg_mn, arg_mx = x.argmin(-1), x.argmax(-1)
    assert np.all(np.take_along_axis(cg, arg_mn[..., None], -1)[..., 0] == 0)
    assert np.all(np.take_along_axis(cg, arg_mx[..., None], -1)[..., 0][nonconst] == qmax)
    # constant groups: all-zero codes and scale 1.0
    assert np.all(cg[~nonconst] == 0)
    assert np.all(scale[~nonconst] == 1.0)
    # scale is the fp16 rounding of range/qmax (numpy does the division and the RNE cast)
    want = ((mx - mn) / np.float32(qmax)).astype(np.float16)
    assert np.array_equal(scale[nonconst], want.astype(np.float32)[nonconst])
    # monotone: larger input never gets a smaller code
    order = np.argsort(x, axis=-1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(cg, order, -1), axis=-1) >= 0)
    # reconstruction error bound: half a step, plus qmax times the fp16 rounding of the step
    khat = oracle.dequantize(c)[:, :T].reshape(R, T, D // gs, gs)
    true_step = (mx - mn).astype(np.float64) / qmax
    bound = scale.astype(np.float64) / 2 + qmax * np.abs(scale - true_step) + 1e-6
    assert np.all(np.abs(khat.astype(np.float64) - x) <= bound[..., None] * (1 + 1e-5))


def test_quantize_exhaustive_two_level_group(oracle):
    """Brute force over a dense set of (min, max) pairs for b=2: a group holding only its
    minimum and maximum must code them 0 and 3; interior points at exact thirds code 1, 2."""
    hs = np.arange(0, 0x7c00, 37, dtype=np.uint16).view(np.float16)
    hs = np.concatenate([hs, -hs])
    rng = np.random.default_rng(5)
    a = rng.choice(hs, 4000)
    b = rng.choice(hs, 4000)
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    keep = hi > lo
    lo, hi = lo[keep], hi[keep]
    T = lo.shape[0]
    k = np.empty((1, T, 64), np.float16)
    k[0, :, 0::2] = lo[:, None]
    k[0, :, 1::2] = hi[:, None]
    c = oracle.Cache(1, T, 64, 2, 32)
    oracle.quantize(c, k)
    code = _unpack(c.codes, 2)[0]
    sc = c.scale.view(np.float16).astype(np.float64)[0, :, 0]
    ok = sc > 0
    assert np.all(code[:, 0::2] == 0)
    # the top code is reached whenever the fp16 step is representable (not flushed to 1.0)
    rng_ = hi.astype(np.float64) - lo.astype(np.float64)
    reach = np.abs(rng_ / sc - 3) < 0.5
    assert np.all(code[reach][:, 1::2] == 3)
    assert reach.mean() > 0.95 and ok.all()


def _one_group_codes(oracle, vals, bits=4, gs=32):
    """Quantise one token whose first group holds `vals` (padded with the group's minimum) and return that
    group's codes, scale and zero."""
    x = np.full((1, 1, 128), np.float16(0.0))
    v = np.asarray(vals, np.float16)
    x[0, 0, :gs] = v.min()
    x[0, 0, :len(v)] = v
    c = oracle.Cache(1, 1, 128, bits, gs)
    oracle.quantize(c, x)
    code = _unpack(c.codes[:, :1], bits)[0, 0, :len(v)]
    return list(code), float(c.scale.view(np.float16)[0, 0, 0]), float(c.zero.view(np.float16)[0, 0, 0])


def test_quantize_rounds_halves_to_even(oracle):
    """Hand-worked: a 4-bit group with minimum 0 and maximum 15 has scale fp16(15 / 15) = 1 and reciprocal 1, so a
    channel's code is rint(x) itself.  2.5 and 3.5 lie exactly between two codes: ties go to the even one, 2 and 4
    (adding one half and truncating would give 3 and 4); likewise 0.5 -> 0, 1.5 -> 2, 13.5 -> 14, 14.5 -> 14."""
    code, scale, zero = _one_group_codes(oracle, [0.0, 15.0, 2.5, 3.5, 0.5, 1.5, 13.5, 14.5, 7.0, 7.25, 7.75])
    assert scale == 1.0 and zero == 0.0
    assert code == [0, 15, 2, 4, 0, 2, 14, 14, 7, 7, 8]
    # 2-bit, group of 64: minimum 0, maximum 3 -> scale 1: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    code, scale, _ = _one_group_codes(oracle, [0.0, 3.0, 0.5, 1.5, 2.5], bits=2, gs=64)
    assert scale == 1.0 and code == [0, 3, 0, 2, 2]


def test_quantize_multiplies_by_the_reciprocal_of_the_scale(oracle):
    """Hand-worked case in which code = rint((x - min) * (1 / scale)), the form this build fixes, differs from
    rint((x - min) / scale).  Group minimum 0, maximum 105/256: scale = fp16(105/256 / 15) = 7/256 exactly.
    x = 91/512: x / scale = 6.5 exactly, a tie, which division would round to the even code 6.  The reciprocal
    1 / scale = 256/7 = 36.5714285714... is not representable; its fp32 rounding is 9586981 * 2^-18 =
    36.57143020629883 (0.43 ulp above).  x times that is 6.50000029057..., which lies above the midpoint
    6.5 + 2^-22 of the two neighbouring fp32 numbers 6.5 and 6.5 + 2^-21, so the product rounds to 6.5 + 2^-21
    and rint gives 7."""
    from fractions import Fraction as F
    inv = F(9586981, 2 ** 18)
    assert abs(inv - F(256, 7)) < F(1, 2 ** 19) and float(np.float32(1) / np.float32(7 / 256)) == float(inv)
    prod = F(91, 512) * inv
    assert prod > F(13, 2) + F(1, 2 ** 22)                       # beyond the fp32 midpoint above 6.5
    code, scale, zero = _one_group_codes(oracle, [0.0, 105 / 256, 91 / 512])
    assert scale == 7 / 256 and zero == 0.0
    assert code == [0, 15, 7]


def test_score_adds_the_four_group_terms_pairwise(oracle):
    """Hand-built cache (codes / scale / zero written directly) whose four group terms are 2^24, 0, 1, 1 before the
    2^-s factor: (t0 + t1) + (t2 + t3) = 2^24 + 2, exactly representable, while adding left to right loses both
    ones (2^24 + 1 rounds back to 2^24 twice).  Query: 1.0 in the first channel of every group, so s = 13,
    qfx = 8192 there, Q_g = 8192 and D_g = 8192 * (first code of the group).
      group 0: code 0, zero 2048           -> fma(scale, 0, 2048 * 8192) = 2^24
      group 1: code 0, zero 0              -> 0
      groups 2, 3: code 1, scale 2^-13, zero 0 -> 2^-13 * 8192 = 1
    z~ = (2^24 + 2) * 2^-13 = 2048 + 2^-12."""
    c = oracle.Cache(1, 1, 128, 4, 32)
    c.n[:] = 1
    h = lambda v: np.array([v], np.float16).view(np.uint16)[0]
    c.scale[0, 0] = [h(1.0), h(1.0), h(2.0 ** -13), h(2.0 ** -13)]
    c.zero[0, 0] = [h(2048.0), h(0.0), h(0.0), h(0.0)]
    c.codes[0, 0, 32] = 1                                        # channel 64 (group 2): low nibble of byte 32
    c.codes[0, 0, 48] = 1                                        # channel 96 (group 3)
    q = np.zeros((1, 128), np.float16)
    q[0, ::32] = 1.0
    qfx, s = oracle.query_fixed(q[0])
    assert s == 13 and list(qfx[::32]) == [8192] * 4 and np.count_nonzero(qfx) == 4
    sel, z = oracle.score(c, q)
    assert float(z[0, 0]) == 2048.0 + 2.0 ** -12
    assert float(sel[0, 0]) == 2048.0 + 2.0 ** -12
    # two groups (2-bit, group 64): t0 + t1 only; 2^24 and 1 -> 2^24 (the one is lost to rounding, once)
    c2 = oracle.Cache(1, 1, 128, 2, 64)
    c2.n[:] = 1
    c2.scale[0, 0] = [h(1.0), h(2.0 ** -13)]
    c2.zero[0, 0] = [h(2048.0), h(0.0)]
    c2.codes[0, 0, 16] = 1                                       # channel 64 (group 1): low crumb of byte 16
    q2 = np.zeros((1, 128), np.float16)
    q2[0, ::64] = 1.0
    _, z2 = oracle.score(c2, q2)
    assert float(z2[0, 0]) == 2048.0


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64), (8, 32)])
def test_fixed_point_score_against_the_plain_fp64_definition(oracle, bits, gs):
    """The plain form of Eq. 2's z~ = q . Q(K)^T (query untouched, fp64) is (a) numpy's matrix product over the
    dequantised keys, and (b) within 2^-14 max|q| sum_c |k^_c| of the fixed-point form: the query's 15-bit
    image is off by at most half a step of 2^-s per channel, and 2^(13-s) <= max|q|."""
    rng = np.random.default_rng(40 + bits)
    R, G, T, D = 2, 4, 257, 128
    k = _keys(rng, R, T)
    q = (rng.standard_normal((R * G, D)) * 0.7).astype(np.float16)
    c = oracle.Cache(R, T + 3, D, bits, gs)
    oracle.quantize(c, k)
    zp = oracle.score_plain(c, q)
    _, z = oracle.score(c, q)
    code = _unpack(c.codes[:, :T], bits).astype(np.float64)
    sc = np.repeat(c.scale[:, :T].view(np.float16).astype(np.float64), gs, axis=-1)
    zr = np.repeat(c.zero[:, :T].view(np.float16).astype(np.float64), gs, axis=-1)
    khat = sc * code + zr                                                     # [R,T,D], independent decode
    for hq in range(R * G):
        r = hq // G
        ref = khat[r] @ q[hq].astype(np.float64)
        assert np.allclose(zp[hq, :T], ref, rtol=1e-12, atol=1e-12)
        assert np.all(zp[hq, T:] == 0)
        mag = np.abs(khat[r]).sum(-1) * np.abs(q[hq].astype(np.float64)).max()
        assert np.all(np.abs(z[hq, :T] - zp[hq, :T]) <= 2.0 ** -14 * mag + 1e-5 * np.abs(zp[hq, :T]) + 1e-6)


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64), (8, 32)])
def test_fixed_point_score_against_the_plain_fp32_form(oracle, bits, gs):
    """The score as one would write it first - fp32, query untouched, ascending fused multiply-add chains - is
    (a) within fp32 rounding of the fp64 definition (at most one rounding per term and per sum:
    (D + 8) 2^-24 sum_c |q_c k^_c| is generous) and (b) within 2^-14 max|q| sum|k^| plus that rounding of the
    fixed-point form the GPU reproduces: the two forms of the same score differ by the query's fixed-point step
    and nothing else."""
    rng = np.random.default_rng(60 + bits)
    R, G, T, D = 2, 4, 300, 128
    k = _keys(rng, R, T)
    q = (rng.standard_normal((R * G, D)) * 1.3).astype(np.float16)
    c = oracle.Cache(R, T + 2, D, bits, gs)
    oracle.quantize(c, k)
    za = oracle.score_fp32(c, q)
    zp = oracle.score_plain(c, q)
    _, zb = oracle.score(c, q)
    code = _unpack(c.codes[:, :T], bits).astype(np.float64)
    sc = np.repeat(c.scale[:, :T].view(np.float16).astype(np.float64), gs, axis=-1)
    zr = np.repeat(c.zero[:, :T].view(np.float16).astype(np.float64), gs, axis=-1)
    absk = np.abs(sc * code) + np.abs(zr)                                    # [R,T,D]: the terms before they cancel
    for hq in range(R * G):
        r = hq // G
        aq = np.abs(q[hq].astype(np.float64))
        rounding = (D + 8) * 2.0 ** -24 * (absk[r] @ aq)
        assert np.all(np.abs(za[hq, :T].astype(np.float64) - zp[hq, :T]) <= rounding + 1e-30)
        step = 2.0 ** -14 * aq.max() * np.abs(sc[r] * code[r] + zr[r]).sum(-1)
        assert np.all(np.abs(za[hq, :T].astype(np.float64) - zb[hq, :T]) <= step + rounding + 2.0 ** -23 * np.abs(zp[hq, :T]))
        assert np.all(za[hq, T:] == 0)


def test_budget_closed_forms(oracle):
    """Table 1a: a g-entry 16-bit index row against a d-entry 16-bit key row is g/d of the
    key budget; the 4-bit and 2-bit code rows of this build occupy the same bytes."""
    g = _golden()
    d = int(g["head_dim"])
    full_key_bytes = d * 2
    assert 64 * g["index_bits"] / 8 / full_key_bytes == g["k_budget_g64"]
    assert 32 * g["index_bits"] / 8 / full_key_bytes == g["k_budget_g32"]
    c4 = oracle.Cache(1, 1, d, 4, 32)
    c2 = oracle.Cache(1, 1, d, 2, 64)
    c8 = oracle.Cache(1, 1, d, 8, 32)
    assert c8.CB / full_key_bytes == g["k_budget_g64"]      # 8-bit codes == paper's g=64 row
    assert c4.CB / full_key_bytes == g["k_budget_g32"]      # 4-bit codes == paper's g=32 row
    assert c2.CB / full_key_bytes == g["k_budget_g32"] / 2
    # totals with values offloaded (V budget 0): K share is half of the KV cache
    assert g["k_budget_g64"] / 2 == g["total_budget_g64"]
    assert g["k_budget_g32"] / 2 == g["total_budget_g32"]
    link = g["link_fraction"] * g["link_n"] * g["link_layers"] * g["link_heads"] * g["link_bytes_each"]
    assert abs(link / 1e6 - g["link_total_MB"]) < 1e-9


# ----------------------------------------------------------------- score ---

def test_query_fixed_properties(oracle):
    rng = np.random.default_rng(1)
    for trial in range(50):
        q = (rng.standard_normal(128) * 10.0 ** rng.integers(-4, 3)).astype(np.float16)
        if trial == 0:
            q[:] = 0
        if trial == 1:
            q[:] = np.float16(6e-8)  # subnormal
        qfx, s = oracle.query_fixed(q)
        qf = q.astype(np.float64)
        amax = np.abs(qf).max()
        if amax == 0:
            assert s == 0 and not qfx.any()
            continue
        assert 2 ** 13 <= amax * 2.0 ** s < 2 ** 14
        assert np.abs(qfx).max() < 2 ** 14
        assert np.all(np.abs(qfx - qf * 2.0 ** s) <= 0.5)
        # the largest element and everything within 3 binades of it is exact
        big = np.abs(qf) >= amax / 8
        assert np.all(qfx[big] == qf[big] * 2.0 ** s)


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64), (8, 32)])
def test_score_against_fp64_dot(oracle, bits, gs):
    """z~ equals q . k_hat evaluated in fp64 up to the query's fixed-point step, and stays
    within the quantisation bound of the exact q . k (closed form: sum_g scale_g/2 * sum|q_c|)."""
    rng = np.random.default_rng(7 + bits)
    R, G, T, D = 2, 4, 300, 128
    k = _keys(rng, R, T)
    q = (rng.standard_normal((R * G, D)) * 1.3).astype(np.float16)
    c = oracle.Cache(R, T, D, bits, gs)
    oracle.quantize(c, k)
    sel, z = oracle.score(c, q)
    khat = oracle.dequantize(c).astype(np.float64)           # [R,T,D]
    qf = q.astype(np.float64)
    scale = c.scale.view(np.float16).astype(np.float64)      # [R,T,NG]
    for r in range(R):
        for g in range(G):
            hq = r * G + g
            _, s = oracle.query_fixed(q[hq])
            ref = khat[r] @ qf[hq]
            fx_bound = 2.0 ** -(s + 1) * np.abs(khat[r]).sum(-1)
            slop = 1e-5 * (np.abs(khat[r]) * np.abs(qf[hq])).sum(-1) + 1e-6
            assert np.all(np.abs(z[hq] - ref) <= fx_bound + slop)
            exact = k[r].astype(np.float64) @ qf[hq]
            qabs = np.abs(qf[hq]).reshape(D // gs, gs).sum(-1)            # [NG]
            qmax = (1 << bits) - 1
            true_step = (k[r].astype(np.float64).reshape(T, D // gs, gs).max(-1)
                         - k[r].astype(np.float64).reshape(T, D // gs, gs).min(-1)) / qmax
            qb = ((scale[r] / 2 + qmax * np.abs(scale[r] - true_step)) * qabs[None, :]).sum(-1)
            assert np.all(np.abs(ref - exact) <= qb * (1 + 1e-6) + 1e-6)
        assert np.array_equal(sel[r], z[r * G:(r + 1) * G].max(0))


def test_score_ranks_like_exact_dot(oracle):
    """The best-scoring token under z~ is the best under the exact fp64 q . k, and a planted
    token (key == the query direction) ranks among the very top."""
    rng = np.random.default_rng(11)
    T, D = 500, 128
    k = _keys(rng, 1, T)
    u = k[0, 123].astype(np.float32)
    q = (u + 0.3 * rng.standard_normal(D)).astype(np.float16)[None]
    c = oracle.Cache(1, T, D, 4, 32)
    oracle.quantize(c, k)
    sel, z = oracle.score(c, q)
    exact = k[0].astype(np.float64) @ q[0].astype(np.float64)
    assert int(z[0].argmax()) == int(exact.argmax())
    assert int((z[0] > z[0, 123]).sum()) == int((exact > exact[123]).sum()) <= 5


# ----------------------------------------------------------------- top-k ---

def test_topk_matches_library_on_distinct(oracle):
    rng = np.random.default_rng(3)
    R, cap = 4, 5000
    sel = rng.permutation(R * cap).reshape(R, cap).astype(np.float32) - 7000.0
    n = np.array([5000, 4999, 17, 1])
    for k in (1, 16, 257, 5000):
        idx, count = oracle.topk(sel, n, k)
        for r in range(R):
            kk = min(k, n[r])
            assert count[r] == kk
            ref = torch.topk(torch.from_numpy(sel[r, :n[r]]), kk).indices.sort().values.numpy()
            assert np.array_equal(idx[r, :kk], ref)
            assert np.all(idx[r, kk:] == -1)


def test_topk_ties(oracle):
    rng = np.random.default_rng(4)
    cap = 3000
    rows = [np.full(cap, 2.5, np.float32),                                   # all equal
            rng.integers(0, 2, cap).astype(np.float32),                      # two-valued
            rng.integers(-3, 4, cap).astype(np.float32) * 0.0,               # +0 / -0 mix
            rng.integers(0, 50, cap).astype(np.float32)]
    rows[2][::3] = -0.0
    sel = np.stack(rows)
    n = np.full(4, cap)
    for k in (1, 100, 1500, 2999):
        idx, count = oracle.topk(sel, n, k)
        for r in range(4):
            # library stable sort on the negated values == (value desc, index asc)
            ref = np.sort(np.argsort(-(sel[r] + 0.0), kind="stable")[:k])
            assert np.array_equal(idx[r], ref)
    idx, _ = oracle.topk(sel, n, 7)
    assert np.array_equal(idx[0], np.arange(7))          # ties -> lowest indices


# ---------------------------------------------------------------- attend ---

def _run_pipeline(oracle, k16, v16, q16, bits, gs, k, G):
    R, T, D = k16.shape
    c = oracle.Cache(R, T, D, bits, gs)
    oracle.quantize(c, k16)
    sel, z = oracle.score(c, q16)
    idx, count = oracle.topk(sel, c.n, k)
    pos = np.tile(np.arange(T, dtype=np.int32), (R, 1))
    y, w = oracle.attend(c, q16, idx, count, pos, v16, 1.0 / math.sqrt(D), want_w=True)
    return c, sel, z, idx, count, y, w


def test_full_selection_8bit_converges_to_exact_attention(oracle):
    """k = n with 8-bit keys reproduces Eq. 1 (analogue of tau = 1 selecting 100%)."""
    assert _golden()["tau_one_selection_ratio"] == 1.0
    rng = np.random.default_rng(21)
    R, G, T, D = 2, 1, 256, 128
    k16 = _keys(rng, R, T)
    v16 = rng.standard_normal((R, T, D)).astype(np.float16)
    q16 = (rng.standard_normal((R * G, D)) * 0.5).astype(np.float16)
    errs = {}
    for bits in (2, 4, 8):
        _, _, _, idx, count, y, w = _run_pipeline(oracle, k16, v16, q16, bits, 32, T, G)
        assert np.all(count == T)
        e = 0.0
        for r in range(R):
            ref = oracle.attention_exact(q16[r], k16[r], v16[r], 1.0 / math.sqrt(D))
            e = max(e, np.abs(y[r] - ref).max() / np.abs(ref).max())
        errs[bits] = e
    assert errs[8] < 2e-2
    assert errs[8] < errs[4] < errs[2]


def test_attention_exact_matches_torch(oracle):
    rng = np.random.default_rng(22)
    T, D = 300, 128
    q = rng.standard_normal(D).astype(np.float16)
    K = rng.standard_normal((T, D)).astype(np.float16)
    V = rng.standard_normal((T, D)).astype(np.float16)
    y = oracle.attention_exact(q, K, V, 1 / math.sqrt(D))
    tq, tK, tV = (torch.from_numpy(a.astype(np.float64)) for a in (q, K, V))
    ref = torch.softmax(tK @ tq / math.sqrt(D), 0) @ tV
    assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("bits,gs", [(4, 32), (2, 64)])
def test_full_selection_is_dense_softmax_over_dequantised_keys(oracle, bits, gs):
    rng = np.random.default_rng(23)
    R, G, T, D = 2, 4, 200, 128
    k16 = _keys(rng, R, T)
    v16 = rng.standard_normal((R, T, D)).astype(np.float16)
    q16 = (rng.standard_normal((R * G, D)) * 0.5).astype(np.float16)
    c, sel, z, idx, count, y, w = _run_pipeline(oracle, k16, v16, q16, bits, gs, T, G)
    khat = torch.from_numpy(oracle.dequantize(c).astype(np.float64))
    for hq in range(R * G):
        r = hq // G
        logits = khat[r] @ torch.from_numpy(q16[hq].astype(np.float64)) / math.sqrt(D)
        a = torch.softmax(logits, 0)
        ref = a @ torch.from_numpy(v16[r].astype(np.float64))
        assert np.abs(y[hq] - ref.numpy()).max() <= 2e-3 * np.abs(ref.numpy()).max()
        assert abs(w[hq].sum() - 1.0) < 1e-5


def test_k_equals_one_returns_argmax_value(oracle):
    rng = np.random.default_rng(24)
    R, T, D = 3, 100, 128
    k16 = _keys(rng, R, T)
    v16 = rng.standard_normal((R, T, D)).astype(np.float16)
    q16 = rng.standard_normal((R, D)).astype(np.float16)
    c, sel, z, idx, count, y, w = _run_pipeline(oracle, k16, v16, q16, 4, 32, 1, 1)
    for r in range(R):
        assert idx[r, 0] == sel[r].argmax()
        assert np.array_equal(y[r], v16[r, idx[r, 0]].astype(np.float32))
        assert w[r, 0] == 1.0


def test_attend_uses_pos_indirection_and_subset_softmax(oracle):
    rng = np.random.default_rng(25)
    R, G, T, D, k = 1, 2, 64, 128, 8
    k16 = _keys(rng, R, T)
    v16 = rng.standard_normal((R, 2 * T, D)).astype(np.float16)
    q16 = rng.standard_normal((R * G, D)).astype(np.float16)
    c = oracle.Cache(R, T, D, 4, 32)
    oracle.quantize(c, k16)
    sel, z = oracle.score(c, q16)
    idx, count = oracle.topk(sel, c.n, k)
    pos = (2 * T - 1 - np.arange(T, dtype=np.int32))[None].copy()     # reversed map into a longer store
    acc = np.full((R, T), 0.5, np.float32)                            # prior accumulated score
    y, w = oracle.attend(c, q16, idx, count, pos, v16, 0.05, acc=acc, want_w=True)
    for hq in range(R * G):
        l = z[hq, idx[0]].astype(np.float64) * np.float64(np.float32(0.05))
        a = np.exp(l - l.max())
        a /= a.sum()
        ref = a @ v16[0, pos[0, idx[0]]].astype(np.float64)
        assert np.allclose(y[hq], ref, rtol=1e-5, atol=1e-6)
        assert np.allclose(w[hq], a, rtol=1e-6)
    # accumulated score: sum over the group's heads, only on selected slots, strictly positive there
    assert np.allclose(acc[0, idx[0]], 0.5 + w.sum(0), rtol=1e-6)
    mask = np.ones(T, bool)
    mask[idx[0]] = False
    assert np.all(acc[0, mask] == 0.5) and np.all(acc[0, idx[0]] > 0.5)
    # logits far beyond exp's range: the softmax must stay finite (max-subtracted form)
    acc2 = np.zeros((R, T), np.float32)
    y2, w2 = oracle.attend(c, q16, idx, count, pos, v16, 50.0, acc=acc2, want_w=True)
    assert (w2 == 0).any()                       # some weights underflow ...
    assert np.all(acc2[0, idx[0]] >= np.float32(G * 1e-30))   # ... yet every selected slot is marked
    for hq in range(R * G):
        l = torch.from_numpy(z[hq, idx[0]].astype(np.float64) * np.float64(np.float32(50.0)))
        assert l.max() > 800
        ref = torch.softmax(l, 0).numpy() @ v16[0, pos[0, idx[0]]].astype(np.float64)
        assert np.all(np.isfinite(y2[hq])) and np.allclose(y2[hq], ref, rtol=1e-5, atol=1e-6)


def test_selection_overlaps_exact_topk(oracle):
    """Sanity on the synthetic workload: the set selected from 4-bit scores overlaps the set an
    exact fp64 q . k would select by > 85%, and the planted tokens of a head share one score."""
    import synth_inputs as S
    w = S.Workload("t", 91, 1, 8, 2, 2048, 4, 32, 128)
    d = S.make_layer(w)
    R = w.batch * w.n_kv_heads
    k16 = d["keys"].numpy().reshape(R, w.n, 128)
    v16 = d["values"].numpy().reshape(R, w.n, 128)
    q16 = d["q"].numpy().reshape(R * w.gqa, 128)
    c, sel, z, idx, count, y, wts = _run_pipeline(oracle, k16, v16, q16, 4, 32, w.k, w.gqa)
    planted = d["planted"].numpy().reshape(R * w.gqa, w.planted)
    for r in range(R):
        exact = np.stack([k16[r].astype(np.float64) @ q16[r * w.gqa + g].astype(np.float64)
                          for g in range(w.gqa)]).max(0)
        ref = set(np.argsort(-exact, kind="stable")[: w.k])
        assert len(ref & set(idx[r])) >= 0.85 * w.k
    for hq in range(R * w.gqa):
        assert len(set(z[hq, planted[hq]])) == 1
        # a planted token scores about |u|^2: far above the bulk of its head's scores
        assert (z[hq] > z[hq, planted[hq][0]]).mean() < 0.1


# ----------------------------------------------------------------- evict ---

def _brute_evict(acc, n, M, Rp):
    if n <= M:
        return list(range(n))
    free = list(range(n - Rp))
    free.sort(key=lambda j: (-acc[j], j))
    return sorted(free[: M - Rp] + list(range(n - Rp, n)))


@pytest.mark.parametrize("n,M,Rp", [(64, 48, 0), (64, 48, 8), (64, 64, 4), (50, 64, 4), (64, 1, 1),
                                    (33, 32, 32), (64, 17, 3)])
def test_evict_brute_force_and_invariants(oracle, n, M, Rp):
    rng = np.random.default_rng(n * 1000 + M * 10 + Rp)
    R, D, cap = 3, 128, 70
    k16 = _keys(rng, R, n)
    c = oracle.Cache(R, cap, D, 4, 32)
    oracle.quantize(c, k16)
    before = c.copy()
    acc = np.zeros((R, cap), np.float32)
    acc[:, :n] = rng.integers(0, 6, (R, n)).astype(np.float32) * 0.25      # many ties
    acc[2, :n] = rng.standard_normal(n).astype(np.float32) ** 2
    pos = np.zeros((R, cap), np.int32)
    pos[:, :n] = rng.permutation(1000)[:n].astype(np.int32)
    acc0, pos0 = acc.copy(), pos.copy()
    kept = oracle.evict(c, acc, pos, M, Rp)
    for r in range(R):
        ref = _brute_evict(acc0[r], n, M, Rp)
        m = len(ref)
        assert c.n[r] == m == min(n, M)
        assert list(kept[r, :m]) == ref and np.all(kept[r, m:] == -1)
        assert np.all(np.diff(kept[r, :m]) > 0)
        if n > M:
            assert set(range(n - Rp, n)).issubset(set(ref))
            ev = sorted(set(range(n - Rp)) - set(ref))
            kp = [j for j in ref if j < n - Rp]
            if ev and kp:
                assert acc0[r, kp].min() >= acc0[r, ev].max()
        assert np.array_equal(c.codes[r, :m], before.codes[r, ref])
        assert np.array_equal(c.scale[r, :m], before.scale[r, ref])
        assert np.array_equal(c.zero[r, :m], before.zero[r, ref])
        assert np.array_equal(acc[r, :m], acc0[r, ref])
        assert np.array_equal(pos[r, :m], pos0[r, ref])
    # idempotent once n <= M
    snap = c.copy()
    acc1, pos1 = acc.copy(), pos.copy()
    oracle.evict(c, acc, pos, M, Rp)
    assert np.array_equal(c.codes, snap.codes) and np.array_equal(acc, acc1) and np.array_equal(pos, pos1)


def test_evict_pos_composition(oracle):
    """Repeated evictions keep pos pointing at the original rows: equals a list filter."""
    rng = np.random.default_rng(77)
    R, D, cap = 1, 128, 40
    c = oracle.Cache(R, cap, D, 4, 32)
    acc = np.zeros((R, cap), np.float32)
    pos = np.zeros((R, cap), np.int32)
    alive = []
    nxt = 0
    for rnd in range(6):
        T = 8
        oracle.quantize(c, _keys(rng, R, T))
        n = int(c.n[0])
        pos[0, n - T:n] = np.arange(nxt, nxt + T)
        acc[0, n - T:n] = 0
        alive += list(range(nxt, nxt + T))
        nxt += T
        acc[0, :n] += rng.integers(0, 4, n).astype(np.float32)
        a0 = acc[0, :n].copy()
        ref = _brute_evict(a0, n, 20, 4)
        oracle.evict(c, acc, pos, 20, 4)
        alive = [alive[j] for j in ref]
        assert list(pos[0, :int(c.n[0])]) == alive


# ------------------------------------------- the paper's un-renormalised weights (Eq. 5) ---

def test_lse_and_global_weights_against_numpy(oracle):
    """lse over all resident tokens against numpy's logsumexp; with it, attend uses softmax_all(l)[selected]
    (Sec. 3.2, Eq. 5: the selected weights are not renormalised), checked against numpy in fp64; with every
    token selected both forms coincide."""
    rng = np.random.default_rng(808)
    R, G, n, k, D = 2, 4, 300, 25, 128
    c = oracle.Cache(R, n + 6, D, 4, 32)
    oracle.quantize(c, _keys(rng, R, n))
    q = (2 * rng.standard_normal((R * G, D))).astype(np.float16)
    V = rng.standard_normal((R, n + 6, D)).astype(np.float16)
    sel, z = oracle.score(c, q)
    sm = 0.11
    L = oracle.lse(z, R, c.n, sm)
    l64 = z[:, :n].astype(np.float32) * np.float32(sm)
    ref = np.log(np.exp(l64.astype(np.float64) - l64.max(1, keepdims=True)).sum(1)) + l64.max(1)
    assert np.allclose(L, ref, rtol=1e-6, atol=1e-6)
    idx, count = oracle.topk(sel, c.n, k)
    pos = np.tile(np.arange(n + 6, dtype=np.int32), (R, 1))
    acc = np.zeros((R, n + 6), np.float32)
    y, w = oracle.attend(c, q, idx, count, pos, V, sm, acc=acc, want_w=True, lse=L)
    acc_ref = np.zeros((R, n + 6))
    for hq in range(R * G):
        r = hq // G
        a_all = np.exp(l64[hq].astype(np.float64) - ref[hq])                     # softmax over all n
        assert abs(a_all.sum() - 1) < 1e-9
        a = a_all[idx[r]]
        assert np.allclose(w[hq], a, rtol=1e-5, atol=1e-12) and w[hq].sum() < 1
        assert np.allclose(y[hq], a @ V[r, idx[r]].astype(np.float64), rtol=1e-5, atol=1e-7)
        acc_ref[r, idx[r]] += a
    assert np.allclose(acc, acc_ref, rtol=1e-5, atol=1e-12)
    # k = n: the two normalisations agree and both are standard attention over the dequantised keys
    idx, count = oracle.topk(sel, c.n, n)
    ya, _ = oracle.attend(c, q, idx, count, pos, V, sm)
    yb, _ = oracle.attend(c, q, idx, count, pos, V, sm, lse=L)
    assert np.allclose(ya, yb, rtol=1e-5, atol=1e-7)
    assert np.all(np.isneginf(oracle.lse(z, R, [0, 0], sm)))
