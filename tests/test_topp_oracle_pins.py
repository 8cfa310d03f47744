"""Pins for the oracle of the paper's selection rule (Eq. 4, oracle/hca_topp_oracle.c): the integer weight
against exp, the selected prefix against a brute-force search and an fp64 softmax, closed forms, the
tau = 1 row of the paper's threshold table.  CPU only."""
import math
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_closed_forms.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_weight_tracks_exp_and_is_monotone(oracle):
    us = -np.concatenate([np.linspace(0, 14, 3000), np.random.default_rng(0).uniform(0, 14, 3000)])
    w = np.array([oracle.topp_weight(u) for u in us], np.float64)
    ref = np.exp(np.float32(us).astype(np.float64)) * 2.0 ** 31
    assert np.all(np.abs(w - ref) <= 2e-5 * ref + 1.0)           # polynomial ~1e-5, truncation to an integer
    order = np.argsort(us)
    assert np.all(np.diff(w[order]) >= 0)
    assert oracle.topp_weight(0.0) == 2 ** 31
    assert oracle.topp_weight(-23.0) == 0 and oracle.topp_weight(-1e30) == 0 and oracle.topp_weight(-math.inf) == 0


def _brute(oracle, v, sm, tau, k_max):
    """Prefix search written out in Python on the same integer weights."""
    n = len(v)
    order = sorted(range(n), key=lambda j: (-float(v[j]), j))
    l = (v.astype(np.float32) * np.float32(sm)).astype(np.float32)
    m = l.max()
    w = [oracle.topp_weight(float(np.float32(l[j] - m))) for j in order]
    Z = sum(w)
    theta = Z if tau >= 1 else max(1, (Z * int(math.ldexp(tau, 64))) >> 64)
    run, ks = 0, n
    for i, x in enumerate(w):
        run += x
        if run >= theta:
            ks = i + 1
            break
    return ks, sorted(order[:min(ks, k_max)]), theta, Z


@pytest.mark.parametrize("tau", [0.3, 0.5, 0.9, 0.99, 1.0])
@pytest.mark.parametrize("sm", [0.0884, 0.5])
def test_prefix_against_brute_force_and_fp64_softmax(oracle, tau, sm):
    rng = np.random.default_rng(int(tau * 100) + int(sm * 1000))
    R, n, cap, k_max = 3, 700, 720, 650
    sel = np.zeros((R, cap), np.float32)
    sel[:, :n] = rng.standard_normal((R, n)).astype(np.float32) * 12
    sel[1, :n] = np.round(sel[1, :n])                                    # ties
    sel[2, 5::50] += 60                                                  # a few dominant tokens
    idx, count, kstar, mass = oracle.topp(sel, [n] * R, sm, tau, k_max)
    for r in range(R):
        ks, ref, theta, Z = _brute(oracle, sel[r, :n], sm, tau, k_max)
        assert kstar[r] == ks and count[r] == min(ks, k_max)
        assert list(idx[r, :count[r]]) == ref and np.all(idx[r, count[r]:] == -1)
        assert int(mass[r, 0]) == theta and int(mass[r, 1]) == Z
        # against an exact softmax: the prefix reaches tau, one token less does not (up to the weight's 1e-5)
        l = sel[r, :n].astype(np.float64) * np.float64(np.float32(sm))
        a = np.exp(l - l.max())
        a /= a.sum()
        order = sorted(range(n), key=lambda j: (-float(sel[r, j]), j))
        cum = np.cumsum(a[order])
        assert cum[ks - 1] >= tau - 1e-4
        if ks > 1:
            assert cum[ks - 2] < tau + 1e-4


def test_closed_forms(oracle):
    gold = _golden()
    n = 1000
    # equal scores: every weight is 2^31, so k* = ceil(tau n) for dyadic tau; ties go to the lower slots
    sel = np.full((1, n), 3.5, np.float32)
    for tau, want in ((0.5, 500), (0.25, 250), (1.0, n)):
        idx, count, kstar, _ = oracle.topp(sel, [n], 0.1, tau, n)
        assert kstar[0] == want and list(idx[0, :want]) == list(range(want))
    # the paper's threshold table: tau = 1 keeps everything (weights within 2^-31 of the maximum all count)
    sel = np.random.default_rng(1).uniform(-50, 50, (1, n)).astype(np.float32)
    idx, count, kstar, _ = oracle.topp(sel, [n], 0.0884, 1.0, n)
    assert kstar[0] / n == gold["tau_one_selection_ratio"] and list(idx[0]) == list(range(n))
    # one dominant token
    sel = np.zeros((1, n), np.float32)
    sel[0, 321] = 400.0
    idx, count, kstar, _ = oracle.topp(sel, [n], 0.0884, 0.9, 8)
    assert kstar[0] == 1 and count[0] == 1 and idx[0, 0] == 321
    # sharper softmax -> shorter prefix
    sel = np.random.default_rng(2).standard_normal((1, n)).astype(np.float32) * 10
    ks = [int(oracle.topp(sel, [n], s, 0.8, n)[2][0]) for s in (0.02, 0.1, 0.5, 2.0)]
    assert ks == sorted(ks, reverse=True) and ks[0] > ks[-1]


def test_clip_gives_the_top_k_set_and_ragged_rows(oracle):
    rng = np.random.default_rng(5)
    cap = 400
    sel = rng.standard_normal((4, cap)).astype(np.float32)
    n = [400, 0, 17, 250]
    idx, count, kstar, _ = oracle.topp(sel, n, 0.05, 0.95, 30)
    ridx, rcount = oracle.topk(sel, n, 30)
    assert list(count) == [30, 0, min(int(kstar[2]), 30), 30] and kstar[1] == 0
    for r in (0, 3):
        assert kstar[r] > 30 and np.array_equal(idx[r], ridx[r])
    assert np.array_equal(idx[2, :count[2]], np.sort(np.argsort(-sel[2, :17], kind="stable")[:count[2]]))


def topp_margin(n, Z):
    """How far the attention mass of the integer form's prefix may lie from the fp64 one (derivation: every integer
    weight is exp(u) 2^31 (1 + d) with |d| <= 3e-5 - polynomial 2e-5, fp32 logit and product roundings the rest -
    minus a truncation below one unit; a prefix sum over Z therefore moves by at most 2 * 3e-5 relative plus n
    units out of Z >= 2^31)."""
    return 6e-5 + n / float(Z)


@pytest.mark.parametrize("tau", [0.3, 0.9, 0.999])
def test_plain_eq4_against_numpy_and_the_integer_form_against_it(oracle, tau):
    """hco_topp_plain is Eq. 4 as written (fp64 softmax, sort, shortest prefix reaching tau): checked against numpy.
    The integer form's k* is then valid for the plain one up to the stated margin: its prefix holds at least
    tau - eps of the plain mass and one slot less holds less than tau + eps."""
    rng = np.random.default_rng(int(tau * 1000))
    R, n, cap = 4, 3000, 3010
    sm = 0.0884
    sel = np.zeros((R, cap), np.float32)
    sel[:, :n] = rng.standard_normal((R, n)).astype(np.float32) * 30
    sel[1, :n] = np.round(sel[1, :n] / 4) * 4                              # heavy ties
    sel[2, :n] *= 0.05                                                     # nearly flat: long prefix
    sel[3, 7] = 900.0                                                      # one dominant token
    ns = [n, n, n, n - 100]
    kp, order, cum = oracle.topp_plain(sel, ns, sm, tau)
    _, _, ks, mass = oracle.topp(sel, ns, sm, tau, n)
    for r in range(R):
        nr = ns[r]
        l = sel[r, :nr].astype(np.float64) * sm
        a = np.exp(l - l.max())
        a /= a.sum()
        o = np.lexsort((np.arange(nr), -sel[r, :nr].astype(np.float64)))
        ref = np.cumsum(a[o])
        assert np.array_equal(order[r, :nr], o)
        assert np.allclose(cum[r, :nr], ref, rtol=1e-12, atol=1e-15)
        want = int(np.argmax(ref >= tau)) + 1 if ref[-1] >= tau else nr
        assert kp[r] == want
        eps = topp_margin(nr, int(mass[r, 1]))
        k = int(ks[r])
        assert cum[r, k - 1] >= tau - eps
        assert k == 1 or cum[r, k - 2] < tau + eps
        # and wherever the plain prefix clears tau by more than the margin on both sides, the two agree
        if cum[r, kp[r] - 1] >= tau + eps and (kp[r] == 1 or cum[r, kp[r] - 2] < tau - eps):
            assert k == kp[r]
    # equal scores: the mass of a prefix is its length over n (closed form)
    flat = np.full((1, 100), 2.0, np.float32)
    kp, _, cum = oracle.topp_plain(flat, [100], 0.3, 0.25)
    assert kp[0] == 25 and np.allclose(cum[0], np.arange(1, 101) / 100, rtol=1e-12)
