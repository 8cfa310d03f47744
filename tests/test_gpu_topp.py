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
