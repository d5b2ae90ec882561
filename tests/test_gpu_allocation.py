"""Parity of the histogram pass and of the heterogeneous sparsity allocation with the oracle."""
import math

import numpy as np
import pytest

import oracle as O
import synth_inputs as SI

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lgn():
    import paper_2006_08173_amd as m
    m.load()
    return m


def to_dev(a: np.ndarray):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


@pytest.mark.parametrize("dtype", [SI.F32, SI.BF16])
def test_histogram_parity(lgn, dtype):
    for n in (0, 1, 3, 7, 255, 4099, 1_000_003, 5_000_000):
        g = SI.lognormal_tensor(n, seed=60 + n % 11, mu=-11.0, sigma=3.0, zero_frac=0.25, dtype=dtype)
        if n > 20:
            sp = np.array([np.inf, -np.inf, np.nan, 1e-45, -3e-39, 3.4e38, -0.0], np.float32)
            g[:7] = sp if dtype == SI.F32 else SI.f32_to_bf16_bits(sp)
        got = lgn.lgn_log_histogram(to_dev(g)).cpu().numpy().view(np.uint64)
        assert np.array_equal(got, O.log_histogram(g)), n


def upload_stats(lgn, stats):
    raw = b"".join(bytes(lgn.LgnStats(s.n, s.nnz, s.n_nonfinite, s.mu / math.log(2.0), 0.0, s.mu, s.sigma,
                                      s.max_abs, s.min_abs_nz, s.status, 0)) for s in stats)
    return torch.from_numpy(np.frombuffer(raw, dtype=np.uint8).copy()).cuda()


def layer_stats(seed=2):
    rng = np.random.default_rng(seed)
    sizes = [256 * c * h * w for c, h, w in ([(512, 7, 7)] * 5 + [(256, 14, 14)] * 5 + [(128, 28, 28)] * 5
                                             + [(64, 56, 56)] * 4 + [(64, 112, 112)])]
    out = []
    for n in sizes:
        nnz = int(n * rng.uniform(0.4, 0.7))
        out.append(O.make_stats(n, nnz, rng.uniform(-16, -8), rng.uniform(1.2, 2.2), 1.0, 1e-30))
    return out


def compare(lgn, stats, hists, S, min_cos, cap, alpha_dtype=0):
    n = len(stats)
    dst = upload_stats(lgn, stats)
    dh = None if hists is None else torch.from_numpy(np.ascontiguousarray(hists).view(np.int64)).cuda()
    dmc = torch.tensor(min_cos, dtype=torch.float64, device="cuda") if len(min_cos) else None
    p_buf, a_buf = lgn.lgn_sparsity_allocate(dst, dh, n, S, dmc, cap, 0.997, alpha_dtype)
    got_p = lgn.read_array(p_buf, lgn.LgnPruneParams, n)
    got_a = lgn.read_array(a_buf, lgn.LgnAlloc, n)
    want_p, want_a = O.sparsity_allocate(stats, hists, S, min_cos, cap, 0.997, alpha_dtype)
    for i in range(n):
        assert np.float32(got_p[i].alpha) == np.float32(want_p[i].alpha), i
        assert got_p[i].status == want_p[i].status and got_a[i].status == want_a[i].status, i
        assert got_p[i].s_pred == pytest.approx(want_p[i].s_pred, abs=1e-12)
        assert got_a[i].sparsity == pytest.approx(want_a[i].sparsity, abs=1e-12)
        assert got_a[i].cosine == pytest.approx(want_a[i].cosine, abs=1e-12)
        assert got_a[i].k == pytest.approx(want_a[i].k, rel=1e-12, abs=1e-12)
    return got_p, got_a


def test_allocation_parity_scenarios(lgn):
    stats = layer_stats()
    for S, min_cos, cap in ((0.9, [], 0.98), (0.9, [0.98] * 5 + [0.95] * 5, 0.98), (0.9, [0.98] * 5 + [0.95] * 5, 0.905),
                            (0.8, [0.999] * 15, 0.97), (0.95, [0.9] * 3, 0.96), (0.5, [0.99] * 20, 0.97)):
        p, a = compare(lgn, stats, None, S, min_cos, cap)
    compare(lgn, stats, None, 0.9, [0.98] * 5, 0.98, alpha_dtype=1)     # bf16 thresholds
    # degenerate layers: empty, point mass, already sparser than asked
    odd = [O.make_stats(1000, 0, float("nan"), float("nan"), 0.0, 0.0, 0, O.ST_EMPTY),
           O.make_stats(1000, 900, -3.0, 0.0, 0.05, 0.05, 0, O.ST_SIGMA0),
           O.make_stats(1000, 50, -5.0, 2.0, 1.0, 1e-9)] + layer_stats(5)[:4]
    compare(lgn, odd, None, 0.9, [0.99, 0.99, 0.99, 0.99], 0.97)


def test_allocation_from_tensors_on_the_device(lgn):
    """Statistics, histograms and allocation for a small network without leaving the device."""
    rng = np.random.default_rng(9)
    layers, devs = [], []
    for i, n in enumerate([40_000, 40_000, 160_000, 160_000, 640_000, 640_000]):
        mu, sigma = float(rng.uniform(-14, -9)), float(rng.uniform(1.3, 2.0))
        g = SI.lognormal_tensor(n, seed=300 + i, mu=mu, sigma=sigma, zero_frac=0.5)
        g[np.abs(g) > math.exp(mu + 2.5 * sigma)] = 0      # truncated, as the paper finds real gradients to be
        layers.append(g)
        devs.append(to_dev(g))
    L = len(layers)
    st_all = torch.empty(L * 72, dtype=torch.uint8, device="cuda")
    h_all = torch.empty(L, lgn.LGN_HIST_BINS, dtype=torch.int64, device="cuda")
    for i, d in enumerate(devs):
        lgn.lgn_stats(d, out=st_all[i * 72:(i + 1) * 72])
        lgn.lgn_log_histogram(d, out=h_all[i])
    dev_stats = lgn.read_array(st_all, lgn.LgnStats, L)
    same_in = [O.make_stats(s.n, s.nnz, s.mu, s.sigma, s.max_abs, s.min_abs_nz, s.n_nonfinite, s.status) for s in dev_stats]
    hists = np.stack([O.log_histogram(g) for g in layers])
    assert np.array_equal(h_all.cpu().numpy().view(np.uint64), hists)
    min_cos = [0.97, 0.97]
    dmc = torch.tensor(min_cos, dtype=torch.float64, device="cuda")
    p_buf, a_buf = lgn.lgn_sparsity_allocate(st_all, h_all, L, 0.9, dmc, 0.97)
    got_p = lgn.read_array(p_buf, lgn.LgnPruneParams, L)
    got_a = lgn.read_array(a_buf, lgn.LgnAlloc, L)
    want_p, want_a = O.sparsity_allocate(same_in, hists, 0.9, min_cos, 0.97)
    total = sum(g.size for g in layers)
    achieved = 0.0
    for i in range(L):
        assert np.float32(got_p[i].alpha) == np.float32(want_p[i].alpha)
        assert got_a[i].status == want_a[i].status
        assert got_a[i].k == pytest.approx(want_a[i].k, rel=1e-12)
        # prune with the allocated threshold: the predicted sparsity and cosine are what comes out
        y = lgn.lgn_prune(devs[i], p_buf[i * 24:(i + 1) * 24], 700 + i, 0).cpu().numpy()
        s_meas = float(np.mean(y == 0))
        assert abs(s_meas - got_a[i].sparsity) < 6e-3
        x = layers[i].astype(np.float64)
        cos = float(x @ y / math.sqrt((x @ x) * (y.astype(np.float64) @ y)))
        # the 0.997-quantile sits a little below the true cut, so the closed form is slightly pessimistic
        assert -0.005 < cos - got_a[i].cosine < 0.045
        achieved += s_meas * layers[i].size / total
    assert abs(achieved - 0.9) < 6e-3 or any(a.status & lgn.LGN_ALLOC_CAPPED for a in got_a)
