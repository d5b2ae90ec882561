"""Parity of the prefix coder (appendix "Encoding") with the oracle: stream bytes and chunk table
bit for bit, decoding on the device returns the input, and the paper's bits-per-value claim holds
on the device output."""
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


def host_table(table, n):
    """The table proper: one entry per chunk, the total and the status (scratch follows it)."""
    nchunks = (n + 4095) // 4096
    return table.cpu().numpy().view(np.uint64)[: nchunks + 2]


def host_stream(buf, table, n):
    t = host_table(table, n)
    return buf.cpu().numpy()[: int(t[-2]) * 4], t


def pruned_like(n, seed, dtype, alpha=2.5e-4):
    """Values as lgn_prune leaves them: many zeros, many +-alpha, the rest lognormal above alpha."""
    rng = np.random.default_rng(seed)
    v = SI.lognormal_tensor(n, seed=seed, mu=-7.0, sigma=2.0, zero_frac=0.0, dtype=SI.F32)
    r = rng.random(n)
    v[r < 0.25] = np.float32(alpha)
    v[r < 0.10] = -np.float32(alpha)
    v[r > 0.45] = 0.0
    if n > 9:
        v[7] = -0.0                                       # sign bit only: long codeword, survives
        v[9] = np.float32(np.nan)
    return v if dtype == SI.F32 else SI.f32_to_bf16_bits(v)


SIZES = [0, 1, 15, 16, 17, 255, 4095, 4096, 4097, 3 * 4096 + 1234, 40 * 4096 + 5]


@pytest.mark.parametrize("dtype", [SI.F32, SI.BF16])
def test_value_streams_match_oracle(lgn, dtype):
    alpha = 2.5e-4 if dtype == SI.F32 else float(SI.bf16_bits_to_f32(SI.f32_to_bf16_bits(np.float32([2.5e-4])))[0])
    p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
    width = 32 if dtype == SI.F32 else 16
    special = O.prefix_special_of_alpha(alpha, width)
    for n in SIZES:
        a = pruned_like(n, 40 + n % 7, dtype, alpha)
        d = to_dev(a)
        buf, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_VALUE, p)
        got, t = host_stream(buf, table, n)
        want, wt, wsub = O.prefix_encode(a, special, with_sub=True)
        assert np.array_equal(t, wt), n
        assert np.array_equal(got, want), n
        assert np.array_equal(lgn.prefix_sub_lengths(table, n).cpu().numpy().view(np.uint16), wsub), n
        back = lgn.lgn_prefix_decode(buf, table, n, lgn.LGN_OUT_VALUE, p,
                                     dtype=lgn.LGN_F32 if dtype == SI.F32 else lgn.LGN_BF16)
        raw = back.view(torch.int32 if dtype == SI.F32 else torch.int16).cpu().numpy()
        assert np.array_equal(raw.view(np.uint32 if dtype == SI.F32 else np.uint16),
                              a.view(np.uint32 if dtype == SI.F32 else np.uint16)), n


@pytest.mark.parametrize("n_bits,e", [(2, 1), (4, 2), (6, 3), (8, 5), (8, 2)])
def test_code_streams_match_oracle(lgn, n_bits, e):
    m = n_bits - 1 - e
    s = -14
    alpha = 3.1e-4
    p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
    f = lgn.upload_struct(lgn.LgnFpParams(n_bits, e, m, s, 0.0, 0, 0))
    special = O.prefix_special_of_code(alpha, e, m, s)
    rng = np.random.default_rng(n_bits * 10 + e)
    for n in SIZES:
        codes = rng.integers(0, 1 << n_bits, n, dtype=np.uint8)
        r = rng.random(n)
        codes[r < 0.3] = special | (rng.integers(0, 2, n, dtype=np.uint8)[r < 0.3] << (n_bits - 1))
        codes[r > 0.5] = 0
        d = to_dev(codes)
        buf, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_CODE8, p, f)
        got, t = host_stream(buf, table, n)
        want, wt, wsub = O.prefix_encode(codes, special, n_bits, with_sub=True)
        assert np.array_equal(t, wt), n
        assert np.array_equal(got, want), n
        assert np.array_equal(lgn.prefix_sub_lengths(table, n).cpu().numpy().view(np.uint16), wsub), n
        back = lgn.lgn_prefix_decode(buf, table, n, lgn.LGN_OUT_CODE8, p, f)
        assert np.array_equal(back.cpu().numpy(), codes), n


def test_code_streams_dense_empty_and_without_special(lgn):
    """Byte codes at the two ends of the density range (every code non-zero: the longest run of the
    encoder's per-thread loop; every code zero) and without a pruning threshold (two classes)."""
    n_bits, e, m, s = 6, 3, 2, -14
    f = lgn.upload_struct(lgn.LgnFpParams(n_bits, e, m, s, 0.0, 0, 0))
    alpha = 3.1e-4
    special = O.prefix_special_of_code(alpha, e, m, s)
    rng = np.random.default_rng(77)
    n = 9 * 4096 + 777
    dense = rng.integers(1, 1 << n_bits, n, dtype=np.uint8)
    dense[rng.random(n) < 0.4] = special
    cases = [(dense, alpha), (np.zeros(n, np.uint8), alpha), (dense, None),
             (np.where(rng.random(n) < 0.03, dense, 0).astype(np.uint8), alpha)]
    for codes, a in cases:
        p = lgn.upload_struct(lgn.LgnPruneParams(a, 0, 0.0, 0.0)) if a is not None else None
        sp = special if a is not None else 0
        d = to_dev(codes)
        buf, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_CODE8, p, f)
        got, t = host_stream(buf, table, n)
        want, wt = O.prefix_encode(codes, sp, n_bits)
        assert np.array_equal(t, wt)
        assert np.array_equal(got, want)
        back = lgn.lgn_prefix_decode(buf, table, n, lgn.LGN_OUT_CODE8, p, f)
        assert np.array_equal(back.cpu().numpy(), codes)


def test_no_special_class_and_small_capacity(lgn):
    a = pruned_like(5 * 4096, 3, SI.F32)
    d = to_dev(a)
    buf, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_VALUE, None)        # no alpha: two classes only
    got, t = host_stream(buf, table, a.size)
    want, wt = O.prefix_encode(a, 0)
    assert np.array_equal(t, wt) and np.array_equal(got, want)
    # a buffer that holds the first three chunks only: they are written, the status entry is set
    cap = int(wt[3]) * 4
    small = torch.full((cap + 64,), 0xEE, dtype=torch.uint8, device="cuda")
    _, table2 = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_VALUE, None, out=small[:cap])
    t2 = host_table(table2, a.size)
    assert t2[-1] == 1 and np.array_equal(t2[:-1], wt[:-1])
    hs = small.cpu().numpy()
    assert np.array_equal(hs[:cap], want[:cap]) and np.all(hs[cap:] == 0xEE)
    with pytest.raises(lgn.LgnError):
        lgn.lgn_prefix_encode(d, lgn.LGN_OUT_PACKED, None)
    with pytest.raises(lgn.LgnError):
        lgn.lgn_prefix_encode(d.view(torch.uint8), lgn.LGN_OUT_CODE8, None, None)


def test_byte_codes_with_dense_and_sparse_stretches(lgn):
    """The decoder takes a step of sixteen byte codes in one of two forms and picks the form for the
    next step from how many non-zero codes the last one held: stretches of dense and of sparse codes
    of many lengths, so that the switch happens at every position of a sub-block, in both
    directions, and differently in the lanes of a wave."""
    n_bits, e, m, s = 6, 3, 2, -14
    f = lgn.upload_struct(lgn.LgnFpParams(n_bits, e, m, s, 0.0, 0, 0))
    alpha = 3.1e-4
    p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
    special = O.prefix_special_of_code(alpha, e, m, s)
    rng = np.random.default_rng(2024)
    n = 37 * 4096 + 301
    dens = np.empty(n)
    i = 0
    while i < n:
        k = int(rng.choice([5, 16, 17, 48, 100, 256, 700, 5000]))
        dens[i:i + k] = rng.choice([0.0, 0.05, 0.15, 0.4, 0.6, 0.9, 1.0])
        i += k
    codes = rng.integers(1, 1 << n_bits, n, dtype=np.uint8)
    codes[rng.random(n) < 0.4] = special
    codes[rng.random(n) >= dens] = 0
    d = to_dev(codes)
    buf, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_CODE8, p, f)
    got, t = host_stream(buf, table, n)
    want, wt, wsub = O.prefix_encode(codes, special, n_bits, with_sub=True)
    assert np.array_equal(t, wt) and np.array_equal(got, want)
    assert np.array_equal(lgn.prefix_sub_lengths(table, n).cpu().numpy().view(np.uint16), wsub)
    back = lgn.lgn_prefix_decode(buf, table, n, lgn.LGN_OUT_CODE8, p, f)
    assert np.array_equal(back.cpu().numpy(), codes)


def test_byte_codes_small_capacity(lgn):
    """Byte codes into a buffer that ends inside the stream: the chunks that fit are written whole,
    nothing is written past the buffer, the table is complete and the status entry is set."""
    n_bits, e, m, s = 6, 3, 2, -14
    f = lgn.upload_struct(lgn.LgnFpParams(n_bits, e, m, s, 0.0, 0, 0))
    alpha = 3.1e-4
    p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
    special = O.prefix_special_of_code(alpha, e, m, s)
    rng = np.random.default_rng(5)
    n = 11 * 4096 + 100
    codes = np.where(rng.random(n) < 0.2, rng.integers(1, 1 << n_bits, n), 0).astype(np.uint8)
    want, wt = O.prefix_encode(codes, special, n_bits)
    d = to_dev(codes)
    cap = int(wt[7]) * 4 + 8                               # chunks 0..6 fit, chunk 7 does not
    small = torch.full((cap + 4096,), 0xEE, dtype=torch.uint8, device="cuda")
    _, table = lgn.lgn_prefix_encode(d, lgn.LGN_OUT_CODE8, p, f, out=small[:cap])
    t = host_table(table, n)
    assert t[-1] == 1 and np.array_equal(t[:-1], wt[:-1])
    hs = small.cpu().numpy()
    assert np.array_equal(hs[: int(wt[7]) * 4], want[: int(wt[7]) * 4])
    assert np.all(hs[cap:] == 0xEE)
    # chunks behind the one that did not fit are skipped too (they start beyond the buffer)
    assert np.all(hs[int(wt[7]) * 4 : cap] == 0xEE)


def test_chain_prune_quantize_encode_config1(lgn):
    """stats+solvers -> fused prune/quantize -> prefix code, parameters never leaving the device."""
    cfg = SI.config_c1()
    g = SI.make(cfg)
    d = to_dev(g)
    st, p, f = lgn.lgn_stats_solve(d, cfg["sparsity"], lgn.LGN_F32, cfg["n_bits"])
    codes = lgn.lgn_prune_quantize_fused(d, p, f, O.ROUND_STOCHASTIC, cfg["rng_seed"], 0, out_kind=O.OUT_CODE8)
    buf, table = lgn.lgn_prefix_encode(codes, lgn.LGN_OUT_CODE8, p, f)
    hp, hf = lgn.read_prune_params(p), lgn.read_fp_params(f)
    special = O.prefix_special_of_code(hp.alpha, hf.e_bits, hf.m_bits, hf.scale_exp)
    hc = codes.cpu().numpy()
    got, t = host_stream(buf, table, g.size)
    want, wt = O.prefix_encode(hc, special, cfg["n_bits"])
    assert np.array_equal(t, wt) and np.array_equal(got, want)
    assert np.array_equal(O.prefix_decode(got, t, g.size, cfg["n_bits"], special), hc)
    bits_per_value = got.size * 8 / g.size
    assert bits_per_value < 2.6                            # 85 % zeros, 6-bit codes for the rest


def test_bits_per_value_claim_on_device(lgn):
    """Appendix "Encoding": relative to fp32, about 4 bits per value at 80 % sparsity and about 2 at
    90 % (lognormal tensor, sigma = 2, no zeros before pruning)."""
    n = 1 << 22
    g = SI.lognormal_tensor(n, seed=12, mu=-10.0, sigma=2.0, zero_frac=0.0, dtype=SI.F32)
    d = to_dev(g)
    for sparsity, claim in ((0.8, 4.0), (0.9, 2.0)):
        st, p, _ = lgn.lgn_stats_solve(d, sparsity)
        y = lgn.lgn_prune(d, p, 5, 0)
        buf, table = lgn.lgn_prefix_encode(y, lgn.LGN_OUT_VALUE, p)
        words = int(host_table(table, n)[-2])
        assert abs(words * 32 / n - claim) < 0.35
        back = lgn.lgn_prefix_decode(buf, table, n, lgn.LGN_OUT_VALUE, p)
        assert torch.equal(back.view(torch.int32), y.view(torch.int32))
