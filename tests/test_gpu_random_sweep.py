"""Seeded random sweep of the streaming entry points: every argument drawn at random within its
documented range (size, element type, threshold, format, scale, rounding, seed, element offset,
output kind), the result compared bit for bit with the CPU oracle.  The fixed grids of the other
parity files cover the corners; this one covers combinations nobody thought of."""
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


def to_dev(a):
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def raw(t, like):
    a = t.cpu().numpy()
    if like.dtype == np.uint16:
        return a.view(np.uint16)
    if like.dtype == np.float16:
        return a.view(np.uint16)
    return a.view(np.uint32) if a.dtype == np.float32 else a


def alpha_in_dtype(alpha, dtype):
    """A threshold that is a value of the tensor's element type (as lgn_threshold would produce)."""
    if dtype == SI.BF16:
        return float(SI.bf16_bits_to_f32(SI.f32_to_bf16_bits(np.float32([alpha])))[0])
    if dtype == SI.F16:
        return float(np.float16(alpha))
    return float(np.float32(alpha))


def draw_case(rng):
    dtype = (SI.F32, SI.BF16, SI.F16)[int(rng.integers(0, 3))]
    n = int(rng.choice([rng.integers(1, 600), rng.integers(600, 70_000), rng.integers(70_000, 400_000)]))
    mu = float(rng.uniform(-14.0, -4.0)) if dtype != SI.F16 else float(rng.uniform(-9.0, -3.0))
    sigma = float(rng.uniform(0.3, 3.0))
    g = SI.lognormal_tensor(n, seed=int(rng.integers(0, 1 << 30)), mu=mu, sigma=sigma,
                            zero_frac=float(rng.uniform(0.0, 0.6)), dtype=dtype)
    nb = int(rng.integers(2, 9))
    e = int(rng.integers(1, nb))
    m = nb - 1 - e
    # scale so that the bulk of the tensor lands inside, below or above the format's range
    s = int(round(mu / np.log(2.0))) + int(rng.integers(-6, 7)) - (1 << (e - 1)) // 2
    alpha = alpha_in_dtype(float(np.exp(mu + sigma * rng.uniform(-1.5, 2.5))), dtype) if rng.random() < 0.9 else 0.0
    rounding = int(rng.integers(0, 2))
    seed = int(rng.integers(0, 1 << 62))
    offset = int(rng.choice([0, 4 * rng.integers(0, 1 << 40), rng.integers(0, 1 << 34),
                             (1 << 34) - 4 * rng.integers(1, 2000)]))   # aligned, unaligned, near a counter carry
    return dtype, g, alpha, e, m, s, rounding, seed, offset


def test_random_sweep_of_the_streaming_calls(lgn):
    rng = np.random.default_rng(777)
    lgn_dtype = {SI.F32: lgn.LGN_F32, SI.BF16: lgn.LGN_BF16, SI.F16: lgn.LGN_F16}
    for case in range(160):
        dtype, g, alpha, e, m, s, rounding, seed, offset = draw_case(rng)
        ctx = (case, dtype, g.size, alpha, e, m, s, rounding, seed, offset)
        d = to_dev(g)
        if dtype == SI.F16:
            d = d.view(torch.float16) if d.dtype != torch.float16 else d
        p = lgn.upload_struct(lgn.LgnPruneParams(alpha, 0, 0.0, 0.0))
        f = lgn.upload_struct(lgn.LgnFpParams(1 + e + m, e, m, s, 0.0, 0, 0))
        kind = (O.OUT_CODE8, O.OUT_PACKED, O.OUT_VALUE)[case % 3]
        want = O.prune_quantize(g, alpha, e, m, s, rounding, seed, offset, kind)
        got = lgn.lgn_prune_quantize_fused(d, p, f, rounding, seed, offset, out_kind=kind, n_bits=1 + e + m,
                                           dtype=lgn_dtype[dtype])
        if kind == O.OUT_VALUE:
            assert np.array_equal(raw(got, g), raw(_as_tensor(want), g)), ctx
        else:
            assert np.array_equal(got.cpu().numpy(), want), ctx
        # the two halves of the composition, every third case each
        if case % 3 == 0:
            wantp = O.prune(g, alpha, seed, offset)
            gotp = lgn.lgn_prune(d, p, seed, offset, dtype=lgn_dtype[dtype])
            assert np.array_equal(raw(gotp, g), raw(_as_tensor(wantp), g)), ctx
        elif case % 3 == 1:
            wantq = O.fp_quantize(g, e, m, s, rounding, seed, offset, O.OUT_CODE8)
            gotq = lgn.lgn_fp_quantize(d, f, rounding, seed, offset, out_kind=O.OUT_CODE8, dtype=lgn_dtype[dtype])
            assert np.array_equal(gotq.cpu().numpy(), wantq), ctx


class _as_tensor:
    """numpy array wrapped so that raw() can treat oracle output like a device result."""

    def __init__(self, a):
        self.a = a

    def cpu(self):
        return self

    def numpy(self):
        return self.a
