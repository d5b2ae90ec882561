"""Pins of the oracle's prefix code (appendix "Encoding"): the printed code table, an independent
decoder written on character strings, the length identity, the chunk container, and the paper's
bits-per-value claim on a synthetic lognormal tensor."""
import math
import os

import numpy as np
import pytest

import oracle as O
import synth_inputs as SI

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "prefix_code_table.txt")


def read_table():
    words, claims = {}, []
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "claim_bits_at_sparsity":
            claims.append((float(t[1]), float(t[2])))
        else:
            words[t[0]] = t[1]
    return words, claims


def bit_string(stream: np.ndarray, first_word: int, n_words: int) -> str:
    """Stream bits as characters: bit k of the stream is bit (k & 7) of byte k >> 3."""
    bits = np.unpackbits(stream[first_word * 4:(first_word + n_words) * 4], bitorder="little")
    return "".join("1" if b else "0" for b in bits)


def lsb_first(v: int, width: int) -> str:
    return "".join("1" if (v >> b) & 1 else "0" for b in range(width))


def string_encode(raw, width, special, words):
    """The code table applied symbol by symbol with string concatenation."""
    out = []
    for v in raw:
        v = int(v)
        mag = v & ((1 << (width - 1)) - 1)
        if v == 0:
            out.append(words["zero"])
        elif special and mag == special:
            out.append(words["minus_alpha"] if v >> (width - 1) else words["plus_alpha"])
        else:
            out.append(words["other"] + lsb_first(v, width))
    return "".join(out)


def string_decode(s, count, width, special, words):
    out, k = [], 0
    for _ in range(count):
        if s.startswith(words["zero"], k):
            out.append(0)
            k += 1
        elif s.startswith(words["plus_alpha"], k):
            out.append(special)
            k += 3
        elif s.startswith(words["minus_alpha"], k):
            out.append(special | 1 << (width - 1))
            k += 3
        else:
            assert s.startswith(words["other"], k)
            k += 2
            out.append(int(s[k:k + width][::-1], 2))
            k += width
    return out, k


def test_code_table_is_prefix_free():
    words, _ = read_table()
    ws = list(words.values())
    for a in ws:
        for b in ws:
            assert a == b or not b.startswith(a)


def test_hand_example_fp32():
    words, _ = read_table()
    a = np.array([0.0, 0.5, -0.5, 1.5, 0.0], np.float32)
    stream, table = O.prefix_encode(a, O.prefix_special_of_alpha(0.5, 32))
    want = (words["zero"] + words["plus_alpha"] + words["minus_alpha"] + words["other"] +
            lsb_first(0x3FC00000, 32) + words["zero"])
    assert len(want) == 1 + 3 + 3 + 34 + 1
    assert list(table) == [0, 2, 0]                       # 42 bits -> two 32-bit words, status 0
    got = bit_string(stream, 0, 2)
    assert got[:len(want)] == want and set(got[len(want):]) <= {"0"}


@pytest.mark.parametrize("width,n_bits", [(32, None), (16, None), (6, 6), (8, 8), (4, 4), (2, 2)])
def test_matches_string_coder_and_round_trips(width, n_bits):
    words, _ = read_table()
    rng = np.random.default_rng(width)
    n = 2 * O.PREFIX_CHUNK + 37                           # three chunks, the last one ragged
    if width == 32:
        vals = rng.standard_normal(n).astype(np.float32)
        special = O.prefix_special_of_alpha(0.25, 32)
        vals[rng.random(n) < 0.2] = 0.25
        vals[rng.random(n) < 0.1] = -0.25
        vals[rng.random(n) < 0.6] = 0.0
        vals[5] = -0.0                                    # not the all-zero pattern: long codeword
        arr = vals
    elif width == 16:
        v32 = rng.standard_normal(n).astype(np.float32)
        v32[rng.random(n) < 0.3] = 0.25
        v32[rng.random(n) < 0.1] = -0.25
        v32[rng.random(n) < 0.5] = 0.0
        arr = SI.f32_to_bf16_bits(v32)
        special = O.prefix_special_of_alpha(0.25, 16)
    else:
        arr = rng.integers(0, 1 << n_bits, n, dtype=np.uint8)
        arr[rng.random(n) < 0.6] = 0
        special = 3 if n_bits > 2 else 1
    raw = arr.view({32: np.uint32, 16: np.uint16}.get(width, np.uint8))
    stream, table, sub = O.prefix_encode(arr, special, n_bits, with_sub=True)
    s2, t2 = O.prefix_encode(arr, special, n_bits)
    assert np.array_equal(s2, stream) and np.array_equal(t2, table)
    nchunks = 3
    assert table.size == nchunks + 2 and table[0] == 0 and table[-1] == 0
    assert stream.size == int(table[nchunks]) * 4
    decoded = []
    for c in range(nchunks):
        part = raw[c * O.PREFIX_CHUNK:(c + 1) * O.PREFIX_CHUNK]
        want = string_encode(part, width, special, words)
        n_words = int(table[c + 1] - table[c])
        assert n_words == (len(want) + 31) // 32          # each chunk starts on a 32-bit boundary
        got = bit_string(stream, int(table[c]), n_words)
        assert got[:len(want)] == want and set(got[len(want):]) <= {"0"}
        vals_c, used = string_decode(got, part.size, width, special, words)
        assert used == len(want)
        decoded += vals_c
        # sub-blocks of 256 elements: the listed lengths are those of the string coder, and decoding
        # can start at each listed position (string decoder from that character on)
        start = 0
        for j in range(16):
            blk = part[j * 256:(j + 1) * 256]
            assert int(sub[16 * c + j]) == len(string_encode(blk, width, special, words))
            vals_b, used_b = string_decode(got[start:], blk.size, width, special, words)
            assert np.array_equal(np.array(vals_b, dtype=raw.dtype), blk) and used_b == int(sub[16 * c + j])
            start += int(sub[16 * c + j])
        assert start == len(want)
    assert sub.size == 16 * nchunks and sub.dtype == np.uint16
    assert np.array_equal(np.array(decoded, dtype=raw.dtype), raw)
    back = O.prefix_decode(stream, table, n, width, special)
    assert np.array_equal(back, raw)
    assert np.array_equal(O.prefix_decode_sub(stream, table, sub, n, width, special), raw)
    # a wrong length anywhere but at the very end derails the sub-block decoder
    bad = sub.copy()
    bad[3] += 1
    assert not np.array_equal(O.prefix_decode_sub(stream, table, bad, n, width, special), raw)


def test_length_identity_and_bound():
    rng = np.random.default_rng(3)
    n = 10 * O.PREFIX_CHUNK
    codes = rng.integers(0, 64, n, dtype=np.uint8)
    codes[rng.random(n) < 0.7] = 0
    special = 9
    stream, table = O.prefix_encode(codes, special, 6)
    for c in range(10):
        part = codes[c * O.PREFIX_CHUNK:(c + 1) * O.PREFIX_CHUNK]
        n0 = int(np.sum(part == 0))
        na = int(np.sum((part & 31) == special))
        bits = n0 + 3 * na + 8 * (part.size - n0 - na)
        assert int(table[c + 1] - table[c]) == (bits + 31) // 32
    assert stream.size <= O.prefix_bound_bytes(n, 6)
    worst = np.full(n, 63, np.uint8)
    s2, _ = O.prefix_encode(worst, special, 6)
    assert s2.size == O.prefix_bound_bytes(n, 6)
    empty_stream, empty_table = O.prefix_encode(np.zeros(0, np.uint8), 1, 6)
    assert empty_stream.size == 0 and list(empty_table) == [0, 0]


@pytest.mark.parametrize("sigma", [2.0])
def test_bits_per_value_claim_of_the_paper(sigma):
    """Pruned fp32 tensor, no prior zeros: about 4 bits per value at 80 % sparsity, about 2 at 90 %,
    and exactly S + 3 f_alpha + 34 f_kept up to the chunk padding."""
    _, claims = read_table()
    n = 1 << 20
    g = SI.lognormal_tensor(n, seed=11, mu=-10.0, sigma=sigma, zero_frac=0.0, dtype=SI.F32)
    st = O.stats(g)
    for sparsity, claimed_bits in claims:
        p = O.threshold(st, sparsity)
        y = O.prune(g, p.alpha, 77, 0)
        stream, table = O.prefix_encode(y, O.prefix_special_of_alpha(p.alpha, 32))
        bits_per_value = stream.size * 8 / n
        f0 = float(np.mean(y == 0))
        fa = float(np.mean(np.abs(y) == np.float32(p.alpha)))
        want = f0 + 3 * fa + 34 * (1 - f0 - fa)
        assert want <= bits_per_value <= want + 32 / O.PREFIX_CHUNK
        assert abs(f0 - sparsity) < 5e-3
        assert abs(bits_per_value - claimed_bits) < 0.35, (sparsity, bits_per_value)
        back = O.prefix_decode(stream, table, n, 32, O.prefix_special_of_alpha(p.alpha, 32))
        assert np.array_equal(back, y.view(np.uint32))
