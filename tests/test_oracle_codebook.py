"""Pins for the oracle's NF codebook and storage formula (Section 2.2; Eq. 3)."""
import math
import os
from statistics import NormalDist

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 6, 7, 8])
def test_codebook_identities(oracle, bits):
    q = oracle.codebook(bits)
    half = 1 << (bits - 1)
    assert q.dtype == np.float32 and q.size == 1 << bits
    assert q[0] == -1.0 and q[-1] == 1.0
    assert q[half - 1] == 0.0                      # p = 1/2 is the 2^(b-1)-th probability
    assert np.all(np.diff(q.astype(np.float64)) > 0)
    assert np.sum(q < 0) == half - 1 and np.sum(q > 0) == half   # asymmetric split


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_codebook_against_library_quantile(oracle, bits):
    # the recipe of Section 2.2 evaluated with an independent inverse normal CDF
    nd = NormalDist()
    delta = 0.5 * (1 / 30 + 1 / 32)
    half = 1 << (bits - 1)
    neg = [delta + i * (0.5 - delta) / (half - 1) for i in range(half)]
    pos = [0.5 + i * (0.5 - delta) / half for i in range(half + 1)]
    probs = neg + pos[1:]
    assert len(probs) == 1 << bits
    assert probs[0] == delta and probs[half - 1] == 0.5 and abs(probs[-1] - (1 - delta)) < 1e-15
    quant = [nd.inv_cdf(p) for p in probs]
    ref = np.array([x / quant[-1] for x in quant])
    ref[half - 1] = 0.0
    q = oracle.codebook(bits).astype(np.float64)
    assert np.max(np.abs(q - ref)) < 1e-7


def test_quantile_function_closed_forms(oracle):
    assert abs(oracle.norm_ppf(0.5)) < 1e-15
    assert abs(oracle.norm_ppf(0.975) - 1.959963984540054) < 1e-12
    assert abs(oracle.norm_ppf(0.8413447460685429) - 1.0) < 1e-12
    assert abs(oracle.norm_ppf(0.1) + oracle.norm_ppf(0.9)) < 1e-12
    # the normalising quantile Phi^-1(1 - delta)
    assert abs(oracle.norm_ppf(1 - 0.5 * (1 / 30 + 1 / 32)) - 1.8481314) < 1e-6


def test_storage_values_printed_in_the_paper(oracle):
    """tests/golden/storage_bits_per_parameter.txt: the bits per parameter the paper prints (three decimals)."""
    rows = [l.split("#")[0].split() for l in open(os.path.join(GOLD, "storage_bits_per_parameter.txt"))]
    rows = [r for r in rows if r]
    seen = 0
    for r in rows:
        if r[0] == "search_space":
            assert int(r[1]) == 3 ** 5
            continue
        b0, b1, b2, blk, sblk, printed = int(r[0]), int(r[1]), r[2], int(r[3]), int(r[4]), r[5]
        assert f"{oracle.storage_bits(1, oracle.config(b0, blk, sblk, b1, b2)):.3f}" == printed
        seen += 1
    assert seen == 2


def test_storage_formula(oracle):
    # Eq. 3 and the two figures the paper quotes: NF-4 (4,8,fp32,64,256) = 4.127, NF-3 = 3.127 bits/param
    assert oracle.storage_bits(1, oracle.config(4, 64, 256, 8, "fp32")) == 4 + 8 / 64 + 32 / (64 * 256)
    assert f"{oracle.storage_bits(1, oracle.config(4, 64, 256)):.3f}" == "4.127"
    assert f"{oracle.storage_bits(1, oracle.config(3, 64, 256)):.3f}" == "3.127"
    n = 4096 * 11008
    c = oracle.config(2, 16, 16, 3, "bf16")
    assert oracle.storage_bits(n, c) == n * (2 + 3 / 16 + 16 / 256)
    # search space of Table 1 has 3^5 members
    grid = [(a, b, c_, d, e) for a in (2, 3, 4) for b in (2, 3, 4) for c_ in ("bf16", "fp16", "fp32")
            for d in (16, 32, 64) for e in (16, 64, 256)]
    assert len(grid) == 243


def test_cast_v_matches_library_rounding(oracle):
    import torch
    rng = np.random.default_rng(5)
    xs = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 10 ** rng.uniform(-8, 4, 2000).astype(np.float32),
                         np.array([0.0, 1.0, 65504.0, 65519.9, 65520.0, 6e-8, 5.96e-8, 2.98e-8, 1e-10, 3.0e38], np.float32)])
    for x in xs:
        x = float(np.float32(abs(x)))
        with np.errstate(over="ignore"):
            assert oracle.cast_v(x, "fp16") == float(np.float32(np.float16(np.float32(x))))
        assert oracle.cast_v(x, "bf16") == float(torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).float())
        assert oracle.cast_v(x, "fp32") == x


def test_pack_layout_by_hand(oracle):
    # little-endian bit stream: code j in bits [j*b, (j+1)*b)
    codes = np.array([1, 2, 3, 4, 5, 6, 7, 0], np.uint8)          # 3 bits each -> 24 bits
    # bit string (LSB first): 100 010 110 001 101 011 111 000
    # byte0 bits0-7 = 1,0,0,0,1,0,1,1 -> 0b11010001 = 0xD1 ; byte1 = 0,0,0,1,1,0,1,0 -> 0b01011000 = 0x58
    # byte2 = 1,1,1,1,1,0,0,0 -> 0b00011111 = 0x1F
    assert oracle.pack(codes, 3).tolist() == [0xD1, 0x58, 0x1F]
    assert oracle.pack(np.array([3, 0, 1, 2], np.uint8), 2).tolist() == [0b10010011]
    assert oracle.pack(np.array([0xA, 0x5, 0xF], np.uint8), 4).tolist() == [0x5A, 0x0F]
    assert oracle.pack(np.array([200, 17], np.uint8), 8).tolist() == [200, 17]
    rng = np.random.default_rng(1)
    for bits in (2, 3, 4, 5, 8):
        c = rng.integers(0, 1 << bits, 1000).astype(np.uint8)
        assert np.array_equal(oracle.unpack(oracle.pack(c, bits), c.size, bits), c)
