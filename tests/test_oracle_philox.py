"""Pins for the oracle's Philox4x32-10 and its dropout lane mapping.

Pin 1 (library routine): the generator class in ATen's PhiloxRNGEngine.h, a header
that ships with the installed PyTorch, is compiled by g++ into a tiny program and
run on the same (seed, counter) pairs.  Its constructor takes (seed, subsequence,
offset) and builds counter = (offset_lo, offset_hi, subsequence_lo, subsequence_hi),
key = (seed_lo, seed_hi): the same layout as the dropout contract with
offset := group index g and subsequence := the contract's `offset`.

Pin 2 (structure): bijectivity on a small counter slice, and avalanche, which any
dropped round constant or swapped word would not necessarily break but a
truncated multiply would; plus the statistical properties the dropout needs.
"""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle

CASES = [
    (0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 1), (1234, 7, 5),
    (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFFFFFFFFFF, 0xFFFFFFFFFFFFFFFF),
    (0x0123456789ABCDEF, 0xFEDCBA9876543210, 0x0F1E2D3C4B5A6978),
    (1 << 32, 1 << 32, 1 << 32), (0xDEADBEEF, 0x100000000 - 1, 0x100000000),
]


def _aten_words(tmp_path, cases):
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    hdr = os.path.join(inc, "ATen", "core", "PhiloxRNGEngine.h")
    if not os.path.exists(hdr):
        pytest.skip("ATen Philox header not present")
    src = tmp_path / "aten_philox.cpp"
    src.write_text(
        "#include <ATen/core/PhiloxRNGEngine.h>\n#include <cstdio>\n#include <cstdlib>\n"
        "int main(int argc,char**argv){for(int i=1;i+2<argc;i+=3){"
        "unsigned long long s=strtoull(argv[i],0,0),q=strtoull(argv[i+1],0,0),o=strtoull(argv[i+2],0,0);"
        "at::Philox4_32 e(s,q,o);unsigned a=e(),b=e(),c=e(),d=e();printf(\"%u %u %u %u\\n\",a,b,c,d);}return 0;}\n")
    exe = tmp_path / "aten_philox"
    subprocess.run(["g++", "-O1", "-std=c++17", f"-I{inc}", str(src), "-o", str(exe)], check=True)
    args = [str(v) for c in cases for v in c]
    out = subprocess.run([str(exe)] + args, check=True, capture_output=True, text=True).stdout
    return [[int(w) for w in line.split()] for line in out.strip().splitlines()]


def test_philox_matches_aten_engine(tmp_path):
    rng = np.random.default_rng(7)
    cases = list(CASES)
    for _ in range(200):
        cases.append(tuple(int(v) for v in rng.integers(0, 2**63, size=3, dtype=np.uint64) * 2 + 1))
    got = _aten_words(tmp_path, cases)
    for (seed, subseq, off), words in zip(cases, got):
        ctr = [off & 0xFFFFFFFF, off >> 32, subseq & 0xFFFFFFFF, subseq >> 32]
        key = [seed & 0xFFFFFFFF, seed >> 32]
        mine = oracle.philox4x32_10(ctr, key)
        assert [int(w) for w in mine] == words, (seed, subseq, off)


def test_philox_is_a_bijection_on_a_counter_slice():
    # a block cipher in counter mode: distinct counters -> distinct 128-bit outputs
    outs = set()
    for c0 in range(4096):
        outs.add(tuple(int(w) for w in oracle.philox4x32_10([c0, 0, 0, 0], [42, 0])))
    assert len(outs) == 4096


def test_philox_avalanche():
    # flipping one input bit flips about half of the 128 output bits
    base = oracle.philox4x32_10([5, 6, 7, 8], [9, 10])
    flips = []
    for word in range(4):
        for bit in (0, 13, 31):
            ctr = [5, 6, 7, 8]
            ctr[word] ^= 1 << bit
            o = oracle.philox4x32_10(ctr, [9, 10])
            flips.append(sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(base, o)))
    assert 48 < np.mean(flips) < 80


def test_dropout_lane_mapping_is_the_contract():
    # element e uses 16-bit lane e%8 of the call for group e//8: word (e%8)//2,
    # low half for even e, high half for odd e; keep iff r16 >= round(p*65536)
    seed, offset, p = 0x1234_5678_9ABC_DEF0, 3, 0.3
    n, e0 = 1000, 5  # start mid-group
    keep = oracle.dropout_mask(n, p, seed, offset, e0=e0)
    t16 = int(np.floor(float(np.float32(p)) * 65536 + 0.5))
    for i in range(n):
        e = e0 + i
        g = e // 8
        w = oracle.philox4x32_10([g & 0xFFFFFFFF, g >> 32, offset, 0], [seed & 0xFFFFFFFF, seed >> 32])
        lane = e % 8
        r16 = (int(w[lane // 2]) >> (16 * (lane % 2))) & 0xFFFF
        assert keep[i] == (1 if r16 >= t16 else 0)


@pytest.mark.parametrize("p", [0.1, 0.3, 0.5])
def test_dropout_keep_rate_and_uniformity(p):
    n = 1 << 20
    keep = oracle.dropout_mask(n, p, 1234, 0)
    t16 = np.floor(float(np.float32(p)) * 65536 + 0.5)
    q = 1 - t16 / 65536
    sigma = np.sqrt(q * (1 - q) / n)
    assert abs(keep.mean() - q) < 4 * sigma
    # per-lane keep rates (8 lanes of a group) are all consistent with q
    lanes = keep.reshape(-1, 8).mean(axis=0)
    assert np.all(np.abs(lanes - q) < 5 * np.sqrt(q * (1 - q) / (n / 8)))
    # per-column uniformity for a [rows, 512] view (chi-square against binomial)
    cols = keep.reshape(-1, 512).sum(axis=0).astype(np.float64)
    rows = n // 512
    chi2 = np.sum((cols - rows * q) ** 2 / (rows * q * (1 - q)))
    assert chi2 < 512 + 5 * np.sqrt(2 * 512)


def test_dropout_offsets_and_seeds_are_independent():
    n, p = 1 << 18, 0.5
    a = oracle.dropout_mask(n, p, 1234, 0)
    b = oracle.dropout_mask(n, p, 1234, 1)
    c = oracle.dropout_mask(n, p, 1235, 0)
    for other in (b, c):
        agree = np.mean(a == other)
        assert abs(agree - 0.5) < 4 * np.sqrt(0.25 / n)


def test_dropout_p_zero_keeps_everything_and_slices_agree():
    assert oracle.dropout_mask(100, 0.0, 1, 2).all()
    full = oracle.dropout_mask(4096, 0.25, 99, 7)
    part = oracle.dropout_mask(1000, 0.25, 99, 7, e0=1003)
    assert np.array_equal(full[1003:2003], part)
