"""Pins of the sparse position code (Sec. 4.3.1): streams worked out by hand from
the paper's description, the bit counts the paper prints (log(1/phi) + 2 bits per
position: 9 bits at phi = 1e-2 and at 1/128, 12 bits at 1e-3), round trips, and a
pure-Python parser written from the receiver's description."""
import os

import numpy as np
import pytest


def bits_of(words, n_bits):
    return "".join(str((int(words[k >> 5]) >> (k & 31)) & 1) for k in range(n_bits))


def python_receiver(bits, d, block_len):
    """The receiver of Sec. 4.3.1, on a string of '0'/'1'."""
    B = max(0, (block_len - 1).bit_length())
    pos, block, k = [], 0, 0
    while k < len(bits):
        if bits[k] == "1":
            off = int(bits[k + 1:k + 1 + B], 2) if B else 0
            pos.append(block * block_len + off)
            k += 1 + B
        else:
            block += 1
            k += 1
    return pos


def test_hand_worked_streams(oracle, golden_dir):
    n = 0
    with open(os.path.join(golden_dir, "position_code_example.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            d, L, pos, stream = line.split()
            idx = np.array([] if pos == "-" else [int(x) for x in pos.split(",")], np.uint32)
            words, n_bits = oracle.codec_encode(idx, int(d), int(L))
            assert bits_of(words, n_bits) == stream, line
            assert oracle.codec_decode(words, n_bits, int(d), int(L), 16).tolist() == idx.tolist()
            assert python_receiver(stream, int(d), int(L)) == idx.tolist()
            n += 1
    assert n == 4


@pytest.mark.parametrize("inv_phi,bits", [(100, 9), (128, 9), (1000, 12)])
def test_bits_per_position_printed_in_paper(oracle, inv_phi, bits):
    """With phi * d positions the stream spends log(1/phi) + 2 bits per position
    (Sec. 2.1, Sec. 3, Sec. 4.3.1)."""
    d = inv_phi * 5000
    rng = np.random.default_rng(inv_phi)
    idx = np.sort(rng.choice(d, d // inv_phi, replace=False)).astype(np.uint32)
    words, n_bits = oracle.codec_encode(idx, d, inv_phi)
    assert n_bits == idx.size * bits
    assert oracle.codec_offset_bits(inv_phi) + 2 == bits
    assert oracle.bits_per_position(float(inv_phi)) == bits          # the formula used for the budgets


@pytest.mark.parametrize("d,L,n", [(1, 1, 1), (17, 1, 9), (1000, 7, 0), (1000, 7, 1000), (100000, 100, 1000),
                                   (123457, 1000, 124), (65536, 64, 5000)])
def test_round_trip_and_python_receiver(oracle, d, L, n):
    rng = np.random.default_rng(d + n)
    idx = np.sort(rng.choice(d, n, replace=False)).astype(np.uint32)
    words, n_bits = oracle.codec_encode(idx, d, L)
    assert n_bits == oracle.codec_stream_bits(n, d, L)
    assert np.array_equal(oracle.codec_decode(words, n_bits, d, L, n), idx)
    if n_bits < 200000:
        assert python_receiver(bits_of(words, n_bits), d, L) == idx.tolist()
    # unused bits of the last word stay zero
    tail = n_bits & 31
    if tail:
        assert int(words[n_bits >> 5]) >> tail == 0


def test_clustered_positions_and_errors(oracle):
    d, L = 5000, 50
    idx = np.arange(1000, 1100, dtype=np.uint32)               # two full blocks, the rest empty
    words, n_bits = oracle.codec_encode(idx, d, L)
    assert np.array_equal(oracle.codec_decode(words, n_bits, d, L, 100), idx)
    with pytest.raises(ValueError):
        oracle.codec_encode(np.array([5, 3], np.uint32), d, L)          # not ascending
    with pytest.raises(ValueError):
        oracle.codec_encode(np.array([5000], np.uint32), d, L)          # outside the vector
    with pytest.raises(ValueError):
        oracle.codec_decode(words, n_bits, d, L, 99)                    # more positions than room
    with pytest.raises(ValueError):
        oracle.codec_decode(words, n_bits - 3, d, L, 100) if bits_of(words, n_bits)[n_bits - 4] == "1" else \
            oracle.codec_decode(np.array([0xFFFFFFFF], np.uint32), 5, 100, 50, 10)   # truncated code
