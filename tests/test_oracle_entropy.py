"""Pins for oracle/kvtc_entropy.py, the byte-wise lossless stage over the packed records (paper, Section "Entropy
coding"): Huffman lengths against a textbook example, brute force and the entropy bound; canonical codes against the
worked example of RFC 1951; the container against a hand-assembled stream; round trips."""
import itertools
import math

import numpy as np
import pytest

import kvtc_entropy as ke


def test_huffman_lengths_textbook_example():
    # the six-letter example of Cormen, Leiserson, Rivest & Stein, "Introduction to Algorithms", section on Huffman codes:
    # frequencies a:45 b:13 c:12 d:16 e:9 f:5 (thousands) -> codeword lengths 1, 3, 3, 3, 4, 4; cost 224 (thousand bits)
    f = [45, 13, 12, 16, 9, 5]
    L = ke.huffman_lengths(f)
    assert L.tolist() == [1, 3, 3, 3, 4, 4]
    assert int(np.dot(f, L)) == 224


@pytest.mark.parametrize("seed", range(6))
def test_huffman_lengths_are_optimal_by_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = 5
    f = rng.integers(1, 30, n)
    best = min(int(np.dot(f, Ls)) for Ls in itertools.product(range(1, n), repeat=n) if sum(2.0 ** -l for l in Ls) <= 1.0 + 1e-12)
    assert int(np.dot(f, ke.huffman_lengths(f))) == best


def test_huffman_is_complete_and_within_one_bit_of_entropy():
    rng = np.random.default_rng(1)
    for _ in range(5):
        f = rng.integers(1, 1000, 256)
        L = ke.huffman_lengths(f)
        assert abs(sum(2.0 ** -int(l) for l in L) - 1.0) < 1e-12                # Kraft equality: a full tree
        pr = f / f.sum()
        H = -(pr * np.log2(pr)).sum()
        avg = float(np.dot(pr, L))
        assert H <= avg + 1e-12 < H + 1.0


def test_limited_lengths_fit_and_stay_a_prefix_code():
    # a geometric histogram whose Huffman tree is a 255-deep chain
    f = np.array([2 ** min(i, 60) for i in range(256)][::-1], dtype=object)
    f = np.array([int(x) if x < 2 ** 62 else 2 ** 62 for x in f], dtype=np.int64)
    assert ke.huffman_lengths(np.maximum(f, 1)).max() > ke.MAX_LEN
    L = ke.limited_lengths(f)
    assert 1 <= L.min() and L.max() <= ke.MAX_LEN
    assert sum(2.0 ** -int(l) for l in L) <= 1.0 + 1e-12
    # zero counts stay encodable
    L0 = ke.limited_lengths(np.array([1000] + [0] * 255))
    assert L0.min() >= 1 and L0.max() <= ke.MAX_LEN and L0[0] == 1


def test_canonical_codes_worked_example_of_the_deflate_specification():
    # RFC 1951, section 3.2.2: alphabet ABCDEFGH with lengths (3, 3, 3, 3, 3, 2, 4, 4) gets codes
    # 010, 011, 100, 101, 110, 00, 1110, 1111
    codes = ke.canonical_codes([3, 3, 3, 3, 3, 2, 4, 4])
    assert codes.tolist() == [0b010, 0b011, 0b100, 0b101, 0b110, 0b00, 0b1110, 0b1111]


def test_canonical_codes_are_prefix_free():
    rng = np.random.default_rng(3)
    L = ke.limited_lengths(rng.integers(0, 5000, 256) ** 2)
    C_ = ke.canonical_codes(L)
    words = sorted(format(int(c), "b").zfill(int(l)) for c, l in zip(C_, L))
    assert len(set(words)) == 256
    for a, b in zip(words, words[1:]):
        assert not b.startswith(a)


def test_container_hand_assembled():
    """One byte position (R = 1), three tokens.  Byte values 0, 1, 2, 3 get lengths 1, 2, 3, 4; the other 252 values get
    12-bit codes, which leaves the code incomplete (Kraft sum below 1) -- allowed.  The container is written out by hand."""
    L = np.full((1, 256), 12, dtype=np.uint8)
    L[0, 0], L[0, 1], L[0, 2], L[0, 3] = 1, 2, 3, 4
    assert sum(2.0 ** -int(l) for l in L[0]) <= 1.0
    codes = ke.canonical_codes(L[0])
    assert codes[:4].tolist() == [0b0, 0b10, 0b110, 0b1110]
    rec = np.array([[1], [0], [2]], dtype=np.uint8)                 # B A C
    blob = ke.encode(rec, L)
    # bit string, first bit first: B = 1 0, A = 0, C = 1 1 0  ->  bits 1,0,0,1,1,0 -> byte 0b011001 = 0x19
    expect = np.array([0, 4], dtype="<u4").tobytes() + np.array([2, 1, 3] + [0] * 61, dtype="<u2").tobytes() + bytes([0x19, 0, 0, 0])
    assert blob == expect
    assert np.array_equal(ke.decode(blob, 3, 1, L), rec)


@pytest.mark.parametrize("T", [1, 63, 64, 65, 200])
def test_round_trip_and_bound(T):
    rng = np.random.default_rng(T)
    R = 24
    # bytes with a different skew per position, like headers next to packed codes
    rec = np.stack([np.minimum(255, rng.geometric(1.0 / (2 + 6 * k), T)) for k in range(R)], axis=1).astype(np.uint8)
    L = ke.calibrate_tables(rec[: max(1, T // 2)])                # tables from a part of the data: the rest has unseen values
    blob = ke.encode(rec, L)
    assert len(blob) <= ke.bound_bytes(T, R)
    assert np.array_equal(ke.decode(blob, T, R, L), rec)
    n_chunks = (T + 63) // 64
    off = np.frombuffer(blob, dtype="<u4", count=n_chunks + 1)
    lb = np.frombuffer(blob, dtype="<u2", count=64 * n_chunks, offset=4 * (n_chunks + 1)).astype(np.int64)
    assert np.all(off % 4 == 0) and np.all(lb[T:] == 0)
    for c in range(n_chunks):
        assert off[c + 1] - off[c] == (lb[64 * c:64 * c + 64].sum() + 31) // 32 * 4
    # the coded size is what the tables say: sum of the code lengths of the bytes
    assert lb.sum() == sum(int(L[k, b]) for row in rec for k, b in enumerate(row))


def test_position_tables_beat_a_position_blind_code_on_structured_records():
    """Records whose first byte is nearly constant and whose second is uniform: one table per position codes them in
    about 1 + 8 bits, a single table for both positions cannot."""
    rng = np.random.default_rng(0)
    T = 4096
    rec = np.stack([np.where(rng.random(T) < 0.95, 7, rng.integers(0, 256, T)), rng.integers(0, 256, T)], axis=1).astype(np.uint8)
    L = ke.calibrate_tables(rec)
    per_pos = sum(int(L[k, b]) for row in rec for k, b in enumerate(row)) / T
    blind = ke.limited_lengths(np.bincount(rec.reshape(-1), minlength=256))
    one_table = sum(int(blind[b]) for b in rec.reshape(-1)) / T
    assert per_pos < 10.0 < one_table


def test_committed_table_bundle_is_what_the_script_writes():
    """The code-length tables the benchmark loads are stored values: for two tensors of the 32-layer cache they must be
    exactly what oracle/make_entropy_tables.py computes, and every table must be a prefix code of at most 12 bits."""
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("make_entropy_tables", os.path.join(root, "oracle", "make_entropy_tables.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    z = np.load(os.path.join(root, "paper_2511_01815_amd", "plans", "c3_entropy_cr16.npz"))["code_len"]
    assert z.shape == (64, 128, 256) and z.dtype == np.uint8
    assert z.min() >= 1 and z.max() <= ke.MAX_LEN
    kraft = (2.0 ** -z.astype(np.float64)).sum(axis=2)
    assert np.all(kraft <= 1.0 + 1e-12)
    np.testing.assert_array_equal(z[0], mod.tables_of(0, 0))           # layer 0, K
    np.testing.assert_array_equal(z[63], mod.tables_of(31, 1))         # layer 31, V
