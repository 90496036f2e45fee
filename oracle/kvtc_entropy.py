"""Lossless stage over the packed records -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.

Paper, Section "Entropy coding": the byte array the quantiser packed is passed through a general
lossless coder on the GPU (DEFLATE in the paper's implementation; appendix "Ablations of lossless
compression" measures what it adds).  DEFLATE itself stays a host-side reference here
(kvtc_oracle.deflate).  This module defines the byte-wise entropy coder that the GPU library runs
in its place, chosen for the structure of THIS byte array: every record has the same layout, so
byte k of a record (the high byte of a group's shift, the third byte of the 4-bit codes, ...) has a
distribution of its own, which a position-blind coder cannot see.  The coder is a static prefix
code per byte position:

  * calibration: for every position k of the record, a histogram of the byte values over the
    calibration records, every count raised to at least 1 (so that every byte value stays
    encodable), Huffman code lengths from it, limited to 12 bits by halving the counts (rounding
    up, at least 1) and rebuilding until the longest code fits;
  * codes are canonical (the rule of RFC 1951, section 3.2.2: shorter codes first, equal lengths in
    symbol order) and are written most significant code bit first into a bit string that fills
    bytes from their least significant bit -- so a table is fully described by its 256 lengths;
  * container of a tensor's T records (chunks of 64 tokens):
        uint32 chunk_off[n_chunks + 1]   byte offset of each chunk's bit string in the payload, then the payload length
        uint16 len_bits[64 * n_chunks]   bits of each token's code string (0 beyond the last token)
        payload                          the chunks' bit strings, each padded with zero bits to a multiple of 4 bytes;
                                         inside a chunk the tokens' strings follow each other bit by bit
    all little-endian.  Decoding a token needs only its chunk's offset and the lengths before it in
    the chunk, so every token decodes independently.

Only the tests and the benchmark's CPU leg may import this module; it shares no code with the GPU library.
"""
from __future__ import annotations

import heapq
from typing import List

import numpy as np

MAX_LEN = 12
CHUNK = 64


def huffman_lengths(freq) -> np.ndarray:
    """Code lengths of a Huffman code for positive weights freq[0..n-1] (n >= 2): repeatedly merge the two lightest
    trees; a symbol's length is the number of merges its tree took part in.  Ties: the tree created earlier (leaves in
    symbol order first) is taken first, which makes the result a function of the weights alone."""
    f = [int(x) for x in freq]
    n = len(f)
    assert n >= 2 and min(f) > 0
    heap = [(f[i], i, (i,)) for i in range(n)]          # (weight, creation order, leaves)
    heapq.heapify(heap)
    depth = [0] * n
    order = n
    while len(heap) > 1:
        w1, _, l1 = heapq.heappop(heap)
        w2, _, l2 = heapq.heappop(heap)
        for s in l1 + l2:
            depth[s] += 1
        heapq.heappush(heap, (w1 + w2, order, l1 + l2))
        order += 1
    return np.array(depth, dtype=np.int64)


def limited_lengths(counts, max_len: int = MAX_LEN) -> np.ndarray:
    """Lengths (1..max_len) of a prefix code over all len(counts) symbols from a histogram: counts of zero are raised to
    one; while the Huffman code is too deep the counts are halved (rounded up) and the code rebuilt."""
    f = np.maximum(np.asarray(counts, dtype=np.int64), 1)
    assert (1 << max_len) >= len(f)
    while True:
        L = huffman_lengths(f)
        if L.max() <= max_len:
            return L
        f = np.maximum((f + 1) // 2, 1)


def canonical_codes(lengths) -> np.ndarray:
    """Code values (as integers whose most significant of `length` bits comes first) assigned by length, then by symbol."""
    lengths = np.asarray(lengths, dtype=np.int64)
    codes = np.zeros(len(lengths), dtype=np.int64)
    code = 0
    for ln in range(1, int(lengths.max()) + 1):
        for s in np.nonzero(lengths == ln)[0]:
            codes[s] = code
            code += 1
        code <<= 1
    return codes


def _reverse_bits(v: int, n: int) -> int:
    r = 0
    for _ in range(n):
        r = (r << 1) | (v & 1)
        v >>= 1
    return r


def calibrate_tables(records: np.ndarray, max_len: int = MAX_LEN) -> np.ndarray:
    """[R, 256] uint8 code lengths, one prefix code per byte position of the record."""
    records = np.ascontiguousarray(records, dtype=np.uint8)
    R = records.shape[1]
    out = np.zeros((R, 256), dtype=np.uint8)
    for k in range(R):
        out[k] = limited_lengths(np.bincount(records[:, k], minlength=256), max_len)
    return out


def bound_bytes(n_tokens: int, record_bytes: int, max_len: int = MAX_LEN) -> int:
    """Largest container any input of this shape can produce."""
    n_chunks = (n_tokens + CHUNK - 1) // CHUNK
    per_chunk = (CHUNK * record_bytes * max_len + 31) // 32 * 4
    return 4 * (n_chunks + 1) + 2 * CHUNK * n_chunks + n_chunks * per_chunk


def encode(records: np.ndarray, lengths: np.ndarray) -> bytes:
    records = np.ascontiguousarray(records, dtype=np.uint8)
    T, R = records.shape
    assert lengths.shape == (R, 256)
    rev = [[_reverse_bits(int(c), int(l)) for c, l in zip(canonical_codes(lengths[k]), lengths[k])] for k in range(R)]
    n_chunks = (T + CHUNK - 1) // CHUNK
    len_bits = np.zeros(CHUNK * n_chunks, dtype=np.uint16)
    chunk_off = np.zeros(n_chunks + 1, dtype=np.uint32)
    payload: List[bytes] = []
    pos_bytes = 0
    for c in range(n_chunks):
        acc, nbits = 0, 0
        for t in range(c * CHUNK, min(T, (c + 1) * CHUNK)):
            start = nbits
            row = records[t]
            for k in range(R):
                b = int(row[k])
                acc |= rev[k][b] << nbits
                nbits += int(lengths[k, b])
            len_bits[t] = nbits - start
        nbytes = (nbits + 31) // 32 * 4
        chunk_off[c] = pos_bytes
        payload.append(acc.to_bytes(nbytes, "little"))
        pos_bytes += nbytes
    chunk_off[n_chunks] = pos_bytes
    return chunk_off.astype("<u4").tobytes() + len_bits.astype("<u2").tobytes() + b"".join(payload)


def decode(blob: bytes, n_tokens: int, record_bytes: int, lengths: np.ndarray) -> np.ndarray:
    """Bit by bit, with the counting form of canonical decoding (how many codes of each length there are, and the
    first code of each length) -- no lookup table."""
    T, R = n_tokens, record_bytes
    n_chunks = (T + CHUNK - 1) // CHUNK
    chunk_off = np.frombuffer(blob, dtype="<u4", count=n_chunks + 1)
    len_bits = np.frombuffer(blob, dtype="<u2", count=CHUNK * n_chunks, offset=4 * (n_chunks + 1))
    base = 4 * (n_chunks + 1) + 2 * CHUNK * n_chunks
    assert len(blob) == base + int(chunk_off[n_chunks])
    # per position: symbols sorted by (length, symbol); count per length
    tables = []
    for k in range(R):
        L = lengths[k].astype(np.int64)
        order = sorted(range(256), key=lambda s: (L[s], s))
        count = np.bincount(L, minlength=MAX_LEN + 2)
        tables.append((order, count))
    out = np.zeros((T, R), dtype=np.uint8)
    for c in range(n_chunks):
        data = int.from_bytes(blob[base + int(chunk_off[c]): base + int(chunk_off[c + 1])], "little")
        pos = 0
        for t in range(c * CHUNK, min(T, (c + 1) * CHUNK)):
            start = pos
            for k in range(R):
                order, count = tables[k]
                code, first, index, ln = 0, 0, 0, 0
                while True:
                    code |= (data >> pos) & 1
                    pos += 1
                    ln += 1
                    n = int(count[ln])
                    if code - n < first:
                        out[t, k] = order[index + (code - first)]
                        break
                    index += n
                    first = (first + n) << 1
                    code <<= 1
            assert pos - start == int(len_bits[t])
    return out
