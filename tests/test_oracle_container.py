"""Pins for the oracle's bitstream writer / reader (h_Hf and its inverse, Sec. II-B (iii))."""
import os

import numpy as np
import pytest

from oracle import co3_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def string_pack(sym, seg_len, seg_book, lens, codes):
    """Reference by string concatenation: returns (words, chunk_offset, sub_bits, payload)."""
    out, offs, subs, payload, e = "", [], [], 0, 0
    for n, bk in zip(seg_len, seg_book):
        for c0 in range(0, n, orc.CHUNK):
            out += "0" * (-len(out) % 32)
            offs.append(len(out))
            nin = min(orc.CHUNK, n - c0)
            for s0 in range(0, orc.CHUNK, orc.SUB):
                piece = "".join(format(int(codes[bk][s]), "b").zfill(int(lens[bk][s]))
                                for s in sym[e + c0 + s0: e + c0 + min(s0 + orc.SUB, nin)]) if s0 < nin else ""
                subs.append(len(piece)); payload += len(piece); out += piece
        e += n
    out += "0" * (-len(out) % 32)
    offs.append(len(out))
    words = [int(out[i:i + 32], 2) for i in range(0, len(out), 32)]
    return words, offs, subs, payload


def test_hand_packed_golden():
    gold = {}
    for line in open(os.path.join(GOLD, "bitstream_hand.txt")):
        if line.startswith("#"):
            continue
        k, *v = line.split()
        gold[k] = v
    lens = np.array([[1, 2, 3, 3]], np.uint8)
    codes = np.array([[0b0, 0b10, 0b110, 0b111]], np.uint64)
    sym = np.array([0, 1, 2, 3] * 16 + [3, 3, 0, 0, 1, 2], np.uint8)
    r = orc.pack(sym, [70], [0], lens, codes)
    assert r["rc"] == 0
    nw = len(gold["words"])
    assert [format(int(x), "08X") for x in r["words"][:nw]] == gold["words"]
    assert not r["words"][nw:].any()
    assert r["chunk_offset"].tolist() == [int(x) for x in gold["chunk_offset"]]
    assert r["sub_bits"][:2].tolist() == [int(x) for x in gold["sub_bits"]] and not r["sub_bits"][2:].any()
    assert r["payload_bits"] == int(gold["payload_bits"][0])


def random_book(rng, A, active=None):
    w = (rng.pareto(0.8, A) * 20 + 1).astype(np.uint64)
    if active is not None:
        w[rng.permutation(A)[active:]] = 0
    return w


@pytest.mark.parametrize("segs", [[1], [63], [64], [65], [4095], [4096], [4097], [3 * 4096 + 70],
                                  [5, 4096, 1, 9000, 64], [0, 100, 0], [20000]])
def test_roundtrip_and_string_reference(segs):
    rng = np.random.default_rng(sum(segs))
    A, nb = 64, 3
    W = np.stack([random_book(rng, A) for _ in range(nb)])
    lens = np.stack([orc.huffman_lengths(w) for w in W])
    codes = np.stack([orc.canonical_codes(l) for l in lens])
    book = [int(rng.integers(0, nb)) for _ in segs]
    d = sum(segs)
    sym = np.concatenate([rng.choice(A, n, p=W[b] / W[b].sum()) for n, b in zip(segs, book)]).astype(np.uint8)
    r = orc.pack(sym, segs, book, lens, codes)
    assert r["rc"] == 0
    words, offs, subs, payload = string_pack(sym.tolist(), segs, book, lens, codes)
    assert r["words"][:len(words)].tolist() == words and not r["words"][len(words):].any()
    assert r["chunk_offset"].tolist() == offs and r["sub_bits"].tolist() == subs
    assert r["payload_bits"] == payload == int(lens[np.repeat(book, segs), sym].astype(np.int64).sum())
    assert np.all(np.diff(r["chunk_offset"].astype(np.int64)) >= 0) and np.all(r["chunk_offset"] % 32 == 0)
    rc, back = orc.unpack(r["words"][:len(words)], d, segs, book, lens, codes, r["chunk_offset"], r["sub_bits"])
    assert rc == 0 and np.array_equal(back, sym)


def test_single_symbol_stream_and_long_codes():
    # one active symbol: 1 bit per element
    lens = np.zeros((1, 16), np.uint8); lens[0, 5] = 1
    codes = np.zeros((1, 16), np.uint64)
    sym = np.full(300, 5, np.uint8)
    r = orc.pack(sym, [300], [0], lens, codes)
    assert r["payload_bits"] == 300 and r["sub_bits"][:5].tolist() == [64, 64, 64, 64, 44]
    rc, back = orc.unpack(r["words"], 300, [300], [0], lens, codes, r["chunk_offset"], r["sub_bits"])
    assert rc == 0 and np.array_equal(back, sym)
    # codes up to 63 bits (weights 1, 1, 2, 4, ...)
    w = np.array([1] + [1 << i for i in range(63)], np.uint64)
    l = orc.huffman_lengths(w)[None, :]; c = orc.canonical_codes(l[0])[None, :]
    rng = np.random.default_rng(5)
    sym = rng.integers(0, 64, 5000).astype(np.uint8)
    r = orc.pack(sym, [5000], [0], l, c)
    words, offs, subs, payload = string_pack(sym.tolist(), [5000], [0], l, c)
    assert r["words"][:len(words)].tolist() == words and r["payload_bits"] == payload
    rc, back = orc.unpack(r["words"], 5000, [5000], [0], l, c, r["chunk_offset"], r["sub_bits"])
    assert rc == 0 and np.array_equal(back, sym)


def test_errors_capacity_nocode_corrupt():
    rng = np.random.default_rng(9)
    w = random_book(rng, 16, active=9)
    l = orc.huffman_lengths(w)[None, :]; c = orc.canonical_codes(l[0])[None, :]
    act = np.flatnonzero(w)
    sym = rng.choice(act, 9000).astype(np.uint8)
    good = orc.pack(sym, [9000], [0], l, c)
    nw = int(good["chunk_offset"][-1]) // 32
    assert orc.pack(sym, [9000], [0], l, c, cap_words=nw)["rc"] == 0
    assert orc.pack(sym, [9000], [0], l, c, cap_words=nw - 2)["rc"] == orc.ERR_CAPACITY
    bad = sym.copy(); bad[17] = int(np.flatnonzero(w == 0)[0])
    assert orc.pack(bad, [9000], [0], l, c)["rc"] == orc.ERR_NOCODE
    # a truncated stream, a wrong sub-chunk length and a misaligned chunk offset are all detected
    args = ([9000], [0], l, c)
    assert orc.unpack(good["words"][:nw - 3], 9000, *args, good["chunk_offset"], good["sub_bits"])[0] == orc.ERR_CORRUPT
    sb = good["sub_bits"].copy(); sb[3] -= 1
    assert orc.unpack(good["words"], 9000, *args, good["chunk_offset"], sb)[0] == orc.ERR_CORRUPT
    co = good["chunk_offset"].copy(); co[1] += 1
    assert orc.unpack(good["words"], 9000, *args, co, good["sub_bits"])[0] == orc.ERR_CORRUPT
