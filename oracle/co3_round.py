"""One CO3 round on the CPU oracle, in the order of Algorithm 1 of the paper (arXiv 2204.08211):
lines 8-10 for every user, then lines 13-14 at the PS.  TEST INFRASTRUCTURE ONLY."""
import time

import numpy as np

from . import co3_oracle as orc


def encode_round(g, m, gamma, E, M, seg_len, seg_book, bias, per_user_books=False, weights=None, timings=None,
                 stochastic_seed=None):
    """g, m: float32 [U, d]; bias: int [U, nseg]; weights: None = build the code from this round's
    histogram (pooled over users per table id, or per user), else uint64 [nbooks, A] fixed weights;
    stochastic_seed: None = closest representative, else the stochastic conversion with that seed.

    Returns a dict with m_new, sym, hist, lens, codes, words (list per user), chunk_offset,
    sub_bits, payload_bits, counters."""
    g = np.asarray(g, np.float32); m = np.asarray(m, np.float32)
    U, d = g.shape
    nseg = len(seg_len)
    A = 1 << (1 + E + M)
    bias = np.asarray(bias, np.int32).reshape(U, nseg)
    bpu = max(seg_book) + 1
    nbooks = bpu * (U if per_user_books else 1)
    tm = timings if timings is not None else {}

    def tick(name, t0):
        tm[name] = tm.get(name, 0.0) + time.perf_counter() - t0

    m_new = np.empty_like(g); sym = np.empty((U, d), np.uint16 if orc.is_wide(E, M) else np.uint8)
    counters = np.zeros(2, np.uint64)
    hist = np.zeros((nbooks, A), np.uint64)
    for u in range(U):                                     # Algorithm 1 lines 8 and 10
        off = 0
        for k, n in enumerate(seg_len):
            t0 = time.perf_counter()
            if stochastic_seed is None:
                mo, s, _, cnt = orc.ef_step(g[u, off:off + n], m[u, off:off + n], gamma, E, M, int(bias[u, k]),
                                            want_q=False)
            else:
                mo, s, _, cnt = orc.ef_step_sr(g[u, off:off + n], m[u, off:off + n], gamma, E, M, int(bias[u, k]),
                                               u, off, stochastic_seed, want_q=False)
            tick("ef_quantize", t0)
            m_new[u, off:off + n] = mo; sym[u, off:off + n] = s; counters += cnt
            t0 = time.perf_counter()
            orc.histogram(s, A, hist[(u * bpu if per_user_books else 0) + seg_book[k]])
            tick("histogram", t0)
            off += n
    t0 = time.perf_counter()
    w = hist if weights is None else np.asarray(weights, np.uint64).reshape(nbooks, A)
    lens = np.stack([orc.huffman_lengths(w[b]) for b in range(nbooks)])
    codes = np.stack([orc.canonical_codes(lens[b]) for b in range(nbooks)])
    tick("codebook", t0)
    words, chunk_offset, sub_bits, payload, rcs = [], [], [], [], []
    for u in range(U):                                     # Algorithm 1 line 9
        books_u = [(u * bpu if per_user_books else 0) + b for b in seg_book]
        t0 = time.perf_counter()
        r = orc.pack(sym[u], seg_len, books_u, lens, codes)
        tick("pack", t0)
        words.append(r["words"][: int(r["chunk_offset"][-1]) // 32])
        chunk_offset.append(r["chunk_offset"]); sub_bits.append(r["sub_bits"]); payload.append(r["payload_bits"])
        rcs.append(r["rc"])
    return dict(m_new=m_new, sym=sym, hist=hist, lens=lens, codes=codes, words=words,
                chunk_offset=np.stack(chunk_offset), sub_bits=np.stack(sub_bits),
                payload_bits=np.array(payload, np.uint64), counters=counters, rc=rcs, nbooks=nbooks, bpu=bpu)


def ps_round(enc, E, M, seg_len, seg_book, bias, per_user_books=False, timings=None):
    """Algorithm 1 lines 13-14: decode every user's stream, then average."""
    U = len(enc["words"])
    d = int(sum(seg_len))
    tm = timings if timings is not None else {}
    sym = np.empty((U, d), np.uint16 if orc.is_wide(E, M) else np.uint8)
    for u in range(U):
        books_u = [(u * enc["bpu"] if per_user_books else 0) + b for b in seg_book]
        t0 = time.perf_counter()
        rc, s = orc.unpack(enc["words"][u], d, seg_len, books_u, enc["lens"], enc["codes"],
                           enc["chunk_offset"][u], enc["sub_bits"][u])
        tm["decode"] = tm.get("decode", 0.0) + time.perf_counter() - t0
        if rc != 0:
            raise ValueError(f"oracle unpack failed for user {u}: {rc}")
        sym[u] = s
    t0 = time.perf_counter()
    avg = orc.aggregate(sym, seg_len, np.asarray(bias, np.int32).reshape(U, len(seg_len)), E, M)
    tm["average"] = tm.get("average", 0.0) + time.perf_counter() - t0
    return sym, avg
