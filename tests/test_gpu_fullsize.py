"""GPU-vs-oracle parity at the full sizes of the five workloads, through the same entry points
and buffers bench.py uses (pytest -m gpu).

The oracle cannot run a whole round of the large workloads in test time, so:
  - some users are checked completely (memory, symbols, sub-chunk bits, chunk offsets, payload,
    and, while the vector is small enough, the whole bitstream);
  - sampled chunks (first, last, layer boundaries, random; for every user) are checked element
    by element: memory, symbols, the chunk's words at the offset the GPU reports, and the PS
    average, which needs every user's symbol of that chunk;
  - what covers everything is checked through properties: histogram rows equal the symbol counts
    and sum to the element counts, the code is an optimal prefix code of the histogram (Kraft
    equality, cost equal to the Huffman cost), chunk offsets are the running sum of the rounded
    sub-chunk bits, the payload is their sum.
Where the oracle has every user's symbols (workloads 1-3) the histogram and the code tables are
compared exactly instead.  The round is then repeated through the single-sweep encoder (the
configuration bench.py's headline times) with the code tables held, checked against the oracle
in the same way, and compared with the first round everywhere; once more with the stochastic
conversion; and, for the workloads whose users the oracle can fit, once more exactly as bench.py's
headline runs it: moment fit, model weights and Huffman build on the device, single-sweep encode
under that model code, PS average.

Inputs are drawn on the device with the seeded generator and copied to the host for the oracle.
The memory the checked round starts from is the result of a first round from m_0 = 0: the GPU
carries it, and the oracle recomputes it from that round's gradients wherever it checks something,
so nothing the oracle computes takes a GPU result as input.  The exponent bias follows the
workload's rule on the first round (v = g, since m_0 = 0) and is held, as in bench.py.  The one
exception is stated where it occurs: the model code's integer weights cannot be reproduced bit for
bit by a second incomplete-gamma routine, so they are compared with the oracle's to a tolerance and
the device's weights then define the code both sides encode with.
"""
import heapq
import time

import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

CHUNK = 4096


def chunk_table(seg_len):
    """(element start, length, segment) of every chunk of one user."""
    out, off = [], 0
    for k, n in enumerate(seg_len):
        for c0 in range(0, n, CHUNK):
            out.append((off + c0, min(CHUNK, n - c0), k))
        off += n
    return out


def huffman_cost(w):
    h = [int(x) for x in w if x > 0]
    if len(h) == 1:
        return h[0]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def check_code_is_optimal(hist, lens, codes):
    act = hist > 0
    assert np.array_equal(lens > 0, act)
    L = lens[act].astype(np.int64)
    if L.size >= 2:
        Lmax = int(L.max())
        assert int(sum(1 << (Lmax - int(l)) for l in L)) == 1 << Lmax          # Kraft equality
    assert int((hist[act].astype(object) * L.astype(object)).sum()) == huffman_cost(hist)
    ref = orc.canonical_codes(lens)                                            # canonical form of these lengths
    assert np.array_equal(ref, codes)


def run_workload(name, full_users, n_random_chunks, full_words_limit=40_000_000, exact_hist=True, gamma=None,
                 full_users_later=None, model_round=False):
    """full_users: users checked completely in the first (three-step) round; full_users_later: in the
    later rounds (default: the same); gamma: another memory-decay coefficient than the workload's
    default; model_round: also the device-fitted model code, as bench.py's headline runs it."""
    import dataclasses
    import torch
    from paper_2204_08211_amd import binding as B
    t_start = time.time()
    w = syn.WORKLOADS[name]
    if gamma is not None:
        w = dataclasses.replace(w, gamma=gamma)
        name = f"{name} gamma={gamma}"
    if full_users_later is None:
        full_users_later = full_users
    dev = torch.device("cuda:0")
    U, d, E, M = w.U, w.d, w.E, w.M
    A = 1 << (1 + E + M)
    stride = (d + 31) // 32 * 32     # rows on 128-byte boundaries, as bench.py lays them out
    seg_len = w.seg_len
    nseg = len(seg_len)
    seg_book = list(range(nseg)) if nseg > 1 else [0]
    seg_off = np.concatenate([[0], np.cumsum(seg_len)]).astype(np.int64)
    print(f"[{name}] U={U} d={d} [1,{E},{M}] nseg={nseg}", flush=True)

    g0 = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    g = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    m = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    out = torch.zeros(d, dtype=torch.float32, device=dev)

    # round 0 (m_0 = 0) only produces a realistic memory; round 1 is the one checked.  The bias is the
    # workload's rule on round 0 (v = g there), held for round 1, where some elements then clamp.
    for u in range(U):
        syn.user_gradient_torch(w, 0, u, dev, out=g0[u, :d])
        syn.user_gradient_torch(w, 1, u, dev, out=g[u, :d])
    mx = np.zeros((U, nseg))
    for k in range(nseg):
        mx[:, k] = g0[:, int(seg_off[k]):int(seg_off[k + 1])].abs().amax(dim=1).cpu().numpy()
    bias = syn.bias_table(mx, E)
    plan = B.Plan(E, M, U, d, bias, seg_len=seg_len, seg_book=seg_book, per_user_books=w.per_user_books)
    books = B.co3_build_codebook(E, M, plan.num_books, None)
    buf = B.RoundBuffers(plan, dev, max_code_len=16)
    B.co3_encode(plan, books, g0, m, m, w.gamma, buf, mode=B.BOOK_EMPIRICAL)
    torch.cuda.synchronize()
    m_in = m.clone()
    buf.status.zero_()
    B.co3_encode(plan, books, g, m, m, w.gamma, buf, mode=B.BOOK_EMPIRICAL)
    B.co3_ps_aggregate(plan, books, buf, out)
    torch.cuda.synchronize()
    print(f"[{name}] GPU rounds done at {time.time() - t_start:.1f}s", flush=True)
    status = buf.status.cpu().numpy()
    assert status[B.STAT_NOCODE] == 0 and status[B.STAT_CAPACITY] == 0 and status[B.STAT_CORRUPT] == 0
    assert status[B.STAT_NONFINITE] == 0

    def oracle_m_in(u, lo, hi, k):
        """The memory after round 0 (from m_0 = 0), elements lo..hi of user u in layer k: the oracle's own."""
        g0h = g0[u, lo:hi].cpu().numpy()
        mo = orc.ef_step(g0h, np.zeros_like(g0h), w.gamma, E, M, int(bias[u, k]), want_q=False)[0]
        assert np.array_equal(mo.view(np.uint32), m_in[u, lo:hi].cpu().numpy().view(np.uint32)), \
            f"memory after round 0, user {u} layer {k}"
        return mo

    def verify(m_res, bf, out_res, first, seed=None, bk=None, tag=None):
        """Check one round's outputs (memory m_res, buffers bf, average out_res) against the oracle.
        first: the three-step encoder's round, which also has symbols, a histogram and fresh code tables;
        otherwise the single-sweep encoder's round with the tables `bk` (default: those of the first
        round) held; seed: that round used the stochastic conversion with this seed."""
        label = name if first else name + " " + (tag or ("single-sweep" if seed is None else "single-sweep stochastic"))
        detailed_users = full_users if first else full_users_later

        def ef(gs, ms, b, u, e_first):
            if seed is None:
                return orc.ef_step(gs, ms, w.gamma, E, M, b, want_q=False)
            return orc.ef_step_sr(gs, ms, w.gamma, E, M, b, u, e_first, seed, want_q=False)
        nch = plan.num_chunks
        ctab = chunk_table(seg_len)
        assert len(ctab) == nch
        hist = buf.hist.cpu().numpy().view(np.uint64)
        lc = [(bk or books).export(b) for b in range(plan.num_books)]
        lens = np.stack([x[0] for x in lc]); codes = np.stack([x[1] for x in lc])
        sub_bits = bf.sub_bits.cpu().numpy().view(np.uint16).reshape(U, nch, 64)
        chunk_offset = bf.chunk_offset.cpu().numpy().view(np.uint64)
        payload = bf.payload_bits.cpu().numpy().view(np.uint64)
        sym_gpu = buf.symbols_2d()
        bpu = max(seg_book) + 1

        def book_of(u, k):
            return (u * bpu if w.per_user_books else 0) + seg_book[k]

        # ---- properties that cover everything ------------------------------------------------
        per_chunk = sub_bits.astype(np.uint64).sum(axis=2)
        rounded = (per_chunk + np.uint64(31)) & ~np.uint64(31)
        expect_off = np.concatenate([np.zeros((U, 1), np.uint64), np.cumsum(rounded, axis=1, dtype=np.uint64)], axis=1)
        assert np.array_equal(chunk_offset, expect_off), "chunk offsets are not the running sum of the rounded sizes"
        assert np.array_equal(payload, per_chunk.sum(axis=1, dtype=np.uint64))
        # histogram rows = counts of the symbols the GPU wrote (torch.bincount as a library count)
        if first:
            counts = np.zeros_like(hist)
            for u in range(U):
                for k in range(nseg):
                    sl = slice(int(seg_off[k]), int(seg_off[k + 1]))
                    counts[book_of(u, k)] += torch.bincount(sym_gpu[u, sl].to(torch.int32), minlength=A).cpu().numpy().astype(np.uint64)
            assert np.array_equal(hist, counts)
            assert int(hist.sum()) == U * d
            for b in range(plan.num_books):
                check_code_is_optimal(hist[b], lens[b], codes[b])
        print(f"[{label}] properties ok at {time.time() - t_start:.1f}s; payload {payload.sum() / (U * d):.4f} bit/element, "
              f"max code length {int(lens.max())}, max offset {int(chunk_offset.max())} bits", flush=True)

        # ---- users checked completely ----------------------------------------------------------
        oracle_hist = np.zeros_like(hist)
        clamped = 0
        full_list = list(range(U)) if exact_hist and first else list(detailed_users)
        for u in full_list:
            gh = g[u, :d].cpu().numpy()
            mh = np.empty(d, np.float32)
            for k in range(nseg):
                mh[int(seg_off[k]):int(seg_off[k + 1])] = oracle_m_in(u, int(seg_off[k]), int(seg_off[k + 1]), k)
            sym_o = np.empty(d, np.uint8)
            detailed = u in detailed_users
            m_gpu = m_res[u, :d].cpu().numpy() if detailed else None
            for k in range(nseg):
                sl = slice(int(seg_off[k]), int(seg_off[k + 1]))
                mo, so, _, cnt = ef(gh[sl], mh[sl], int(bias[u, k]), u, int(seg_off[k]))
                sym_o[sl] = so
                clamped += int(cnt[1])
                orc.histogram(so, A, oracle_hist[book_of(u, k)])
                if detailed:
                    assert np.array_equal(mo.view(np.uint32), m_gpu[sl].view(np.uint32)), f"memory of user {u}, layer {k}"
            if detailed:
                if first:
                    assert np.array_equal(sym_o, sym_gpu[u].cpu().numpy()), f"symbols of user {u}"
                # sub-chunk bits from the oracle's symbols and the exported lengths
                for k in range(nseg):
                    lo, hi = int(seg_off[k]), int(seg_off[k + 1])
                    if hi == lo:
                        continue
                    L = lens[book_of(u, k)][sym_o[lo:hi]].astype(np.uint32)
                    nck = (hi - lo + CHUNK - 1) // CHUNK
                    pad = np.zeros(nck * CHUNK, np.uint32); pad[:hi - lo] = L
                    c_first = sum((int(n) + CHUNK - 1) // CHUNK for n in seg_len[:k])
                    assert np.array_equal(pad.reshape(nck, 64, 64).sum(axis=2), sub_bits[u, c_first:c_first + nck]), \
                        f"sub-chunk bits of user {u}, layer {k}"
                if d <= full_words_limit and exact_hist:
                    pass  # the whole bitstream is compared below, once the oracle's own code is known
            print(f"[{label}] user {u} {'checked' if detailed else 'counted'} at {time.time() - t_start:.1f}s", flush=True)
            if detailed and (d <= full_words_limit or (first and full_words_limit < 0)):
                # whole bitstream of this user with the exported tables (they are checked against the
                # oracle's own tables below when the oracle has the full histogram)
                r = orc.pack(sym_o, seg_len, [book_of(u, k) for k in range(nseg)], lens, codes)
                assert r["rc"] == 0
                nw = int(r["chunk_offset"][-1]) // 32
                assert np.array_equal(r["chunk_offset"], chunk_offset[u])
                assert np.array_equal(r["words"][:nw], bf.words[u, :nw].cpu().numpy().view(np.uint32)), f"bitstream of user {u}"
                assert r["payload_bits"] == int(payload[u])
            del gh, mh, sym_o
        if exact_hist and first:
            assert np.array_equal(hist, oracle_hist), "histogram"
            for b in range(plan.num_books):
                lo, co = orc.codebook(oracle_hist[b])
                assert np.array_equal(lo, lens[b]) and np.array_equal(co, codes[b]), f"code table {b}"
            assert clamped == int(status[B.STAT_CLAMPED])

        # ---- sampled chunks, every user ----------------------------------------------------------
        rng = np.random.default_rng(syn.seed_for(w.cfg, 999, 0))
        picks = {0, nch - 1}
        for k in range(nseg):   # chunks next to layer boundaries
            c_first = sum((int(n) + CHUNK - 1) // CHUNK for n in seg_len[:k])
            picks.update({c_first, max(c_first - 1, 0)})
        picks.update(int(x) for x in rng.integers(0, nch, n_random_chunks))
        # the chunks of every user that straddle 2^32 stream bits, if any
        for u in range(U):
            j = int(np.searchsorted(chunk_offset[u], np.uint64(1 << 32)))
            if 0 < j < nch:
                picks.update({j - 1, j})
        picks = sorted(picks)
        for c in picks:
            e0, n, k = ctab[c]
            syms = np.empty((U, n), np.uint8)
            for u in range(U):
                gh = g[u, e0:e0 + n].cpu().numpy(); mh = oracle_m_in(u, e0, e0 + n, k)
                mo, so, _, _ = ef(gh, mh, int(bias[u, k]), u, e0)
                assert np.array_equal(mo.view(np.uint32), m_res[u, e0:e0 + n].cpu().numpy().view(np.uint32)), (c, u)
                if first:
                    assert np.array_equal(so, sym_gpu[u, e0:e0 + n].cpu().numpy()), (c, u)
                syms[u] = so
                bk = book_of(u, k)
                r = orc.pack(so, [n], [0], lens[bk][None, :], codes[bk][None, :])
                assert r["rc"] == 0
                nw = int(r["chunk_offset"][-1]) // 32
                w0 = int(chunk_offset[u, c]) // 32
                assert np.array_equal(r["words"][:nw], bf.words[u, w0:w0 + nw].cpu().numpy().view(np.uint32)), (c, u)
                assert np.array_equal(r["sub_bits"][:64], sub_bits[u, c]), (c, u)
                assert int(chunk_offset[u, c + 1]) - int(chunk_offset[u, c]) == nw * 32
            avg = orc.aggregate(syms, [n], bias[:, k:k + 1], E, M)
            got = out_res[e0:e0 + n].cpu().numpy()
            vals = np.stack([np.array([orc.value(s, E, M, int(bias[u, k])) for s in range(A)])[syms[u]] for u in range(U)])
            scale = np.maximum(np.abs(avg), np.abs(vals).mean(axis=0))
            assert np.all(np.abs(got.astype(np.float64) - avg) <= 1e-6 * scale), f"PS average in chunk {c}"
            assert np.array_equal(got.view(np.uint32), avg.view(np.uint32)), f"PS average (bitwise) in chunk {c}"
        print(f"[{label}] {len(picks)} sampled chunks x {U} users ok at {time.time() - t_start:.1f}s", flush=True)

    verify(m, buf, out, True)

    # The same round again through the single-sweep encoder (the configuration bench.py's headline
    # times) with the code tables held: starts from the same memory, writes to buffers of its own.
    m2 = m_in.clone()
    buf2 = B.RoundBuffers(plan, dev, max_code_len=16)
    out2 = torch.zeros(d, dtype=torch.float32, device=dev)
    buf2.chunk_offset.fill_(-1); buf2.sub_bits.fill_(-1); buf2.payload_bits.fill_(-1)
    B.co3_encode(plan, books, g, m2, m2, w.gamma, buf2, mode=B.BOOK_FIXED, single_sweep=True)
    B.co3_ps_aggregate(plan, books, buf2, out2)
    torch.cuda.synchronize()
    status2 = buf2.status.cpu().numpy()
    assert status2[B.STAT_NOCODE] == 0 and status2[B.STAT_CAPACITY] == 0 and status2[B.STAT_CORRUPT] == 0
    assert status2[B.STAT_STALLED] == 0 and status2[B.STAT_NONFINITE] == 0
    assert status2[B.STAT_CLAMPED] == status[B.STAT_CLAMPED]
    verify(m2, buf2, out2, False)
    # and, since both encoders were just checked against the oracle where it reaches, everywhere else
    # against each other
    assert torch.equal(m2, m) and torch.equal(out2, out)
    assert torch.equal(buf2.chunk_offset, buf.chunk_offset) and torch.equal(buf2.sub_bits, buf.sub_bits)
    assert torch.equal(buf2.payload_bits, buf.payload_bits)
    for u in range(U):
        nw = int(buf.chunk_offset[u, -1].item()) // 32
        assert torch.equal(buf2.words[u, :nw], buf.words[u, :nw]), f"stream of user {u}"
    print(f"[{name}] single-sweep round identical to the three-step round at {time.time() - t_start:.1f}s", flush=True)

    # Once more with the stochastic conversion (single-sweep encoder, tables held): every element draws its
    # dither from its index, user and the seed, so the oracle can check any chunk on its own.
    # The dither reaches symbols the closest-representative round never produced, so the held code is
    # rebuilt with a weight of at least one for every producible symbol.
    seed = 0xC03 + w.cfg
    hist_all = buf.hist.cpu().numpy().view(np.uint64).copy()
    producible = np.array([not np.isnan(orc.value(s, E, M, 10)) for s in range(A)])
    hist_all[:, producible] += np.uint64(1)
    books_sr = B.co3_build_codebook(E, M, plan.num_books, hist_all)
    m3 = m_in.clone()
    B.co3_encode(plan, books_sr, g, m3, m3, w.gamma, buf2, mode=B.BOOK_FIXED, single_sweep=True, stochastic_seed=seed)
    B.co3_ps_aggregate(plan, books_sr, buf2, out2)
    torch.cuda.synchronize()
    status3 = buf2.status.cpu().numpy()
    assert status3[B.STAT_NOCODE] == 0 and status3[B.STAT_CAPACITY] == 0 and status3[B.STAT_CORRUPT] == 0
    assert status3[B.STAT_STALLED] == 0
    assert not torch.equal(m3, m2)
    verify(m3, buf2, out2, False, seed=seed, bk=books_sr)

    # The model refresh at full size: moment fit of v = g + gamma m_in for every user and layer.  The oracle
    # (two-pass fp64 moments of its own v) checks every user when it can afford to, else the first full ones.
    from oracle import co3_gennorm_fit as fitm
    params = B.co3_gennorm_fit(plan, g, m_in, w.gamma)
    torch.cuda.synchronize()
    par = params.cpu().numpy()
    fit_users = list(range(U)) if model_round else (list(full_users) if full_users else [0])[:2]
    ref_par = np.zeros((U, nseg, 4))
    for u in fit_users:
        gh = g[u, :d].cpu().numpy()
        mh = np.empty(d, np.float32)
        for k in range(nseg):
            mh[int(seg_off[k]):int(seg_off[k + 1])] = oracle_m_in(u, int(seg_off[k]), int(seg_off[k + 1]), k)
        ref = fitm.fit_round(gh[None, :], mh[None, :], w.gamma, seg_len)[0]
        ref_par[u] = ref
        for k in range(nseg):
            if ref[k, 1] == 0.0:
                assert par[u, k, 1] == 0.0 and par[u, k, 2] == 0.0
                continue
            sigma = ref[k, 1] * float(np.sqrt(fitm.variance_factor(ref[k, 2])))
            assert abs(par[u, k, 0] - ref[k, 0]) <= 1e-11 * sigma, (u, k)
            assert abs(par[u, k, 3] / ref[k, 3] - 1.0) <= 1e-9, (u, k, par[u, k, 3], ref[k, 3])
            assert abs(par[u, k, 2] / ref[k, 2] - 1.0) <= 1e-9 and abs(par[u, k, 1] / ref[k, 1] - 1.0) <= 1e-9, (u, k)
        del gh, mh
    print(f"[{name}] moment fit of users {fit_users} equals the oracle's at {time.time() - t_start:.1f}s; "
          f"beta in [{par[:, :, 2].min():.3f}, {par[:, :, 2].max():.3f}]", flush=True)
    if not model_round:
        return

    # The round as bench.py's headline runs it: the model code designed on the device (fit above ->
    # mixture weights -> Huffman build, no host step), held, and the single-sweep encoder under it.  Every
    # producible symbol has a weight of at least one, so this code has far longer codewords than the
    # histogram's.  The device's integer weights are held to |dw| <= 1 + 1e-9 w against the oracle's own
    # (from its own fit); the oracle's Huffman construction on the device's weights must then give the
    # device's tables, and the streams are checked against the oracle under those tables.
    weights_t = B.co3_model_weights_device(plan, params)
    books_m = B.co3_build_codebook(E, M, plan.num_books, None)
    B.co3_build_codebook_device(books_m, weights_t, buf2.status)
    torch.cuda.synchronize()
    wts = weights_t.cpu().numpy().view(np.uint64)
    ref_w = fitm.pooled_model_weights(E, M, bias, ref_par, seg_len, seg_book, w.per_user_books)
    assert np.array_equal(wts > 0, ref_w > 0)
    dw = np.abs(wts.astype(np.float64) - ref_w.astype(np.float64))
    assert np.all(dw <= 1.0 + 1e-9 * ref_w.astype(np.float64)), dw.max()
    for b in range(plan.num_books):
        lo, co = orc.codebook(wts[b])
        ld, cd = books_m.export(b)
        assert np.array_equal(lo, ld) and np.array_equal(co, cd), f"model code table {b}"
    m4 = m_in.clone()
    buf2.status.zero_()
    buf2.chunk_offset.fill_(-1); buf2.sub_bits.fill_(-1); buf2.payload_bits.fill_(-1)
    B.co3_encode(plan, books_m, g, m4, m4, w.gamma, buf2, mode=B.BOOK_FIXED, single_sweep=True)
    B.co3_ps_aggregate(plan, books_m, buf2, out2)
    torch.cuda.synchronize()
    status4 = buf2.status.cpu().numpy()
    assert status4[B.STAT_NOCODE] == 0 and status4[B.STAT_CAPACITY] == 0 and status4[B.STAT_CORRUPT] == 0
    assert status4[B.STAT_STALLED] == 0 and status4[B.STAT_CODELEN] == 0
    assert status4[B.STAT_CLAMPED] == status[B.STAT_CLAMPED]
    assert torch.equal(m4, m) and torch.equal(out2, out)       # memory and average do not depend on the code
    verify(m4, buf2, out2, False, bk=books_m, tag="single-sweep, device-fitted model code")
    bits_model = float(buf2.payload_bits.cpu().numpy().astype(np.float64).sum()) / (U * d)
    bits_emp = float(buf.payload_bits.cpu().numpy().astype(np.float64).sum()) / (U * d)
    print(f"[{name}] model code {bits_model:.4f} bit/element, histogram code {bits_emp:.4f}; clamped "
          f"{int(status[B.STAT_CLAMPED])} of {U * d}", flush=True)
    assert bits_model <= 1.02 * bits_emp


def test_cfg1_full():
    run_workload("cfg1", full_users=[0], n_random_chunks=24, model_round=True)


def test_cfg2_full():
    run_workload("cfg2", full_users=[0, 9], n_random_chunks=24, model_round=True)


@pytest.mark.parametrize("gamma", syn.WORKLOADS["cfg3"].gammas)
def test_cfg3_full(gamma):
    # the workload bench.py times, at each memory-decay coefficient the workload names
    run_workload("cfg3", full_users=[0, 15], n_random_chunks=24, gamma=gamma, model_round=True)


def test_cfg4_full():
    # 16 layers with their own bias and code table; one user checked completely
    run_workload("cfg4", full_users=[3], n_random_chunks=16, exact_hist=False, full_words_limit=0)


def test_cfg5_full():
    # more than 2^32 stream bits per user and more than 2^32 elements in the batch; user 0 is checked
    # completely (memory, symbols, sub-chunk bits, every stream word) in the three-step round
    run_workload("cfg5", full_users=[0], full_users_later=[], n_random_chunks=24, exact_hist=False,
                 full_words_limit=-1)
