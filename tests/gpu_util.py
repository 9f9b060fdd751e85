"""Helpers of the GPU parity tests: run one round through the C ABI, run it on the oracle,
compare element by element."""
import numpy as np

import co3_synth as syn
from oracle import co3_oracle as orc
from oracle import co3_round as oround


def special_values(E, M, bias, rng, n):
    """fp32 probes around every representative and midpoint, plus zeros, denormals, huge values."""
    g = orc.grid(E, M, bias)
    mids = (g[:-1] + g[1:]) / 2
    with np.errstate(over="ignore"):
        base = np.concatenate([g, mids]).astype(np.float32)
        pts = np.concatenate([base, np.nextafter(base, np.float32(np.inf)), np.nextafter(base, np.float32(0)),
                              np.array([0.0, 1e-45, 3e-39, 1.1754944e-38, 1e-30, g[-1] * 1.5, g[-1] * 4, 1e30],
                                       np.float32)])
    pts = pts[np.isfinite(pts)]
    pts = np.concatenate([pts, -pts])
    return rng.choice(pts, n).astype(np.float32)


def _sym_numpy(t):
    """Symbols as the oracle holds them: uint8, or uint16 for alphabets above 8 bits (torch has them as int16)."""
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def gpu_round(plan_kwargs, g, m, gamma, mode, weights=None, words_stride=None, max_code_len=32, want_decode=True,
              books=None, buf=None, single_sweep=False, stochastic_seed=None, single_sweep_hist=False):
    """One encode (+ decode + aggregate) through the binding.  Returns (dict of numpy arrays, objects).
    single_sweep: fixed code, no symbols and no histogram requested (they stay as they were)."""
    import torch
    from paper_2204_08211_amd import binding as B
    dev = torch.device("cuda:0")
    plan = B.Plan(**plan_kwargs)
    U, d = plan.U, plan.d
    stride = (d + 3) // 4 * 4
    gt = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    mt = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    gt[:, :d] = torch.from_numpy(np.ascontiguousarray(g)).to(dev)
    mt[:, :d] = torch.from_numpy(np.ascontiguousarray(m)).to(dev)
    if books is None:
        books = B.co3_build_codebook(plan.E, plan.M, plan.num_books, weights)
    if buf is None:
        buf = B.RoundBuffers(plan, dev, words_stride=words_stride, max_code_len=max_code_len)
    buf.status.zero_()
    if single_sweep:  # outputs the call must overwrite
        buf.payload_bits.fill_(-1); buf.chunk_offset.fill_(-1); buf.sub_bits.fill_(-1)
    if single_sweep_hist:
        buf.hist.fill_(-7)   # the call must overwrite it
    B.co3_encode(plan, books, gt, mt, mt, gamma, buf, mode=mode, single_sweep=single_sweep,
                 stochastic_seed=stochastic_seed, single_sweep_hist=single_sweep_hist)
    torch.cuda.synchronize()
    out = dict(
        m_new=mt[:, :d].cpu().numpy(), sym=_sym_numpy(buf.symbols_2d()),
        hist=buf.hist.cpu().numpy().view(np.uint64), chunk_offset=buf.chunk_offset.cpu().numpy().view(np.uint64),
        sub_bits=buf.sub_bits.cpu().numpy().view(np.uint16), payload_bits=buf.payload_bits.cpu().numpy().view(np.uint64),
        words=buf.words.cpu().numpy().view(np.uint32), status_encode=buf.status.cpu().numpy().copy(),
    )
    lc = [books.export(b) for b in range(plan.num_books)]
    out["lens"] = np.stack([x[0] for x in lc]); out["codes"] = np.stack([x[1] for x in lc])
    if want_decode:
        sym2 = torch.full((plan.symbols_bytes,), 255, dtype=torch.uint8, device=dev)
        q = torch.full((U, stride), float("nan"), dtype=torch.float32, device=dev)
        B.co3_decode(plan, books, buf, symbols=sym2, q=q)
        avg = torch.full((d,), float("nan"), dtype=torch.float32, device=dev)
        B.co3_ps_aggregate(plan, books, buf, avg)
        torch.cuda.synchronize()
        out["dec_sym"] = _sym_numpy(B.symbols_2d(plan, sym2))
        out["dec_q"] = q[:, :d].cpu().numpy()
        out["avg"] = avg.cpu().numpy()
        out["status"] = buf.status.cpu().numpy().copy()
    return out, (plan, books, buf, gt, mt)


def oracle_round(plan_kwargs, g, m, gamma, weights=None, stochastic_seed=None):
    E, M = plan_kwargs["E"], plan_kwargs["M"]
    U, d = g.shape
    seg_len = plan_kwargs.get("seg_len") or [d]
    seg_book = plan_kwargs.get("seg_book") or [0] * len(seg_len)
    bias = np.broadcast_to(np.asarray(plan_kwargs["bias"], np.int32), (U, len(seg_len)))
    pub = bool(plan_kwargs.get("per_user_books", False))
    enc = oround.encode_round(g, m, gamma, E, M, seg_len, seg_book, bias, pub, weights, stochastic_seed=stochastic_seed)
    sym, avg = oround.ps_round(enc, E, M, seg_len, seg_book, bias, pub)
    enc["dec_sym"] = sym
    enc["avg"] = avg
    vals = np.empty(g.shape, np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            lut = np.array([orc.value(s, E, M, int(bias[u, k])) for s in range(1 << (1 + E + M))])
            vals[u, off:off + n] = lut[sym[u, off:off + n]]
        off += n
    enc["dec_q"] = vals
    return enc


def assert_bits_equal(a, b, what):
    a = np.ascontiguousarray(a); b = np.ascontiguousarray(b)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    av = a.view(np.uint32) if a.dtype == np.float32 else a
    bv = b.view(np.uint32) if b.dtype == np.float32 else b
    if not np.array_equal(av, bv):
        bad = np.flatnonzero(av.ravel() != bv.ravel())
        raise AssertionError(f"{what}: {bad.size} of {av.size} differ, first at {bad[:5]}: "
                             f"gpu {a.ravel()[bad[:5]]} oracle {b.ravel()[bad[:5]]}")


def compare_round(gpu, ref, d, decode=True, avg_exact=True, single_sweep=False):
    """Bit-exact for symbols, histograms, codebooks, offsets, bitstreams and the fp32 memory;
    the PS average within 1e-6 relative (and, since the GPU sums in fp64 in the oracle's order,
    normally identical)."""
    if not single_sweep:  # the single-sweep encoder produces neither
        assert_bits_equal(gpu["sym"], ref["sym"], "symbols")
        assert_bits_equal(gpu["hist"], ref["hist"], "histogram")
    assert_bits_equal(gpu["m_new"], ref["m_new"], "memory m'")
    assert_bits_equal(gpu["lens"], ref["lens"], "code lengths")
    assert_bits_equal(gpu["codes"], ref["codes"], "codes")
    assert_bits_equal(gpu["chunk_offset"], ref["chunk_offset"], "chunk offsets")
    assert_bits_equal(gpu["sub_bits"], ref["sub_bits"], "sub-chunk bits")
    assert_bits_equal(gpu["payload_bits"], ref["payload_bits"], "payload bits")
    for u, w in enumerate(ref["words"]):
        assert_bits_equal(gpu["words"][u, :w.size], w, f"bitstream of user {u}")
    assert int(gpu["status_encode"][0]) == int(ref["counters"][0])
    assert int(gpu["status_encode"][1]) == int(ref["counters"][1])
    assert int(gpu["status_encode"][6]) == 0, "single-sweep encoder stalled"
    if decode:
        assert_bits_equal(gpu["dec_sym"], ref["dec_sym"], "decoded symbols")
        assert_bits_equal(gpu["dec_q"], ref["dec_q"], "decoded values")
        U = gpu["dec_q"].shape[0]
        scale = np.maximum(np.abs(ref["avg"]), np.abs(ref["dec_q"]).mean(axis=0))
        assert np.all(np.abs(gpu["avg"].astype(np.float64) - ref["avg"]) <= 1e-6 * scale), "PS average"
        if avg_exact:
            assert_bits_equal(gpu["avg"], ref["avg"], "PS average (bitwise)")
        assert int(gpu["status"][5]) == 0, "decoder flagged corruption"
