"""GPU-vs-oracle parity through the C ABI (pytest -m gpu).  Bit-exact for symbols, histograms,
codebooks, bit offsets, bitstreams and the fp32 error memory; 1e-6 relative for the PS average."""
import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_oracle as orc
import gpu_util as gu

pytestmark = pytest.mark.gpu

BOOK_FIXED, BOOK_EMPIRICAL = 0, 1


def make_inputs(rng, U, d, E, M, bias, beta=1.0, alpha=1e-3, specials=0.2, mem_scale=0.5):
    g = np.stack([syn.gennorm_numpy(rng, d, beta, alpha) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, beta, alpha * mem_scale) for _ in range(U)])
    if specials:
        for u in range(U):
            idx = rng.choice(d, int(d * specials), replace=False)
            g[u, idx] = gu.special_values(E, M, bias, rng, idx.size)
            m[u, idx[: idx.size // 2]] = 0
    return g, m


@pytest.mark.parametrize("E,M,d", [(3, 0, 5 * 2048 + 123), (4, 1, 4096 * 3 + 70), (4, 3, 40000), (3, 2, 4095),
                                   (5, 2, 2049), (2, 1, 64), (2, 5, 10000), (7, 0, 9000)])
def test_single_user_adversarial(E, M, d):
    print(f"case E={E} M={M} d={d}", flush=True)
    rng = np.random.default_rng(E * 1000 + M * 10 + d)
    bias = min((2 ** E - 2) + 9, 100)          # top binade 2^-9 (2^26 for the 7-bit exponent)
    g, m = make_inputs(rng, 1, d, E, M, bias)
    kw = dict(E=E, M=M, U=1, d=d, bias=[[bias]])
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    ref = gu.oracle_round(kw, g, m, 0.9)
    gu.compare_round(gpu, ref, d)


def test_nonfinite_inputs():
    E, M, d, bias = 4, 3, 7000, 20
    rng = np.random.default_rng(1)
    g, m = make_inputs(rng, 2, d, E, M, bias)
    g[0, [0, 5, 4096, 6999]] = [np.nan, np.inf, -np.inf, np.nan]
    m[1, [17, 18]] = [np.inf, np.nan]
    kw = dict(E=E, M=M, U=2, d=d, bias=[[bias], [bias]])
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    ref = gu.oracle_round(kw, g, m, 0.9)
    assert int(ref["counters"][0]) == 6
    gu.compare_round(gpu, ref, d)


def test_extreme_bias_denormal_range():
    # smallest supported scale: the subnormal row of the format lies in fp32's denormal range
    E, M, d, bias = 4, 3, 20000, 127
    rng = np.random.default_rng(2)
    top = orc.grid(E, M, bias)[-1]
    g = (rng.standard_normal((1, d)) * top / 3).astype(np.float32)
    g[0, :4000] = gu.special_values(E, M, bias, rng, 4000)
    m = (rng.standard_normal((1, d)) * top / 8).astype(np.float32)
    kw = dict(E=E, M=M, U=1, d=d, bias=[[bias]])
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    ref = gu.oracle_round(kw, g, m, 0.9)
    gu.compare_round(gpu, ref, d)
    # and the largest supported scale
    bias = (2 ** E - 2) - 100
    top = orc.grid(E, M, bias)[-1]
    g = (rng.standard_normal((1, d)) * top / 3).astype(np.float32)
    m = (rng.standard_normal((1, d)) * top / 8).astype(np.float32)
    kw = dict(E=E, M=M, U=1, d=d, bias=[[bias]])
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    gu.compare_round(gpu, gu.oracle_round(kw, g, m, 0.9), d)


@pytest.mark.parametrize("per_user", [False, True])
def test_multi_user_multi_segment(per_user):
    E, M, U = 3, 2, 3
    seg_len = [1, 63, 4097, 0, 2048 * 3 + 5, 64, 9001, 4096]
    seg_book = [0, 1, 2, 0, 1, 3, 2, 0]
    d = sum(seg_len)
    rng = np.random.default_rng(7 + per_user)
    bias = rng.integers(8, 20, (U, len(seg_len))).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 8)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 30)
        off += n
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book, per_user_books=per_user)
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    ref = gu.oracle_round(kw, g, m, 0.9)
    gu.compare_round(gpu, ref, d)


def test_fixed_model_codebook():
    # code designed from the GenNorm model (Sec. IV-A (ii)); weights come from the oracle's model
    E, M, U, d = 4, 3, 2, 30000
    rng = np.random.default_rng(11)
    g = np.stack([syn.gennorm_numpy(rng, d, 0.9, 1e-3) for _ in range(U)])
    m = np.zeros_like(g)
    bias = syn.bias_for_max(np.abs(g).max(), E)
    w, _, _ = orc.gennorm_weights(E, M, bias, 0.0, 1e-3, 0.9)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], max_code_len=64)
    ref = gu.oracle_round(kw, g, m, 0.9, weights=w[None, :])
    gu.compare_round(gpu, ref, d)
    assert ref["lens"].max() > 11


def test_long_codes_slow_paths():
    # weights 1, 1, 2, 4, ... give codes of up to 63 bits: exercises the 64-bit encode and the
    # canonical-search decode paths
    E, M, U, d = 4, 1, 1, 6000
    A = 64
    nm = orc.num_magnitudes(E, M)
    emit = np.array([s for s in range(A) if (s & 31) < nm and s != 32])
    w = np.zeros(A, np.uint64)
    w[emit] = np.array([1] + [1 << i for i in range(emit.size - 1)], np.uint64)
    rng = np.random.default_rng(13)
    bias = 16
    grid = orc.grid(E, M, bias)
    k = rng.integers(0, nm, d)
    g = (grid[k] * rng.choice([-1.0, 1.0], d)).astype(np.float32)[None, :]
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]])
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], max_code_len=64)
    ref = gu.oracle_round(kw, g, m, 0.9, weights=w[None, :])
    assert ref["lens"].max() >= 57
    gu.compare_round(gpu, ref, d)


def test_iterations_carry_memory_cfg1_recipe():
    # workload 1 at reduced d: fresh gradient per iteration, memory carried, bias per iteration
    w = syn.WORKLOADS["cfg1"].scaled(d=3 * 4096 + 999)
    m = np.zeros((1, w.d), np.float32)
    for it in range(w.iters):
        g = syn.user_gradient_numpy(w, it, 0)[None, :]
        v = g + np.float32(w.gamma) * m
        bias = syn.bias_for_max(np.abs(v).max(), w.E)
        kw = dict(E=w.E, M=w.M, U=1, d=w.d, bias=[[bias]])
        gpu, _ = gu.gpu_round(kw, g, m, w.gamma, BOOK_EMPIRICAL)
        ref = gu.oracle_round(kw, g, m, w.gamma)
        gu.compare_round(gpu, ref, w.d)
        m = ref["m_new"]


def test_in_place_and_determinism():
    E, M, U, d, bias = 4, 3, 4, 50000, 18
    rng = np.random.default_rng(17)
    g, m = make_inputs(rng, U, d, E, M, bias, specials=0.05)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    a, _ = gu.gpu_round(kw, g, m, 0.5, BOOK_EMPIRICAL)
    b, _ = gu.gpu_round(kw, g, m, 0.5, BOOK_EMPIRICAL)
    for key in ("sym", "m_new", "hist", "words", "chunk_offset", "sub_bits", "avg"):
        gu.assert_bits_equal(a[key], b[key], key)


def test_error_paths_capacity_nocode_corrupt():
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U, d, bias = 4, 1, 1, 20000, 16
    rng = np.random.default_rng(19)
    g = syn.gennorm_numpy(rng, d, 1.0, 2.0 ** -12)[None, :]
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]])
    ref = gu.oracle_round(kw, g, m, 0.9)
    need = ref["words"][0].size
    # stream buffer two chunks short: the last chunks are skipped and counted, nothing is written past it
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL, words_stride=need - 700, want_decode=False)
    assert int(gpu["status_encode"][B.STAT_CAPACITY]) >= 1
    gu.assert_bits_equal(gpu["chunk_offset"], ref["chunk_offset"], "offsets still exact")
    # fixed code that lacks symbols which occur
    w = ref["hist"][0].copy(); w[np.argsort(w)[-3]] = 0
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], want_decode=False)
    assert int(gpu["status_encode"][B.STAT_NOCODE]) == int(ref["hist"][0][np.argsort(ref["hist"][0])[-3]])
    # corrupt stream / index: the decoder flags it and stays inside the buffers
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    assert int(gpu["status"][B.STAT_CORRUPT]) == 0
    buf.sub_bits[0, 5] += 3
    buf.words[0, 100:140] = -1
    buf.status.zero_()
    out = torch.zeros(d, dtype=torch.float32, device="cuda:0")
    B.co3_ps_aggregate(plan, books, buf, out)
    torch.cuda.synchronize()
    assert int(buf.status[B.STAT_CORRUPT].item()) >= 1


# ---- single-sweep encoder (fixed code, symbols never stored) ------------------------------------

def _single_sweep_case(kw, g, m, gamma, max_code_len=32, weights=None):
    """Code from the oracle's own histogram of this input (or `weights`), then both sides encode
    with that fixed code; the GPU side through the single-sweep entry."""
    if weights is None:
        weights = gu.oracle_round(kw, g, m, gamma)["hist"]
    ref = gu.oracle_round(kw, g, m, gamma, weights=weights)
    gpu, _ = gu.gpu_round(kw, g, m, gamma, BOOK_FIXED, weights=weights, max_code_len=max_code_len,
                          single_sweep=True)
    gu.compare_round(gpu, ref, kw["d"], single_sweep=True)
    return gpu, ref


@pytest.mark.parametrize("E,M,d", [(3, 0, 5 * 2048 + 123), (4, 3, 40000), (3, 2, 4095), (2, 1, 1), (4, 3, 4096 * 4),
                                   (4, 2, 4096 * 9 + 1)])
def test_single_sweep_single_user(E, M, d):
    rng = np.random.default_rng(100 + d)
    bias = 14 if E == 4 else (6 if E == 3 else 2)
    g, m = make_inputs(rng, 1, d, E, M, bias, alpha=orc.grid(E, M, bias)[-1] / 6)
    kw = dict(E=E, M=M, U=1, d=d, bias=[[bias]])
    _single_sweep_case(kw, g, m, 0.9)


@pytest.mark.parametrize("per_user", [False, True])
def test_single_sweep_multi_user_multi_segment(per_user):
    # layers that start at unaligned elements, empty and tiny layers, several tables
    E, M, U = 3, 2, 3
    seg_len = [1, 63, 4097, 0, 2048 * 3 + 5, 64, 9001, 4096, 4096 * 5, 7]
    seg_book = [0, 1, 2, 0, 1, 3, 2, 0, 1, 3]
    d = sum(seg_len)
    rng = np.random.default_rng(27 + per_user)
    bias = rng.integers(8, 20, (U, len(seg_len))).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 8)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 30)
        off += n
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book, per_user_books=per_user)
    _single_sweep_case(kw, g, m, 0.9)


def test_single_sweep_many_workgroups():
    # enough chunks that the encoder takes four chunks per workgroup (smaller inputs get one), and more
    # than 64 workgroups per user, so that the look-back walks several windows of entries
    E, M, U = 4, 3, 8
    d = 4096 * 4 * 261 + 4096 + 17
    rng = np.random.default_rng(31)
    g = np.stack([syn.gennorm_numpy(rng, d, 1.0, 1e-3) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, 1.0, 3e-4) for _ in range(U)])
    bias = syn.bias_for_max(np.abs(g + np.float32(0.9) * m).max(), E)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    _single_sweep_case(kw, g, m, 0.9)


def test_single_sweep_one_chunk_per_workgroup_many_entries():
    # the small form (one chunk per workgroup) with more than 64 look-back entries per user
    E, M, U = 4, 3, 2
    d = 4096 * 150 + 17
    rng = np.random.default_rng(32)
    g = np.stack([syn.gennorm_numpy(rng, d, 1.0, 1e-3) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, 1.0, 3e-4) for _ in range(U)])
    bias = syn.bias_for_max(np.abs(g + np.float32(0.9) * m).max(), E)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    _single_sweep_case(kw, g, m, 0.9)


def test_single_sweep_long_codes_and_model_code():
    E, M, U, d = 4, 1, 1, 6000
    A = 64
    nm = orc.num_magnitudes(E, M)
    emit = np.array([s for s in range(A) if (s & 31) < nm and s != 32])
    w = np.zeros(A, np.uint64)
    w[emit] = np.array([1] + [1 << i for i in range(emit.size - 1)], np.uint64)
    rng = np.random.default_rng(13)
    bias = 16
    grid = orc.grid(E, M, bias)
    k = rng.integers(0, nm, d)
    g = (grid[k] * rng.choice([-1.0, 1.0], d)).astype(np.float32)[None, :]
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]])
    _, ref = _single_sweep_case(kw, g, m, 0.9, max_code_len=64, weights=w[None, :])
    assert ref["lens"].max() >= 57
    # GenNorm-model code (Sec. IV-A (ii)) on GenNorm data
    E, M, U, d = 4, 3, 2, 30000
    g = np.stack([syn.gennorm_numpy(rng, d, 0.9, 1e-3) for _ in range(U)])
    m = np.zeros_like(g)
    bias = syn.bias_for_max(np.abs(g).max(), E)
    w, _, _ = orc.gennorm_weights(E, M, bias, 0.0, 1e-3, 0.9)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    _single_sweep_case(kw, g, m, 0.9, max_code_len=64, weights=w[None, :])


def test_single_sweep_capacity_and_nocode():
    E, M, U, d, bias = 4, 3, 2, 4096 * 6 + 100, 18
    rng = np.random.default_rng(41)
    g, m = make_inputs(rng, U, d, E, M, bias, specials=0.0, alpha=2e-3)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    ref = gu.oracle_round(kw, g, m, 0.5)
    small = int(ref["chunk_offset"][0][3] // 32) + 5   # room for three chunks and a bit
    gpu, _ = gu.gpu_round(kw, g, m, 0.5, BOOK_FIXED, weights=ref["hist"], words_stride=small,
                          want_decode=False, single_sweep=True)
    assert int(gpu["status_encode"][3]) >= 1
    gu.assert_bits_equal(gpu["chunk_offset"], ref["chunk_offset"], "chunk offsets")
    gu.assert_bits_equal(gpu["words"][0, : int(ref["chunk_offset"][0][3] // 32)],
                         ref["words"][0][: int(ref["chunk_offset"][0][3] // 32)], "chunks that fit")
    w = ref["hist"].copy()
    third = np.argsort(ref["hist"][0])[-3]
    w[0, third] = 0
    gpu, _ = gu.gpu_round(kw, g, m, 0.5, BOOK_FIXED, weights=w, want_decode=False, single_sweep=True)
    assert int(gpu["status_encode"][2]) == int(ref["hist"][0][third])


def test_single_sweep_bounded_wait_gives_up():
    # The look-back's wait is bounded.  With the bound set to zero from the host a workgroup gives up at the
    # first predecessor entry that is not there yet: it writes no stream words, leaves its chunk offsets
    # untouched and is counted, and so are the workgroups behind it that meet its entry.  Every kernel
    # still ends normally; memory, sub-chunk bits and payload are complete; and whatever was written to
    # the streams is what the oracle writes there.
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U = 4, 3, 4
    d = 4096 * 4 * 300 + 4096 + 17
    rng = np.random.default_rng(77)
    g = np.stack([syn.gennorm_numpy(rng, d, 1.0, 1e-3) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, 1.0, 3e-4) for _ in range(U)])
    bias = syn.bias_for_max(np.abs(g + np.float32(0.9) * m).max(), E)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    weights = gu.oracle_round(kw, g, m, 0.9)["hist"]
    ref = gu.oracle_round(kw, g, m, 0.9, weights=weights)
    B.set_lookback_polls(0)
    try:
        gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=weights, single_sweep=True,
                                                       want_decode=False)
    finally:
        B.set_lookback_polls(B.LOOKBACK_POLLS_DEFAULT)
    stalled = int(gpu["status_encode"][B.STAT_STALLED])
    nch = plan.num_chunks
    print(f"{stalled} workgroups gave up", flush=True)
    assert stalled > 0
    gu.assert_bits_equal(gpu["m_new"], ref["m_new"], "memory m'")
    gu.assert_bits_equal(gpu["sub_bits"], ref["sub_bits"], "sub-chunk bits")
    gu.assert_bits_equal(gpu["payload_bits"], ref["payload_bits"], "payload bits")
    untouched = np.uint64(0xFFFFFFFFFFFFFFFF)
    skipped = 0
    for u in range(U):
        co = gpu["chunk_offset"][u]
        expect = np.zeros(buf.words_stride, np.uint32)       # the buffer starts out as zeros
        for c in range(nch):
            if co[c] == untouched:
                skipped += 1
                continue
            assert co[c] == ref["chunk_offset"][u][c], (u, c)
            w0, w1 = int(ref["chunk_offset"][u][c]) // 32, int(ref["chunk_offset"][u][c + 1]) // 32
            expect[w0:w1] = ref["words"][u][w0:w1]
        assert co[nch] in (untouched, ref["chunk_offset"][u][nch])
        gu.assert_bits_equal(gpu["words"][u], expect, f"stream of user {u}: written chunks as the oracle's, the rest untouched")
    # chunks are skipped by whole workgroups of four
    assert skipped >= stalled and skipped <= 4 * stalled
    # and with the default bound the same call completes
    gpu2, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=weights, single_sweep=True, want_decode=False)
    gu.compare_round(gpu2, ref, d, decode=False, single_sweep=True)


def test_device_builder_refuses_the_sentinel_weight():
    # 2^64 - 1 is the device merge's "queue exhausted" mark; as a weight it is refused before the merge
    # (the host builder refuses it too: the weights sum to 2^64 - 1 or more): counted, table left empty
    import torch
    from paper_2204_08211_amd import binding as B
    E, M = 3, 2
    A = 1 << (1 + E + M)
    w = np.zeros((2, A), np.uint64)
    w[0, 1] = 1; w[0, 2] = np.uint64(0xFFFFFFFFFFFFFFFF)
    w[1, :8] = np.arange(1, 9, dtype=np.uint64)              # a sound table next to it
    with pytest.raises(B.Co3Error) as ei:
        B.co3_build_codebook(E, M, 2, w)
    assert ei.value.code == B.ERR_ARG
    books = B.co3_build_codebook(E, M, 2, None)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int64, device="cuda:0")
    wt = torch.from_numpy(w.view(np.int64)).to("cuda:0")
    B.co3_build_codebook_device(books, wt, status)
    torch.cuda.synchronize()
    assert int(status[B.STAT_CODELEN].item()) == 1
    lens0, codes0 = books.export(0)
    assert not lens0.any() and not codes0.any()
    lens1, codes1 = books.export(1)
    lo, co = orc.codebook(w[1])
    assert np.array_equal(lens1, lo) and np.array_equal(codes1, co)


# ---- PS model update fused into the average (Algorithm 1 line 14) -------------------------------

@pytest.mark.parametrize("U,eta,with_out", [(1, 1.0, True), (3, 0.1, True), (10, 0.05, False), (16, 0.3, True)])
def test_ps_model_update(U, eta, with_out):
    import torch
    from paper_2204_08211_amd import binding as B
    E, M = 4, 3
    seg_len = [4096 * 2 + 5, 0, 3000, 4096]
    seg_book = [0, 1, 1, 0]
    d = sum(seg_len)
    rng = np.random.default_rng(50 + U)
    bias = rng.integers(12, 18, (U, len(seg_len))).astype(np.int32)
    g = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, orc.grid(E, M, int(bias[u, k]))[-1] / 10)
        off += n
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book)
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    ref = gu.oracle_round(kw, g, m, 0.9)
    gu.compare_round(gpu, ref, d)
    w0 = rng.normal(0, 1e-2, d).astype(np.float32)
    w_ref = orc.model_update(ref["dec_sym"], seg_len, bias, E, M, eta, w0)
    w_t = torch.from_numpy(w0.copy()).to(gt.device)
    out = torch.full((d,), float("nan"), dtype=torch.float32, device=gt.device) if with_out else None
    B.co3_ps_aggregate(plan, books, buf, out, model=w_t, eta=eta)
    torch.cuda.synchronize()
    gu.assert_bits_equal(w_t.cpu().numpy(), w_ref, "updated model")
    if with_out:
        gu.assert_bits_equal(out.cpu().numpy(), ref["avg"], "PS average")
    # two steps in a row equal two oracle steps
    B.co3_ps_aggregate(plan, books, buf, out, model=w_t, eta=eta)
    torch.cuda.synchronize()
    gu.assert_bits_equal(w_t.cpu().numpy(), orc.model_update(ref["dec_sym"], seg_len, bias, E, M, eta, w_ref),
                         "model after two updates")


# ---- stochastic fp conversion (dithered Q, Sec. II-B (ii)) --------------------------------------

@pytest.mark.parametrize("E,M,d,seed", [(3, 0, 5 * 2048 + 123, 1), (4, 3, 40000, 0xDEADBEEF12345678), (2, 1, 4095, 7),
                                        (5, 2, 4096 * 4 + 1, 2 ** 63 + 5), (5, 5, 2048 * 9 + 3, 11), (4, 7, 4097, 2 ** 40)])
def test_stochastic_single_user_both_encoders(E, M, d, seed):
    # the last two: 16-bit symbols (whole tiles of the vector path and a ragged end; a tile-sized vector plus one)
    rng = np.random.default_rng(300 + d)
    bias = {2: 2, 3: 6, 4: 14, 5: 22}[E]
    g, m = make_inputs(rng, 1, d, E, M, bias, alpha=orc.grid(E, M, bias)[-1] / 6)
    # the zero/subnormal row and tiny inputs
    tiny = orc.grid(E, M, bias)[1]
    g[0, :500] = rng.uniform(-2 * tiny, 2 * tiny, 500).astype(np.float32)
    g[0, 500:520] = np.array([1e-45, -1e-45, 3e-39, -3e-39, 0.0] * 4, np.float32)
    m[0, :520] = 0
    kw = dict(E=E, M=M, U=1, d=d, bias=[[bias]])
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL, stochastic_seed=seed)
    ref = gu.oracle_round(kw, g, m, 0.9, stochastic_seed=seed)
    gu.compare_round(gpu, ref, d)
    # the same dithers in the single-sweep encoder
    gpu1, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=ref["hist"], single_sweep=True, stochastic_seed=seed)
    ref1 = gu.oracle_round(kw, g, m, 0.9, weights=ref["hist"], stochastic_seed=seed)
    gu.compare_round(gpu1, ref1, d, single_sweep=True)
    # another seed gives another stream; the closest-representative mode is untouched by the seed
    other = gu.oracle_round(kw, g, m, 0.9, stochastic_seed=seed + 1)
    assert not np.array_equal(other["sym"], ref["sym"])


@pytest.mark.parametrize("E,M", [(3, 2), (3, 6)])
def test_stochastic_multi_user_multi_segment(E, M):
    U = 3
    seg_len = [1, 63, 4097, 0, 2048 * 3 + 5, 64, 9001, 4096, 4096 * 5, 7]
    seg_book = [0, 1, 2, 0, 1, 3, 2, 0, 1, 3]
    d = sum(seg_len)
    rng = np.random.default_rng(401)
    bias = rng.integers(8, 20, (U, len(seg_len))).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 8)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 30)
        off += n
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book, per_user_books=False)
    seed = 20240229
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL, stochastic_seed=seed)
    ref = gu.oracle_round(kw, g, m, 0.9, stochastic_seed=seed)
    gu.compare_round(gpu, ref, d)
    gpu1, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=ref["hist"], single_sweep=True, stochastic_seed=seed)
    ref1 = gu.oracle_round(kw, g, m, 0.9, weights=ref["hist"], stochastic_seed=seed)
    gu.compare_round(gpu1, ref1, d, single_sweep=True)


# ---- degenerate sizes ----------------------------------------------------------------------------

@pytest.mark.parametrize("d", [0, 1, 2, 3, 5, 63, 64, 65])
def test_tiny_vectors_both_encoders(d):
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U, bias = 3, 2, 3, 6
    rng = np.random.default_rng(600 + d)
    g = rng.laplace(0, 0.3, (U, d)).astype(np.float32)
    m = rng.laplace(0, 0.1, (U, d)).astype(np.float32)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    if d == 0:
        # nothing to encode: empty streams, zero payload, offsets [0]; the calls must still succeed
        plan = B.Plan(**kw)
        books = B.co3_build_codebook(E, M, plan.num_books, None)
        buf = B.RoundBuffers(plan, "cuda:0")
        z = torch.zeros((U, 4), dtype=torch.float32, device="cuda:0")
        out = torch.zeros(4, dtype=torch.float32, device="cuda:0")
        for single in (False, True):
            buf.chunk_offset.fill_(-1); buf.payload_bits.fill_(-1); buf.hist.fill_(12345)
            B.co3_encode(plan, books, z, z, z, 0.9, buf, mode=B.BOOK_FIXED if single else B.BOOK_EMPIRICAL,
                         single_sweep=single)
            B.co3_ps_aggregate(plan, books, buf, out)
            torch.cuda.synchronize()
            assert buf.chunk_offset.cpu().numpy().tolist() == [[0]] * U
            assert buf.payload_bits.cpu().numpy().tolist() == [0] * U
            if not single:   # the histogram is an output of the three-step encoder: cleared even when nothing is counted
                assert not buf.hist.cpu().numpy().any()
        return
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
    ref = gu.oracle_round(kw, g, m, 0.9)
    gu.compare_round(gpu, ref, d)
    gpu1, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=ref["hist"], single_sweep=True)
    ref1 = gu.oracle_round(kw, g, m, 0.9, weights=ref["hist"])
    gu.compare_round(gpu1, ref1, d, single_sweep=True)


# ---- real-valued scale on top of the integer bias (eq. (exp bias) with b in R) --------------------

def _gain_case(single_sweep, U=3, E=4, M=3):
    import torch
    from oracle import co3_bias_model as bm
    from paper_2204_08211_amd import binding as B
    A = 1 << (1 + E + M)
    sym_t = np.uint16 if A > 256 else np.uint8
    seg_len = [4096 * 2 + 77, 0, 4096 * 3, 1000]
    seg_book = [0, 1, 1, 0]
    nseg = len(seg_len)
    d = sum(seg_len)
    rng = np.random.default_rng(900 + single_sweep)
    # per (user, layer): a GenNorm model, its real-valued optimum of eq. (exp bias), split into bias and gain
    bias = np.zeros((U, nseg), np.int32); gain = np.ones((U, nseg), np.float32); inv_gain = np.ones((U, nseg), np.float32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            beta, alpha = 0.7 + 0.3 * u, 10.0 ** (-3 + 0.5 * k)
            b, _ = bm.best_real_scale(bm.signed_set(E, M, (1 << (E - 1)) - 1), alpha, beta, lo=-30, hi=10, step=0.25)
            bias[u, k], gain[u, k], inv_gain[u, k] = bm.split_real_scale(E, b)
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, beta, alpha)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, alpha / 5)
        off += n
    assert np.any(gain != 1.0)
    g[0, :6] = [np.nan, np.inf, -np.inf, 1e30, -1e30, 0.0]
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book)
    gamma = 0.9
    # the oracle: Algorithm 1 lines 8-10 with the scaled set, then the code of its own histogram
    sym = np.empty((U, d), sym_t); m_ref = np.empty_like(g); q_ref = np.empty_like(g)
    counters = np.zeros(2, np.uint64)
    hist = np.zeros((2, A), np.uint64)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            mo, so, qo, cnt = orc.ef_step_gain(g[u, off:off + n], m[u, off:off + n], gamma, E, M, int(bias[u, k]),
                                               gain[u, k], inv_gain[u, k])
            sym[u, off:off + n] = so; m_ref[u, off:off + n] = mo; q_ref[u, off:off + n] = qo; counters += cnt
            orc.histogram(so, A, hist[seg_book[k]])
        off += n
    lens = np.stack([orc.huffman_lengths(hist[b]) for b in range(2)])
    codes = np.stack([orc.canonical_codes(lens[b]) for b in range(2)])
    avg_ref = orc.aggregate_gain(sym, seg_len, bias, inv_gain, E, M)
    # the library
    dev = torch.device("cuda:0")
    plan = B.Plan(**kw)
    plan.set_gain(gain, inv_gain)
    stride = (d + 3) // 4 * 4
    gt = torch.zeros((U, stride), dtype=torch.float32, device=dev); gt[:, :d] = torch.from_numpy(g).to(dev)
    mt = torch.zeros((U, stride), dtype=torch.float32, device=dev); mt[:, :d] = torch.from_numpy(m).to(dev)
    buf = B.RoundBuffers(plan, dev, max_code_len=32)
    if single_sweep:
        books = B.co3_build_codebook(E, M, plan.num_books, hist)
        B.co3_encode(plan, books, gt, mt, mt, gamma, buf, mode=B.BOOK_FIXED, single_sweep=True)
    else:
        books = B.co3_build_codebook(E, M, plan.num_books, None)
        B.co3_encode(plan, books, gt, mt, mt, gamma, buf, mode=B.BOOK_EMPIRICAL)
    qd = torch.full((U, stride), float("nan"), dtype=torch.float32, device=dev)
    symd = torch.full((plan.symbols_bytes,), 255, dtype=torch.uint8, device=dev)
    avg = torch.full((d,), float("nan"), dtype=torch.float32, device=dev)
    B.co3_decode(plan, books, buf, symbols=symd, q=qd)
    B.co3_ps_aggregate(plan, books, buf, avg)
    torch.cuda.synchronize()
    gu.assert_bits_equal(mt[:, :d].cpu().numpy(), m_ref, "memory m'")
    if not single_sweep:
        gu.assert_bits_equal(buf.symbols_2d().cpu().numpy().view(sym_t), sym, "symbols")
        gu.assert_bits_equal(buf.hist.cpu().numpy().view(np.uint64), hist, "histogram")
    for b in range(2):
        lb, cb = books.export(b)
        assert np.array_equal(lb, lens[b]) and np.array_equal(cb, codes[b])
    for u in range(U):
        r = orc.pack(sym[u], seg_len, seg_book, lens, codes)
        nw = int(r["chunk_offset"][-1]) // 32
        gu.assert_bits_equal(buf.words[u, :nw].cpu().numpy().view(np.uint32), r["words"][:nw], f"bitstream of user {u}")
    gu.assert_bits_equal(B.symbols_2d(plan, symd).cpu().numpy().view(sym_t), sym, "decoded symbols")
    gu.assert_bits_equal(qd[:, :d].cpu().numpy(), q_ref, "decoded values")
    gu.assert_bits_equal(avg.cpu().numpy(), avg_ref, "PS average")
    st = buf.status.cpu().numpy()
    assert int(st[0]) == int(counters[0]) == 3 and int(st[1]) == int(counters[1])
    # not defined together with the stochastic conversion; and switching the scale off restores the plain step
    with pytest.raises(B.Co3Error):
        B.co3_encode(plan, books, gt, mt, mt, gamma, buf, mode=B.BOOK_FIXED, single_sweep=True, stochastic_seed=1)
    if A > 256:   # the reference loops below use the byte oracle's entry points
        return
    plan.set_gain(None, None)
    mt[:, :d] = torch.from_numpy(m).to(dev)
    B.co3_encode(plan, books, gt, mt, mt, gamma, buf, mode=B.BOOK_EMPIRICAL)
    torch.cuda.synchronize()
    n0 = seg_len[0]
    mo, so, _, _ = orc.ef_step(g[1, :n0], m[1, :n0], gamma, E, M, int(bias[1, 0]), want_q=False)
    gu.assert_bits_equal(mt[1, :n0].cpu().numpy(), mo, "memory m' with the scale switched off")
    gu.assert_bits_equal(buf.symbols_2d()[1, :n0].cpu().numpy().view(sym_t), so, "symbols with the scale switched off")


@pytest.mark.parametrize("single_sweep,U", [(False, 3), (True, 3), (True, 7)])
def test_real_valued_scale_both_encoders(single_sweep, U):
    # U = 7: the PS average takes the kernel for five or more users (values scaled from one table)
    _gain_case(single_sweep, U)


@pytest.mark.parametrize("single_sweep", [False, True])
def test_real_valued_scale_wide_alphabet(single_sweep):
    _gain_case(single_sweep, 3, E=5, M=5)


# ---- alphabets wider than one byte (9 to 12 symbol bits, 16-bit symbols) ---------------------------------

@pytest.mark.parametrize("E,M,d", [(5, 6, 4096 * 3 + 77), (4, 5, 4095), (3, 5, 1), (5, 3, 4096 * 2), (5, 6, 3 * 2 ** 20 + 4097)])
def test_wide_alphabets_both_encoders(E, M, d):
    import torch
    from paper_2204_08211_amd import binding as B
    U = 3
    A = 1 << (1 + E + M)
    seg_len = [d] if d < 5000 else [4097, 0, d - 4097 - 63, 63]
    seg_book = [0] if d < 5000 else [0, 1, 1, 0]
    nseg = len(seg_len)
    rng = np.random.default_rng(1200 + E * 10 + M)
    bias = rng.integers(12, 18, (U, nseg)).astype(np.int32) + (8 if E == 5 else 0)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 0.9, top / 40)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 200)
        off += n
    if d > 10:
        g[0, :5] = [np.nan, np.inf, 1e30, -1e30, 0.0]
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book)
    gamma = 0.9
    ref = gu.oracle_round(kw, g, m, gamma)
    assert ref["sym"].dtype == np.uint16

    dev = torch.device("cuda:0")
    plan = B.Plan(**kw)
    assert plan.wide and plan.A == A
    stride = (d + 3) // 4 * 4
    gt = torch.zeros((U, stride), dtype=torch.float32, device=dev); gt[:, :d] = torch.from_numpy(g).to(dev)

    def run(mode, books, single_sweep):
        mt = torch.zeros((U, stride), dtype=torch.float32, device=dev); mt[:, :d] = torch.from_numpy(m).to(dev)
        buf = B.RoundBuffers(plan, dev, max_code_len=40)
        buf.chunk_offset.fill_(-1); buf.sub_bits.fill_(-1); buf.payload_bits.fill_(-1)
        B.co3_encode(plan, books, gt, mt, mt, gamma, buf, mode=mode, single_sweep=single_sweep)
        symd = torch.full((plan.symbols_bytes,), 255, dtype=torch.uint8, device=dev)
        qd = torch.full((U, stride), float("nan"), dtype=torch.float32, device=dev)
        avg = torch.full((d,), float("nan"), dtype=torch.float32, device=dev)
        B.co3_decode(plan, books, buf, symbols=symd, q=qd)
        B.co3_ps_aggregate(plan, books, buf, avg)
        torch.cuda.synchronize()
        gu.assert_bits_equal(mt[:, :d].cpu().numpy(), ref["m_new"], "memory m'")
        if not single_sweep:
            gu.assert_bits_equal(buf.symbols_2d().cpu().numpy().view(np.uint16), ref["sym"], "symbols")
            gu.assert_bits_equal(buf.hist.cpu().numpy().view(np.uint64), ref["hist"], "histogram")
        for b in range(plan.num_books):
            lb, cb = books.export(b)
            assert np.array_equal(lb, ref["lens"][b]) and np.array_equal(cb, ref["codes"][b]), f"code table {b}"
        gu.assert_bits_equal(buf.chunk_offset.cpu().numpy().view(np.uint64), ref["chunk_offset"], "chunk offsets")
        gu.assert_bits_equal(buf.sub_bits.cpu().numpy().view(np.uint16), ref["sub_bits"], "sub-chunk bits")
        gu.assert_bits_equal(buf.payload_bits.cpu().numpy().view(np.uint64), ref["payload_bits"], "payload bits")
        for u, wds in enumerate(ref["words"]):
            gu.assert_bits_equal(buf.words[u, :wds.size].cpu().numpy().view(np.uint32), wds, f"bitstream of user {u}")
        gu.assert_bits_equal(B.symbols_2d(plan, symd).cpu().numpy().view(np.uint16), ref["dec_sym"], "decoded symbols")
        gu.assert_bits_equal(qd[:, :d].cpu().numpy(), ref["dec_q"], "decoded values")
        gu.assert_bits_equal(avg.cpu().numpy(), ref["avg"], "PS average")
        st = buf.status.cpu().numpy()
        assert int(st[0]) == int(ref["counters"][0]) and int(st[1]) == int(ref["counters"][1])
        assert not st[2:].any()
        # the PS update fused into the average (Algorithm 1 line 14)
        w0 = np.random.default_rng(1250).normal(0, 1e-2, d).astype(np.float32)
        w_t = torch.from_numpy(w0.copy()).to(dev)
        B.co3_ps_aggregate(plan, books, buf, None, model=w_t, eta=0.37)
        torch.cuda.synchronize()
        gu.assert_bits_equal(w_t.cpu().numpy(), orc.model_update(ref["dec_sym"], seg_len, bias, E, M, 0.37, w0),
                             "updated model")

    # the code built on the device from this round's counts, then the same code built on the host and held
    books = B.co3_build_codebook(E, M, plan.num_books, None)
    run(B.BOOK_EMPIRICAL, books, False)
    held = B.co3_build_codebook(E, M, plan.num_books, ref["hist"])
    run(B.BOOK_FIXED, held, True)
    # the held code without a symbol buffer, this round's counts asked for as well
    mt = torch.zeros((U, stride), dtype=torch.float32, device=dev); mt[:, :d] = torch.from_numpy(m).to(dev)
    buf = B.RoundBuffers(plan, dev, max_code_len=40)
    buf.hist.fill_(-1)
    B.co3_encode(plan, held, gt, mt, mt, gamma, buf, mode=B.BOOK_FIXED, single_sweep=True, single_sweep_hist=True)
    torch.cuda.synchronize()
    gu.assert_bits_equal(buf.hist.cpu().numpy().view(np.uint64), ref["hist"], "histogram beside the held code")
    gu.assert_bits_equal(mt[:, :d].cpu().numpy(), ref["m_new"], "memory m'")
    for u, wds in enumerate(ref["words"]):
        gu.assert_bits_equal(buf.words[u, :wds.size].cpu().numpy().view(np.uint32), wds, f"bitstream of user {u}")


@pytest.mark.parametrize("stochastic", [False, True])
def test_wide_held_code_with_layers_on_the_tile_grid(stochastic):
    # layers that start at multiples of 2048 elements (the held code's chunk sizes are then summed in the first
    # sweep): one of two chunks, one of half a chunk, an empty one, one with another table and a ragged end; a
    # symbol without a code among them
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U = 4, 5, 3
    A = 1 << (1 + E + M)
    seg_len = [4096 * 2, 2048, 0, 4096 + 2048 + 100]
    seg_book = [0, 1, 0, 1]
    d = sum(seg_len)
    rng = np.random.default_rng(2100)
    bias = rng.integers(10, 14, (U, 4)).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 50)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 300)
        off += n
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book)
    seed = 77 if stochastic else None
    first = gu.oracle_round(kw, g, m, 0.9, stochastic_seed=seed)            # its histograms are the held code's weights
    ref = gu.oracle_round(kw, g, m, 0.9, weights=first["hist"], stochastic_seed=seed)
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=first["hist"], max_code_len=40, stochastic_seed=seed)
    gu.compare_round(gpu, ref, d)
    assert int(gpu["status_encode"][B.STAT_NOCODE]) == 0
    w0 = first["hist"].copy()
    victim = int(np.argsort(w0[1])[-5])
    w0[1, victim] = 0
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w0, max_code_len=40, want_decode=False, stochastic_seed=seed)
    assert int(gpu["status_encode"][B.STAT_NOCODE]) == int(first["hist"][1, victim])


@pytest.mark.parametrize("U,per_user", [(1, False), (17, False), (9, True)])
def test_wide_user_counts_through_the_average(U, per_user):
    # one user; more users than a workgroup of the average has wavefronts (several passes per wavefront), with one
    # set of tables and with a set per user; two layers with their own tables, a ragged last chunk
    E, M = 4, 5
    seg_len = [4096 + 9, 4096 * 2 - 1]
    d = sum(seg_len)
    rng = np.random.default_rng(1900 + U)
    bias = rng.integers(10, 14, (U, 2)).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 50)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 300)
        off += n
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=[0, 1], per_user_books=per_user)
    ref = gu.oracle_round(kw, g, m, 0.9)
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL, max_code_len=40)
    gu.compare_round(gpu, ref, d)


def test_wide_long_codes_per_user_tables_and_device_builder():
    # weights 1, 1, 2, 4, ... on the symbols that occur give codes of up to 61 bits (both halves of the coder's
    # 64-bit append, the decoder's search by length); a table per user; the device builder on the same weights
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U, d = 4, 4, 2, 9000
    A = 1 << (1 + E + M)
    rng = np.random.default_rng(1301)
    bias = np.array([[9], [11]], np.int32)
    w = np.zeros((U, A), np.uint64)
    g = np.empty((U, d), np.float32)
    for u in range(U):
        grid = orc.grid(E, M, int(bias[u, 0]))
        mags = rng.choice(np.arange(1, grid.size), 31, replace=False)
        emit = np.concatenate([mags, mags + (A >> 1)])                     # both signs
        w[u, emit] = np.array([1] + [1 << i for i in range(emit.size - 1)], np.uint64)[rng.permutation(emit.size)]
        k = rng.choice(mags, d)
        g[u] = (grid[k] * rng.choice([-1.0, 1.0], d)).astype(np.float32)
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, per_user_books=True)
    ref = gu.oracle_round(kw, g, m, 0.9, weights=w)
    assert ref["lens"].max() >= 57
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w, max_code_len=64, want_decode=False)
    for key, what in [("m_new", "memory"), ("lens", "code lengths"), ("codes", "codes"), ("chunk_offset", "chunk offsets"),
                      ("sub_bits", "sub-chunk bits"), ("payload_bits", "payload bits")]:
        gu.assert_bits_equal(gpu[key], ref[key], what)
    gu.assert_bits_equal(buf.symbols_2d().cpu().numpy().view(np.uint16), ref["sym"], "symbols")
    for u, wds in enumerate(ref["words"]):
        gu.assert_bits_equal(gpu["words"][u, :wds.size], wds, f"bitstream of user {u}")
    symd = torch.zeros(plan.symbols_bytes, dtype=torch.uint8, device="cuda:0")
    avg = torch.zeros(d, dtype=torch.float32, device="cuda:0")
    B.co3_decode(plan, books, buf, symbols=symd)
    B.co3_ps_aggregate(plan, books, buf, avg)
    torch.cuda.synchronize()
    gu.assert_bits_equal(B.symbols_2d(plan, symd).cpu().numpy().view(np.uint16), ref["dec_sym"], "decoded symbols")
    gu.assert_bits_equal(avg.cpu().numpy(), ref["avg"], "PS average")
    assert int(buf.status[B.STAT_CORRUPT].item()) == 0

    # the device builder gives the host builder's tables; a table holding the sentinel weight is refused and left empty
    w3 = np.concatenate([w, np.zeros((1, A), np.uint64)]); w3[2, 7] = 1; w3[2, 9] = np.uint64(0xFFFFFFFFFFFFFFFF)
    dev_books = B.co3_build_codebook(E, M, 3, None)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int64, device="cuda:0")
    B.co3_build_codebook_device(dev_books, torch.from_numpy(w3.view(np.int64)).to("cuda:0"), status)
    torch.cuda.synchronize()
    assert int(status[B.STAT_CODELEN].item()) == 1
    for b in range(2):
        lb, cb = dev_books.export(b)
        assert np.array_equal(lb, ref["lens"][b]) and np.array_equal(cb, ref["codes"][b])
    lb, cb = dev_books.export(2)
    assert not lb.any() and not cb.any()
    with pytest.raises(B.Co3Error):
        B.co3_build_codebook(E, M, 3, w3)


@pytest.mark.parametrize("per_user", [False, True])
def test_wide_decoder_second_level_tables(per_user):
    # a code with 500 magnitudes of about 10 bits, 1400 of 12 to 16 (more 12-bit prefixes hold only longer codes
    # than the decoder has second-level tables: some of these codes are found there, the rest by search) and 24 of
    # up to 40 bits; every symbol with a code about equally often in the data; the host's tables and the device's
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U, d = 5, 6, 3, 4096 * 7 + 300
    A = 1 << (1 + E + M)
    rng = np.random.default_rng(1800)
    bias = np.full((U, 1), 20, np.int32)
    grid = orc.grid(E, M, 20)
    perm = rng.permutation(np.arange(1, grid.size))
    freq, mid, rare = perm[:500], perm[500:1900], perm[1900:1924]
    w = np.zeros(A, np.uint64)
    w[freq] = 64 << 24
    w[mid] = rng.integers(2, 17, mid.size).astype(np.uint64) << 24
    w[rare] = np.array([1] + [1 << i for i in range(rare.size - 1)], np.uint64)[rng.permutation(rare.size)]
    w[(A >> 1):] = w[:(A >> 1)]                                            # both signs
    used = np.concatenate([freq, mid, rare])
    g = (grid[rng.choice(used, (U, d))] * rng.choice([-1.0, 1.0], (U, d))).astype(np.float32)
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, per_user_books=per_user)
    wt = np.repeat(w[None, :], U if per_user else 1, axis=0)
    ref = gu.oracle_round(kw, g, m, 0.9, weights=wt)
    lens = ref["lens"][0]
    n12 = int((np.ldexp(1.0, 12 - lens[(lens > 12)].astype(int))).sum())   # 12-bit prefixes under the longer codes
    assert n12 > 300 and (lens[mid] >= 13).sum() > 1000 and lens[mid].max() <= 17 and lens[rare].max() >= 36
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=wt, max_code_len=64, want_decode=False)
    for u, wds in enumerate(ref["words"]):
        gu.assert_bits_equal(gpu["words"][u, :wds.size], wds, f"bitstream of user {u}")

    def check(books, what):
        buf.status.zero_()
        symd = torch.zeros(plan.symbols_bytes, dtype=torch.uint8, device="cuda:0")
        avg = torch.zeros(d, dtype=torch.float32, device="cuda:0")
        B.co3_decode(plan, books, buf, symbols=symd)
        B.co3_ps_aggregate(plan, books, buf, avg)
        torch.cuda.synchronize()
        gu.assert_bits_equal(B.symbols_2d(plan, symd).cpu().numpy().view(np.uint16), ref["dec_sym"], f"decoded symbols, {what}")
        gu.assert_bits_equal(avg.cpu().numpy(), ref["avg"], f"PS average, {what}")
        assert int(buf.status[B.STAT_CORRUPT].item()) == 0

    check(books, "tables built on the host")
    dev_books = B.co3_build_codebook(E, M, plan.num_books, None)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int64, device="cuda:0")
    B.co3_build_codebook_device(dev_books, torch.from_numpy(wt.view(np.int64)).to("cuda:0"), status)
    torch.cuda.synchronize()
    assert not status.cpu().numpy().any()
    check(dev_books, "tables built on the device")


def test_wide_coder_rows_overflow_and_mixed_chunks():
    # a fixed code whose frequent symbols are not the data's: chunks of 18 bits per element (a lane's codewords
    # do not fit its LDS row: appended at their final offsets instead), chunks of about 10 (the row coder), a chunk
    # that mixes both, a ragged last chunk, at an odd element offset so that the symbols start mid-word
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U = 4, 5, 2
    A = 1 << (1 + E + M)
    rng = np.random.default_rng(1600)
    bias = np.array([[10, 10], [10, 10]], np.int32)
    grid = orc.grid(E, M, 10)
    light = rng.choice(np.arange(1, grid.size), 128, replace=False)         # magnitudes the table holds as rare
    w = np.full(A, 1 << 12, np.uint64)
    w[light] = 1; w[light + (A >> 1)] = 1
    heavy = np.setdiff1d(np.arange(1, grid.size), light)
    seg_len = [4097, 4096 * 3 + 1000]
    d = sum(seg_len)
    g = np.empty((U, d), np.float32)
    for u in range(U):
        k = rng.choice(heavy, d)
        k[4097 + 0:4097 + 4096] = rng.choice(light, 4096)                   # a whole chunk of rare symbols
        k[4097 + 4096 + 2000:4097 + 4096 + 2200] = rng.choice(light, 200)   # a chunk with some lanes of them
        k[-500:] = rng.choice(light, 500)                                   # the ragged chunk's end
        g[u] = (grid[k] * rng.choice([-1.0, 1.0], d)).astype(np.float32)
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=[0, 0])
    ref = gu.oracle_round(kw, g, m, 0.9, weights=w[None, :])
    lens = ref["lens"][0]
    assert lens[light].min() >= 17 and lens.max() <= 25 and lens[heavy].max() <= 11
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], max_code_len=25,
                                                   want_decode=False)
    for key, what in [("m_new", "memory"), ("chunk_offset", "chunk offsets"), ("sub_bits", "sub-chunk bits"),
                      ("payload_bits", "payload bits")]:
        gu.assert_bits_equal(gpu[key], ref[key], what)
    for u, wds in enumerate(ref["words"]):
        gu.assert_bits_equal(gpu["words"][u, :wds.size], wds, f"bitstream of user {u}")
    avg = torch.zeros(d, dtype=torch.float32, device="cuda:0")
    B.co3_ps_aggregate(plan, books, buf, avg)
    torch.cuda.synchronize()
    gu.assert_bits_equal(avg.cpu().numpy(), ref["avg"], "PS average")
    assert int(buf.status[B.STAT_CORRUPT].item()) == 0 and int(gpu["status_encode"][B.STAT_NOCODE]) == 0


def test_wide_coder_few_long_codes_in_a_chunk():
    # a code whose rare symbols have codewords of 26 to 45 bits (beyond what the coder's LDS entries hold), and a
    # handful of them per chunk: in one lane (first element, last element, two in a row), in lanes at both ends of
    # the wavefront, in as many lanes as are coded again one by one and in one more (the chunk's plain loops), in the
    # ragged last chunk; then the same with one of those symbols left without a code: counted, nothing else
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U = 5, 5, 2
    A = 1 << (1 + E + M)
    rng = np.random.default_rng(1700)
    bias = np.array([[20], [20]], np.int32)
    grid = orc.grid(E, M, 20)
    rare = rng.choice(np.arange(1, grid.size), 34, replace=False)
    w = np.full(A, 1 << 36, np.uint64)
    w[rare] = np.array([1] + [1 << i for i in range(rare.size - 1)], np.uint64); w[rare + (A >> 1)] = w[rare]
    common = np.setdiff1d(np.arange(1, grid.size), rare)
    long_ = rare[np.asarray(orc.huffman_lengths(w))[rare] >= 26]
    assert long_.size >= 20
    d = 4096 * 7 + 1500
    put = {0: [0, 4095],                               # chunk 0: lane 0's first element, lane 63's last
           1: [64 * 7 + 3, 64 * 7 + 4, 64 * 8],        # chunk 1: two in a row in lane 7, lane 8's first
           2: [5, 64 * 20 + 63, 64 * 41 + 31, 64 * 63],          # chunk 2: four lanes
           3: [64 * l + 9 for l in (1, 2, 30, 31, 62)],          # chunk 3: five lanes
           4: list(range(64 * 13, 64 * 14)),                     # chunk 4: every element of lane 13
           7: [0, 64 * 23 + 27]}                                 # the ragged chunk: lane 0, and its last element
    g = np.empty((U, d), np.float32)
    ks = []
    for u in range(U):
        k = rng.choice(common, d)
        for c, where in put.items():
            k[4096 * c + np.array(where)] = rng.choice(long_, len(where))
        ks.append(k)
        g[u] = (grid[k] * rng.choice([-1.0, 1.0], d)).astype(np.float32)
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=bias)
    ref = gu.oracle_round(kw, g, m, 0.9, weights=w[None, :])
    lens = ref["lens"][0]
    assert lens[long_].min() >= 26 and lens[long_].max() >= 44 and lens[common].max() <= 12
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], max_code_len=64,
                                                   want_decode=False)
    for key, what in [("m_new", "memory"), ("chunk_offset", "chunk offsets"), ("sub_bits", "sub-chunk bits"),
                      ("payload_bits", "payload bits")]:
        gu.assert_bits_equal(gpu[key], ref[key], what)
    for u, wds in enumerate(ref["words"]):
        gu.assert_bits_equal(gpu["words"][u, :wds.size], wds, f"bitstream of user {u}")
    avg = torch.zeros(d, dtype=torch.float32, device="cuda:0")
    B.co3_ps_aggregate(plan, books, buf, avg)
    torch.cuda.synchronize()
    gu.assert_bits_equal(avg.cpu().numpy(), ref["avg"], "PS average")
    assert int(buf.status[B.STAT_CORRUPT].item()) == 0 and int(gpu["status_encode"][B.STAT_NOCODE]) == 0

    victim = int(ks[0][4096 * 2 + 5])                  # occurs in a chunk whose lanes are coded again one by one
    w0 = w.copy(); w0[victim] = 0; w0[victim + (A >> 1)] = 0
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w0[None, :], max_code_len=64, want_decode=False)
    assert int(gpu["status_encode"][B.STAT_NOCODE]) == sum(int((k == victim).sum()) for k in ks)


@pytest.mark.parametrize("E,M", [(2, 1), (3, 2), (4, 3), (5, 2), (3, 5), (4, 5), (4, 6), (5, 6)])
def test_device_builders_against_the_oracle(E, M):
    # the builders' sort, merge in rounds with ties, depths and canonical ranks at byte and wide alphabet sizes:
    # tables of many equal weights, of one and two symbols, of distinct powers of two (a path), of counts as a
    # round gives them, of few symbols spread over the alphabet, and an empty one
    import torch
    from paper_2204_08211_amd import binding as B
    A = 1 << (1 + E + M)
    rng = np.random.default_rng(1500 + A)
    tabs = []
    tabs.append(rng.integers(0, 4, A).astype(np.uint64))                          # ties everywhere, some unused
    tabs.append(np.ones(A, np.uint64))                                            # all equal: a full tree
    one = np.zeros(A, np.uint64); one[A - 3] = 5; tabs.append(one)
    two = np.zeros(A, np.uint64); two[0] = 7; two[A - 1] = 7; tabs.append(two)
    npath = min(40, A // 2)
    path = np.zeros(A, np.uint64); idx = rng.choice(A, npath, replace=False)
    path[idx] = np.uint64(1) << np.arange(npath, dtype=np.uint64); tabs.append(path)
    geo = np.floor(1e9 * np.exp(-np.abs(np.arange(A) - A / 2) / (A / 40))).astype(np.uint64); tabs.append(geo)
    nfew = min(100, A // 2)
    few = np.zeros(A, np.uint64); few[rng.choice(A, nfew, replace=False)] = rng.integers(1, 1000, nfew).astype(np.uint64)
    tabs.append(few)
    big = rng.integers(1, 1 << 50, A).astype(np.uint64); tabs.append(big)
    fib = np.zeros(A, np.uint64); nf = min(A, 60); a_, b_ = 1, 1
    for i in range(nf):
        fib[(7 * i) % A if A > 60 else i] = a_; a_, b_ = b_, a_ + b_
    tabs.append(fib)                                                              # the deepest tree for its weights
    tabs.append(np.zeros(A, np.uint64))
    w = np.stack(tabs)
    books = B.co3_build_codebook(E, M, len(tabs), None)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int64, device="cuda:0")
    B.co3_build_codebook_device(books, torch.from_numpy(w.view(np.int64)).to("cuda:0"), status)
    torch.cuda.synchronize()
    assert int(status[B.STAT_CODELEN].item()) == 0
    for b, wt in enumerate(tabs):
        lens, codes = books.export(b)
        if not wt.any():
            assert not lens.any() and not codes.any()
            continue
        rl, rc = orc.codebook(wt)
        gu.assert_bits_equal(lens, rl, f"code lengths of table {b}")
        gu.assert_bits_equal(codes, rc, f"codes of table {b}")


@pytest.mark.parametrize("E,M", [(4, 3), (5, 5)])
def test_device_builders_weights_that_overflow(E, M):
    # sums of 2^64 and of 2^64 - 1 (the queues' sentinel) are refused and counted, the table left empty; the
    # largest sum that fits is coded; tables are independent of each other
    import torch
    from paper_2204_08211_amd import binding as B
    A = 1 << (1 + E + M)
    w = np.zeros((4, A), np.uint64)
    w[0, 3] = w[0, A - 2] = np.uint64(1) << np.uint64(63)                       # 2^64
    w[1, 3] = np.uint64(1) << np.uint64(63); w[1, 9] = (np.uint64(1) << np.uint64(63)) - np.uint64(1)   # 2^64 - 1
    w[2, 1] = w[2, 5] = w[2, 7] = np.uint64(1) << np.uint64(62)                 # 3 x 2^62: fits
    w[3, :40] = np.arange(1, 41, dtype=np.uint64)
    books = B.co3_build_codebook(E, M, 4, None)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int64, device="cuda:0")
    B.co3_build_codebook_device(books, torch.from_numpy(w.view(np.int64)).to("cuda:0"), status)
    torch.cuda.synchronize()
    assert int(status[B.STAT_CODELEN].item()) == 2
    for b in (0, 1):
        lens, codes = books.export(b)
        assert not lens.any() and not codes.any()
    for b in (2, 3):
        lens, codes = books.export(b)
        rl, rc = orc.codebook(w[b])
        gu.assert_bits_equal(lens, rl, f"code lengths of table {b}")
        gu.assert_bits_equal(codes, rc, f"codes of table {b}")


def test_wide_error_paths_capacity_nocode_corrupt():
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U, d, bias = 5, 4, 1, 20000, 24
    rng = np.random.default_rng(1302)
    g = syn.gennorm_numpy(rng, d, 1.0, 2.0 ** -6)[None, :]
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]])
    ref = gu.oracle_round(kw, g, m, 0.9)
    need = ref["words"][0].size
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL, words_stride=need - 1500, want_decode=False)
    assert int(gpu["status_encode"][B.STAT_CAPACITY]) >= 1
    gu.assert_bits_equal(gpu["chunk_offset"], ref["chunk_offset"], "offsets still exact")
    w = ref["hist"][0].copy(); victim = np.argsort(w)[-3]; w[victim] = 0
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], want_decode=False)
    assert int(gpu["status_encode"][B.STAT_NOCODE]) == int(ref["hist"][0][victim])
    gpu, (plan, books, buf, gt, mt) = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL, want_decode=False)
    buf.sub_bits[0, 5] += 3
    buf.words[0, 100:140] = -1
    buf.chunk_offset[0, 3] += 32 * (1 << 40)          # an index entry far outside the stream buffer
    buf.status.zero_()
    out = torch.zeros(d, dtype=torch.float32, device="cuda:0")
    symd = torch.zeros(plan.symbols_bytes, dtype=torch.uint8, device="cuda:0")
    B.co3_ps_aggregate(plan, books, buf, out)
    B.co3_decode(plan, books, buf, symbols=symd)
    torch.cuda.synchronize()
    assert int(buf.status[B.STAT_CORRUPT].item()) >= 2


# ---- single-sweep encoder that also counts the symbols ------------------------------------------------------

@pytest.mark.parametrize("per_user,seed", [(False, None), (True, None), (False, 77)])
def test_single_sweep_with_histogram(per_user, seed):
    # several layers at arbitrary offsets (aligned, shifted and ragged chunks), an empty layer, a shared table
    E, M, U = 4, 2, 3
    seg_len = [4096 * 2 + 5, 0, 4096 * 3, 777, 4096 + 4095]
    seg_book = [0, 1, 1, 2, 0]
    d = sum(seg_len)
    rng = np.random.default_rng(1400 + int(per_user))
    bias = rng.integers(12, 16, (U, len(seg_len))).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.1, top / 30)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 300)
        off += n
    g[1, 3:6] = [np.nan, np.inf, -1e30]
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book, per_user_books=per_user)
    weights = gu.oracle_round(kw, g, m, 0.9)["hist"] + 1          # a held code that is not this round's
    ref = gu.oracle_round(kw, g, m, 0.9, weights=weights, stochastic_seed=seed)
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=weights, single_sweep=True, single_sweep_hist=True,
                          stochastic_seed=seed)
    gu.compare_round(gpu, ref, d, single_sweep=True)
    gu.assert_bits_equal(gpu["hist"], ref["hist"], "histogram of the single sweep")


def test_single_sweep_with_histogram_many_workgroups_and_empty():
    import torch
    from paper_2204_08211_amd import binding as B
    # the four-chunks-per-workgroup form (above 2048 workgroups) with whole, aligned chunks
    E, M, U, d = 4, 3, 4, 4096 * 4 * 600
    rng = np.random.default_rng(1402)
    g = (rng.standard_normal((U, d)) * 1e-3).astype(np.float32)
    m = np.zeros_like(g)
    bias = 20
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    sym = np.stack([orc.ef_step(g[u], m[u], 0.9, E, M, bias, want_q=False)[1] for u in range(U)])
    hist = np.bincount(sym.ravel(), minlength=256).astype(np.uint64)[None, :]
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=hist + 1, single_sweep=True, single_sweep_hist=True,
                          want_decode=False)
    gu.assert_bits_equal(gpu["hist"], hist, "histogram of the single sweep")
    assert int(gpu["status_encode"][6]) == 0
    # no elements: the counts are cleared
    plan = B.Plan(E=E, M=M, U=2, d=0, bias=[[bias]] * 2)
    books = B.co3_build_codebook(E, M, plan.num_books, hist + 1)
    buf = B.RoundBuffers(plan, "cuda:0")
    z = torch.zeros((2, 4), dtype=torch.float32, device="cuda:0")
    buf.hist.fill_(12345); buf.payload_bits.fill_(-1)
    B.co3_encode(plan, books, z, z, z, 0.9, buf, mode=B.BOOK_FIXED, single_sweep=True, single_sweep_hist=True)
    torch.cuda.synchronize()
    assert not buf.hist.cpu().numpy().any() and buf.payload_bits.cpu().numpy().tolist() == [0, 0]


@pytest.mark.parametrize("U", [5, 9])
def test_long_codes_through_the_many_user_average(U):
    # codes of up to 63 bits decoded by the PS kernel for five or more users (rare path: boundary search and the
    # exact 64-bit window), different biases per user, a ragged last chunk
    E, M, d = 4, 1, 4096 * 2 + 1500
    A = 64
    nm = orc.num_magnitudes(E, M)
    emit = np.array([s for s in range(A) if (s & 31) < nm and s != 32])
    w = np.zeros(A, np.uint64)
    w[emit] = np.array([1] + [1 << i for i in range(emit.size - 1)], np.uint64)
    rng = np.random.default_rng(1500 + U)
    bias = rng.integers(12, 20, (U, 1)).astype(np.int32)
    g = np.empty((U, d), np.float32)
    for u in range(U):
        grid = orc.grid(E, M, int(bias[u, 0]))
        k = rng.integers(0, nm, d)
        g[u] = (grid[k] * rng.choice([-1.0, 1.0], d)).astype(np.float32)
    m = np.zeros_like(g)
    kw = dict(E=E, M=M, U=U, d=d, bias=bias)
    gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_FIXED, weights=w[None, :], max_code_len=64)
    ref = gu.oracle_round(kw, g, m, 0.9, weights=w[None, :])
    assert ref["lens"].max() >= 57
    gu.compare_round(gpu, ref, d)


def test_extreme_biases_through_the_many_user_average():
    # the PS kernel for five or more users forms a value as (pattern at bias 0) x 2^-bias: at bias 127 the format's
    # subnormal row lies in fp32's denormal range, at the other end the values reach 2^100; biases of the users a
    # few apart, so that the fp64 sums stay exact
    E, M, d = 4, 3, 4096 + 777
    for base in (127 - 5, (2 ** E - 2) - 100):
        U = 6
        rng = np.random.default_rng(1600 + base % 97)
        bias = (base + rng.integers(0, 6, (U, 1))).astype(np.int32)
        g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
        for u in range(U):
            b = int(bias[u, 0])
            top = orc.grid(E, M, b)[-1]
            g[u] = (rng.standard_normal(d) * top / 3).astype(np.float32)
            g[u, :1500] = gu.special_values(E, M, b, rng, 1500)
            m[u] = (rng.standard_normal(d) * top / 8).astype(np.float32)
        kw = dict(E=E, M=M, U=U, d=d, bias=bias)
        gpu, _ = gu.gpu_round(kw, g, m, 0.9, BOOK_EMPIRICAL)
        gu.compare_round(gpu, gu.oracle_round(kw, g, m, 0.9), d)
