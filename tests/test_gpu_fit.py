"""GPU-vs-oracle parity of the GenNorm moment fit and the model code's weights (pytest -m gpu).

Floating point: the GPU sums raw moments in one sweep in a fixed order, the oracle takes central
moments in two passes with NumPy's pairwise sums, and the two use different log-gamma routines.
Tolerances, from the arithmetic: mean within 1e-12 of the sample's standard deviation; kurtosis,
alpha and beta within 1e-9 relative for samples with |mean| <= sigma (the raw-moment route loses
about (mean/sigma)^4 ulps); weights within 1 + 1e-9 w of the oracle's SciPy-based ones (the floor
of p 2^40 may fall on either side).  The fitted model's code is then used by the single-sweep
encoder, whose streams are compared bit for bit with the oracle's encoding under the same tables.
"""
import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_gennorm_fit as fitm
from oracle import co3_oracle as orc
import gpu_util as gu

pytestmark = pytest.mark.gpu


def gpu_fit(kw, g, m, gamma):
    import torch
    from paper_2204_08211_amd import binding as B
    dev = torch.device("cuda:0")
    plan = B.Plan(**kw)
    U, d = plan.U, plan.d
    stride = (d + 3) // 4 * 4
    gt = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    mt = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    gt[:, :d] = torch.from_numpy(np.ascontiguousarray(g)).to(dev)
    mt[:, :d] = torch.from_numpy(np.ascontiguousarray(m)).to(dev)
    params = B.co3_gennorm_fit(plan, gt, mt, gamma)
    weights = B.co3_model_weights_device(plan, params)
    torch.cuda.synchronize()
    return plan, params.cpu().numpy(), weights.cpu().numpy().view(np.uint64), (gt, mt, params, weights)


def check_params(got, ref, sigma_floor=0.0):
    assert got.shape == ref.shape
    for idx in np.ndindex(ref.shape[:2]):
        mu_r, a_r, b_r, k_r = ref[idx]
        mu_g, a_g, b_g, k_g = got[idx]
        if a_r == 0.0:
            assert a_g == 0.0 and b_g == 0.0 and k_g == 0.0, idx
            assert abs(mu_g - mu_r) <= 1e-12 * max(abs(mu_r), 1e-30), idx
            continue
        sigma = a_r * np.sqrt(float(fitm.variance_factor(b_r)))
        assert abs(mu_g - mu_r) <= 1e-12 * sigma, (idx, mu_g, mu_r)
        assert abs(k_g / k_r - 1.0) <= 1e-9, (idx, k_g, k_r)
        assert abs(b_g / b_r - 1.0) <= 1e-9, (idx, b_g, b_r)
        assert abs(a_g / a_r - 1.0) <= 1e-9, (idx, a_g, a_r)


def check_weights(got, ref):
    assert got.shape == ref.shape
    assert np.array_equal(got > 0, ref > 0)
    g = got.astype(np.float64); r = ref.astype(np.float64)
    assert np.all(np.abs(g - r) <= 1.0 + 1e-9 * r), np.abs(g - r).max()


@pytest.mark.parametrize("beta,alpha,d,E,M", [(0.7, 1e-3, 4096 * 5 + 123, 4, 3), (1.0, 2e-3, 4095, 4, 3),
                                              (1.5, 1e-4, 4096 * 33, 4, 3), (2.0, 1e-2, 100_000, 4, 3),
                                              (0.9, 1e-3, 4096 * 3 + 5, 5, 6), (1.3, 3e-3, 9000, 3, 5)])
def test_fit_single_layer(beta, alpha, d, E, M):
    # the last two: alphabets of 12 and 9 bits (the model's weights for up to 4096 symbols)
    U = 2
    rng = np.random.default_rng(int(beta * 100) + d)
    g = np.stack([syn.gennorm_numpy(rng, d, beta, alpha) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, beta, alpha * 0.4) for _ in range(U)])
    bias = syn.bias_for_max(np.abs(g + np.float32(0.9) * m).max(), E)
    kw = dict(E=E, M=M, U=U, d=d, bias=[[bias]] * U)
    _, par, w, _ = gpu_fit(kw, g, m, 0.9)
    ref = fitm.fit_round(g, m, 0.9, [d])
    check_params(par, ref)
    check_weights(w, fitm.pooled_model_weights(E, M, [[bias]] * U, ref, [d], [0], False))


@pytest.mark.parametrize("per_user", [False, True])
def test_fit_layers_empty_constant_and_shared_tables(per_user):
    E, M, U = 3, 2, 3
    seg_len = [1, 63, 4097, 0, 2048 * 3 + 5, 64, 9001, 4096, 4096 * 5, 7]
    seg_book = [0, 1, 2, 0, 1, 3, 2, 0, 1, 3]
    d = sum(seg_len)
    rng = np.random.default_rng(91 + per_user)
    bias = rng.integers(8, 20, (U, len(seg_len))).astype(np.int32)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            top = orc.grid(E, M, int(bias[u, k]))[-1]
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 0.8 + 0.3 * u, top / 8)
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, top / 30)
        off += n
    g[1, 64:64 + 4097] = 0.25; m[1, 64:64 + 4097] = 0.0          # a constant layer: variance 0
    kw = dict(E=E, M=M, U=U, d=d, bias=bias, seg_len=seg_len, seg_book=seg_book, per_user_books=per_user)
    _, par, w, _ = gpu_fit(kw, g, m, 0.9)
    ref = fitm.fit_round(g, m, 0.9, seg_len)
    assert ref[0, 3, 1] == 0.0 and ref[1, 2, 1] == 0.0 and ref[0, 0, 1] == 0.0  # empty, constant, one element
    check_params(par, ref)
    check_weights(w, fitm.pooled_model_weights(E, M, bias, ref, seg_len, seg_book, per_user))


def test_fit_closed_form_samples():
    # {-1 (p), 0, +1 (p)} scaled: kurtosis 1/(2p) exactly; p = 1/12 is Laplace's 6, p = 1/6 the Normal's 3
    E, M = 4, 3
    d = 4096 * 3
    x = np.zeros((2, d), np.float32)
    x[0, : d // 12] = 0.5; x[0, d // 12: d // 6] = -0.5
    x[1, : d // 6] = 0.5; x[1, d // 6: d // 3] = -0.5
    kw = dict(E=E, M=M, U=2, d=d, bias=[[14]] * 2)
    _, par, _, _ = gpu_fit(kw, x, np.zeros_like(x), 0.9)
    assert abs(par[0, 0, 3] - 6.0) < 1e-12 and abs(par[0, 0, 2] - 1.0) < 1e-9
    assert abs(par[0, 0, 1] - 0.5 * np.sqrt(1.0 / 12.0)) < 1e-10 and par[0, 0, 0] == 0.0
    assert abs(par[1, 0, 3] - 3.0) < 1e-12 and abs(par[1, 0, 2] - 2.0) < 1e-9
    assert abs(par[1, 0, 1] - 0.5 * np.sqrt(2.0 / 3.0)) < 1e-10


def test_fit_is_deterministic_and_gamma_zero_ignores_memory():
    E, M, U, d = 4, 3, 3, 4096 * 7 + 11
    rng = np.random.default_rng(3)
    g = np.stack([syn.gennorm_numpy(rng, d, 0.9, 1e-3) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, 1.2, 1e-2) for _ in range(U)])
    kw = dict(E=E, M=M, U=U, d=d, bias=[[14]] * U)
    _, a, wa, _ = gpu_fit(kw, g, m, 0.0)
    _, b, wb, _ = gpu_fit(kw, g, np.zeros_like(m), 0.0)
    assert np.array_equal(a.view(np.uint64), b.view(np.uint64)) and np.array_equal(wa, wb)
    _, c, _, _ = gpu_fit(kw, g, m, 0.0)
    assert np.array_equal(a.view(np.uint64), c.view(np.uint64))


def test_fitted_model_code_drives_the_single_sweep_encoder():
    # fit on the device -> weights on the device -> code tables on the device -> single-sweep encode;
    # the oracle encodes with the tables the device built (exported), so every stream bit is compared
    import torch
    from paper_2204_08211_amd import binding as B
    w = syn.WORKLOADS["cfg3"].scaled(d=4096 * 9 + 77, U=4)
    g = np.stack([syn.user_gradient_numpy(w, 0, u) for u in range(w.U)])
    m = np.stack([syn.user_gradient_numpy(w, 1, u) for u in range(w.U)]) * np.float32(0.3)
    v = g + np.float32(w.gamma) * m
    bias = np.array([[syn.bias_for_max(np.abs(v[u]).max(), w.E)] for u in range(w.U)], np.int32)
    kw = dict(E=w.E, M=w.M, U=w.U, d=w.d, bias=bias)
    plan, par, wts, (gt, mt, params_t, weights_t) = gpu_fit(kw, g, m, w.gamma)
    ref_par = fitm.fit_round(g, m, w.gamma, [w.d])
    check_params(par, ref_par)
    ref_w = fitm.pooled_model_weights(w.E, w.M, bias, ref_par, [w.d], [0], False)
    check_weights(wts, ref_w)
    books = B.co3_build_codebook(w.E, w.M, plan.num_books, None)
    buf = B.RoundBuffers(plan, gt.device, max_code_len=64)
    B.co3_build_codebook_device(books, weights_t, buf.status)
    torch.cuda.synchronize()
    lens_dev, codes_dev = books.export(0)
    lens_o, codes_o = orc.codebook(wts[0])                 # the oracle's Huffman code of the device's weights
    assert np.array_equal(lens_dev, lens_o) and np.array_equal(codes_dev, codes_o)
    gpu, _ = gu.gpu_round(kw, g, m, w.gamma, 0, books=books, buf=buf, single_sweep=True)
    ref = gu.oracle_round(kw, g, m, w.gamma, weights=wts)
    gu.compare_round(gpu, ref, w.d, single_sweep=True)
    # the model code costs little more than the code of the round's own histogram
    emp = gu.oracle_round(kw, g, m, w.gamma)
    assert ref["payload_bits"].sum() <= 1.01 * emp["payload_bits"].sum()


@pytest.mark.parametrize("E,M", [(4, 3), (4, 6)])
def test_model_bias_on_the_device_and_a_round_with_it(E, M):
    # fit -> bias from the model (eq. (exp bias) with integer b) -> installed in the plan -> weights ->
    # code -> single-sweep encode -> PS average, all without the host; the oracle repeats every step.
    # (4, 6): an alphabet of 11 bits
    import torch
    from oracle import co3_bias_model as bm
    from paper_2204_08211_amd import binding as B
    U = 3
    seg_len = [4096 * 2 + 100, 0, 4096 * 3, 777]
    seg_book = [0, 1, 1, 0]
    d = sum(seg_len)
    rng = np.random.default_rng(123)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, 0.7 + 0.4 * u, 10.0 ** (-4 + k))
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, 10.0 ** (-5 + k))
        off += n
    gamma = 0.9
    start_bias = np.full((U, len(seg_len)), 14, np.int32)
    kw = dict(E=E, M=M, U=U, d=d, bias=start_bias, seg_len=seg_len, seg_book=seg_book, per_user_books=False)
    plan, par, _, (gt, mt, params_t, _) = gpu_fit(kw, g, m, gamma)
    ref_par = fitm.fit_round(g, m, gamma, seg_len)
    check_params(par, ref_par)
    bias_t, err_t = B.co3_model_bias_device(plan, params_t, install=True)
    torch.cuda.synchronize()
    bias_gpu = bias_t.cpu().numpy(); err_gpu = err_t.cpu().numpy()
    bias_ref, err_ref = bm.bias_table(E, M, ref_par)
    assert np.array_equal(bias_gpu, bias_ref), (bias_gpu, bias_ref)
    live = err_ref > 0
    assert np.all(np.abs(err_gpu[live] / err_ref[live] - 1.0) < 1e-8) and np.all(err_gpu[~live] == 0.0)
    assert bias_ref[0, 1] == 7                              # the empty layer: no model, IEEE bias
    # the library's host routine agrees with its device kernel
    for u in range(U):
        for k in range(len(seg_len)):
            assert B.co3_bias_from_model(E, M, *par[u, k, :3])[0] == bias_gpu[u, k]
    # weights and code for the new biases, then a whole round under them
    weights_t = B.co3_model_weights_device(plan, params_t)
    torch.cuda.synchronize()
    wts = weights_t.cpu().numpy().view(np.uint64)
    check_weights(wts, fitm.pooled_model_weights(E, M, bias_ref, ref_par, seg_len, seg_book, False))
    books = B.co3_build_codebook(E, M, plan.num_books, None)
    buf = B.RoundBuffers(plan, gt.device, max_code_len=64)
    B.co3_build_codebook_device(books, weights_t, buf.status)
    out = torch.zeros(d, dtype=torch.float32, device=gt.device)
    m_new = mt.clone()
    B.co3_encode(plan, books, gt, m_new, m_new, gamma, buf, mode=B.BOOK_FIXED, single_sweep=True)
    B.co3_ps_aggregate(plan, books, buf, out)
    torch.cuda.synchronize()
    kw_ref = dict(kw, bias=bias_ref)
    ref = gu.oracle_round(kw_ref, g, m, gamma, weights=wts)
    gu.assert_bits_equal(m_new[:, :d].cpu().numpy(), ref["m_new"], "memory m'")
    gu.assert_bits_equal(buf.chunk_offset.cpu().numpy().view(np.uint64), ref["chunk_offset"], "chunk offsets")
    for u, wds in enumerate(ref["words"]):
        gu.assert_bits_equal(buf.words[u, :wds.size].cpu().numpy().view(np.uint32), wds, f"bitstream of user {u}")
    gu.assert_bits_equal(out.cpu().numpy(), ref["avg"], "PS average")
    st = buf.status.cpu().numpy()
    assert st[B.STAT_NOCODE] == 0 and st[B.STAT_CORRUPT] == 0 and st[B.STAT_STALLED] == 0
    # the model's bias clips far less than one element in a thousand
    assert st[B.STAT_CLAMPED] < 1e-3 * U * d


@pytest.mark.parametrize("E,M", [(2, 1), (3, 2), (4, 3), (5, 2), (4, 5), (5, 6)])
def test_real_valued_scale_on_the_device_and_a_round_with_it(E, M):
    # eq. (exp bias) with real b for every (user, layer) on the device: against the oracle's evaluation of the
    # returned triple, the oracle's own optimum over real b, the library's host routine; a layer without a model;
    # then bias and scale installed from device memory and a whole round under them, against the oracle's
    # scaled conversion.  (5, 2): many binades, the integer bias stays where no real scale gains.  (4, 5), (5, 6): 10
    # and 12 bits
    import math
    import torch
    from scipy import special
    from oracle import co3_bias_model as bm
    from paper_2204_08211_amd import binding as B
    U = 3
    seg_len = [4096 + 50, 3000]
    d = sum(seg_len)
    A = 1 << (1 + E + M)
    sym_t = np.uint16 if A > 256 else np.uint8
    betas = [0.7, 1.0, 1.4]
    sigmas = [[3e-3, 0.2], [1.0, 1e-3], [5.0, 0.05]]
    par = np.zeros((U, 2, 4))
    for u in range(U):
        for k in range(2):
            beta = betas[u]
            par[u, k, 1] = sigmas[u][k] * math.sqrt(math.exp(special.gammaln(1.0 / beta) - special.gammaln(3.0 / beta)))
            par[u, k, 2] = beta
    par[0, 1, :] = 0.0                                   # no model for this layer
    par[2, 1, 0] = 0.3 * sigmas[2][1]                    # a mean that is not zero
    ieee = (1 << (E - 1)) - 1
    dev = torch.device("cuda:0")
    kw = dict(E=E, M=M, U=U, d=d, bias=np.full((U, 2), ieee, np.int32), seg_len=seg_len, seg_book=[0, 1])
    plan = B.Plan(**kw)
    params_t = torch.from_numpy(par).to(dev)
    bias_t, pairs_t, err_t = B.co3_model_scale_device(plan, params_t, install=True)
    torch.cuda.synchronize()
    bias = bias_t.cpu().numpy(); pairs = pairs_t.cpu().numpy(); err = err_t.cpu().numpy()
    reps = bm.signed_set(E, M, ieee)
    scaled_somewhere = False
    for u in range(U):
        for k in range(2):
            mu, alpha, beta = par[u, k, :3]
            gn, ig = float(pairs[u, k, 0]), float(pairs[u, k, 1])
            if alpha == 0.0:
                assert bias[u, k] == ieee and (gn, ig) == (1.0, 1.0) and err[u, k] == 0.0
                continue
            hb, hg, hi, he = B.co3_scale_from_model(E, M, mu, alpha, beta)
            # (the minimum is flat: the sums' rounding, taken in another order on the host, moves its place by up to
            # 1e-4 binades and its value by nothing that shows)
            assert hb == bias[u, k] and abs(ig / hi - 1.0) < 1e-3 and abs(err[u, k] / he - 1.0) < 1e-8, (u, k, ig, hi)
            assert np.float32(gn) == np.float32(1.0) / np.float32(ig)
            assert 2 ** -0.5 * (1 - 1e-6) <= ig <= 2 ** 0.5 * (1 + 1e-6)
            b_lib = (ieee - int(bias[u, k])) + math.log2(ig)
            assert abs(bm.scaled_sq_error(reps, b_lib, mu, alpha, beta) / err[u, k] - 1.0) < 1e-6, (u, k)
            b_int, err_int = B.co3_bias_from_model(E, M, mu, alpha, beta)
            assert err[u, k] <= err_int * (1 + 1e-12)
            if mu == 0.0:
                lo = (ieee - int(bias[u, k])) - 3.0
                b_opt, err_opt = bm.best_real_scale(reps, alpha, beta, lo=lo, hi=lo + 6.0)
                assert abs(err[u, k] / err_opt - 1.0) < 1e-5, (u, k, b_lib, b_opt)
            ob, og, oi = bm.split_real_scale(E, b_lib)
            assert ob == bias[u, k] and abs(float(oi) / ig - 1.0) < 1e-6
            scaled_somewhere = scaled_somewhere or ig != 1.0
    assert scaled_somewhere or E == 5

    # a round under the installed bias and scale
    rng = np.random.default_rng(900 + 10 * E + M)
    g = np.empty((U, d), np.float32); m = np.empty((U, d), np.float32)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            g[u, off:off + n] = syn.gennorm_numpy(rng, n, betas[u], sigmas[u][k])
            m[u, off:off + n] = syn.gennorm_numpy(rng, n, 1.0, sigmas[u][k] / 20)
        off += n
    gain = np.ascontiguousarray(pairs[:, :, 0]); inv_gain = np.ascontiguousarray(pairs[:, :, 1])
    sym = np.empty((U, d), sym_t); m_ref = np.empty_like(g)
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            mo, so, qo, cnt = orc.ef_step_gain(g[u, off:off + n], m[u, off:off + n], 0.9, E, M, int(bias[u, k]),
                                               gain[u, k], inv_gain[u, k])
            sym[u, off:off + n] = so; m_ref[u, off:off + n] = mo
        off += n
    avg_ref = orc.aggregate_gain(sym, seg_len, bias, inv_gain, E, M)
    stride = (d + 3) // 4 * 4
    gt = torch.zeros((U, stride), dtype=torch.float32, device=dev); gt[:, :d] = torch.from_numpy(g).to(dev)
    mt = torch.zeros((U, stride), dtype=torch.float32, device=dev); mt[:, :d] = torch.from_numpy(m).to(dev)
    buf = B.RoundBuffers(plan, dev, max_code_len=40)
    books = B.co3_build_codebook(E, M, plan.num_books, None)
    B.co3_encode(plan, books, gt, mt, mt, 0.9, buf, mode=B.BOOK_EMPIRICAL)
    avg = torch.full((d,), float("nan"), dtype=torch.float32, device=dev)
    B.co3_ps_aggregate(plan, books, buf, avg)
    torch.cuda.synchronize()
    gu.assert_bits_equal(mt[:, :d].cpu().numpy(), m_ref, "memory m'")
    gu.assert_bits_equal(buf.symbols_2d().cpu().numpy().view(sym_t), sym, "symbols")
    gu.assert_bits_equal(avg.cpu().numpy(), avg_ref, "PS average")
    # a scale installed from device memory counts as one: no stochastic conversion until it is removed
    with pytest.raises(B.Co3Error):
        B.co3_encode(plan, books, gt, mt, mt, 0.9, buf, mode=B.BOOK_EMPIRICAL, stochastic_seed=3)
    plan.set_gain(None, None)
    B.co3_encode(plan, books, gt, mt, mt, 0.9, buf, mode=B.BOOK_EMPIRICAL, stochastic_seed=3)
    torch.cuda.synchronize()
