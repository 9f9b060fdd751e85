"""Algorithm 1 as a closed loop on a synthetic strongly convex objective (pytest -m gpu): users'
gradients of f_u(w) = 1/2 sum_i a_i (w_i - c_{u,i})^2 at the PS model, CO3 encode with error
feedback, PS decode + model update, for several iterations.  The oracle runs the same loop on the
CPU; memories, streams and the model must stay identical bit for bit in every iteration.  The
gradient itself is two fp32 element-wise operations, done by torch on the device and by NumPy on
the host (both IEEE, no fusion).  Also checks what the loop is for: the loss falls, and with the
memory (gamma > 0) the compressed run ends closer to the uncompressed one than without it
(Sec. IV-A (iii))."""
import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_oracle as orc
from oracle import co3_round as oround
import gpu_util as gu

pytestmark = pytest.mark.gpu


def objective(rng, U, d):
    a = rng.uniform(0.5, 2.0, d).astype(np.float32)
    c = (rng.normal(0, 1.0, (1, d)) + rng.normal(0, 0.3, (U, d))).astype(np.float32)
    return a, c


def loss(a, c, w):
    return float(np.mean(0.5 * a.astype(np.float64) * (w.astype(np.float64)[None, :] - c) ** 2))


@pytest.mark.parametrize("gamma", [0.0, 0.9])
def test_closed_loop_matches_the_oracle(gamma):
    import torch
    from paper_2204_08211_amd import binding as B
    E, M, U, T, eta = 3, 0, 3, 8, 0.4          # a coarse format ([1,3,0]: 13 values) so that the memory matters
    seg_len = [4096 * 2 + 17, 1000]
    seg_book = [0, 1]
    d = sum(seg_len)
    nseg = len(seg_len)
    rng = np.random.default_rng(2024)
    a, c = objective(rng, U, d)
    dev = torch.device("cuda:0")
    stride = (d + 3) // 4 * 4
    a_t = torch.from_numpy(a).to(dev); c_t = torch.from_numpy(c).to(dev)
    w_t = torch.zeros(d, dtype=torch.float32, device=dev)
    m_t = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    g_t = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    w_o = np.zeros(d, np.float32)
    m_o = np.zeros((U, d), np.float32)
    w_plain = np.zeros(d, np.float32)          # uncompressed reference: w - eta * mean gradient, fp64
    bias0 = np.full((U, nseg), 3, np.int32)
    plan = B.Plan(E, M, U, d, bias0, seg_len=seg_len, seg_book=seg_book)
    books = B.co3_build_codebook(E, M, plan.num_books, None)
    buf = B.RoundBuffers(plan, dev, max_code_len=32)
    losses = [loss(a, c, w_o)]
    for t in range(T):
        # users: gradient at the current model (Algorithm 1 line 7)
        g_t[:, :d] = a_t[None, :] * (w_t[None, :] - c_t)
        g_o = a[None, :] * (w_o[None, :] - c)
        gu.assert_bits_equal(g_t[:, :d].cpu().numpy(), g_o, f"gradients, iteration {t}")
        # bias per user and layer from the corrected gradient (host rule of the workloads)
        v = g_o + np.float32(gamma) * m_o
        bias = np.zeros((U, nseg), np.int32)
        off = 0
        for k, n in enumerate(seg_len):
            bias[:, k] = [syn.bias_for_max(np.abs(v[u, off:off + n]).max(), E) for u in range(U)]
            off += n
        plan.set_bias(bias)
        # lines 8-10 for all users, then lines 13-14 at the PS
        buf.status.zero_()
        B.co3_encode(plan, books, g_t, m_t, m_t, gamma, buf, mode=B.BOOK_EMPIRICAL)
        B.co3_ps_aggregate(plan, books, buf, None, model=w_t, eta=eta)
        torch.cuda.synchronize()
        enc = oround.encode_round(g_o, m_o, gamma, E, M, seg_len, seg_book, bias, False, None)
        sym, _ = oround.ps_round(enc, E, M, seg_len, seg_book, bias, False)
        w_o = orc.model_update(sym, seg_len, bias, E, M, eta, w_o)
        m_o = enc["m_new"]
        gu.assert_bits_equal(m_t[:, :d].cpu().numpy(), m_o, f"memory, iteration {t}")
        for u, wds in enumerate(enc["words"]):
            gu.assert_bits_equal(buf.words[u, :wds.size].cpu().numpy().view(np.uint32), wds, f"stream {u}, iteration {t}")
        gu.assert_bits_equal(w_t.cpu().numpy(), w_o, f"model, iteration {t}")
        w_plain = (w_plain.astype(np.float64) - eta * np.mean(a[None, :].astype(np.float64) *
                                                                (w_plain.astype(np.float64)[None, :] - c), axis=0)).astype(np.float32)
        losses.append(loss(a, c, w_o))
    assert losses[-1] < 0.5 * losses[0]
    gap = float(np.sqrt(np.mean((w_o.astype(np.float64) - w_plain) ** 2)))
    test_closed_loop_matches_the_oracle.gaps[gamma] = gap
    if len(test_closed_loop_matches_the_oracle.gaps) == 2:
        g0, g9 = test_closed_loop_matches_the_oracle.gaps[0.0], test_closed_loop_matches_the_oracle.gaps[0.9]
        assert g9 < g0, (g0, g9)               # error feedback brings the compressed run closer


test_closed_loop_matches_the_oracle.gaps = {}
