#!/usr/bin/env python3
"""Algorithm 1 as a closed loop through the library, on a synthetic strongly convex objective:
U users hold f_u(w) = 1/2 sum_i a_i (w_i - c_{u,i})^2; every iteration each user sends the CO3
encoding of its gradient at the PS model, the PS decodes, averages and updates the model.  The
GenNorm model, the exponent bias (eq. (exp bias)) and the Huffman code are refreshed on the device
every `--refresh` iterations and held in between, as the paper holds them for several epochs
(Sec. VI).  The users' gradients carry seeded noise.  Prints, per format and memory-decay
coefficient gamma, the excess loss after T iterations, its ratio to that of uncompressed SGD on
the same noise, and the bits per element sent (--real-scale: with the real-valued scale of eq. (exp bias)
instead of the integer bias) (Sec. VI discusses the
choice of gamma; Sec. IV-A (iii) the role of the memory).

With --theorem the loop runs in the setting of Theorem 1 of the appendix instead: memory without decay
(gamma = 1), step size 1 / sqrt(T), the averaged iterate (1/T) sum_t w_t, for a sweep of T.  Printed per format
and T: the excess loss of the averaged iterate, the right-hand side of the theorem's bound with its three terms
(mu = min a_i, L = max a_i, G^2 the largest squared gradient norm met, all for the objective summed over
coordinates), and the mean squared memory per element in units of the fitted GenNorm scale squared beside the
2^(4 - 2 mant) + 0.3 of the lemma on the quantization error (stated there for a unit-scale gradient).

    python -m paper_2204_08211_amd.examples.closed_loop [--d 1000000] [--users 8] [--iters 200]
    python -m paper_2204_08211_amd.examples.closed_loop --theorem [--d 200000] [--users 8]
"""
import argparse

import numpy as np
import torch

from paper_2204_08211_amd import binding as B


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--d", type=int, default=1_000_000)
    p.add_argument("--users", type=int, default=8)
    p.add_argument("--iters", type=int, default=200)
    p.add_argument("--refresh", type=int, default=10)
    p.add_argument("--noise", type=float, default=0.1, help="standard deviation of the noise added to every user gradient")
    p.add_argument("--eta", type=float, default=0.2)
    p.add_argument("--stochastic", action="store_true")
    p.add_argument("--real-scale", action="store_true",
                   help="eq. (exp bias) with real b: bias and gain of every user from co3_model_scale_device at each refresh")
    p.add_argument("--theorem", action="store_true", help="sweep T in the setting of Theorem 1 (gamma 1, eta 1/sqrt(T), averaged iterate)")
    a = p.parse_args()
    dev = torch.device("cuda:0")
    U, d, T = a.users, a.d, a.iters
    gen = torch.Generator(device=dev); gen.manual_seed(2204_08211)
    coef = torch.rand(d, device=dev, generator=gen) * 1.5 + 0.5                         # a_i in [0.5, 2]
    centre = torch.randn(1, d, device=dev, generator=gen) + 0.3 * torch.randn(U, d, device=dev, generator=gen)
    stride = (d + 3) // 4 * 4

    def loss(w):
        return float((0.5 * coef.double() * (w.double()[None, :] - centre.double()) ** 2).mean())

    def gradients(w, t, out):
        """Stochastic gradients of the users at w: the exact ones plus seeded noise (the same for every run)."""
        ng = torch.Generator(device=dev); ng.manual_seed(1000 + t)
        out[:, :d] = coef[None, :] * (w[None, :] - centre) + a.noise * torch.randn(U, d, device=dev, generator=ng)

    g = torch.zeros((U, stride), device=dev)
    if a.theorem:
        theorem_sweep(a, dev, coef, centre, loss, gradients, g)
        return
    w_plain = torch.zeros(d, device=dev)
    for t in range(T):
        gradients(w_plain, t, g)
        w_plain -= a.eta * g[:, :d].mean(dim=0)
    l_star = loss((coef[None, :] * centre).sum(0) / (U * coef))      # minimiser: the mean centre
    l_plain = loss(w_plain)
    l_0 = loss(torch.zeros(d, device=dev))
    print(f"U={U} d={d} T={T} eta={a.eta} noise={a.noise} refresh every {a.refresh}: loss at w=0 {l_0:.5f}, optimum {l_star:.5f}, "
          f"uncompressed after T: excess {l_plain - l_star:.3e}")
    print(f"{'format':>10} {'gamma':>6} {'excess loss':>12} {'/ uncompressed excess':>22} {'bit/element':>12} {'clamped':>10}")
    for E, M in ((2, 1), (3, 0), (4, 3), (5, 2)):
        for gamma in (0.0, 0.5, 0.7, 0.9, 1.0):
            plan = B.Plan(E, M, U, d, [[(1 << (E - 1)) - 1]] * U)
            books = B.co3_build_codebook(E, M, plan.num_books, None)
            buf = B.RoundBuffers(plan, dev, max_code_len=64)
            w = torch.zeros(d, device=dev)
            m = torch.zeros((U, stride), device=dev)
            bits = 0.0
            for t in range(T):
                gradients(w, t, g)
                if t % a.refresh == 0:                                  # fit -> bias -> weights -> code, all on the device
                    params = B.co3_gennorm_fit(plan, g, m, gamma)
                    if a.real_scale:                                    # the argmins over real b, on the device as well
                        B.co3_model_scale_device(plan, params, install=True)
                    else:
                        B.co3_model_bias_device(plan, params, install=True)
                    B.co3_build_codebook_device(books, B.co3_model_weights_device(plan, params), buf.status)
                B.co3_encode(plan, books, g, m, m, gamma, buf, mode=B.BOOK_FIXED, single_sweep=True,
                             stochastic_seed=(t + 1) if a.stochastic else None)
                B.co3_ps_aggregate(plan, books, buf, None, model=w, eta=a.eta)
                bits += float(buf.payload_bits.sum().item())
            st = buf.status.cpu().numpy()
            assert st[B.STAT_NOCODE] == 0 and st[B.STAT_CORRUPT] == 0 and st[B.STAT_STALLED] == 0 and st[B.STAT_CAPACITY] == 0
            ex = loss(w) - l_star
            print(f"{'[1,%d,%d]' % (E, M):>10} {gamma:6.2f} {ex:12.3e} {ex / max(l_plain - l_star, 1e-300):22.3f} "
                  f"{bits / (T * U * d):12.3f} {int(st[B.STAT_CLAMPED]):10d}")


def theorem_sweep(a, dev, coef, centre, loss, gradients, g):
    """Theorem 1 (appendix): E L(w_bar_T) - L* <= (|w_0 - w*|^2 + G^2) / sqrt(T) + (mu + 2 L)(2^(4 - 2 mant) + 0.3) / T."""
    U, d = a.users, a.d
    stride = g.shape[1]
    mean_centre = (coef[None, :] * centre).sum(0) / (U * coef)
    l_star = loss(mean_centre) * d                                # the objective summed over coordinates
    mu, L = float(coef.min()), float(coef.max())
    dist0 = float((mean_centre.double() ** 2).sum())               # w_0 = 0
    print(f"U={U} d={d} noise={a.noise} mu={mu:.3f} L={L:.3f} |w0-w*|^2={dist0:.4e}, gamma=1, eta=1/sqrt(T), refresh every {a.refresh}")
    print(f"{'format':>10} {'T':>6} {'excess loss':>12} {'bound':>12} {'= dist/sqrtT':>13} {'+ G^2/sqrtT':>12} {'+ quant/T':>10} "
          f"{'E m^2/alpha^2':>14} {'lemma':>8} {'bit/element':>12}")
    for E, M in ((2, 1), (3, 0), (4, 3), (5, 2)):
        for T in (16, 64, 256, 1024):
            eta = 1.0 / np.sqrt(T)
            plan = B.Plan(E, M, U, d, [[(1 << (E - 1)) - 1]] * U)
            books = B.co3_build_codebook(E, M, plan.num_books, None)
            buf = B.RoundBuffers(plan, dev, max_code_len=64)
            w = torch.zeros(d, device=dev)
            w_bar = torch.zeros(d, device=dev, dtype=torch.float64)
            m = torch.zeros((U, stride), device=dev)
            bits = 0.0; g2 = 0.0; mem = 0.0
            for t in range(T):
                w_bar += w.double() / T
                g2 = max(g2, float(((coef * (w - mean_centre)).double() ** 2).sum()))
                gradients(w, t, g)
                if t % a.refresh == 0:
                    params = B.co3_gennorm_fit(plan, g, m, 1.0)
                    B.co3_model_bias_device(plan, params, install=True)
                    B.co3_build_codebook_device(books, B.co3_model_weights_device(plan, params), buf.status)
                    alpha2 = float((params[..., 1].double() ** 2).mean())
                B.co3_encode(plan, books, g, m, m, 1.0, buf, mode=B.BOOK_FIXED, single_sweep=True)
                B.co3_ps_aggregate(plan, books, buf, None, model=w, eta=eta)
                bits += float(buf.payload_bits.sum().item())
                mem += float((m[:, :d].double() ** 2).mean()) / alpha2 / T
            st = buf.status.cpu().numpy()
            assert st[B.STAT_NOCODE] == 0 and st[B.STAT_CORRUPT] == 0 and st[B.STAT_STALLED] == 0 and st[B.STAT_CAPACITY] == 0
            ex = loss(w_bar.float()) * d - l_star
            lemma = 2.0 ** (4 - 2 * M) + 0.3
            terms = (dist0 / np.sqrt(T), g2 / np.sqrt(T), (mu + 2 * L) * lemma / T)
            print(f"{'[1,%d,%d]' % (E, M):>10} {T:6d} {ex:12.4e} {sum(terms):12.4e} {terms[0]:13.4e} {terms[1]:12.4e} {terms[2]:10.3e} "
                  f"{mem:14.4f} {lemma:8.3f} {bits / (T * U * d):12.3f}")


if __name__ == "__main__":
    main()
