"""A whole round (co3_encode + co3_ps_aggregate) captured in a HIP graph and replayed (pytest -m gpu).
The library clears its counters with fill kernels, not memset nodes, so the sequence may be
captured; every replay, with fresh inputs written into the captured buffers and eager work and
synchronisations in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest

import co3_synth as syn
import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("single_sweep,E,M", [(False, 4, 3), (True, 4, 3), (False, 5, 5)])
def test_round_in_a_graph_equals_eager(single_sweep, E, M):
    # (5, 5): 16-bit symbols, the code rebuilt per round (the model code below is for alphabets of up to 8 bits)
    import torch
    from paper_2204_08211_amd import binding as B
    U, d = 4, 4096 * 11 + 321
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    stride = (d + 3) // 4 * 4
    bias0 = 16 if E == 4 else 24
    plan = B.Plan(E, M, U, d, [[bias0]] * U)
    # a model code (every producible symbol has a codeword) for the fixed mode; rebuilt per round otherwise
    books = B.co3_build_codebook(E, M, plan.num_books,
                                 B.co3_gennorm_weights(E, M, 16, 0.0, 5e-3, 1.0)[None, :] if single_sweep else None)
    buf = B.RoundBuffers(plan, dev, max_code_len=64)
    g = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    m = torch.zeros((U, stride), dtype=torch.float32, device=dev)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    mode = B.BOOK_FIXED if single_sweep else B.BOOK_EMPIRICAL

    def fresh(it):
        return torch.from_numpy(np.stack([syn.gennorm_numpy(rng, d, 1.0, 2e-3 * (1 + it)) for _ in range(U)])).to(dev)

    def step():   # the binding enqueues on torch's current stream
        B.co3_encode(plan, books, g, m, m, 0.9, buf, mode=mode, single_sweep=single_sweep)
        B.co3_ps_aggregate(plan, books, buf, out)

    g[:, :d] = fresh(0)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                              # warm-up on the capture stream
        side.synchronize()
        m.zero_()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    m_eager = torch.zeros_like(m)
    for it in range(4):
        g[:, :d] = fresh(it + 1)
        # eager reference on copies of the state the replay starts from
        m_ref = m.clone()
        buf_ref = B.RoundBuffers(plan, dev, max_code_len=64)
        out_ref = torch.zeros_like(out)
        B.co3_encode(plan, books, g, m_ref, m_ref, 0.9, buf_ref, mode=mode, single_sweep=single_sweep)
        B.co3_ps_aggregate(plan, books, buf_ref, out_ref)
        torch.cuda.synchronize()
        buf.words.zero_(); out.fill_(float("nan"))             # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(m, m_ref), f"memory, replay {it}"
        assert torch.equal(buf.chunk_offset, buf_ref.chunk_offset) and torch.equal(buf.sub_bits, buf_ref.sub_bits)
        assert torch.equal(buf.payload_bits, buf_ref.payload_bits)
        for u in range(U):
            nw = int(buf_ref.chunk_offset[u, -1].item()) // 32
            assert torch.equal(buf.words[u, :nw], buf_ref.words[u, :nw]), f"stream {u}, replay {it}"
        assert torch.equal(out, out_ref), f"average, replay {it}"
        if not single_sweep:
            assert torch.equal(buf.hist, buf_ref.hist)
    st = buf.status.cpu().numpy()
    assert st[B.STAT_NOCODE] == 0 and st[B.STAT_CORRUPT] == 0 and st[B.STAT_STALLED] == 0 and st[B.STAT_CAPACITY] == 0
