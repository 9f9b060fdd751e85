#!/usr/bin/env python3
"""CO3 codec benchmark on one MI355X.

One "step" = one whole CO3 round for all U users: co3_encode (error correction, fp conversion,
memory update, Huffman coding into the chunked bitstream) followed by co3_ps_aggregate (decode all
streams, dequantize, average).  Inputs are synthetic GenNorm gradients resident in
HBM before the timed region; the memory m is carried from step to step and the gradients rotate
through a small pre-generated pool.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--book empirical|model]

--book model (default, the headline): the paper's operating mode.  The Huffman code is designed
once, off the timed path, from the GenNorm model of g + gamma m (Sec. IV-A (ii)) and held, as the
paper holds its fitted parameters for several epochs; the user side is then the library's
single-sweep encoder (symbols never reach HBM).  The design of that code (device moment fit, mixture
weights, Huffman build) is timed on its own and reported as "model_refresh".  --book empirical: every round builds its code on
the device from that round's pooled symbol histogram (quantize sweep, code build, coding sweep).
Whichever is not the headline is measured too and reported under "other_book".
"""
import argparse
import dataclasses
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # vector lane-operations per second (non-packed), in 10^12


def counter_figures(workload):
    """Per-kernel figures from rocprofv3 --pmc runs (HBM bytes per launch, vector instructions per element, LDS
    bank-conflict share), read from profiles/<workload>_counters.json.  That file records the digest of the library
    sources it was measured on; for any other build the figures are not quoted (None)."""
    from paper_2204_08211_amd import build as hip_build
    path = os.path.join(ROOT, "profiles", f"{workload}_counters.json")
    if not os.path.exists(path):
        return None, "no counter file for this workload"
    with open(path) as fh:
        c = json.load(fh)
    if c.get("source_digest") != hip_build.source_digest():
        return None, "counter file was measured on other sources"
    return c, None


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--workload", default="cfg3", help="cfg1..cfg5 of BASELINE.json (default: the one the target is quoted on)")
    p.add_argument("--book", default="model", choices=["empirical", "model"])
    p.add_argument("--gamma", type=float, default=None,
                   help="memory-decay coefficient (default: the workload's; the others it names are reported under gamma_sweep)")
    p.add_argument("--no-gamma-sweep", action="store_true", help="skip the workload's other memory-decay coefficients")
    p.add_argument("--model-encoder", default="sweep", choices=["sweep", "three"],
                   help="encoder for --book model: the single-sweep kernel (symbols never stored) or the three-step one")
    p.add_argument("--stochastic", action="store_true",
                   help="stochastic fp conversion (dithered Q) instead of the closest representative; a new seed per step")
    p.add_argument("--row-align", type=int, default=32,
                   help="users' rows of g and m start at multiples of this many elements (the library asks for a multiple "
                        "of 4; 32 = 128 bytes keeps every 16 KB chunk on cache-line boundaries)")
    p.add_argument("--sweep-hist", action="store_true",
                   help="the single-sweep encoder also counts the symbols (histogram output with a held code)")
    p.add_argument("--format", default=None, metavar="E,M",
                   help="run the workload in the format [1, E, M] instead of its own; an alphabet of more than 8 bits "
                        "takes the library's 16-bit-symbol kernels")
    p.add_argument("--per-user-books", action="store_true", help="every user its own code tables instead of pooled ones")
    p.add_argument("--graph", action="store_true",
                   help="replay the step from HIP graphs (one per gradient set of the pool) instead of launching eagerly")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-other-book", action="store_true", help="measure only the headline code-table mode")
    p.add_argument("--ignore-status", action="store_true", help="tuning runs only: do not stop on codec error counters")
    p.add_argument("--pool", type=int, default=2, help="pre-generated gradient sets to rotate through")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="run plain device copies of a known size instead (reference for rocprofv3 --pmc byte counters)")
    return p.parse_args()


def calibrate_copy():
    """Five plain copies of 1 GiB: what FETCH_SIZE / WRITE_SIZE read for 2^30 bytes in, 2^30 out."""
    import torch
    n = 1 << 28
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy": True, "bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n, "copies": 5}))


def cpu_baseline(w, it0_host, bias_host):
    """The oracle as it stands, single thread, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import co3_round as oround
    g = it0_host
    U, d = g.shape
    m = np.zeros_like(g)
    tm = {}
    seg_book = list(range(len(w.seg_len))) if w.nseg > 1 else [0]
    t0 = time.perf_counter()
    enc = oround.encode_round(g, m, w.gamma, w.E, w.M, w.seg_len, seg_book, bias_host[:U], False, None, tm)
    t_enc = time.perf_counter() - t0
    oround.ps_round(enc, w.E, w.M, w.seg_len, seg_book, bias_host[:U], False, tm)
    t_all = time.perf_counter() - t0
    return dict(value=U * d / t_all / 1e9, unit="GElem/s", cores=1, kind="oracle",
                sample=f"users 0..{U - 1} of {w.U} at full d={d}, one round (encode+decode+average), "
                       f"{t_all:.1f} s; encode alone {U * d / t_enc / 1e6:.2f} MElem/s",
                stages_s={k: round(v, 3) for k, v in tm.items()})


ENC_KERNELS = ["k_zero_u64", "k_quantize", "k_reduce_hist", "k_build_books", "k_chunk_bits", "k_scan_chunks", "k_pack",
               "k_encode_fused"]


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (users are a batch on that GPU); --gpus {a.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)
    if a.calibrate_copy:
        calibrate_copy()
        return
    import numpy as np
    import torch
    import co3_synth as syn
    from paper_2204_08211_amd import binding as B

    w = syn.WORKLOADS[a.workload]
    if a.per_user_books:
        w = dataclasses.replace(w, per_user_books=True)
    wide = False
    if a.format:
        E, M = (int(x) for x in a.format.split(","))
        w = dataclasses.replace(w, E=E, M=M, name=f"{w.name} in [1,{E},{M}]")
        wide = 1 + E + M > 8
    sweep_gammas = [] if (a.gamma is not None or a.no_gamma_sweep) else [x for x in w.gammas if x != w.gamma]
    if a.gamma is not None:
        w = dataclasses.replace(w, gamma=a.gamma)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    U, d = w.U, w.d
    stride = (d + a.row_align - 1) // a.row_align * a.row_align   # elements between users' rows (the library asks for a multiple of 4)
    nseg = len(w.seg_len)
    seg_book = list(range(nseg)) if nseg > 1 else [0]
    seg_off = np.concatenate([[0], np.cumsum(w.seg_len)]).astype(np.int64)
    elems = U * d

    # inputs: pool of gradient sets, memory starts at zero (m_0 = 0)
    pool = []
    for it in range(a.pool):
        g = torch.zeros((U, stride), dtype=torch.float32, device=dev)
        for u in range(U):
            syn.user_gradient_torch(w, it, u, dev, out=g[u, :d])
        pool.append(g)
    m = torch.zeros((U, stride), dtype=torch.float32, device=dev)

    # exponent bias: the workload's rule on iteration 0 (v = g since m_0 = 0), per user and segment;
    # held for the whole run like the paper holds b_t for several epochs
    mx = np.zeros((U, nseg))
    for k in range(nseg):
        mx[:, k] = pool[0][:, seg_off[k]:seg_off[k + 1]].abs().amax(dim=1).cpu().numpy()
    bias = syn.bias_table(mx, w.E)

    plan = B.Plan(w.E, w.M, U, d, bias, seg_len=w.seg_len, seg_book=seg_book, per_user_books=w.per_user_books)
    buf = B.RoundBuffers(plan, dev, max_code_len=16)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    counter = [0]

    def measure(books, mode, label, single_sweep=False, gamma=None):
        gamma = w.gamma if gamma is None else gamma

        def eager_step(idx):
            B.co3_encode(plan, books, pool[idx], m, m, gamma, buf, mode=mode, single_sweep=single_sweep,
                         stochastic_seed=(1000 + counter[0]) if a.stochastic else None,
                         single_sweep_hist=single_sweep and a.sweep_hist)
            B.co3_ps_aggregate(plan, books, buf, out)

        graphs = []
        if a.graph:   # one captured step per gradient set; the seed of a stochastic run is then fixed per set
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for idx in range(a.pool):
                    eager_step(idx)
                    side.synchronize()
                    gr = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gr, stream=side):
                        eager_step(idx)
                    graphs.append(gr)
            torch.cuda.synchronize()

        def step():
            idx = counter[0] % a.pool
            if graphs:
                graphs[idx].replay()
            else:
                eager_step(idx)
            counter[0] += 1
        for _ in range(a.warmup):
            step()
        torch.cuda.synchronize()
        buf.status.zero_()
        torch.cuda.synchronize()
        B.profile_begin()
        ev0 = torch.cuda.Event(enable_timing=True)
        ev1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(a.steps):
            step()
        ev1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        dev_ms = ev0.elapsed_time(ev1)
        kt = B.profile_end()
        ksteps = a.steps
        if graphs:   # replays launch nothing through the library: per-kernel times from a few eager steps
            ksteps = 5
            B.profile_begin()
            for i in range(ksteps):
                eager_step(i % a.pool)
            kt = B.profile_end()
        status = buf.status.cpu().numpy().tolist()
        if (status[B.STAT_CAPACITY] or status[B.STAT_NOCODE] or status[B.STAT_CORRUPT] or status[B.STAT_CODELEN]
                or status[B.STAT_STALLED]) \
                and not a.ignore_status:
            print(f"bench.py: codec reported errors ({label}): status={status}", file=sys.stderr)
            sys.exit(1)
        ms_per_step = max(wall_ms, dev_ms) / a.steps
        payload = buf.payload_bits.cpu().numpy().astype(np.float64)
        container_bits = float(buf.chunk_offset[:, -1].cpu().numpy().astype(np.float64).sum()) \
            + 64.0 * U * (plan.num_chunks + 1) + 16.0 * U * plan.num_chunks * 64
        bpe = float(payload.sum()) / elems
        per_launch = {k: v[0] / v[1] for k, v in kt.items()}
        enc_ms = sum(kt[k][0] for k in ENC_KERNELS if k in kt) / ksteps
        dec_ms = kt["k_aggregate"][0] / ksteps
        enc_alg = (12.0 + bpe / 8.0) * elems   # read g, read m, write m', write codewords
        return dict(ms_per_step=ms_per_step, kt=kt, per_launch=per_launch, bpe=bpe, status=status,
                    summary={
                        "book": label, "ms_per_step": round(ms_per_step, 4),
                        "gelem_s": round(elems / (ms_per_step * 1e-3) / 1e9, 3),
                        "encode": {"ms": round(enc_ms, 4), "gelem_s": round(elems / enc_ms / 1e6, 2),
                                   "hbm_frac_algorithmic": round(enc_alg / (enc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                   "bytes_per_element_algorithmic": round(12.0 + bpe / 8.0, 3)},
                        "decode_average": {"ms": round(dec_ms, 4), "gelem_s": round(elems / dec_ms / 1e6, 2),
                                           "hbm_frac_algorithmic": round((bpe / 8.0 + 4.0 / U) * elems / (dec_ms * 1e-3)
                                                                         / 1e9 / HBM_PEAK_GBS, 4)},
                        "bits_per_element": {"payload": round(bpe, 4), "container": round(container_bits / elems, 4)},
                        "kernel_ms_per_launch": {k: round(v, 4) for k, v in per_launch.items()},
                    })

    refresh = {}

    def model_books(gamma=None, refresh=refresh):
        """Code tables of the GenNorm model of v = g + gamma m, all on the device and off the timed path (the
        paper holds the fitted parameters for several epochs): moment fit per user and layer, mixture weights
        per table, Huffman build.  Its cost is reported as "model_refresh"."""
        gamma = w.gamma if gamma is None else gamma
        books = B.co3_build_codebook(w.E, w.M, plan.num_books, None)
        ws = torch.empty(int(B.lib().co3_plan_fit_workspace_bytes(plan.handle)), dtype=torch.uint8, device=dev)
        params = torch.zeros((U, nseg, 4), dtype=torch.float64, device=dev)
        weights = torch.zeros((plan.num_books, plan.A), dtype=torch.int64, device=dev)
        for rep in range(3):   # the last repetition is the one timed
            torch.cuda.synchronize()
            if rep == 2:
                B.profile_begin()
            t0 = time.perf_counter()
            B.co3_gennorm_fit(plan, pool[0], m, gamma, params=params, workspace=ws)
            # the model's own exponent bias (eq. (exp bias)) is computed and timed but not installed: the
            # workload prescribes the bias rule "top binade covers max|v|"
            model_bias, _ = B.co3_model_bias_device(plan, params, install=False)
            B.co3_model_weights_device(plan, params, weights=weights)
            B.co3_build_codebook_device(books, weights, buf.status)
            torch.cuda.synchronize()
            if rep == 2:
                kt = B.profile_end()
                refresh.update(ms=round((time.perf_counter() - t0) * 1e3, 4),
                               kernel_ms={k: round(v[0] / v[1], 4) for k, v in kt.items()},
                               moments_sweep_hbm_frac=round(8.0 * elems / (kt["k_moments"][0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
        p = params.cpu().numpy()
        refresh.update(beta_fit_range=[round(float(p[:, :, 2].min()), 4), round(float(p[:, :, 2].max()), 4)],
                       model_bias_minus_workload_bias=[int(x) for x in
                                                       (model_bias.cpu().numpy() - bias).ravel()[:16]])
        return books

    def settle(gamma):
        """m_0 = 0, then enough rounds for the memory to reach its steady state under this decay coefficient
        (a clamped element's remainder drains by a factor gamma per round) before a model of v is fitted."""
        m.zero_()
        n = int(min(400, math.ceil(4.0 / max(1.0 - gamma, 1e-2))))
        for _ in range(n):
            B.co3_encode(plan, emp_books, pool[counter[0] % a.pool], m, m, gamma, buf, mode=B.BOOK_EMPIRICAL)
            counter[0] += 1
        torch.cuda.synchronize()
        return n

    runs = {}
    model_code = None
    order = ["empirical", "model"] if a.book == "empirical" else ["model", "empirical"]
    if a.no_other_book:
        order = order[:1]
    emp_books = B.co3_build_codebook(w.E, w.M, plan.num_books, None)
    settle_rounds = settle(w.gamma)
    for label in order:
        if label == "empirical":
            runs[label] = measure(emp_books, B.BOOK_EMPIRICAL, "empirical")
        else:
            model_code = model_books()
            runs[label] = measure(model_code, B.BOOK_FIXED, "model", single_sweep=a.model_encoder == "sweep")

    head = runs[a.book]
    kt, per_launch, bpe = head["kt"], head["per_launch"], head["bpe"]
    sb = 2.0 if wide else 1.0             # bytes of a stored symbol
    alg_bytes = {  # algorithmic bytes per element of each kernel
        "k_quantize": 12.0 + sb,          # read g, read m, write m', write symbol
        "k_chunk_bits": sb,               # read symbol
        "k_pack": sb + bpe / 8.0,         # read symbol, write codewords
        "k_aggregate": bpe / 8.0 + 4.0 / U,
        "k_encode_fused": 12.0 + bpe / 8.0,   # read g, read m, write m', write codewords
    }
    dom = max(per_launch, key=lambda k: kt[k][0])
    ach = alg_bytes.get(dom, 0.0) * elems / (per_launch[dom] * 1e-3) / 1e9
    counters, counters_note = counter_figures(a.workload + (f"_fp1{w.E}{w.M}" if a.format else ""))
    ck = (counters or {}).get("kernels", {})
    roof = dict(bound="hbm", kernel=dom, achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                frac=round(ach / HBM_PEAK_GBS, 4), traffic=ck.get(dom, {}).get("traffic_bytes"),
                bytes_per_element=alg_bytes.get(dom), avg_launch_ms=round(per_launch[dom], 4))
    if counters_note:
        roof["traffic_note"] = counters_note
    if dom == "k_aggregate":
        roof["note"] = "the decoder is bound by its serial table-lookup chain (integer ALU / LDS latency), not by HBM"
    roof["kernels"] = {k: {"achieved_GBs": round(alg_bytes[k] * elems / (per_launch[k] * 1e-3) / 1e9, 1),
                           "frac": round(alg_bytes[k] * elems / (per_launch[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                       for k in alg_bytes if k in per_launch}
    for k, entry in roof["kernels"].items():
        # what the counters say about the binding unit: vector instructions per element (SQ_INSTS_VALU x 64 /
        # elements) and the share of the launch the vector ALUs would need for them at the nominal issue rate
        # (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz); this is an occupancy of the unit, not a roofline fraction
        if k in ck and ck[k].get("valu_per_element") is not None:
            vpe = ck[k]["valu_per_element"]
            entry.update(valu_per_element=vpe, lds_bank_conflict_share=ck[k].get("lds_conflict_share"),
                         valu_busy=round(vpe * elems / (per_launch[k] * 1e-3) / 1e12 / ALU_PEAK_TOPS, 4))
    if "k_aggregate" in roof["kernels"]:
        roof["kernels"]["k_aggregate"]["gsymbols_s"] = round(elems / (per_launch["k_aggregate"] * 1e-3) / 1e9, 2)
    res = {
        "metric": "CO3 encode+decode GElem/s and % HBM roofline on 1 MI355X; bits/element",
        "value": head["summary"]["gelem_s"], "unit": "GElem/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": head["summary"]["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32+u16" if wide else "f32+u8",
        "data": "synthetic GenNorm gradients (seeded torch device generator; recipe in co3_synth.py)",
        "config": {"workload": f"{w.name}: U={U} d={d} [1,{w.E},{w.M}] gamma={w.gamma} nseg={nseg} book={a.book} "
                               f"({'per-user' if w.per_user_books else 'pooled over users'})",
                   "elements_per_step": elems},
        "roofline": roof,
        "encode": head["summary"]["encode"],
        "decode_average": head["summary"]["decode_average"],
        "bits_per_element": head["summary"]["bits_per_element"],
        "kernel_ms_per_launch": head["summary"]["kernel_ms_per_launch"],
        "status": head["status"],
    }
    if refresh:
        res["model_refresh"] = refresh
    # co3_decode on its own (symbols of every user back to HBM), streams of the last measured round
    last_books = model_code if order[-1] == "model" else emp_books
    sym_out = torch.empty(plan.symbols_bytes, dtype=torch.uint8, device=dev)
    B.co3_decode(plan, last_books, buf, symbols=sym_out)
    torch.cuda.synchronize()
    B.profile_begin()
    for _ in range(3):
        B.co3_decode(plan, last_books, buf, symbols=sym_out)
    kd = B.profile_end()
    res["decode_symbols"] = {"ms": round(kd["k_decode"][0] / kd["k_decode"][1], 4),
                             "gelem_s": round(elems / (kd["k_decode"][0] / kd["k_decode"][1]) / 1e6, 2)}
    del sym_out
    others = [runs[k]["summary"] for k in runs if k != a.book]
    if others:
        res["other_book"] = others[0]
    res["settle_rounds"] = settle_rounds
    res["source_digest"] = __import__("paper_2204_08211_amd.build", fromlist=["x"]).source_digest()
    # the workload's other memory-decay coefficients: the same two measurements from a memory settled under each
    if sweep_gammas:
        sweep = {}
        for gm in sweep_gammas:
            n = settle(gm)
            mb = model_books(gm, refresh={})
            r_model = measure(mb, B.BOOK_FIXED, "model", single_sweep=a.model_encoder == "sweep", gamma=gm)
            r_emp = measure(emp_books, B.BOOK_EMPIRICAL, "empirical", gamma=gm)
            sweep[str(gm)] = {
                "settle_rounds": n,
                "model": {k: r_model["summary"][k] for k in ("ms_per_step", "gelem_s", "encode", "decode_average", "bits_per_element")},
                "empirical": {k: r_emp["summary"][k] for k in ("ms_per_step", "gelem_s", "encode", "decode_average", "bits_per_element")},
                "clamped_per_step": round(r_model["status"][B.STAT_CLAMPED] / a.steps, 1),
                "encode_fused_hbm_frac": round((12.0 + r_model["bpe"] / 8.0) * elems / (r_model["per_launch"]["k_encode_fused"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                if "k_encode_fused" in r_model["per_launch"] else None,
            }
            del mb
        res["gamma_sweep"] = sweep
    res["clamped_per_step"] = round(head["status"][B.STAT_CLAMPED] / a.steps, 1)
    if not a.no_cpu_baseline:
        ns = min(U, max(1, int(200e6 // d)))   # about 10-15 s of single-thread oracle work
        host = pool[0][:ns, :d].cpu().numpy()
        res["cpu_baseline"] = cpu_baseline(w, host, bias)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
