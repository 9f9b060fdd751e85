#!/usr/bin/env python3
"""Turn rocprofv3 output of bench.py runs into the short summaries kept under profiles/.

Inputs (folders of CSV files that rocprofv3 wrote, plus the JSON line bench.py printed in the same run):

  --stats DIR   rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o <workload> -- python3 bench.py ...
                (DIR/<workload>_kernel_stats.csv, DIR/bench.json = bench.py's stdout of that run)
  --pmc DIR     four counter runs, one counter each (rocprofv3 does not split counters over passes):
                rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -o bench_FETCH_SIZE -- python3 bench.py ...
                rocprofv3 --pmc WRITE_SIZE ...                          -o bench_WRITE_SIZE ...
                and the same two on plain device copies of 2^30 bytes (bench.py --calibrate-copy), -o copy_FETCH_SIZE /
                copy_WRITE_SIZE: what the counters read for a known number of bytes gives bytes per count
  --sq DIR      two runs of at most 8 SQ counters each, -o set1 / set2 (instruction mix, LDS bank conflicts, waits)

Outputs in --out: <workload>_kernel_stats.md, <workload>_hbm_traffic.md, <workload>_sq_counters.md and
<workload>_counters.json.  The JSON carries the digest of the library sources (paper_2204_08211_amd.build.
source_digest) it was measured on; bench.py quotes its figures only for a build with the same digest.
"""
import argparse
import collections
import csv
import json
import os

from paper_2204_08211_amd import build as hip_build


# kernels whose name in the library's event timing (co3_profile_end) differs from the function's
TIMING_NAME = {"k_pack_chunk": "k_pack", "k_chunk_bits_hist": "k_chunk_bits",
               # the kernels for 16-bit symbols are timed under the names of the steps they take
               "k_quantize_wide": "k_quantize", "k_reduce_hist_wide": "k_reduce_hist", "k_build_books_wide": "k_build_books",
               "k_chunk_bits_wide": "k_chunk_bits", "k_pack_wide": "k_pack", "k_aggregate_wide": "k_aggregate",
               "k_decode_wide": "k_decode", "k_zero_wide": "k_zero_u64"}


def short_name(kernel):
    """'void co3::k_encode_fused<false, 4>(...)' -> ('k_encode_fused', 'co3::k_encode_fused<false, 4>'); the first is
    the name bench.py reports the kernel under."""
    full = kernel.split("(")[0].replace("void ", "").strip()
    k = full.replace("co3::", "").split("<")[0]
    return TIMING_NAME.get(k, k), full


def per_kernel_average(path):
    """{short name: {counter: average per launch}}, {short name: full name}, {short name: launches} of a
    rocprofv3 counter_collection CSV."""
    vals = collections.defaultdict(lambda: collections.defaultdict(list))
    names = {}
    for r in csv.DictReader(open(path)):
        if "co3::" not in r["Kernel_Name"] and "copyBuffer" not in r["Kernel_Name"]:
            continue
        k, full = short_name(r["Kernel_Name"])
        names[k] = full
        vals[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
    avg = {k: {c: sum(v) / len(v) for c, v in cs.items()} for k, cs in vals.items()}
    calls = {k: max(len(v) for v in cs.values()) for k, cs in vals.items()}
    return avg, names, calls


def main():
    p = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    p.add_argument("--workload", default="cfg3")
    p.add_argument("--stats")
    p.add_argument("--pmc")
    p.add_argument("--sq")
    p.add_argument("--out", default="profiles")
    p.add_argument("--bench-args", default="--no-cpu-baseline", help="the bench.py arguments of the runs, for the record")
    a = p.parse_args()
    wl = a.workload
    os.makedirs(a.out, exist_ok=True)
    counters = {"source_digest": hip_build.source_digest(), "workload": wl, "kernels": {}}
    bj = None

    if a.stats:
        bj = json.loads(open(os.path.join(a.stats, "bench.json")).read().strip().splitlines()[-1])
        rows = list(csv.DictReader(open(os.path.join(a.stats, f"{wl}_kernel_stats.csv"))))
        out = [f"# rocprofv3 kernel statistics: libco3 kernels, workload {bj['config']['workload']}\n",
               "Command (on the MI355X box, from /tmp with TMPDIR=/tmp):\n",
               f"    rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -o {wl} -- python3 bench.py {a.bench_args}",
               f"    python3 -m paper_2204_08211_amd.profile_summary --workload {wl} --stats <dir> ...\n",
               "bench.py designs the model code on the device (k_moments, k_fit_params, k_model_bias_*, k_model_weights, "
               "k_build_books), measures the headline (model code held: " +
               ("k_zero_fused, k_encode_fused, k_aggregate" if "k_encode_fused" in bj["kernel_ms_per_launch"] else
                "for 16-bit symbols the three coding steps with the symbols in the workspace, then k_aggregate_wide") +
               "), the workload's other memory-decay coefficients, then the path with the code rebuilt every round (k_zero_u64, "
               "k_quantize, k_reduce_hist, k_build_books, k_chunk_bits, k_scan_chunks, k_pack, k_aggregate; the *_wide kernels "
               "for 16-bit symbols) and co3_decode (k_decode).  Times in microseconds.\n",
               "| kernel | calls | average | min | max | share of all GPU time (incl. input generation) |", "|---|---|---|---|---|---|"]
        for r in rows:
            if "co3::" not in r["Name"]:
                continue
            _, full = short_name(r["Name"])
            out.append(f"| {full} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | "
                       f"{float(r['MaxNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} % |")
        out.append("\nbench.py's own HIP-event timing in the same run (ms per launch):\n")
        out.append("    headline (model code held): " + json.dumps(bj["kernel_ms_per_launch"]))
        if "other_book" in bj:
            out.append("    code rebuilt every round:   " + json.dumps(bj["other_book"]["kernel_ms_per_launch"]))
        if "model_refresh" in bj:
            out.append("    model refresh:              " + json.dumps(bj["model_refresh"]["kernel_ms"]))
        e = bj["encode"]
        out.append(f"\nHeadline step {bj['ms_per_step']} ms, {bj['value']} GElem/s; encode {e['ms']} ms = "
                   f"{e['hbm_frac_algorithmic'] * 100:.1f} % of 8 TB/s on {e['bytes_per_element_algorithmic']} B/element; "
                   f"decode + average {bj['decode_average']['ms']} ms.")
        if "other_book" in bj:
            ob = bj["other_book"]
            out.append(f"Code rebuilt every round: step {ob['ms_per_step']} ms, {ob['gelem_s']} GElem/s; encode "
                       f"{ob['encode']['ms']} ms = {ob['encode']['hbm_frac_algorithmic'] * 100:.1f} %; decode + average "
                       f"{ob['decode_average']['ms']} ms.")
        out.append(f"\nLibrary sources: digest {counters['source_digest']}.")
        open(os.path.join(a.out, f"{wl}_kernel_stats.md"), "w").write("\n".join(out) + "\n")

    elems = bj["config"]["elements_per_step"] if bj else None

    if a.pmc:
        F, names, calls = per_kernel_average(os.path.join(a.pmc, "bench_FETCH_SIZE_counter_collection.csv"))
        W, _, _ = per_kernel_average(os.path.join(a.pmc, "bench_WRITE_SIZE_counter_collection.csv"))
        cfa, _, _ = per_kernel_average(os.path.join(a.pmc, "copy_FETCH_SIZE_counter_collection.csv"))
        cwa, _, _ = per_kernel_average(os.path.join(a.pmc, "copy_WRITE_SIZE_counter_collection.csv"))
        cf = cfa["__amd_rocclr_copyBuffer"]["FETCH_SIZE"]
        cw = cwa["__amd_rocclr_copyBuffer"]["WRITE_SIZE"]
        ff, fw = 1048576.0 / cf, 1048576.0 / cw          # KiB per count
        lines = [f"# HBM traffic of the libco3 kernels, workload {wl}\n",
                 "Two counter runs (one counter each) and the same two on plain device copies of 2^30 bytes, on the MI355X box "
                 "from /tmp with TMPDIR=/tmp:\n"]
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            lines.append(f"    rocprofv3 --pmc {c} --output-format csv -d <dir> -o bench_{c} -- python3 bench.py --steps 3 --warmup 1 {a.bench_args}")
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            lines.append(f"    rocprofv3 --pmc {c} --output-format csv -d <dir> -o copy_{c} -- python3 bench.py --calibrate-copy")
        lines.append(f"    python3 -m paper_2204_08211_amd.profile_summary --workload {wl} --pmc <dir> ...")
        lines.append(f"\nCalibration: a copy that reads and writes 1 048 576 KiB shows FETCH_SIZE = {cf:.0f} and WRITE_SIZE = {cw:.0f}: "
                     f"bytes = FETCH_SIZE x {ff:.3f} KiB, WRITE_SIZE x {fw:.3f} KiB.\n")
        alg = {}
        if bj:
            bpe = bj["bits_per_element"]["payload"]
            d = elems // int(bj["config"]["workload"].split("U=")[1].split()[0])
            stream = elems * bpe / 8
            sb = 2 if bj.get("dtype", "").endswith("u16") else 1   # bytes of a stored symbol
            alg = {"k_encode_fused": (8 * elems, 4 * elems + stream), "k_quantize": (8 * elems, (4 + sb) * elems),
                   "k_chunk_bits": (sb * elems if sb == 2 else 0, 0),   # (the byte path sizes chunks from their counts)
                   "k_pack": (sb * elems, stream), "k_aggregate": (stream, 4 * d),
                   "k_decode": (stream, sb * elems), "k_moments": (8 * elems, 0)}
            lines.append(f"Averages per launch; MB = 10^6 bytes; payload {bpe:.3f} bit/element; {elems} elements per launch.  "
                         "Algorithmic bytes: g and m read, m' written, the bitstream written (encoders); symbols written "
                         "(k_quantize) or read (k_pack); the bitstream read and the average written (k_aggregate).\n")
        lines.append("| kernel | launches | FETCH_SIZE | WRITE_SIZE | read MB | written MB | algorithmic read MB | algorithmic written MB | traffic / algorithmic |")
        lines.append("|---|---|---|---|---|---|---|---|---|")
        for k in sorted(F):
            if k.startswith("__amd"):
                continue
            f = F[k].get("FETCH_SIZE", 0.0)
            w = W.get(k, {}).get("WRITE_SIZE", 0.0)
            rb, wb = f * ff * 1024, w * fw * 1024
            counters["kernels"].setdefault(k, {})["traffic_bytes"] = round(rb + wb)
            counters["kernels"][k]["traffic_read_bytes"] = round(rb)
            counters["kernels"][k]["traffic_written_bytes"] = round(wb)
            if k in alg and sum(alg[k]) > 0:
                ar, aw = alg[k]
                lines.append(f"| {names[k]} | {calls[k]} | {f:.1f} | {w:.1f} | {rb / 1e6:.1f} | {wb / 1e6:.1f} | {ar / 1e6:.1f} | {aw / 1e6:.1f} | "
                             f"{(rb + wb) / (ar + aw):.3f} |")
            else:
                lines.append(f"| {names[k]} | {calls[k]} | {f:.1f} | {w:.1f} | {rb / 1e6:.1f} | {wb / 1e6:.1f} |  |  |  |")
        lines.append(f"\nLibrary sources: digest {counters['source_digest']}.")
        open(os.path.join(a.out, f"{wl}_hbm_traffic.md"), "w").write("\n".join(lines) + "\n")

    if a.sq:
        A, names, _ = per_kernel_average(os.path.join(a.sq, "set1_counter_collection.csv"))
        B, _, _ = per_kernel_average(os.path.join(a.sq, "set2_counter_collection.csv"))
        ms = {}
        if bj:
            ms.update(bj.get("model_refresh", {}).get("kernel_ms", {}))
            ms.update(bj.get("other_book", {}).get("kernel_ms_per_launch", {}))
            ms.update(bj["kernel_ms_per_launch"])
            if "decode_symbols" in bj:
                ms["k_decode"] = bj["decode_symbols"]["ms"]
        set1 = "SQ_WAVES SQ_BUSY_CYCLES SQ_INSTS_VALU SQ_ACTIVE_INST_VALU SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT SQ_WAIT_INST_LDS SQ_ACTIVE_INST_LDS"
        set2 = "SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_ACTIVE_INST_ANY SQ_INSTS_SALU SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_LDS_IDX_ACTIVE"
        lines = [f"# SQ counters of the libco3 kernels, workload {wl}: instruction mix, LDS bank conflicts, waiting\n",
                 "Two counter runs (at most 8 SQ counters each), on the MI355X box from /tmp with TMPDIR=/tmp:\n",
                 f"    rocprofv3 --pmc {set1} --output-format csv -d <dir> -o set1 -- python3 bench.py --steps 3 --warmup 1 {a.bench_args}",
                 f"    rocprofv3 --pmc {set2} --output-format csv -d <dir> -o set2 -- python3 bench.py --steps 3 --warmup 1 {a.bench_args}",
                 f"    python3 -m paper_2204_08211_amd.profile_summary --workload {wl} --sq <dir> ...\n",
                 "Averages per launch, in millions (wavefront instructions; SQ_WAVE_CYCLES, SQ_WAIT_ANY and SQ_ACTIVE_INST_ANY in "
                 "units of four clocks summed over wavefronts).  Derived: VALU per element = SQ_INSTS_VALU x 64 / elements; "
                 "VALU busy = SQ_INSTS_VALU x 4 clocks / (1024 SIMDs x launch time x 2.4 GHz); LDS busy = SQ_LDS_IDX_ACTIVE / "
                 "(256 CUs x launch time x 2.4 GHz); conflict share = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE; waiting = "
                 "SQ_WAIT_ANY / SQ_WAVE_CYCLES (share of a resident wavefront's time spent in s_waitcnt).\n",
                 "| kernel | launch ms | waves | VALU | SALU | LDS | VMEM rd | VMEM wr | LDS_IDX_ACTIVE | LDS_BANK_CONFLICT | VALU per element | VALU busy | LDS busy | conflict share | waiting |",
                 "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
        for k in sorted(A):
            if k.startswith("__amd"):
                continue
            x, y = A[k], B.get(k, {})
            valu, idx, conf = x.get("SQ_INSTS_VALU", 0.0), y.get("SQ_LDS_IDX_ACTIVE", 0.0), x.get("SQ_LDS_BANK_CONFLICT", 0.0)
            if valu < 1e6:
                continue     # fill and scan kernels: nothing to read from these counters
            t = ms.get(k)
            vpe = valu * 64 / elems if elems else None
            share = conf / idx if idx else 0.0
            busy = valu * 4 / (1024 * t * 1e-3 * 2.4e9) if t else None
            lbusy = idx / (256 * t * 1e-3 * 2.4e9) if t else None
            wait = y.get("SQ_WAIT_ANY", 0.0) / y["SQ_WAVE_CYCLES"] if y.get("SQ_WAVE_CYCLES") else None
            counters["kernels"].setdefault(k, {}).update(
                valu_per_element=round(vpe, 2) if vpe is not None else None, lds_conflict_share=round(share, 3),
                wait_share=round(wait, 3) if wait is not None else None)
            pct = lambda v: f"{v * 100:.0f} %" if v is not None else ""
            lines.append(f"| {names[k]} | {t if t is not None else ''} | {x.get('SQ_WAVES', 0) / 1e6:.3f} | {valu / 1e6:.1f} | "
                         f"{y.get('SQ_INSTS_SALU', 0) / 1e6:.1f} | {x.get('SQ_INSTS_LDS', 0) / 1e6:.1f} | {y.get('SQ_INSTS_VMEM_RD', 0) / 1e6:.2f} | "
                         f"{y.get('SQ_INSTS_VMEM_WR', 0) / 1e6:.2f} | {idx / 1e6:.1f} | {conf / 1e6:.1f} | "
                         f"{vpe:.1f} | {pct(busy)} | {pct(lbusy)} | {pct(share)} | {pct(wait)} |")
        lines.append(f"\nLibrary sources: digest {counters['source_digest']}.")
        open(os.path.join(a.out, f"{wl}_sq_counters.md"), "w").write("\n".join(lines) + "\n")

    if a.pmc or a.sq:
        with open(os.path.join(a.out, f"{wl}_counters.json"), "w") as fh:
            json.dump(counters, fh, indent=1, sort_keys=True)
            fh.write("\n")
    print(json.dumps(counters, indent=1, sort_keys=True))


if __name__ == "__main__":
    main()
