"""The measurement helpers that run on the host: how rocprofv3's kernel names map to the names the library times its
steps under, the per-kernel averages of a counter file, and when bench.py quotes a counter file (CPU only)."""
import json
import os

import bench
from paper_2204_08211_amd import build as hip_build
from paper_2204_08211_amd import profile_summary as ps


def test_kernel_names_map_to_the_timed_steps():
    cases = {
        "void co3::k_encode_fused<false, 4, 5, false>(co3::Layout, float const*)": ("k_encode_fused", "co3::k_encode_fused<false, 4, 5, false>"),
        "co3::k_pack_chunk(co3::Layout)": ("k_pack", "co3::k_pack_chunk"),
        "co3::k_chunk_bits_hist(co3::Layout)": ("k_chunk_bits", "co3::k_chunk_bits_hist"),
        "void co3::k_quantize_wide<false, true>(co3::Layout)": ("k_quantize", "co3::k_quantize_wide<false, true>"),
        "void co3::k_aggregate_wide<false>(co3::Layout)": ("k_aggregate", "co3::k_aggregate_wide<false>"),
        "co3::k_decode_wide(co3::Layout)": ("k_decode", "co3::k_decode_wide"),
        "co3::k_zero_wide(unsigned long*, unsigned long)": ("k_zero_u64", "co3::k_zero_wide"),
        "co3::k_moments(co3::Layout)": ("k_moments", "co3::k_moments"),
    }
    for name, want in cases.items():
        assert ps.short_name(name) == want, name


def test_per_kernel_average_of_a_counter_file(tmp_path):
    path = tmp_path / "c.csv"
    rows = [("co3::k_pack_wide(co3::Layout)", "FETCH_SIZE", 10.0), ("co3::k_pack_wide(co3::Layout)", "FETCH_SIZE", 30.0),
            ("co3::k_pack_chunk(co3::Layout)", "FETCH_SIZE", 50.0), ("at::native::fill(float*)", "FETCH_SIZE", 999.0),
            ("__amd_rocclr_copyBuffer", "FETCH_SIZE", 7.0)]
    path.write_text("Kernel_Name,Counter_Name,Counter_Value\n" + "".join(f'"{k}",{c},{v}\n' for k, c, v in rows))
    avg, names, calls = ps.per_kernel_average(str(path))
    # both coders are timed as k_pack: their launches are averaged together; kernels of other libraries are left out
    assert avg["k_pack"]["FETCH_SIZE"] == 30.0 and calls["k_pack"] == 3
    assert avg["__amd_rocclr_copyBuffer"]["FETCH_SIZE"] == 7.0
    assert set(avg) == {"k_pack", "__amd_rocclr_copyBuffer"}


def test_counter_file_is_quoted_only_for_the_sources_it_was_measured_on(tmp_path, monkeypatch):
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    os.makedirs(tmp_path / "profiles")
    assert bench.counter_figures("cfgX") == (None, "no counter file for this workload")
    digest = hip_build.source_digest()
    (tmp_path / "profiles" / "cfgX_counters.json").write_text(json.dumps({"source_digest": digest, "kernels": {}}))
    got, note = bench.counter_figures("cfgX")
    assert note is None and got["source_digest"] == digest
    (tmp_path / "profiles" / "cfgX_counters.json").write_text(json.dumps({"source_digest": "0" * 64, "kernels": {}}))
    assert bench.counter_figures("cfgX") == (None, "counter file was measured on other sources")


def test_source_digest_covers_every_kernel_source_and_the_header():
    csrc = os.path.join(os.path.dirname(hip_build.__file__), "csrc")
    listed = set(hip_build.SOURCES)
    on_disk = {f for f in os.listdir(csrc) if f.endswith((".hip", ".cpp"))}
    assert listed == on_disk            # nothing is compiled that the digest does not read, and the reverse
    assert len(hip_build.source_digest()) == 64
