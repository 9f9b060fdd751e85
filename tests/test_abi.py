"""The C-ABI library loads and exports every symbol include/co3.h declares (no compute calls:
this runs without a GPU)."""
import ctypes
import os
import re
import subprocess

from paper_2204_08211_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "co3.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(co3_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert "co3_build_codebook" in names and "co3_encode" in names and "co3_decode" in names \
        and "co3_ps_aggregate" in names
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_status_strings():
    assert binding.status_string(0) == "CO3_OK" and binding.status_string(-4) == "CO3_ERR_CODELEN"


def test_struct_layouts_match_the_header(tmp_path):
    # compile a C program against include/co3.h that prints sizeof / offsetof, compare with ctypes
    structs = {"co3_segment": binding.Segment, "co3_encode_args": binding.EncodeArgs,
               "co3_decode_args": binding.DecodeArgs, "co3_aggregate_args": binding.AggregateArgs,
               "co3_format": binding.Format, "co3_gennorm_params": binding.GennormParams}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "co3.h"', 'int main(void){']
    for cname, st in structs.items():
        lines.append(f'printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in st._fields_:
            lines.append(f'printf("{cname}.{fname} %zu\\n", offsetof({cname}, {fname}));')
    lines.append("return 0;}")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, st in structs.items():
        assert int(out[cname]) == ctypes.sizeof(st), cname
        for fname, _ in st._fields_:
            assert int(out[f"{cname}.{fname}"]) == getattr(st, fname).offset, (cname, fname)


def test_host_side_argument_checks_need_no_gpu():
    L = binding.lib()
    out = ctypes.c_void_p()
    # exp_bits = 1 makes the exponent set empty; 1 + exp + mant > 12 is more than the widest alphabet provided for
    assert L.co3_plan_create(binding.Format(1, 2), 1, 10, 0, None, (ctypes.c_int32 * 1)(3), 0, ctypes.byref(out)) == binding.ERR_FORMAT
    assert L.co3_plan_create(binding.Format(6, 6), 1, 10, 0, None, (ctypes.c_int32 * 1)(3), 0, ctypes.byref(out)) == binding.ERR_FORMAT
    # bias outside the supported range
    assert L.co3_plan_create(binding.Format(4, 3), 1, 10, 0, None, (ctypes.c_int32 * 1)(200), 0, ctypes.byref(out)) == binding.ERR_FORMAT
    # segments that do not tile [0, d)
    segs = (binding.Segment * 2)(binding.Segment(0, 4, 0, 0), binding.Segment(5, 5, 0, 0))
    assert L.co3_plan_create(binding.Format(4, 3), 1, 10, 2, ctypes.cast(segs, ctypes.c_void_p),
                             (ctypes.c_int32 * 2)(3, 3), 0, ctypes.byref(out)) == binding.ERR_ARG
    assert L.co3_encode(None, None, None) == binding.ERR_ARG
    assert L.co3_plan_num_chunks(None) == 0
    # no users, too many users (they are a grid dimension)
    assert L.co3_plan_create(binding.Format(4, 3), 0, 10, 0, None, (ctypes.c_int32 * 1)(14), 0, ctypes.byref(out)) == binding.ERR_ARG
    assert L.co3_plan_create(binding.Format(4, 3), 70000, 10, 0, None, (ctypes.c_int32 * 1)(14), 0, ctypes.byref(out)) == binding.ERR_ARG
    # null arguments of the model routines; host model routines with impossible parameters
    assert L.co3_gennorm_fit(None, None, None, 0, 0.9, None, None, 0, None) == binding.ERR_ARG
    assert L.co3_model_weights_device(None, None, None, None) == binding.ERR_ARG
    assert L.co3_model_bias_device(None, None, None, None, None, 0, None) == binding.ERR_ARG
    assert L.co3_plan_set_bias_device(None, None, None) == binding.ERR_ARG
    b = ctypes.c_int32(0)
    e = ctypes.c_double(0.0)
    assert L.co3_bias_from_model(binding.Format(4, 3), 0.0, -1.0, 1.0, ctypes.byref(b), ctypes.byref(e)) == binding.ERR_ARG
    assert L.co3_bias_from_model(binding.Format(1, 3), 0.0, 1.0, 1.0, ctypes.byref(b), ctypes.byref(e)) == binding.ERR_FORMAT
    assert L.co3_plan_fit_workspace_bytes(None) == 0 and L.co3_plan_bias_workspace_bytes(None) == 0
