"""Host-side checks of libst3.so that need no GPU: exported symbols, schedule helpers,
closed-form accounting, and argument validation (error paths enqueue nothing)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from conftest import ROOT, read_table
from oracle import st3_oracle as orc
from paper_2412_20105_amd import binding as st3
from paper_2412_20105_amd import pipeline
from workloads import WORKLOADS


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "st3.h")).read()
    return sorted(set(re.findall(r"ST3_EXPORT[^;(]*?\b(st3_\w+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 16 and set(names) == set(st3.EXPORTED)
    lib = st3.lib()
    for n in names:
        assert getattr(lib, n) is not None
    assert st3.st3_version() >> 8 >= 1
    assert lib.st3_status_string(0) == b"ok"
    assert b"workspace" in lib.st3_status_string(3)


def test_diagnostic_block_is_inert_without_the_environment_switch():
    """A process that loads the library without ST3_DEBUG=1 cannot flip its process-wide switches."""
    import subprocess
    import sys
    code = ("import ctypes as C; L = C.CDLL(%r); L.st3_debug_enabled.restype = C.c_int; "
            "print(L.st3_debug_enabled(), L.st3_debug_set_attend_tile(8), L.st3_debug_set_prefill_path(1), "
            "L.st3_profile_enable(4), L.st3_profile_read(None, None, None, None))" % st3.LIB_PATH)
    env = {k: v for k, v in os.environ.items() if k != "ST3_DEBUG"}
    out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, check=True).stdout.split()
    assert out == ["0", "2", "2", "2", "2"]                 # ST3_ERR_UNSUPPORTED from every setter
    env["ST3_DEBUG"] = "1"
    out = subprocess.run([sys.executable, "-c", code.replace("L.st3_profile_enable(4), L.st3_profile_read(None, None, None, None)", "0, 0")],
                         env=env, capture_output=True, text=True, check=True).stdout.split()
    assert out == ["1", "0", "0", "0", "0"]
    assert st3.st3_debug_enabled()                          # this process: switched on by conftest.py


def test_schedule_helpers_match_oracle_on_all_workloads():
    for w in WORKLOADS.values():
        assert np.array_equal(np.array(pipeline.keep_table_for(w)), orc.schedule_for(w)), w.name


def test_pvtp_helper_reproduces_printed_tables():
    for L, S, R, P, Cbp in (tuple(map(int, r)) for r in read_table("pvtp_stride_tables.txt")):
        keep = st3.st3_schedule_pvtp(L, 576, 3, S, P, R)
        assert keep == orc.keep_pvtp(L, 576, S, P, R)
        assert keep[-1] == 576 * Cbp // 10000 and keep[2] == 576 and keep[3] == 288
        # an exactly divisible count makes the last-layer ratio itself visible
        assert st3.st3_schedule_pvtp(L, 10000, 3, S, P, R)[-1] == Cbp


def test_anneal_helper_variants():
    keep0 = [600, 100, 7, 0]
    for kind, code, param in (("cos", st3.ST3_ANNEAL_COS, 90), ("linear", st3.ST3_ANNEAL_LINEAR, 50),
                              ("exp", st3.ST3_ANNEAL_EXP, 20), ("drop", st3.ST3_ANNEAL_DROP, 4)):
        got = np.array(st3.st3_schedule_anneal(code, param, 120, keep0))
        assert np.array_equal(got, orc.keep_anneal(keep0, 120, kind, param)), kind
    none = st3.st3_schedule_anneal(st3.ST3_ANNEAL_NONE, 1.0, 3, [5, 2])
    assert none == [[5] * 4, [2] * 4]


def test_kv_bytes_closed_form():
    assert st3.st3_kv_bytes(16, 32, 128, st3.ST3_BF16, [632] * 32) == orc.kv_bytes(16, 32, 128, 2, [632] * 32)
    assert st3.st3_kv_bytes(16, 40, 128, st3.ST3_BF16, [631] * 40) / 2 ** 30 == pytest.approx(7.70, abs=0.005)
    assert st3.st3_kv_bytes(1, 4, 64, st3.ST3_F32, [64, 32]) == 2 * 4 * 64 * 4 * 96


def test_workspace_bytes_monotone_and_rejects_bad_shapes():
    sh = st3.make_shape(2, 4, 64, st3.ST3_F32)
    a = st3.st3_workspace_bytes(sh, 100, 64, 1)
    b = st3.st3_workspace_bytes(sh, 1000, 64, 1)
    c = st3.st3_workspace_bytes(sh, 1000, 640, 4)
    assert 0 < a <= b <= c
    assert st3.st3_workspace_bytes(st3.make_shape(2, 4, 96, st3.ST3_F32), 100, 64, 1) == 0
    assert st3.st3_workspace_bytes(st3.make_shape(0, 4, 64, st3.ST3_F32), 100, 64, 1) == 0


def test_argument_errors_are_reported_before_any_launch():
    lib = st3.lib()
    sh = st3.make_shape(1, 4, 64, st3.ST3_F32)
    bad = st3.make_shape(1, 4, 80, st3.ST3_F32)
    fake = 0x1000                                  # aligned, never dereferenced on an error path
    kv = st3.KvLayer(fake, fake, 4 * 128 * 64, 128 * 64, 64, 128)
    seg = st3.Segments(8, 64, 100, fake, fake)
    # unsupported head_dim
    assert lib.st3_decode_attention(C.byref(bad), fake, C.byref(kv), C.byref(seg), fake, None, 0, fake, 1 << 30,
                                    None) == st3.ST3_ERR_UNSUPPORTED
    # null q
    assert lib.st3_decode_attention(C.byref(sh), None, C.byref(kv), C.byref(seg), fake, None, 0, fake, 1 << 30,
                                    None) == st3.ST3_ERR_INVALID_ARG
    # workspace too small
    assert lib.st3_decode_attention(C.byref(sh), fake, C.byref(kv), C.byref(seg), fake, None, 0, fake, 16,
                                    None) == st3.ST3_ERR_WORKSPACE_TOO_SMALL
    # lengths beyond capacity
    seg_big = st3.Segments(8, 64, 129, fake, fake)
    assert lib.st3_decode_attention(C.byref(sh), fake, C.byref(kv), C.byref(seg_big), fake, None, 0, fake, 1 << 30,
                                    None) == st3.ST3_ERR_INVALID_ARG
    # append into a full cache
    seg_full = st3.Segments(8, 64, 128, fake, fake)
    assert lib.st3_kv_append(C.byref(sh), C.byref(kv), C.byref(seg_full), fake, fake, None) == st3.ST3_ERR_INVALID_ARG
    # misaligned K pointer
    kv_mis = st3.KvLayer(fake + 4, fake, 4 * 128 * 64, 128 * 64, 64, 128)
    assert lib.st3_kv_append(C.byref(sh), C.byref(kv_mis), C.byref(seg), fake, fake, None) == st3.ST3_ERR_INVALID_ARG
    # top-k with k > n, and n beyond the supported size
    assert lib.st3_select_topk(fake, 10, None, 0, 1, None, 10, 11, None, fake, 11, None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_select_topk(fake, 20000, None, 0, 1, None, 20000, 5, None, fake, 5, None) == st3.ST3_ERR_UNSUPPORTED
    # compaction with a row size that is not a multiple of 4
    assert lib.st3_compact_rows(fake, 1, 1, 0, 0, 8, 6, fake, 4, 4, 8, 0, None) == st3.ST3_ERR_INVALID_ARG
    # select-compact with a bad mode / negative count
    assert lib.st3_select_compact_layer(C.byref(sh), C.byref(kv), C.byref(seg), fake, fake, 64, 10, 7, fake, 1 << 30,
                                        None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_select_compact_layer(C.byref(sh), C.byref(kv), C.byref(seg), fake, fake, 64, -1, 0, fake, 1 << 30,
                                        None) == st3.ST3_ERR_INVALID_ARG
    # prefill: segment layout outside the sequence, window too large
    t4 = st3.Tensor4(fake, 4 * 128 * 64, 128 * 64, 64)
    assert lib.st3_prefill_attention(C.byref(sh), C.byref(t4), C.byref(t4), C.byref(t4), 100, 50, 60, 1, C.byref(t4),
                                     None, 0, fake, 1 << 30, None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_prefill_attention(C.byref(sh), C.byref(t4), C.byref(t4), C.byref(t4), 100, 8, 64, 17, C.byref(t4),
                                     None, 0, fake, 1 << 30, None) == st3.ST3_ERR_INVALID_ARG
    # whole-step call: a lazy layer that wants the mass while its source does not ask for one is refused
    ws_bytes = st3.st3_workspace_bytes(sh, 128, 64, 1)
    steps = (st3.LayerStep * 2)()
    for i, s in enumerate(steps):
        s.kv = st3.KvLayer(None if i else fake, fake, 4 * 128 * 64, 128 * 64, 64, 128)
        s.seg = st3.Segments(8, 64, 100, fake, fake)
        s.score_col, s.id_col, s.col_stride = fake + 0x1000 * i, fake + 0x100000 + 0x1000 * i, 64
        s.keep_after, s.inherit_from = 60, -1 if i == 0 else 0
        s.q, s.k_new, s.v_new, s.out = fake, fake, fake, fake
        s.vis_mass, s.mass_stride = (None, 0) if i == 0 else (fake, 64)
        s.workspace, s.workspace_bytes = fake + 0x10000000 * (i + 1), ws_bytes
    assert lib.st3_decode_step(C.byref(sh), 2, steps, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    steps[1].inherit_from = 1                       # a layer cannot inherit from itself or from a later layer
    assert lib.st3_decode_step(C.byref(sh), 2, steps, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    # the step in two parts: the same refusals, layer by layer and for the plans; a layer index outside the array
    assert lib.st3_decode_layer_attend(C.byref(sh), 2, steps, 1, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_decode_layer_attend(C.byref(sh), 2, steps, 2, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_decode_layer_attend(C.byref(sh), 2, steps, -1, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_decode_layer_attend(C.byref(bad), 2, steps, 0, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_UNSUPPORTED
    assert lib.st3_decode_plans(C.byref(sh), 2, steps, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_decode_plans(C.byref(sh), 0, steps, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    steps[1].inherit_from = -1
    steps[1].kv = steps[0].kv
    assert lib.st3_decode_plans(C.byref(sh), 2, steps, 7, None) == st3.ST3_ERR_INVALID_ARG            # no such mode
    steps[0].seg = st3.Segments(8, 64, 128, fake, fake)                                                 # no room for the appended row
    assert lib.st3_decode_layer_attend(C.byref(sh), 2, steps, 0, st3.ST3_HOLE_FILL, None) == st3.ST3_ERR_INVALID_ARG
    # the allocation-free decode attention: null query; a shape whose scratch does not fit the library's array
    assert lib.st3_decode_attention_noalloc(C.byref(sh), None, C.byref(kv), C.byref(seg), fake, None, 0,
                                            None) == st3.ST3_ERR_INVALID_ARG
    big = st3.make_shape(64, 40, 128, st3.ST3_BF16)
    cap = 4096
    kv_big = st3.KvLayer(fake, fake, 40 * cap * 128, cap * 128, 128, cap)
    seg_b = st3.Segments(8, 64, 100, fake, fake)
    assert st3.st3_workspace_bytes(big, cap, 64, 1) > st3.ST3_NOALLOC_SCRATCH_BYTES
    assert lib.st3_decode_attention_noalloc(C.byref(big), fake, C.byref(kv_big), C.byref(seg_b), fake, None, 0,
                                            None) == st3.ST3_ERR_WORKSPACE_TOO_SMALL
    # schedule helpers
    assert lib.st3_schedule_pvtp(32, 576, 3, 0, 5000, 100, fake) == st3.ST3_ERR_INVALID_ARG
    assert lib.st3_schedule_anneal(0, C.c_double(0.0), 4, fake, 2, fake) == st3.ST3_ERR_INVALID_ARG


def test_ctypes_structures_have_the_layout_the_c_header_declares(tmp_path):
    """Compiles a few lines of plain C against include/st3.h (also proving the header is valid C) and
    compares sizeof / offsetof of every structure with the ctypes mirror in the binding."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    structs = {"st3_attn_shape": st3.AttnShape, "st3_tensor4": st3.Tensor4, "st3_kv_layer": st3.KvLayer,
               "st3_segments": st3.Segments, "st3_gather_pair": st3.GatherPair, "st3_layer_step": st3.LayerStep}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "st3.h"', 'int main(void) {']
    for cname, ct in structs.items():
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in ct._fields_:
            lines.append(f'  printf("{cname}.{fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, ct in structs.items():
        assert int(got[cname]) == C.sizeof(ct), cname
        for fname, _ in ct._fields_:
            assert int(got[f"{cname}.{fname}"]) == getattr(ct, fname).offset, f"{cname}.{fname}"
    # enumerators the binding repeats as plain integers
    enums = {"ST3_KV_E4M3": st3.ST3_KV_E4M3, "ST3_E4M3": st3.ST3_E4M3, "ST3_HOLE_FILL": st3.ST3_HOLE_FILL,
             "ST3_BF16": st3.ST3_BF16, "ST3_ERR_WORKSPACE_TOO_SMALL": st3.ST3_ERR_WORKSPACE_TOO_SMALL,
             "ST3_ANNEAL_NONE": st3.ST3_ANNEAL_NONE, "ST3_MAX_GATHER": st3.ST3_MAX_GATHER}
    src2 = tmp_path / "enums.c"
    src2.write_text('#include <stdio.h>\n#include "st3.h"\nint main(void) {\n' +
                    "".join(f'  printf("{k} %d\\n", (int){k});\n' for k in enums) + "  return 0;\n}\n")
    exe2 = tmp_path / "enums"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src2), "-o", str(exe2)], check=True)
    got2 = dict(l.split() for l in subprocess.run([str(exe2)], check=True, capture_output=True, text=True).stdout.splitlines())
    for k, v in enums.items():
        assert int(got2[k]) == v, k
