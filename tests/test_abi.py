"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before touching
the device."""
import ctypes as C
import os
import subprocess
import re

import pytest

from paper_2605_22269_amd import binding as mk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good_cfg(**kw):
    base = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, tokens_per_frame=49, frames_per_segment=8,
                superpatches_per_frame=4, dtype=mk.MUKV_F32, keep_ratio=0.25, alpha=0.7, causal=1, score_layer=-1,
                max_frames=64, max_chunk_frames=8, max_questions=2, device_id=0, att_path=0, batch_chunks=0,
                refine_margin=-1.0, overlap_copy=0)
    base.update(kw)
    return mk.mukv_config(**base)


def test_header_symbols_are_exported():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("mukv.h", "mukv_measure.h"))
    declared = set(re.findall(r"^(?:int|const char \*)\s*(mukv_\w+)\(", text, flags=re.M))
    assert declared == set(mk.EXPORTS)
    lib = mk.load()
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_covers_every_status():
    lib = mk.load()
    seen = {lib.mukv_strerror(s).decode() for s in range(0, -6, -1)}
    assert len(seen) == 6 and "unknown status" not in seen
    assert lib.mukv_strerror(-99).decode() == "unknown status"


@pytest.mark.parametrize("field,value,status", [
    ("n_layers", 0, mk.MUKV_ERR_INVALID_ARG),
    ("keep_ratio", 0.0, mk.MUKV_ERR_INVALID_ARG),
    ("keep_ratio", 1.5, mk.MUKV_ERR_INVALID_ARG),
    ("keep_ratio", 0.01, mk.MUKV_ERR_INVALID_ARG),      # kappa would be 0
    ("alpha", -0.1, mk.MUKV_ERR_INVALID_ARG),
    ("dtype", 7, mk.MUKV_ERR_INVALID_ARG),
    ("n_q_heads", 5, mk.MUKV_ERR_SHAPE),                 # not a multiple of n_kv_heads
    ("superpatches_per_frame", 50, mk.MUKV_ERR_SHAPE),
    ("score_layer", 2, mk.MUKV_ERR_SHAPE),
    ("head_dim", 48, mk.MUKV_ERR_UNSUPPORTED),
    ("head_dim", 256, mk.MUKV_ERR_UNSUPPORTED),
    ("tokens_per_frame", 8193, mk.MUKV_ERR_UNSUPPORTED),
    ("max_frames", 0, mk.MUKV_ERR_INVALID_ARG),
    ("batch_chunks", -1, mk.MUKV_ERR_INVALID_ARG),
    ("batch_chunks", 65, mk.MUKV_ERR_UNSUPPORTED),
    ("overlap_copy", 2, mk.MUKV_ERR_INVALID_ARG),
])
def test_create_rejects_bad_config_on_the_host(field, value, status):
    lib = mk.load()
    cfg = good_cfg(**{field: value})
    h = C.c_void_p()
    assert lib.mukv_create(C.byref(cfg), C.byref(h)) == status
    assert not h.value


def test_null_arguments():
    lib = mk.load()
    cfg = good_cfg()
    assert lib.mukv_create(None, C.byref(C.c_void_p())) == mk.MUKV_ERR_INVALID_ARG
    assert lib.mukv_create(C.byref(cfg), None) == mk.MUKV_ERR_INVALID_ARG
    assert lib.mukv_destroy(None) == mk.MUKV_OK
    assert lib.mukv_reset(None) == mk.MUKV_ERR_INVALID_ARG
    assert lib.mukv_flush(None) == mk.MUKV_ERR_INVALID_ARG
    st = mk.mukv_strides(1, 1, 1)
    assert lib.mukv_compress_chunk(None, None, None, C.byref(st), None, None, None, 1, None, None) == mk.MUKV_ERR_INVALID_ARG
    prm = mk.mukv_retrieve_params(0, 1, 1, 0, -1, 0, 0.3)
    assert lib.mukv_retrieve(None, None, None, 1, C.byref(prm), None, None, None, None, None) == mk.MUKV_ERR_INVALID_ARG
    assert lib.mukv_gather_kv(None, None, 1, 1, 0, None, None, None, None) == mk.MUKV_ERR_INVALID_ARG
    assert lib.mukv_get_state(None, None) == mk.MUKV_ERR_INVALID_ARG


def test_binding_struct_sizes_match_header_layout(tmp_path):
    # 8 int32 | 2 double | 8 int32 | double | int32 (+ tail padding)
    assert C.sizeof(mk.mukv_config) == 8 * 4 + 2 * 8 + 8 * 4 + 8 + 8
    assert C.sizeof(mk.mukv_retrieve_params) == 6 * 4 + 8
    assert C.sizeof(mk.mukv_strides) == 24
    assert C.sizeof(mk.mukv_state) == 4 * 8 + 2 * 4 + 12 * 8 + 8
    # and against the header itself, through the C compiler: sizes and every field offset
    structs = {"mukv_config": mk.mukv_config, "mukv_retrieve_params": mk.mukv_retrieve_params,
               "mukv_strides": mk.mukv_strides, "mukv_state": mk.mukv_state,
               "mukv_signals_out": mk.mukv_signals_out, "mukv_profile": mk.mukv_profile}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "mukv.h"', '#include "mukv_measure.h"', 'int main(void) {']
    for name, st in structs.items():
        lines.append(f'printf("{name} %zu\\n", sizeof({name}));')
        for fname, _ in st._fields_:
            lines.append(f'printf("{name}.{fname} %zu\\n", offsetof({name}, {fname}));')
    lines += ['return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for name, st in structs.items():
        assert int(out[name]) == C.sizeof(st), name
        for fname, _ in st._fields_:
            assert int(out[f"{name}.{fname}"]) == getattr(st, fname).offset, f"{name}.{fname}"
