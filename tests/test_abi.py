"""The C-ABI libraries load and export every symbol include/*.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="tango.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tango_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2308_00890_amd import build as b

    if b.is_stale():
        b.build()
    return ctypes.CDLL(b.LIB)


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert "tango_quantize" in names and "tango_qspmm_bwd" in names and len(names) >= 19
    for n in names:
        assert hasattr(lib, n), n


def test_benchaid_header_symbols_are_exported(lib):
    """The harness's measurement aids are a library and a header of their own; tango.h holds the method only."""
    from paper_2308_00890_amd import benchaid, build as b

    aid = ctypes.CDLL(b.AID_LIB)
    names = declared_symbols("tango_benchaid.h")
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["tango.h", "tango_benchaid.h"]
    assert names == sorted(benchaid.SIGNATURES) and len(names) == 5
    for n in names:
        assert hasattr(aid, n), n
        assert not hasattr(lib, n), "measurement aid exported by the method's library: " + n
        assert n not in declared_symbols()


def test_binding_lists_every_symbol():
    from paper_2308_00890_amd import binding

    assert sorted(binding.SIGNATURES) == declared_symbols()
    for n in declared_symbols():
        assert callable(getattr(binding, n)), n


def test_version_and_status_strings(lib):
    lib.tango_status_string.restype = ctypes.c_char_p
    assert lib.tango_version() >= 100
    assert lib.tango_status_string(0) == b"ok"
    for code in range(-6, 0):
        assert len(lib.tango_status_string(code)) > 3


def test_argument_validation_needs_no_gpu(lib):
    # validation happens on the host before any launch
    lib.tango_quantize.restype = ctypes.c_int
    rc = lib.tango_quantize(None, ctypes.c_size_t(8), 7, ctypes.c_uint64(0), ctypes.c_uint64(0), None, None, None, None,
                            ctypes.c_size_t(0), None)
    assert rc == -3  # bad rounding enum
    rc = lib.tango_quantize(None, ctypes.c_size_t(8), 0, ctypes.c_uint64(0), ctypes.c_uint64(0), None, None, None, None,
                            ctypes.c_size_t(0), None)
    assert rc == -1  # NULL tensors


def test_layer_struct_layouts_match_the_header(tmp_path):
    """The ctypes mirrors of tango_gat_layer / tango_gcn_layer / tango_graph have the C compiler's sizes and offsets."""
    import subprocess

    from paper_2308_00890_amd import binding

    src = tmp_path / "layout.c"
    fields = {
        "tango_graph": ["n_nodes", "n_edges", "in_ptr", "out_eid"],
        "tango_gat_layer": ["g", "slope", "seed", "H", "absmax_Hp", "alpha_q", "grad_out", "dalpha", "da_dst", "fused",
                            "row_lse", "absmax_alpha", "ws", "ws_bytes"],
        "tango_gcn_layer": ["g", "f_out", "seed", "w_q", "Hp", "grad_out", "dH", "ws", "ws_bytes", "w_q_src_order"],
        "tango_typed_layer": ["g_dst", "g_src", "n_types", "seed", "w_q", "Hp", "dH", "ws", "ws_bytes", "w_q_src_order"],
    }
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "tango.h"', "int main(void){"]
    for st, fs in fields.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (st, st))
        for f in fs:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (st, f, st, f))
    lines.append("return 0;}")
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = dict(l.split() for l in subprocess.check_output([str(exe)]).decode().splitlines())
    for st, fs in fields.items():
        cls = getattr(binding, st)
        assert int(out[st]) == ctypes.sizeof(cls), st
        for f in fs:
            assert int(out["%s.%s" % (st, f)]) == getattr(cls, f).offset, (st, f)
