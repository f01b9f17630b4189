"""CPU-side checks of the C-ABI library: it loads and exports every symbol the header declares."""
import ctypes
import os
import re

import paper_2101_05600_amd as m

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ctcbs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ctcbs_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(os.path.join(ROOT, "paper_2101_05600_amd", "libctcbs.so")):
        m.build()
    L = m.lib()
    names = declared_symbols()
    assert set(names) == set(m.EXPORTS), (names, m.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_config_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "ctcbs.h")).read()
    body = text[text.index("typedef struct {", text.index("Search configuration")):]
    body = body[:body.index("} ctcbs_config_t;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|float|void\*)\s+([a-z_0-9]+);", body)
    assert fields == [f[0] for f in m.Config._fields_]
    out = text[text.index("typedef struct {", text.index("Views of one step")):]
    out = out[:out.index("} ctcbs_step_out_t;")]
    out = re.sub(r"/\*.*?\*/", "", out, flags=re.S)
    fields = re.findall(r"\b(?:const\s+)?(?:int32_t|float|uint8_t)\s*\*?\s*([a-z_0-9]+);", out)
    assert fields == [f[0] for f in m.StepOut._fields_]


def test_strerror_needs_no_gpu():
    assert m.ctcbs_strerror(0) == "ok"
    assert "capacity" in m.ctcbs_strerror(m.ECAP)
    assert "unknown" in m.ctcbs_strerror(-99)
