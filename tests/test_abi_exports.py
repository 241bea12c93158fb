"""CPU-side checks of the C-ABI library: it loads and exports every function the
header declares.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rnnt_beam.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rnnt_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_core_calls():
    names = declared_functions()
    for n in ("rnnt_beam_create", "rnnt_beam_decode", "rnnt_beam_results", "rnnt_lm_create"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2506_00185_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2506_00185_amd import build
        build.build()
    lib = ctypes.CDLL(binding.library_path())
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == declared_functions()


def test_binding_fails_loudly_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import synth_inputs as S
    from paper_2506_00185_amd import BeamDecoder, RnntBeamError
    c = S.config(1)
    with pytest.raises(RnntBeamError):
        BeamDecoder(c, S.make_weights(c))


def test_config_struct_matches_header_field_order():
    from paper_2506_00185_amd.binding import _Config
    text = open(HEADER).read()
    body = re.search(r"typedef struct \{(.*?)\} rnnt_config_t;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        names = decl.split(None, 1)[1]
        for n in names.split(","):
            fields.append(re.sub(r"\[.*\]", "", n).strip())
    assert fields == [f[0] for f in _Config._fields_]
