"""CPU-side checks of the C-ABI library: it loads and exports every function the
header declares, fails loudly without a GPU, and its host logic (the block -> work item
mapping of the per-step launches) is right.  No GPU call is made here."""
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


@pytest.mark.parametrize("a_tiles,a_m,b_begin,b_end,b_m", [(33, 4, 44, 80, 4), (20, 4, 0, 44, 4), (33, 8, 12, 80, 8),
                                                           (64, 8, 0, 0, 0), (1, 1, 0, 0, 0), (3, 2, 5, 6, 7),
                                                           (0, 0, 0, 80, 1), (9, 16, 79, 80, 12)])
def test_block_map_covers_every_item_once_on_the_xcd_of_its_tile(a_tiles, a_m, b_begin, b_end, b_m):
    """Host logic of the per-step launches: every (role, n-tile, m-tile) item exactly once, on a block whose index
    is congruent to the n-tile modulo 8 (one weight slice, one L2), grid a multiple of 8 and no larger than
    8 x the fullest XCD needs."""
    from paper_2506_00185_amd.binding import block_map
    grid, role, nt, mt = block_map(a_tiles, a_m, b_begin, b_end, b_m)
    assert grid % 8 == 0
    want = {(0, n, m) for n in range(a_tiles) for m in range(a_m)} | {(1, n, m) for n in range(b_begin, b_end)
                                                                      for m in range(b_m)}
    got = [(int(r), int(n), int(m)) for r, n, m in zip(role, nt, mt) if r >= 0]
    assert len(got) == len(set(got)) == len(want) and set(got) == want
    for bid, (r, n) in enumerate(zip(role, nt)):
        if r >= 0:
            assert n % 8 == bid % 8
    per_xcd = [sum(1 for (r, n, m) in want if n % 8 == x) for x in range(8)]
    assert grid == 8 * max(per_xcd)
    # within an XCD the items of role 0 come before those of role 1 (what the selection tail's producers rely on)
    for x in range(8):
        roles = [int(role[b]) for b in range(x, grid, 8) if role[b] >= 0]
        assert roles == sorted(roles)
