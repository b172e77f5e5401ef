"""The C-ABI library loads and exports every symbol include/gbt.h declares
(no compute calls: this runs without a GPU)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_1806_11248_amd as g
    if not os.path.exists(g.LIB_PATH):
        from paper_1806_11248_amd import build
        build.build()
    return g.load()


def test_header_symbols_are_exported(lib):
    import paper_1806_11248_amd as g
    hdr = open(os.path.join(ROOT, "include", "gbt.h")).read()
    declared = sorted(set(re.findall(r"GBT_API[^;(]*?\b(gbt_\w+)\s*\(", hdr)))
    assert len(declared) >= 20
    assert sorted(g.SYMBOLS) == declared
    for s in declared:
        assert hasattr(lib, s), s


def test_host_only_calls(lib):
    import paper_1806_11248_amd as g
    assert lib.gbt_version().decode().startswith("libgbt")
    # Sec. 2.2: bit length of the largest symbol
    for mv, b in {0: 1, 1: 1, 15: 4, 63: 6, 255: 8, 256: 9, 65535: 16}.items():
        assert g.bits_for(mv) == b
    assert g.packed_words(10_000, 8, 4) * 4 == 40_004
    assert g.packed_words(115_000_000, 13, 8) == (115_000_000 * 13 * 8 + 31) // 32 + 1
    assert lib.gbt_grow_tree_workspace_bytes(1000, 8, 4, 16, 3) > 1000 * 16
    assert lib.gbt_grow_tree_workspace_bytes(1000, 8, 4, 16, 99) == 0     # unsupported depth
    assert lib.gbt_partition_workspace_bytes(10_000) >= 40_000
    # sparse rows: an even number of entries plus the slack that word-wise readers may touch
    assert lib.gbt_sparse_capacity(0) == 32 and lib.gbt_sparse_capacity(5) == 38 and lib.gbt_sparse_capacity(-1) == 0
    assert lib.gbt_grow_tree_sparse_workspace_bytes(1000, 5000, 50, 256, 8) > 2 * 5000 * 2
    # 76,800 global bin ids take 32-bit entries; more than 2^28 ids are no valid shape
    assert lib.gbt_grow_tree_sparse_workspace_bytes(1000, 5000, 300, 256, 8) > 2 * 5000 * 4
    assert lib.gbt_grow_tree_sparse_workspace_bytes(1000, 5000, 5000, 60_000, 8) == 0
    assert lib.gbt_sparse_entry_bytes(256, 256) == 2 and lib.gbt_sparse_entry_bytes(300, 256) == 4
    assert lib.gbt_sparse_entry_bytes(5000, 60_000) == 0 and lib.gbt_sparse_entry_bytes(0, 256) == 0
    # loss-guided growth keeps histograms for the nodes it expands ahead of their turn
    assert (lib.gbt_grow_tree_lossguide_workspace_bytes(1000, 8, 4, 16, 64)
            > lib.gbt_grow_tree_workspace_bytes(1000, 8, 4, 16, 6))
    assert lib.gbt_grow_tree_lossguide_workspace_bytes(1000, 8, 4, 16, 0) == 0
    # a null context is refused, not dereferenced
    assert lib.gbt_destroy(None) == g.binding.EINVAL
    assert lib.gbt_gradients(None, 0, None, None, 0, None) == g.binding.EINVAL


def test_struct_layouts_match_header():
    import ctypes as C
    import paper_1806_11248_amd as g
    assert C.sizeof(g.binding.Split) == 72
    assert C.sizeof(g.binding.Params) == 48
    assert C.sizeof(g.binding.Tree) == 8 + 11 * 8
    # four 8-byte arrays over GBT_PROF_CLASSES = 8 classes, four over GBT_PROF_LEVELS = 18 depths
    assert C.sizeof(g.binding.Profile) == 8 * (4 * len(g.binding.PROF_CLASSES) + 4 * g.binding.PROF_LEVELS) == 8 * (4 * 8 + 4 * 18)


def test_every_environment_switch_is_documented_in_the_header():
    """gbt_create reads GBT_TUNE_* switches; each has to be listed, with its default, in include/gbt.h."""
    import glob
    import re
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    read = set()
    for path in glob.glob(os.path.join(root, "paper_1806_11248_amd", "csrc", "*")):
        read |= set(re.findall(r'getenv\("([A-Z0-9_]+)"\)', open(path).read()))
    assert read, "no switches found: has the source moved?"
    header = open(os.path.join(root, "include", "gbt.h")).read()
    missing = sorted(v for v in read if not re.search(r"\b%s\b\s+\[" % v, header))
    assert not missing, f"undocumented environment switches: {missing}"
