"""Host-side checks that need no GPU: the C-ABI library loads and exports what the header declares."""
import os
import re

import numpy as np

from paper_1809_00832_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "treelstm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_entry_point():
    names = declared_functions()
    assert "tl_create" in names and "tl_forward" in names and "tl_destroy" in names
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_error_strings():
    assert binding.tl_strerror(binding.TL_OK) == "ok"
    assert "malformed" in binding.tl_strerror(binding.TL_ESTRUCT)
    assert "progress" in binding.tl_strerror(binding.TL_ESTALL)


def test_config_struct_layout_matches_header():
    # 8 ints then 6 pointers, natural alignment
    assert binding.tl_config.emb.offset == 32 and binding.tl_config.v.offset == 72
    assert ctypes_sizeof() == 80


def ctypes_sizeof():
    import ctypes
    return ctypes.sizeof(binding.tl_config)


def test_generator_is_deterministic_and_shaped_as_documented():
    a, b = synth.workload("sentence"), synth.workload("sentence")
    assert np.array_equal(a.trees.left, b.trees.left) and np.array_equal(a.params.u, b.params.u)
    t = a.trees
    assert t.n_trees == 25 and t.n_nodes == 2 * t.n_leaves - t.n_trees
    sizes = np.diff(t.tree_off)
    leaves = (sizes + 1) // 2
    assert leaves.min() >= 5 and leaves.max() <= 50
    assert (t.left[t.tree_off[:-1]] >= 0).all()          # pre-order: every root comes first
    assert (t.left[t.left >= 0] > np.flatnonzero(t.left >= 0)).all()   # children after parents
    p = a.params
    assert p.emb.shape == (20000, 300) and p.u.shape == (300, 750) and p.w_leaf.shape == (300, 450)
    assert (p.b[150:450] == 1).all() and not p.b[:150].any() and not p.b[450:].any()
    bound = np.sqrt(6.0 / (300 + 750))
    assert np.abs(p.u).max() <= bound and np.abs(p.u).max() > 0.99 * bound
    assert abs(float(p.emb.std()) - 0.1) < 1e-3
    s = synth.workload("stress").trees
    assert s.n_trees == 64 and s.n_nodes == 64 * 2047


def test_splitmix_reference_values():
    """First outputs of SplitMix64 with state 0 (published test vector of the generator)."""
    s = synth.Stream.__new__(synth.Stream)
    s.key, s.ctr = 0, 0
    assert [int(x) for x in s.u64(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
