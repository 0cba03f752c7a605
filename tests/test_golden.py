"""Stored values: the paper's printed constants and an oracle drift guard."""
import os

import numpy as np

import oracle
from taper_inputs import (fill_values_numpy, structure_config1, structure_config2, structure_config3,
                          structure_config5)

G = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def paper_constants():
    d = {}
    for line in open(os.path.join(G, "paper_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            d[line[0]] = float(line[1])
    return d


def test_workload_shapes_follow_the_paper():
    c = paper_constants()
    for st in (structure_config2(), structure_config3(), structure_config5(k=4)):
        assert st.shape.n_q_heads == c["n_q_heads"] and st.shape.n_kv_heads == c["n_kv_heads"]
        assert int((st.prefix_len + st.suffix_len).max()) <= c["max_context"]
    # config 3 widths are uniform on 4..8: inside the paper's fanout range around P50=4 .. P90=7
    st = structure_config3()
    widths = np.bincount(st.branch_group)[16:]
    assert widths.min() >= c["fanout_p50"] and widths.max() <= c["fanout_p90"] + 1
    # a branch with no private tokens owns no private page
    ints = oracle.resolve(16, st.block_table, st.branch_group, st.prefix_len, st.suffix_len, want_slots=False)
    assert np.all(ints.n_suffix_pages[st.suffix_len == 0] == c["empty_branch_blocks"])


def test_config5_is_nested_in_k():
    a, b = structure_config5(k=2), structure_config5(k=16)
    assert a.n_seqs == 96 + 32 * 3 and b.n_seqs == 96 + 32 * 17
    # the branches admitted at k=2 are the first three of each request at k=16, on the same pages
    for g in range(96, 128):
        ra = np.flatnonzero(a.branch_group == g)
        rb = np.flatnonzero(b.branch_group == g)[:3]
        w = a.block_table.shape[1]
        assert np.array_equal(a.suffix_len[ra], b.suffix_len[rb])
        assert np.array_equal(a.block_table[ra], b.block_table[rb][:, :w])


def test_oracle_matches_stored_config1_values():
    b = fill_values_numpy(structure_config1())
    st, sh = b.structure, b.structure.shape
    out, lse, _, _ = oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, b.q, b.kv,
                                      st.block_table, st.prefix_len, st.suffix_len)
    n = 0
    for line in open(os.path.join(G, "config1_oracle.txt")):
        if line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "bt":
            continue
        s, h = int(f[0]), int(f[1])
        got = np.array([lse[s, h], out[s, h, 0], out[s, h, 21], out[s, h, 63]])
        assert np.allclose(got, np.array([float(x) for x in f[2:]]), rtol=1e-13, atol=1e-15)
        n += 1
    assert n == 20
