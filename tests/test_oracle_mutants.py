"""The pins must be able to fail: plant plausible mistakes in *copies* of the
oracle source (CPU only) and check that the library-softmax pin rejects each."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from taper_inputs import AttnShape, fill_values_numpy, structure_custom
from tests.test_oracle_pins import library_attention

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "taper_oracle.c")

MUTANTS = {
    "dropped_scale": ("x[t] = scale * acc;", "x[t] = acc;"),
    "gqa_modulo_instead_of_division": ("hk = h / g;", "hk = h % Hkv;"),
    "suffix_starts_at_floor_page": ("int npp = (int)ceil_div(prefix_len, P);", "int npp = prefix_len / P;"),
    "k_tile_read_row_major": ("return tile + (int64_t)(d / 8) * (P * 8) + tok * 8 + d % 8;",
                              "return tile + (int64_t)tok * D + d;"),
    "v_tile_read_like_k": ("return tile + (int64_t)(tok / 4) * (4 * D) + d * 4 + tok % 4;",
                           "return tile + (int64_t)(d / 8) * (P * 8) + tok * 8 + d % 8;"),
    "k_and_v_swapped": ("int64_t tile = ((page * 2 + is_v) * Hkv + hk)", "int64_t tile = ((page * 2 + 1 - is_v) * Hkv + hk)"),
    "max_not_subtracted_and_sign": ("x[t] = exp(x[t] - m);", "x[t] = exp(m - x[t]);"),
    "last_token_dropped": ("for (int t = 0; t < n; ++t) { x[t] = exp(x[t] - m); Z += x[t]; }",
                           "for (int t = 0; t < n; ++t) { x[t] = exp(x[t] - m); if (t == n - 1 && n > 1) x[t] = 0; Z += x[t]; }"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pin_rejects_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    c = tmp_path / "mutant.c"
    c.write_text(src.replace(old, new))
    so = tmp_path / "mutant.so"
    subprocess.check_call(["gcc", "-O1", "-fPIC", "-shared", "-std=c99", "-o", str(so), str(c), "-lm"])
    lib = ctypes.CDLL(str(so))
    sh = AttnShape(8, 2, 16, 8)
    b = fill_values_numpy(structure_custom(sh, [(21, [0]), (13, [0, 5, 9]), (8, [3])], seed=21))
    st = b.structure
    out = np.zeros((st.n_seqs, sh.n_q_heads, sh.head_dim))
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    lib.taper_oracle_attention(
        ctypes.c_int(st.n_seqs), ctypes.c_int(sh.n_q_heads), ctypes.c_int(sh.n_kv_heads), ctypes.c_int(sh.head_dim),
        ctypes.c_int(sh.page_size), ctypes.c_double(sh.scale), p(b.q), p(b.kv), p(st.block_table),
        ctypes.c_int(st.block_table.shape[1]), p(st.prefix_len), p(st.suffix_len), p(out), None, None, ctypes.c_int(1))
    ref, _ = library_attention(b)
    assert np.max(np.abs(out - ref)) > 1e-6, f"mutant {name} slipped through the pin"
