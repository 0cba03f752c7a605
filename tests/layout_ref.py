"""Test-side statement of the pool layout, written as array shapes.

The pool is [n_pages][2 (K,V)][Hkv][page*D] bf16.  A K tile viewed as an array
has shape [D/8][page][8] (dims grouped by 8); a V tile has shape
[page/4][D][4] (tokens grouped by 4, transposed).  This helper builds the
element index by reshaping an arange, so it shares no formula with the oracle
or with the HIP code.
"""
import numpy as np


class PoolView:
    def __init__(self, n_kv_heads, head_dim, page_size):
        self.Hkv, self.D, self.P = n_kv_heads, head_dim, page_size
        tile = page_size * head_dim
        ar = np.arange(tile, dtype=np.int64)
        # k_idx[tok, d] / v_idx[tok, d]: offset inside the tile
        self.k_idx = ar.reshape(head_dim // 8, page_size, 8).transpose(1, 0, 2).reshape(page_size, head_dim)
        self.v_idx = ar.reshape(page_size // 4, head_dim, 4).transpose(0, 2, 1).reshape(page_size, head_dim)
        self.tile = tile

    def k_off(self, page, hk, tok, d):
        return ((page * 2 + 0) * self.Hkv + hk) * self.tile + self.k_idx[tok, d]

    def v_off(self, page, hk, tok, d):
        return ((page * 2 + 1) * self.Hkv + hk) * self.tile + self.v_idx[tok, d]

    def k_rows(self, kv_flat, page, hk):
        """[page_size, D] view (copy) of K for one page / kv head."""
        base = ((page * 2 + 0) * self.Hkv + hk) * self.tile
        return kv_flat[base + self.k_idx]

    def v_rows(self, kv_flat, page, hk):
        base = ((page * 2 + 1) * self.Hkv + hk) * self.tile
        return kv_flat[base + self.v_idx]


def dense_context(st, kv_bits, s, hk):
    """Gather sequence s's visible K and V rows, in logical order, as float64
    [n, D] arrays, straight from the block table (prefix pages, then private
    pages starting at entry ceil(prefix/page))."""
    from taper_inputs import f32_from_bf16_bits

    sh = st.shape
    pv = PoolView(sh.n_kv_heads, sh.head_dim, sh.page_size)
    flat = kv_bits.reshape(-1)
    P = sh.page_size
    npre, nsuf = int(st.prefix_len[s]), int(st.suffix_len[s])
    npp = -(-npre // P)
    ks, vs = [], []
    for seg_len, first in ((npre, 0), (nsuf, npp)):
        for j in range(-(-seg_len // P)):
            page = int(st.block_table[s, first + j])
            take = min(P, seg_len - j * P)
            ks.append(pv.k_rows(flat, page, hk)[:take])
            vs.append(pv.v_rows(flat, page, hk)[:take])
    if not ks:
        return np.zeros((0, sh.head_dim)), np.zeros((0, sh.head_dim))
    k = f32_from_bf16_bits(np.concatenate(ks)).astype(np.float64)
    v = f32_from_bf16_bits(np.concatenate(vs)).astype(np.float64)
    return k, v
