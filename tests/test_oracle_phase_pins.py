"""Pins of the oracle's reduce-phase attention (contexts made of several private
segments, §3.1 reduce visibility) and KV append, against an independent statement of
the pool layout (tests/layout_ref.py), scipy's softmax, and the already pinned
two-segment oracle."""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import scipy.special

import oracle
from taper_inputs import (AttnShape, bf16_bits_from_f32, f32_from_bf16_bits, fill_values_numpy, reduce_structure,
                          structure_custom)
from tests.layout_ref import PoolView

SMALL = AttnShape(4, 2, 16, 4)
QWEN = AttnShape(64, 8, 128, 16)


def parallel_batch(shape, seed=5, spare=40):
    reqs = [(13, [0]), (10, [0, 3, 4, 9]), (7, [5, 1, 0]), (6, [2])]
    st = structure_custom(shape, reqs, seed=seed)
    st = structure_custom(shape, reqs, seed=seed, n_pool_pages=st.n_pool_pages + spare)  # room for the reduce tokens
    return fill_values_numpy(st)


def dense_segments(seg, kv_bits, s, hk):
    """K and V rows of sequence s in logical order, gathered page by page with the test-side layout."""
    sh = seg.shape
    pv = PoolView(sh.n_kv_heads, sh.head_dim, sh.page_size)
    flat = kv_bits.reshape(-1)
    P = sh.page_size
    pieces = [int(seg.prefix_len[s])] + [int(x) for x in seg.seg_len[seg.seg_start[s]:seg.seg_start[s + 1]]]
    entry = 0
    ks, vs = [], []
    for n in pieces:
        for j in range(-(-n // P)):
            page = int(seg.block_table[s, entry + j])
            take = min(P, n - j * P)
            ks.append(pv.k_rows(flat, page, hk)[:take])
            vs.append(pv.v_rows(flat, page, hk)[:take])
        entry += -(-n // P)
    k = f32_from_bf16_bits(np.concatenate(ks)).astype(np.float64)
    v = f32_from_bf16_bits(np.concatenate(vs)).astype(np.float64)
    return k, v


def run_segments(seg, q, kv):
    sh = seg.shape
    return oracle.attention_segments(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, q, kv,
                                     seg.block_table, seg.prefix_len, seg.seg_start, seg.seg_len)


def reduce_case(shape, keep=(), seed=5):
    b = parallel_batch(shape, seed)
    seg = reduce_structure(b.structure, z_len=[3, 6, 0, 9], seed=seed + 1, keep_parallel=keep)
    rng = np.random.Generator(np.random.PCG64(seed + 2))
    q = bf16_bits_from_f32(rng.standard_normal((seg.n_seqs, shape.n_q_heads, shape.head_dim), dtype=np.float32))
    return b, seg, q


def library_segments(seg, q, kv):
    sh = seg.shape
    out = np.zeros((seg.n_seqs, sh.n_q_heads, sh.head_dim))
    lse = np.zeros((seg.n_seqs, sh.n_q_heads))
    qf = f32_from_bf16_bits(q).astype(np.float64)
    for s in range(seg.n_seqs):
        for h in range(sh.n_q_heads):
            k, v = dense_segments(seg, kv, s, h // sh.gqa)
            x = (k @ qf[s, h]) * sh.scale
            out[s, h] = scipy.special.softmax(x) @ v
            lse[s, h] = scipy.special.logsumexp(x)
    return out, lse


@pytest.mark.parametrize("shape,keep", [(SMALL, ()), (SMALL, (1,)), (QWEN, ()), (QWEN, (2,))])
def test_reduce_attention_matches_library_softmax(shape, keep):
    b, seg, q = reduce_case(shape, keep)
    out, lse = run_segments(seg, q, b.kv)
    ref, ref_lse = library_segments(seg, q, b.kv)
    assert np.max(np.abs(out - ref)) <= 1e-12 and np.max(np.abs(lse - ref_lse)) <= 1e-12


def test_reduce_sequence_sees_prefix_all_branches_in_order_and_own_tokens():
    """The slot list is exactly: the prefix's slots, then every branch's private slots in branch order (the very
    slots the parallel phase resolved for them), then the reduce tokens' slots."""
    b, seg, _ = reduce_case(SMALL)
    par = b.structure
    ints = oracle.resolve(4, par.block_table, par.branch_group, par.prefix_len, par.suffix_len)
    ctx, npriv, slots = oracle.resolve_segments(4, seg.block_table, seg.prefix_len, seg.seg_start, seg.seg_len)
    z = [3, 6, 0, 9]
    for g in range(par.n_groups):
        members = np.flatnonzero(par.branch_group == g)
        pl = int(par.prefix_len[members[0]])
        want = list(ints.slots[members[0], :pl])
        for s in members:
            want += list(ints.slots[s, pl : pl + int(par.suffix_len[s])])
        got = list(slots[g, : ctx[g]])
        assert got[: len(want)] == want
        assert len(got) == len(want) + z[g]
        tail = got[len(want):]
        assert len(set(tail)) == len(tail) and not set(tail) & set(int(x) for x in ints.slots.ravel() if x >= 0)
        # the reduce tokens sit on fresh pages, consecutive inside a page
        assert all(t % 4 == i % 4 for i, t in enumerate(tail))
        assert npriv[g] == sum(-(-int(par.suffix_len[s]) // 4) for s in members) + -(-z[g] // 4)


def test_one_segment_per_sequence_is_the_parallel_phase():
    b = parallel_batch(QWEN)
    st = b.structure
    seg_start = np.arange(st.n_seqs + 1, dtype=np.int32)
    ints = oracle.resolve(16, st.block_table, st.branch_group, st.prefix_len, st.suffix_len)
    ctx, npriv, slots = oracle.resolve_segments(16, st.block_table, st.prefix_len, seg_start, st.suffix_len)
    assert np.array_equal(ctx, ints.ctx_len) and np.array_equal(npriv, ints.n_suffix_pages)
    assert np.array_equal(slots, ints.slots)
    out, lse = oracle.attention_segments(64, 8, 128, 16, QWEN.scale, b.q, b.kv, st.block_table, st.prefix_len, seg_start,
                                         st.suffix_len)
    ref, ref_lse, _, _ = oracle.attention(64, 8, 128, 16, QWEN.scale, b.q, b.kv, st.block_table, st.prefix_len, st.suffix_len)
    assert np.array_equal(out, ref) and np.array_equal(lse, ref_lse)


def test_every_branch_is_visible_to_the_reduce_token_and_to_no_sibling():
    b, seg, q = reduce_case(SMALL)
    par = b.structure
    base, _ = run_segments(seg, q, b.kv)
    pv = PoolView(2, 16, 4)
    members = np.flatnonzero(par.branch_group == 1)  # the request with 4 branches
    pl = int(par.prefix_len[members[0]])
    for s in members:
        if par.suffix_len[s] == 0:
            continue
        kv2 = b.kv.copy()
        page = int(par.block_table[s, -(-pl // 4)])
        for hk in range(2):
            kv2.reshape(-1)[pv.v_off(page, hk, 0, np.arange(16))] ^= 0x8000  # flip the sign of the branch's first V row
        out2, _ = run_segments(seg, q, kv2)
        assert np.max(np.abs(out2[1] - base[1])) > 1e-6, "reduce token does not see the branch"
        others = [g for g in range(seg.n_seqs) if g != 1]
        assert np.array_equal(out2[others], base[others])
        sib = oracle.attention(4, 2, 16, 4, SMALL.scale, b.q, kv2, par.block_table, par.prefix_len, par.suffix_len)[0]
        sib0 = oracle.attention(4, 2, 16, 4, SMALL.scale, b.q, b.kv, par.block_table, par.prefix_len, par.suffix_len)[0]
        for t in members:
            assert (t == s) != np.array_equal(sib[t], sib0[t])  # only the branch itself changes (Lemma 1)


def test_order_of_segments_does_not_change_the_sum():
    """Softmax attention has no positional term here: listing the branches in another order (with the block
    table rearranged to match) gives the same result up to summation order -- every token counted once."""
    b, seg, q = reduce_case(QWEN)
    out, _ = run_segments(seg, q, b.kv)
    s = 1
    P = 16
    lens = [int(x) for x in seg.seg_len[seg.seg_start[s]:seg.seg_start[s + 1]]]
    npp = -(-int(seg.prefix_len[s]) // P)
    pages, e = [], npp
    for n in lens:
        pages.append(list(seg.block_table[s, e : e + -(-n // P)]))
        e += -(-n // P)
    order = [3, 0, 4, 2, 1]
    bt = seg.block_table.copy()
    bt[s, npp:e] = [p for i in order for p in pages[i]]
    sl = seg.seg_len.copy()
    sl[seg.seg_start[s]:seg.seg_start[s + 1]] = [lens[i] for i in order]
    out2, _ = oracle.attention_segments(64, 8, 128, 16, QWEN.scale, q, b.kv, bt, seg.prefix_len, seg.seg_start, sl)
    assert np.max(np.abs(out2 - out)) <= 1e-12 and np.array_equal(out2[0], out[0])


def test_kv_append_writes_exactly_the_new_rows():
    sh = QWEN
    b = parallel_batch(sh)
    st = b.structure
    pv = PoolView(8, 128, 16)
    rng = np.random.Generator(np.random.PCG64(9))
    k_new = bf16_bits_from_f32(rng.standard_normal((st.n_seqs, 8, 128), dtype=np.float32))
    v_new = bf16_bits_from_f32(rng.standard_normal((st.n_seqs, 8, 128), dtype=np.float32))
    # the slot after each sequence's last private token; sequences whose private part fills its pages get a fresh page
    used = set(int(x) for x in st.block_table.ravel() if x >= 0)
    fresh = iter(p for p in range(st.n_pool_pages) if p not in used)
    slot = np.zeros(st.n_seqs, np.int64)
    for s in range(st.n_seqs):
        npp, sl = -(-int(st.prefix_len[s]) // 16), int(st.suffix_len[s])
        page = int(st.block_table[s, npp + sl // 16]) if sl % 16 else next(fresh)
        slot[s] = page * 16 + sl % 16
    kv = b.kv.copy()
    oracle.kv_append(8, 128, 16, k_new, v_new, slot, kv)
    changed = np.flatnonzero(kv.ravel() != b.kv.ravel())
    want = []
    d = np.arange(128)
    for s in range(st.n_seqs):
        for hk in range(8):
            page, tok = int(slot[s]) // 16, int(slot[s]) % 16
            assert np.array_equal(kv.ravel()[pv.k_off(page, hk, tok, d)], k_new[s, hk])
            assert np.array_equal(kv.ravel()[pv.v_off(page, hk, tok, d)], v_new[s, hk])
            want += list(pv.k_off(page, hk, tok, d)) + list(pv.v_off(page, hk, tok, d))
    assert set(changed) <= set(want)  # (a new value may equal the old garbage by chance)
    assert len(changed) > 0.99 * len(want)


SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "taper_oracle.c")
MUTANTS = {
    "segment_pages_rounded_down": ("            entry += (int)ceil_div(seg_len[k], P);\n            priv_pages",
                                   "            entry += seg_len[k] / P;\n            priv_pages"),
    "last_segment_dropped": ("for (int k = seg_start[s]; k < seg_start[s + 1]; ++k) {\n            for (int j = 0; j < seg_len[k]; ++j, ++t)",
                             "for (int k = seg_start[s]; k < seg_start[s + 1] - (seg_start[s + 1] - seg_start[s] > 1); ++k) {\n            for (int j = 0; j < seg_len[k]; ++j, ++t)"),
    "segments_packed_without_fresh_pages": ("slots[s * slots_stride + t] = (int64_t)row[entry + j / P] * P + j % P;",
                                            "slots[s * slots_stride + t] = (int64_t)row[(t / P)] * P + t % P;"),
    "append_writes_v_with_k_layout": ("kv_pool[kv_elem(1, page, hk, tok, d, Hkv, D, P)] = v_new",
                                      "kv_pool[kv_elem(0, page, hk, tok, d, Hkv, D, P) + (int64_t)Hkv * P * D] = v_new"),
    "append_off_by_one_token": ("int tok = (int)(slot[s] % P);\n                kv_pool", "int tok = (int)((slot[s] + 1) % P);\n                kv_pool"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    c = tmp_path / "mutant.c"
    c.write_text(src.replace(old, new))
    so = tmp_path / "mutant.so"
    subprocess.check_call(["gcc", "-O1", "-fPIC", "-shared", "-std=c99", "-o", str(so), str(c), "-lm"])
    saved = oracle.oracle._lib
    oracle.oracle._lib = ctypes.CDLL(str(so))
    oracle.oracle._lib.taper_oracle_resolve.restype = ctypes.c_int
    oracle.oracle._lib.taper_oracle_attention.restype = ctypes.c_int
    try:
        failed = []
        for pin in (lambda: test_reduce_attention_matches_library_softmax(QWEN, ()),
                    test_reduce_sequence_sees_prefix_all_branches_in_order_and_own_tokens,
                    test_one_segment_per_sequence_is_the_parallel_phase, test_kv_append_writes_exactly_the_new_rows):
            try:
                pin()
            except Exception:  # noqa: BLE001
                failed.append(pin)
        assert failed, f"mutant {name} slipped through every pin"
    finally:
        oracle.oracle._lib = saved
