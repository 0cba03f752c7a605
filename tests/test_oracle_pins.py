"""Pins for the CPU oracle: everything here is fixed by the mathematics or by
the paper's setting, never by the oracle itself or by the GPU path.

Paper passages: visibility rule and shared prefix blocks (§3.1), schedule
invariance (Lemma 1, App. A), memory accounting (App. C), model shape (App. D).
"""
import math

import numpy as np
import pytest
import scipy.special

import oracle
from taper_inputs import (AttnShape, Batch, bf16_bits_from_f32, f32_from_bf16_bits, fill_values_numpy,
                          structure_config1, structure_custom)
from tests.layout_ref import PoolView, dense_context

SMALL = AttnShape(4, 2, 16, 4)  # tiny heads / pages so brute force stays readable


def run_oracle(b: Batch, **kw):
    st, sh = b.structure, b.structure.shape
    return oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, b.q, b.kv,
                            st.block_table, st.prefix_len, st.suffix_len, **kw)


def library_attention(b: Batch):
    """softmax(q K^T * scale) V per (sequence, head) with scipy's softmax on a dense gather."""
    st, sh = b.structure, b.structure.shape
    out = np.zeros((st.n_seqs, sh.n_q_heads, sh.head_dim))
    lse = np.zeros((st.n_seqs, sh.n_q_heads))
    qf = f32_from_bf16_bits(b.q).astype(np.float64)
    for s in range(st.n_seqs):
        for h in range(sh.n_q_heads):
            k, v = dense_context(st, b.kv, s, h // sh.gqa)
            x = (k @ qf[s, h]) * sh.scale
            out[s, h] = scipy.special.softmax(x) @ v
            lse[s, h] = scipy.special.logsumexp(x)
    return out, lse


def mixed_small(seed=7, shape=SMALL):
    reqs = [(13, [0]), (10, [0, 3, 4, 9]), (1, [0]), (8, [5, 1]), (6, [0])]
    return fill_values_numpy(structure_custom(shape, reqs, seed=seed))


# ------------------------------------------------------------------ library
def test_matches_library_softmax_config1():
    b = fill_values_numpy(structure_config1())
    out, lse, wsum, _ = run_oracle(b)
    ref, ref_lse = library_attention(b)
    assert np.max(np.abs(out - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    assert np.max(np.abs(lse - ref_lse)) <= 1e-12
    assert np.max(np.abs(wsum - 1.0)) <= 1e-13


def test_matches_library_softmax_qwen_shape_unaligned():
    sh = AttnShape(64, 8, 128, 16)
    reqs = [(37, [0]), (50, [0, 7, 16, 21]), (16, [1])]  # prefix ends mid-page; suffix starts on a fresh page
    b = fill_values_numpy(structure_custom(sh, reqs, seed=11))
    out, lse, wsum, _ = run_oracle(b)
    ref, ref_lse = library_attention(b)
    assert np.max(np.abs(out - ref)) <= 1e-12
    assert np.max(np.abs(lse - ref_lse)) <= 1e-12
    assert np.max(np.abs(wsum - 1.0)) <= 1e-13


# ------------------------------------------------------------------ closed forms
def test_single_key_returns_its_value_exactly():
    st = structure_custom(SMALL, [(1, [0]), (1, [0, 1])], seed=3)
    b = fill_values_numpy(st)
    out, _, _, _ = run_oracle(b)
    for s in range(st.n_seqs):
        for h in range(SMALL.n_q_heads):
            k, v = dense_context(st, b.kv, s, h // SMALL.gqa)
            if len(k) == 1:
                assert np.array_equal(out[s, h], v[0])


def test_identical_keys_return_mean_value():
    st = structure_custom(SMALL, [(9, [0]), (6, [0, 5])], seed=4)
    b = fill_values_numpy(st)
    pv = PoolView(SMALL.n_kv_heads, SMALL.head_dim, SMALL.page_size)
    flat = b.kv.reshape(-1)
    key = bf16_bits_from_f32(np.linspace(-1, 1, SMALL.head_dim).astype(np.float32))
    for page in range(st.n_pool_pages):
        for hk in range(SMALL.n_kv_heads):
            for tok in range(SMALL.page_size):
                flat[pv.k_off(page, hk, tok, np.arange(SMALL.head_dim))] = key
    out, _, _, _ = run_oracle(b)
    for s in range(st.n_seqs):
        for h in range(SMALL.n_q_heads):
            _, v = dense_context(st, b.kv, s, h // SMALL.gqa)
            assert np.max(np.abs(out[s, h] - v.mean(axis=0))) <= 1e-14


def test_zero_query_averages_valid_tokens_only():
    """q = 0 gives the plain mean of V over the n visible tokens; the invalid
    tail slots of partial pages hold +-1e30 and must not leak in."""
    st = structure_custom(SMALL, [(7, [0]), (5, [0, 2, 6])], seed=5)
    b = fill_values_numpy(st)
    b.q[:] = 0
    poison_invalid_slots(b, 1e30)
    out, _, _, _ = run_oracle(b)
    for s in range(st.n_seqs):
        for h in range(SMALL.n_q_heads):
            _, v = dense_context(st, b.kv, s, h // SMALL.gqa)
            assert np.max(np.abs(out[s, h] - v.mean(axis=0))) <= 1e-14


def poison_invalid_slots(b: Batch, val: float):
    """Overwrite every slot no sequence may read (tail of partial pages and
    unreferenced pages) with +-val."""
    st, sh = b.structure, b.structure.shape
    pv = PoolView(sh.n_kv_heads, sh.head_dim, sh.page_size)
    valid = np.zeros((st.n_pool_pages, sh.page_size), bool)
    P = sh.page_size
    for s in range(st.n_seqs):
        npre, nsuf = int(st.prefix_len[s]), int(st.suffix_len[s])
        npp = -(-npre // P)
        for t in range(npre):
            valid[st.block_table[s, t // P], t % P] = True
        for j in range(nsuf):
            valid[st.block_table[s, npp + j // P], j % P] = True
    flat = b.kv.reshape(-1)
    pos = bf16_bits_from_f32(np.array([val], np.float32))[0]
    neg = bf16_bits_from_f32(np.array([-val], np.float32))[0]
    d = np.arange(sh.head_dim)
    for page in range(st.n_pool_pages):
        for tok in range(P):
            if not valid[page, tok]:
                for hk in range(sh.n_kv_heads):
                    flat[pv.k_off(page, hk, tok, d)] = np.where(d % 2 == 0, pos, neg)
                    flat[pv.v_off(page, hk, tok, d)] = np.where(d % 2 == 0, neg, pos)


def test_dominant_key_selects_its_slot():
    """One key aligned with q and scaled up takes all the weight; V rows are
    one-hot codes of (page, token), so the output names the physical slot."""
    sh = AttnShape(2, 1, 128, 16)
    st = structure_custom(sh, [(24, [0]), (20, [3, 20])], seed=6, n_pool_pages=7)
    b = fill_values_numpy(st)
    pv = PoolView(1, 128, 16)
    flat = b.kv.reshape(-1)
    d = np.arange(128)
    # V[page, tok] = one-hot at index page*16+tok (7 pages * 16 = 112 <= 128)
    one = bf16_bits_from_f32(np.array([1.0], np.float32))[0]
    for page in range(7):
        for tok in range(16):
            flat[pv.v_off(page, 0, tok, d)] = np.where(d == page * 16 + tok, one, 0).astype(np.uint16)
    ints = oracle.resolve(16, st.block_table, st.branch_group, st.prefix_len, st.suffix_len)
    rng = np.random.default_rng(0)
    for s in range(st.n_seqs):
        npre, nsuf = int(st.prefix_len[s]), int(st.suffix_len[s])
        picks = [int(rng.integers(0, npre))] + ([npre + int(rng.integers(0, nsuf))] if nsuf else [])
        b.q[s, 1] = b.q[s, 0]
        qv = f32_from_bf16_bits(b.q[s, 0]).astype(np.float64)
        for t_star in picks:
            # physical slot of logical position t_star, by hand from the block table
            if t_star < npre:
                page, tok = int(st.block_table[s, t_star // 16]), t_star % 16
            else:
                j = t_star - npre
                page, tok = int(st.block_table[s, -(-npre // 16) + j // 16]), j % 16
            saved = flat[pv.k_off(page, 0, tok, d)].copy()
            flat[pv.k_off(page, 0, tok, d)] = bf16_bits_from_f32((200.0 * qv / np.linalg.norm(qv)).astype(np.float32))
            out, _, _, _ = run_oracle(b)
            flat[pv.k_off(page, 0, tok, d)] = saved
            for h in (0, 1):
                code = out[s, h]
                assert int(np.argmax(code)) == page * 16 + tok
                assert code[page * 16 + tok] > 1 - 1e-9
            assert int(ints.slots[s, t_star]) == page * 16 + tok


# ------------------------------------------------------------------ brute force
def test_brute_force_explicit_term_lists():
    """S = 3 sequences, contexts of 1..5 tokens, D = 8: the visible (k, v)
    pairs are literal lists; every term is written out and summed with fsum."""
    sh = AttnShape(2, 1, 8, 4)
    rng = np.random.default_rng(42)
    rb = lambda *shape: f32_from_bf16_bits(bf16_bits_from_f32(rng.standard_normal(shape).astype(np.float32))).astype(np.float64)
    prefix_kv = [(rb(8), rb(8)) for _ in range(3)]  # request B's shared prefix: 3 tokens
    branch0_kv = []  # branch with no private tokens
    branch1_kv = [(rb(8), rb(8)) for _ in range(2)]
    serial_kv = [(rb(8), rb(8)) for _ in range(5)]
    visible = [serial_kv, prefix_kv + branch0_kv, prefix_kv + branch1_kv]
    st = structure_custom(sh, [(5, [0]), (3, [0, 2])], seed=9, n_pool_pages=9)
    b = fill_values_numpy(st)
    pv = PoolView(1, 8, 4)
    flat = b.kv.reshape(-1)
    d = np.arange(8)

    def put(page, tok, kv):
        flat[pv.k_off(page, 0, tok, d)] = bf16_bits_from_f32(kv[0].astype(np.float32))
        flat[pv.v_off(page, 0, tok, d)] = bf16_bits_from_f32(kv[1].astype(np.float32))

    bt = st.block_table
    for t, kv in enumerate(serial_kv):
        put(bt[0, t // 4], t % 4, kv)
    for t, kv in enumerate(prefix_kv):
        put(bt[1, 0], t, kv)
    assert bt[2, 0] == bt[1, 0]  # one set of prefix blocks
    for j, kv in enumerate(branch1_kv):
        put(bt[2, 1], j, kv)  # private tokens start on entry ceil(3/4) = 1
    out, lse, _, _ = run_oracle(b)
    qf = f32_from_bf16_bits(b.q).astype(np.float64)
    scale = 1.0 / math.sqrt(8)
    for s in range(3):
        for h in range(2):
            xs = [scale * math.fsum(float(qf[s, h, i]) * float(k[i]) for i in range(8)) for k, _ in visible[s]]
            m = max(xs)
            ws = [math.exp(x - m) for x in xs]
            Z = math.fsum(ws)
            for i in range(8):
                expect = math.fsum(w * float(v[i]) for w, (_, v) in zip(ws, visible[s])) / Z
                assert abs(out[s, h, i] - expect) <= 1e-15 * max(1.0, abs(expect)) + 1e-15
            assert abs(lse[s, h] - (m + math.log(Z))) <= 1e-14


# ------------------------------------------------------------------ invariances
def test_split_then_merge_equals_monolithic():
    """The identity the GPU design relies on, checked in fp64 without sharing
    code with it: attention over the prefix alone and over the private tokens
    alone, merged through their log-sum-exps, equals one pass over both."""
    sh = SMALL
    st = structure_custom(sh, [(10, [3, 4, 9])], seed=8)
    b = fill_values_numpy(st)
    out, lse, _, _ = run_oracle(b)
    # prefix only: same rows with suffix_len = 0
    o_p, l_p, _, _ = oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, b.q, b.kv,
                                      st.block_table, st.prefix_len, np.zeros_like(st.suffix_len))
    # private tokens only: drop the prefix entries from each row
    npp = -(-int(st.prefix_len[0]) // sh.page_size)
    bt_s = np.ascontiguousarray(st.block_table[:, npp:])
    o_s, l_s, _, _ = oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, b.q, b.kv,
                                      bt_s, st.suffix_len, np.zeros_like(st.suffix_len))
    m = np.maximum(l_p, l_s)
    wp, ws = np.exp(l_p - m), np.exp(l_s - m)
    merged = (wp[..., None] * o_p + ws[..., None] * o_s) / (wp + ws)[..., None]
    assert np.max(np.abs(merged - out)) <= 1e-12
    assert np.max(np.abs(m + np.log(wp + ws) - lse)) <= 1e-12


def test_page_permutation_invariance_is_bit_exact():
    b = mixed_small()
    st = b.structure
    out0, _, _, _ = run_oracle(b)
    perm = np.random.default_rng(1).permutation(st.n_pool_pages)  # old page p moves to perm[p]
    kv2 = np.empty_like(b.kv)
    kv2[perm] = b.kv
    bt2 = st.block_table.copy()
    bt2[bt2 >= 0] = perm[bt2[bt2 >= 0]]
    out1, _, _, _ = oracle.attention(SMALL.n_q_heads, SMALL.n_kv_heads, SMALL.head_dim, SMALL.page_size, SMALL.scale,
                                     b.q, kv2, bt2, st.prefix_len, st.suffix_len)
    assert np.array_equal(out0, out1)


def test_sibling_independence_is_bit_exact():
    """Lemma 1: a branch's output does not depend on which siblings run in the
    same step, nor on their order."""
    b = mixed_small()
    st = b.structure
    out0, _, _, _ = run_oracle(b)
    members = [s for s in range(st.n_seqs) if st.branch_group[s] == 1]
    assert len(members) == 4
    for keep in ([members[2]], [members[3], members[0]], members[::-1]):
        rows = np.array(keep)
        out1, _, _, _ = oracle.attention(SMALL.n_q_heads, SMALL.n_kv_heads, SMALL.head_dim, SMALL.page_size,
                                         SMALL.scale, b.q[rows], b.kv, st.block_table[rows], st.prefix_len[rows],
                                         st.suffix_len[rows])
        assert np.array_equal(out1, out0[rows])


def test_gqa_head_mapping():
    b = mixed_small()
    g = SMALL.gqa
    b.q[:, 1] = b.q[:, 0]  # heads 0,1 share KV head 0
    b.q[:, g] = b.q[:, 0]  # head g reads KV head 1
    out, _, _, _ = run_oracle(b)
    assert np.array_equal(out[:, 0], out[:, 1])
    assert not np.array_equal(out[:, 0], out[:, g])


def test_garbage_invariance_is_bit_exact():
    b = mixed_small()
    out0, _, _, _ = run_oracle(b)
    poison_invalid_slots(b, 1e30)
    out1, _, _, _ = run_oracle(b)
    assert np.array_equal(out0, out1)


# ------------------------------------------------------------------ integer side
def independent_slots(st):
    """Table-first resolver: walk every block-table entry and say which logical
    positions of which sequences it carries (the inverse of the oracle's
    position-first lookup)."""
    P = st.shape.page_size
    S = st.n_seqs
    ctx = st.prefix_len.astype(np.int64) + st.suffix_len
    slots = np.full((S, int(ctx.max())), -1, np.int64)
    for s in range(S):
        npre, nsuf = int(st.prefix_len[s]), int(st.suffix_len[s])
        npp = -(-npre // P)
        for j in range(st.block_table.shape[1]):
            page = int(st.block_table[s, j])
            if j < npp:
                lo, hi = j * P, min(npre, (j + 1) * P)
                slots[s, lo:hi] = page * P + np.arange(hi - lo)
            elif j < npp + -(-nsuf // P):
                jj = j - npp
                lo, hi = jj * P, min(nsuf, (jj + 1) * P)
                slots[s, npre + lo : npre + hi] = page * P + np.arange(hi - lo)
    return slots


@pytest.mark.parametrize("maker", [structure_config1, lambda: mixed_small().structure])
def test_integer_side(maker):
    st = maker()
    P = st.shape.page_size
    ints = oracle.resolve(P, st.block_table, st.branch_group, st.prefix_len, st.suffix_len)
    assert np.array_equal(ints.ctx_len, st.prefix_len + st.suffix_len)
    assert np.array_equal(ints.n_prefix_pages, -(-st.prefix_len // P))
    # memory accounting (App. C): a branch costs blocks(private tokens); none when it has produced nothing
    assert np.array_equal(ints.n_suffix_pages, -(-st.suffix_len // P))
    assert np.all(ints.n_suffix_pages[st.suffix_len == 0] == 0)
    assert np.array_equal(ints.slots, independent_slots(st))
    # group CSR
    gs = ints.group_start
    assert gs[0] == 0 and gs[-1] == st.n_seqs and ints.n_groups == st.n_groups
    for g in range(ints.n_groups):
        assert np.all(st.branch_group[gs[g] : gs[g + 1]] == g)
    # one set of prefix blocks per request: members resolve identical prefix slots
    for g in range(ints.n_groups):
        a = gs[g]
        npre = int(st.prefix_len[a])
        for s in range(a + 1, gs[g + 1]):
            assert np.array_equal(ints.slots[s, :npre], ints.slots[a, :npre])


def test_config1_matches_the_stated_setting():
    st = structure_config1()
    assert st.n_seqs == 5 and st.n_pool_pages == 64
    assert list(st.prefix_len) == [256, 192, 192, 192, 192]
    assert list(st.suffix_len) == [0, 0, 8, 17, 32]
    ints = oracle.resolve(16, st.block_table, st.branch_group, st.prefix_len, st.suffix_len)
    assert list(ints.n_prefix_pages) == [16, 12, 12, 12, 12]
    assert list(ints.n_suffix_pages) == [0, 0, 1, 2, 2]
    assert st.unique_tokens == 256 + 192 + 57
    used = np.unique(st.block_table[st.block_table >= 0])
    assert len(used) == 16 + 12 + 5


def test_resolve_rejects_bad_groups():
    st = structure_config1()
    bad = st.branch_group.copy()
    bad[2] = 3
    with pytest.raises(ValueError):
        oracle.resolve(16, st.block_table, bad, st.prefix_len, st.suffix_len)
