"""ctypes front end of the C oracle (argument marshalling only)."""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "taper_oracle.c")
_LIB = os.path.join(_HERE, "libtaper_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over (sequence, head))."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.taper_oracle_resolve.restype = ctypes.c_int
        _lib.taper_oracle_attention.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


@dataclasses.dataclass
class OracleInts:
    n_groups: int
    ctx_len: np.ndarray
    n_prefix_pages: np.ndarray
    n_suffix_pages: np.ndarray
    group_start: np.ndarray  # [G+1]
    slots: Optional[np.ndarray]  # int64 [S, max_ctx], -1 past the end


def resolve(page_size: int, block_table, branch_group, prefix_len, suffix_len, want_slots: bool = True) -> OracleInts:
    lib = _load()
    bt = _i32(block_table)
    S = bt.shape[0]
    grp, pl, sl = _i32(branch_group), _i32(prefix_len), _i32(suffix_len)
    ctx = np.zeros(S, np.int32)
    npp = np.zeros(S, np.int32)
    nsp = np.zeros(S, np.int32)
    gs = np.zeros(S + 1, np.int32)
    slots = None
    stride = 0
    if want_slots:
        stride = int((pl.astype(np.int64) + sl).max()) if S else 0
        slots = np.zeros((S, stride), np.int64)
    G = lib.taper_oracle_resolve(
        ctypes.c_int(S), ctypes.c_int(page_size), _p(bt), ctypes.c_int(bt.shape[1]), _p(grp), _p(pl), _p(sl),
        _p(ctx), _p(npp), _p(nsp), _p(gs), _p(slots), ctypes.c_int64(stride))
    if G < 0:
        raise ValueError("malformed branch_group (ids must start at 0 and grow by steps of 1, members contiguous)")
    return OracleInts(G, ctx, npp, nsp, gs[: G + 1].copy(), slots)


def attention(n_q_heads: int, n_kv_heads: int, head_dim: int, page_size: int, scale: float,
              q_bits: np.ndarray, kv_bits: np.ndarray, block_table, prefix_len, suffix_len,
              n_threads: int = 0, want_lse: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray], np.ndarray, int]:
    """Returns (out fp64 [S,Hq,D], lse fp64 [S,Hq] or None, weights_sum fp64 [S,Hq], threads used)."""
    lib = _load()
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    kv = np.ascontiguousarray(kv_bits, dtype=np.uint16)
    bt = _i32(block_table)
    pl, sl = _i32(prefix_len), _i32(suffix_len)
    S = bt.shape[0]
    assert q.shape == (S, n_q_heads, head_dim), q.shape
    assert kv.size % (2 * n_kv_heads * page_size * head_dim) == 0
    out = np.zeros((S, n_q_heads, head_dim), np.float64)
    lse = np.zeros((S, n_q_heads), np.float64) if want_lse else None
    wsum = np.zeros((S, n_q_heads), np.float64)
    used = lib.taper_oracle_attention(
        ctypes.c_int(S), ctypes.c_int(n_q_heads), ctypes.c_int(n_kv_heads), ctypes.c_int(head_dim),
        ctypes.c_int(page_size), ctypes.c_double(scale), _p(q), _p(kv), _p(bt), ctypes.c_int(bt.shape[1]),
        _p(pl), _p(sl), _p(out), _p(lse), _p(wsum), ctypes.c_int(n_threads))
    return out, lse, wsum, used


# ----------------------------------------------------------------------------- reduce phase, KV append
def resolve_segments(page_size: int, block_table, prefix_len, seg_start, seg_len, want_slots: bool = True):
    """Sequences whose private context is a list of segments (each on fresh pages).
    Returns (ctx_len int32 [S], n_private_pages int32 [S], slots int64 [S, max_ctx] or None)."""
    lib = _load()
    bt = _i32(block_table)
    S = bt.shape[0]
    pl, ss, sl = _i32(prefix_len), _i32(seg_start), _i32(seg_len)
    assert len(ss) == S + 1 and ss[0] == 0 and ss[-1] == len(sl)
    ctx = np.zeros(S, np.int32)
    npriv = np.zeros(S, np.int32)
    totals = pl.astype(np.int64) + np.array([sl[ss[s]:ss[s + 1]].sum() for s in range(S)], np.int64)
    stride = int(totals.max()) if (S and want_slots) else 0
    slots = np.zeros((S, stride), np.int64) if want_slots else None
    lib.taper_oracle_resolve_segments(ctypes.c_int(S), ctypes.c_int(page_size), _p(bt), ctypes.c_int(bt.shape[1]), _p(pl),
                                      _p(ss), _p(sl), _p(ctx), _p(npriv), _p(slots), ctypes.c_int64(stride))
    assert np.array_equal(ctx, totals)
    return ctx, npriv, slots


def attention_slots(n_q_heads: int, n_kv_heads: int, head_dim: int, page_size: int, scale: float, q_bits, kv_bits,
                    slots, ctx_len, n_threads: int = 0):
    """Attention over explicit slot lists.  Returns (out fp64 [S,Hq,D], lse fp64 [S,Hq])."""
    lib = _load()
    lib.taper_oracle_attention_slots.restype = ctypes.c_int
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    kv = np.ascontiguousarray(kv_bits, dtype=np.uint16)
    sl = np.ascontiguousarray(slots, dtype=np.int64)
    cl = _i32(ctx_len)
    S = sl.shape[0]
    assert q.shape == (S, n_q_heads, head_dim)
    out = np.zeros((S, n_q_heads, head_dim), np.float64)
    lse = np.zeros((S, n_q_heads), np.float64)
    lib.taper_oracle_attention_slots(ctypes.c_int(S), ctypes.c_int(n_q_heads), ctypes.c_int(n_kv_heads), ctypes.c_int(head_dim),
                                     ctypes.c_int(page_size), ctypes.c_double(scale), _p(q), _p(kv), _p(sl),
                                     ctypes.c_int64(sl.shape[1]), _p(cl), _p(out), _p(lse), ctypes.c_int(n_threads))
    return out, lse


def attention_segments(n_q_heads, n_kv_heads, head_dim, page_size, scale, q_bits, kv_bits, block_table, prefix_len,
                       seg_start, seg_len, n_threads: int = 0):
    ctx, _, slots = resolve_segments(page_size, block_table, prefix_len, seg_start, seg_len)
    return attention_slots(n_q_heads, n_kv_heads, head_dim, page_size, scale, q_bits, kv_bits, slots, ctx, n_threads)


def kv_append(n_kv_heads: int, head_dim: int, page_size: int, k_new_bits, v_new_bits, slot, kv_bits: np.ndarray) -> None:
    """Writes the new K/V rows (uint16 [S,Hkv,D]) into `kv_bits` (modified in place) at slot[s]."""
    lib = _load()
    k = np.ascontiguousarray(k_new_bits, dtype=np.uint16)
    v = np.ascontiguousarray(v_new_bits, dtype=np.uint16)
    sl = np.ascontiguousarray(slot, dtype=np.int64)
    S = len(sl)
    assert k.shape == v.shape == (S, n_kv_heads, head_dim)
    assert kv_bits.dtype == np.uint16 and kv_bits.flags.c_contiguous
    lib.taper_oracle_kv_append(ctypes.c_int(S), ctypes.c_int(n_kv_heads), ctypes.c_int(head_dim), ctypes.c_int(page_size),
                               _p(k), _p(v), _p(sl), _p(kv_bits))
