"""Thin ctypes binding of libtaper_attn.so: argument marshalling only.

Every step of the decode-step attention runs in the HIP library; this module
converts numpy / torch arguments to pointers and sizes.  torch is used for
device memory and streams, nothing else.  There is no fallback: if the library
is missing or fails to load, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtaper_attn.so")

TAPER_OK, TAPER_EINVAL, TAPER_EBLOCK, TAPER_EGROUP, TAPER_ELEN, TAPER_EHIP, TAPER_ENOMEM = 0, -1, -2, -3, -4, -5, -6

EXPORTED = [
    "taper_create", "taper_destroy", "taper_plan_build", "taper_plan_free", "taper_plan_export",
    "taper_plan_resolve_slots_host", "taper_plan_resolve_slots", "taper_decode_step_attention",
    "taper_decode_step_attention_simple", "taper_step_latency_probe", "taper_kernel_times", "taper_kernel_times_layers",
    "taper_strerror", "taper_last_error",
    "taper_plan_build_segments", "taper_append_slots", "taper_kv_append", "taper_branch_blocks",
    "taper_predictor_fit", "taper_predictor_eval", "taper_predictor_mape", "taper_window_create",
    "taper_window_destroy", "taper_window_push", "taper_window_size", "taper_window_fit", "taper_admit_step",
    "taper_predictor_fit_monotone", "taper_window_fit_monotone",
    "taper_stream_read_probe", "taper_reserve", "taper_decode_step_attention_static",
]


class taper_attn_config(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int), ("n_kv_heads", ctypes.c_int), ("head_dim", ctypes.c_int),
                ("page_size", ctypes.c_int), ("scale", ctypes.c_float), ("device", ctypes.c_int),
                ("partial_format", ctypes.c_int)]


class taper_work_item(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("seq0", "n_branch", "page0", "n_tokens", "part_base", "kind", "part", "merge0")]


class taper_merge_entry(ctypes.Structure):
    _fields_ = [("first_row", ctypes.c_int32), ("rows_per_head", ctypes.c_int32)]


_I32P = ctypes.POINTER(ctypes.c_int32)


class taper_plan_view(ctypes.Structure):
    _fields_ = [("n_seqs", ctypes.c_int32), ("n_groups", ctypes.c_int32), ("ctx_len", _I32P),
                ("n_prefix_pages", _I32P), ("n_suffix_pages", _I32P), ("group_start", _I32P),
                ("seg_start", _I32P), ("seg_len", _I32P), ("seg_page0", _I32P),
                ("n_items", ctypes.c_int32), ("items", ctypes.POINTER(taper_work_item)),
                ("n_pool_items", ctypes.c_int32),
                ("n_parts_shared", ctypes.c_int32), ("n_parts_private", ctypes.c_int32), ("part_start", _I32P),
                ("merge_start", _I32P), ("merge", ctypes.POINTER(taper_merge_entry)),
                ("n_partial_rows", ctypes.c_int64), ("tokens_unique", ctypes.c_int64),
                ("tokens_logical", ctypes.c_int64), ("workspace_id", ctypes.c_int32),
                ("workspace_rows", ctypes.c_int64)]


class taper_plan_options(ctypes.Structure):
    _fields_ = [("target_workgroups", ctypes.c_int32), ("share_prefix", ctypes.c_int32),
                ("max_branches_per_item", ctypes.c_int32), ("shared_cost_pct", ctypes.c_int32),
                ("shared_item_cost", ctypes.c_int32), ("private_item_cost", ctypes.c_int32),
                ("private_merge_cost", ctypes.c_int32), ("solo_item_tokens", ctypes.c_int32),
                ("min_share_tokens", ctypes.c_int32), ("pool_pct", ctypes.c_int32), ("pool_item_tokens", ctypes.c_int32),
                ("small_step_grid", ctypes.c_int32), ("scatter_sub_groups", ctypes.c_int32)]


class taper_probe_result(ctypes.Structure):
    _fields_ = [("us_min", ctypes.c_double), ("us_median", ctypes.c_double), ("us_mean", ctypes.c_double),
                ("n_tokens", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("l_context", ctypes.c_int64),
                ("kv_bytes_unique", ctypes.c_int64), ("kv_bytes_logical", ctypes.c_int64),
                ("gbps_unique", ctypes.c_double), ("gbps_logical", ctypes.c_double)]


class taper_predictor(ctypes.Structure):
    _fields_ = [("a", ctypes.c_double), ("b", ctypes.c_double), ("c", ctypes.c_double)]


class taper_admission_options(ctypes.Structure):
    _fields_ = [("rho", ctypes.c_double), ("utility_kind", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class taper_admission_result(ctypes.Structure):
    _fields_ = [("t0_ms", ctypes.c_double), ("budget_ms", ctypes.c_double), ("t_pred_ms", ctypes.c_double),
                ("n_tokens", ctypes.c_int64), ("l_context", ctypes.c_int64), ("evaluations", ctypes.c_int64),
                ("admitted", ctypes.c_int64)]


UTILITY_KINDS = {"linear": 0, "concave": 1, "table": 2}
PARTIAL_FORMATS = {"f16_scaled": 0, "f32": 1}


class TaperError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"taper_attn status {status}: {message}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_2605_06914_amd/build.py); there is no fallback path")
    try:  # share torch's HIP runtime (same soname) when torch is importable
        import torch  # noqa: F401
    except Exception:  # pragma: no cover - torch is only needed for device work
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.taper_create.argtypes = [ctypes.POINTER(taper_attn_config), ctypes.POINTER(vp)]
    lib.taper_destroy.argtypes = [vp]
    lib.taper_destroy.restype = None
    lib.taper_reserve.argtypes = [vp, ci, i64]
    lib.taper_plan_build.argtypes = [vp, ci, vp, ci, vp, vp, vp, i64, ctypes.POINTER(taper_plan_options), vp,
                                     ctypes.POINTER(vp)]
    lib.taper_plan_build_segments.argtypes = [vp, ci, vp, ci, vp, vp, vp, vp, i64, ctypes.POINTER(taper_plan_options), vp,
                                              ctypes.POINTER(vp)]
    lib.taper_append_slots.argtypes = [ci, vp, ci, vp, vp, vp, ci, i64, vp, vp]
    lib.taper_kv_append.argtypes = [vp, ci, vp, vp, vp, vp, vp]
    lib.taper_branch_blocks.argtypes = [i64, ci]
    lib.taper_branch_blocks.restype = i64
    lib.taper_plan_free.argtypes = [vp]
    lib.taper_plan_free.restype = None
    lib.taper_plan_export.argtypes = [vp, ctypes.POINTER(taper_plan_view)]
    lib.taper_plan_resolve_slots_host.argtypes = [vp, vp, i64]
    lib.taper_plan_resolve_slots.argtypes = [vp, vp, vp, i64, vp]
    lib.taper_decode_step_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.taper_decode_step_attention_simple.argtypes = [vp, ci, vp, vp, i64, vp, ci, vp, vp, vp, vp, vp]
    lib.taper_decode_step_attention_static.argtypes = [vp, ci, vp, vp, i64, vp, ci, vp, vp, vp, vp, vp]
    lib.taper_step_latency_probe.argtypes = [vp, vp, ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                             ci, ci, vp, ctypes.POINTER(taper_probe_result)]
    lib.taper_kernel_times.argtypes = [vp, vp, vp, vp, vp, ci, ci, vp, ctypes.POINTER(ctypes.c_double)]
    lib.taper_kernel_times_layers.argtypes = [vp, vp, ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ci, ci,
                                              vp, ctypes.POINTER(ctypes.c_double)]
    lib.taper_stream_read_probe.argtypes = [vp, vp, i64, i64, ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double)]
    dp, f64 = ctypes.POINTER(ctypes.c_double), ctypes.c_double
    pp = ctypes.POINTER(taper_predictor)
    lib.taper_predictor_fit.argtypes = [i64, vp, vp, vp, pp, dp]
    lib.taper_predictor_fit_monotone.argtypes = [i64, vp, vp, vp, pp, dp]
    lib.taper_window_fit_monotone.argtypes = [vp, pp, dp]
    lib.taper_predictor_eval.argtypes = [pp, f64, f64]
    lib.taper_predictor_eval.restype = f64
    lib.taper_predictor_mape.argtypes = [pp, i64, vp, vp, vp, dp]
    lib.taper_window_create.argtypes = [ctypes.c_int32, ctypes.POINTER(vp)]
    lib.taper_window_destroy.argtypes = [vp]
    lib.taper_window_destroy.restype = None
    lib.taper_window_push.argtypes = [vp, f64, f64, f64]
    lib.taper_window_size.argtypes = [vp]
    lib.taper_window_size.restype = ctypes.c_int32
    lib.taper_window_fit.argtypes = [vp, pp, dp]
    lib.taper_admit_step.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, ctypes.POINTER(taper_admission_options),
                                     vp, ctypes.POINTER(taper_admission_result)]
    lib.taper_strerror.argtypes = [ci]
    lib.taper_strerror.restype = ctypes.c_char_p
    lib.taper_last_error.restype = ctypes.c_char_p
    for name in EXPORTED:
        getattr(lib, name)
    _lib = lib
    return lib


def _check(status: int):
    if status != TAPER_OK:
        lib = load_library()
        msg = lib.taper_last_error().decode() or lib.taper_strerror(status).decode()
        raise TaperError(status, msg)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(t) -> int:
    """Device pointer of a torch tensor, or a raw int."""
    return int(t) if isinstance(t, int) else int(t.data_ptr())


def _dev(t, what: str, numel: int, dtype: str, device: int) -> int:
    """Device pointer of tensor `t` after checking what the C ABI cannot see from a bare pointer: element
    type, contiguity, device and size (an undersized, strided or wrong-device tensor would become an
    out-of-bounds access inside the kernel).  A raw int is passed through: the caller vouches for it."""
    if isinstance(t, int):
        return t
    if str(t.dtype).rsplit(".", 1)[-1] != dtype:
        raise TaperError(TAPER_EINVAL, f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TaperError(TAPER_EINVAL, f"{what} must be contiguous")
    if t.device.type != "cuda" or (t.device.index or 0) != device:
        raise TaperError(TAPER_EINVAL, f"{what} must live on cuda:{device}, got {t.device}")
    if t.numel() < numel:
        raise TaperError(TAPER_EINVAL, f"{what} holds {t.numel()} elements, the step needs {numel}")
    return int(t.data_ptr())


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(stream) if isinstance(stream, int) else int(stream.cuda_stream)


class Plan:
    """One decode step's integer metadata (taper_plan)."""

    def __init__(self, ctx: "Context", handle: int, n_seqs: int = 0, n_pool_pages: int = 0):
        self.ctx, self._h = ctx, handle
        self.n_seqs, self.n_pool_pages = int(n_seqs), int(n_pool_pages)

    def free(self):
        # a plan hands its buffers back to its context, so it must be freed first
        if self._h and self.ctx._h:
            load_library().taper_plan_free(self._h)
        self._h = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def export(self) -> dict:
        """taper_plan_export, copied into numpy arrays."""
        v = taper_plan_view()
        _check(load_library().taper_plan_export(self._h, ctypes.byref(v)))
        S, G = v.n_seqs, v.n_groups
        n_parts = v.n_parts_shared + v.n_parts_private
        arr = lambda p, n: np.ctypeslib.as_array(p, shape=(n,)).copy() if n else np.zeros(0, np.int32)
        items = np.ctypeslib.as_array(ctypes.cast(v.items, _I32P), shape=(v.n_items, 8)).copy()
        n_merge = int(arr(v.merge_start, S + 1)[-1])
        seg_start = arr(v.seg_start, S + 1)
        n_seg = int(seg_start[-1])
        merge = np.ctypeslib.as_array(ctypes.cast(v.merge, _I32P), shape=(n_merge, 2)).copy()
        return dict(n_seqs=S, n_groups=G, ctx_len=arr(v.ctx_len, S), n_prefix_pages=arr(v.n_prefix_pages, S),
                    n_suffix_pages=arr(v.n_suffix_pages, S), group_start=arr(v.group_start, G + 1),
                    seg_start=seg_start, seg_len=arr(v.seg_len, n_seg), seg_page0=arr(v.seg_page0, n_seg),
                    items=items, item_fields=[f[0] for f in taper_work_item._fields_],
                    n_pool_items=v.n_pool_items, n_parts_shared=v.n_parts_shared, n_parts_private=v.n_parts_private,
                    part_start=arr(v.part_start, n_parts + 1), merge_start=arr(v.merge_start, S + 1), merge=merge,
                    n_partial_rows=int(v.n_partial_rows), tokens_unique=int(v.tokens_unique),
                    tokens_logical=int(v.tokens_logical), workspace_id=int(v.workspace_id),
                    workspace_rows=int(v.workspace_rows))

    def resolve_slots_host(self, stride: int) -> np.ndarray:
        S = self.export()["n_seqs"]
        out = np.zeros((S, stride), np.int64)
        _check(load_library().taper_plan_resolve_slots_host(self._h, out.ctypes.data, stride))
        return out

    def resolve_slots(self, slots_dev, stride: int, stream=None):
        ptr = _dev(slots_dev, "slots", self.n_seqs * int(stride), "int64", self.ctx.cfg.device)
        _check(load_library().taper_plan_resolve_slots(self.ctx._h, self._h, ptr, stride, _stream(stream)))


class Context:
    """taper_ctx: shape + workspace.  device=-1 gives a host-only context."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, page_size: int = 16,
                 scale: Optional[float] = None, device: int = 0, partial_format="f16_scaled"):
        lib = load_library()
        pf = PARTIAL_FORMATS[partial_format] if isinstance(partial_format, str) else int(partial_format)
        cfg = taper_attn_config(n_q_heads, n_kv_heads, head_dim, page_size,
                                float(scale if scale is not None else head_dim ** -0.5), device, pf)
        h = ctypes.c_void_p()
        _check(lib.taper_create(ctypes.byref(cfg), ctypes.byref(h)))
        self._h = h.value
        self.cfg = cfg

    def close(self):
        if self._h:
            load_library().taper_destroy(self._h)
            self._h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reserve(self, max_seqs: int, max_partial_rows: int):
        """Size the workspace ahead of time so that no later plan_build allocates."""
        _check(load_library().taper_reserve(self._h, int(max_seqs), int(max_partial_rows)))

    def plan_build(self, block_table, branch_group, prefix_len, suffix_len, n_pool_pages: int,
                   target_workgroups: int = 0, share_prefix: bool = True, max_branches_per_item: int = 0,
                   shared_cost_pct: int = 0, shared_item_cost: int = 0, private_item_cost: int = 0,
                   pool_pct: int = 0, pool_item_tokens: int = 0, private_merge_cost: int = 0, solo_item_tokens: int = 0,
                   min_share_tokens: int = 0, scatter_sub_groups: bool = False, small_step_grid: int = 0, stream=None) -> Plan:
        bt = _i32(block_table)
        grp, pl, sl = _i32(branch_group), _i32(prefix_len), _i32(suffix_len)
        if bt.ndim != 2 or not (len(grp) == len(pl) == len(sl) == bt.shape[0]):
            raise TaperError(TAPER_EINVAL, "block_table must be [S, max_blocks] and the per-sequence arrays length S")
        opts = taper_plan_options(target_workgroups, int(share_prefix), max_branches_per_item, shared_cost_pct,
                                  shared_item_cost, private_item_cost, private_merge_cost, solo_item_tokens,
                                  min_share_tokens, pool_pct, pool_item_tokens, small_step_grid, int(scatter_sub_groups))
        h = ctypes.c_void_p()
        st = 0 if self.cfg.device < 0 else _stream(stream)
        _check(load_library().taper_plan_build(self._h, bt.shape[0], bt.ctypes.data, bt.shape[1], grp.ctypes.data,
                                               pl.ctypes.data, sl.ctypes.data, int(n_pool_pages), ctypes.byref(opts),
                                               st, ctypes.byref(h)))
        return Plan(self, h.value, bt.shape[0], n_pool_pages)

    def plan_build_segments(self, block_table, branch_group, prefix_len, seg_start, seg_len, n_pool_pages: int,
                            stream=None, **options) -> Plan:
        """Plan for sequences that see their prefix and then a list of private segments (reduce phase)."""
        bt = _i32(block_table)
        grp, pl, ss, sl = _i32(branch_group), _i32(prefix_len), _i32(seg_start), _i32(seg_len)
        if bt.ndim != 2 or not (len(grp) == len(pl) == bt.shape[0] == len(ss) - 1) or (len(ss) and ss[-1] != len(sl)):
            raise TaperError(TAPER_EINVAL, "block_table must be [S, max_blocks], seg_start length S + 1 ending at len(seg_len)")
        names = ["target_workgroups", "share_prefix", "max_branches_per_item", "shared_cost_pct", "shared_item_cost",
                 "private_item_cost", "private_merge_cost", "solo_item_tokens", "min_share_tokens", "pool_pct",
                 "pool_item_tokens", "small_step_grid", "scatter_sub_groups"]
        vals = {n: 0 for n in names}
        vals["share_prefix"] = 1
        for k, v in options.items():
            if k not in vals:
                raise TypeError(f"unknown plan option {k}")
            vals[k] = int(v)
        opts = taper_plan_options(*[vals[n] for n in names])
        h = ctypes.c_void_p()
        st = 0 if self.cfg.device < 0 else _stream(stream)
        _check(load_library().taper_plan_build_segments(self._h, bt.shape[0], bt.ctypes.data, bt.shape[1], grp.ctypes.data,
                                                        pl.ctypes.data, ss.ctypes.data, sl.ctypes.data if len(sl) else None,
                                                        int(n_pool_pages), ctypes.byref(opts), st, ctypes.byref(h)))
        return Plan(self, h.value, bt.shape[0], n_pool_pages)

    # elements of the tensors of a step of n_seqs sequences over a pool of n_pool_pages pages
    def _qo_elems(self, n_seqs: int) -> int:
        return int(n_seqs) * self.cfg.n_q_heads * self.cfg.head_dim

    def _kv_row_elems(self, n_seqs: int) -> int:
        return int(n_seqs) * self.cfg.n_kv_heads * self.cfg.head_dim

    def _pool_elems(self, n_pool_pages: int) -> int:
        return int(n_pool_pages) * 2 * self.cfg.n_kv_heads * self.cfg.page_size * self.cfg.head_dim

    def _step_ptrs(self, n_seqs, n_pool_pages, q, kv_pages, out, lse=None):
        d = self.cfg.device
        return (_dev(q, "q", self._qo_elems(n_seqs), "bfloat16", d),
                _dev(kv_pages, "kv_pages", self._pool_elems(n_pool_pages), "bfloat16", d),
                _dev(out, "out", self._qo_elems(n_seqs), "bfloat16", d),
                _dev(lse, "lse", int(n_seqs) * self.cfg.n_q_heads, "float32", d) if lse is not None else None)

    def kv_append(self, k_new, v_new, slots_dev, kv_pages, n_seqs: int, stream=None, n_pool_pages: int = 0):
        """n_pool_pages (optional): the pool's size, so that the pool tensor's size can be checked too."""
        d = self.cfg.device
        _check(load_library().taper_kv_append(self._h, int(n_seqs),
                                              _dev(k_new, "k_new", self._kv_row_elems(n_seqs), "bfloat16", d),
                                              _dev(v_new, "v_new", self._kv_row_elems(n_seqs), "bfloat16", d),
                                              _dev(slots_dev, "slots", int(n_seqs), "int64", d),
                                              _dev(kv_pages, "kv_pages", self._pool_elems(n_pool_pages), "bfloat16", d),
                                              _stream(stream)))

    def decode_step_attention(self, plan: Plan, q, kv_pages, out, lse=None, stream=None):
        pq, pkv, pout, plse = self._step_ptrs(plan.n_seqs, plan.n_pool_pages, q, kv_pages, out, lse)
        _check(load_library().taper_decode_step_attention(self._h, plan._h, pq, pkv, pout, plse, _stream(stream)))

    def decode_step_attention_simple(self, q, kv_pages, n_pool_pages, block_table, branch_group, prefix_len,
                                     suffix_len, out, stream=None):
        bt = _i32(block_table)
        grp, pl, sl = _i32(branch_group), _i32(prefix_len), _i32(suffix_len)
        pq, pkv, pout, _ = self._step_ptrs(bt.shape[0], n_pool_pages, q, kv_pages, out)
        _check(load_library().taper_decode_step_attention_simple(
            self._h, bt.shape[0], pq, pkv, int(n_pool_pages), bt.ctypes.data, bt.shape[1],
            grp.ctypes.data, pl.ctypes.data, sl.ctypes.data, pout, _stream(stream)))

    def decode_step_attention_static(self, q, kv_pages, n_pool_pages, block_table, branch_group, prefix_len,
                                     suffix_len, out, stream=None):
        """The same step through the library's static scratch array: allocates nothing, enqueues only."""
        bt = _i32(block_table)
        grp, pl, sl = _i32(branch_group), _i32(prefix_len), _i32(suffix_len)
        pq, pkv, pout, _ = self._step_ptrs(bt.shape[0], n_pool_pages, q, kv_pages, out)
        _check(load_library().taper_decode_step_attention_static(
            self._h, bt.shape[0], pq, pkv, int(n_pool_pages), bt.ctypes.data, bt.shape[1],
            grp.ctypes.data, pl.ctypes.data, sl.ctypes.data, pout, _stream(stream)))

    def step_latency_probe(self, plan: Plan, q_layers: Sequence, kv_layers: Sequence, out_layers: Sequence,
                           warmup: int = 10, iters: int = 50, stream=None) -> taper_probe_result:
        n = len(q_layers)
        assert len(kv_layers) == n and len(out_layers) == n
        for l in range(n):
            self._step_ptrs(plan.n_seqs, plan.n_pool_pages, q_layers[l], kv_layers[l], out_layers[l])
        mk = lambda ts: (ctypes.c_void_p * n)(*[_ptr(t) for t in ts])
        res = taper_probe_result()
        _check(load_library().taper_step_latency_probe(self._h, plan._h, n, mk(q_layers), mk(kv_layers),
                                                       mk(out_layers), warmup, iters, _stream(stream),
                                                       ctypes.byref(res)))
        return res

    def kernel_times(self, plan: Plan, q, kv_pages, out, warmup: int = 5, iters: int = 20, stream=None):
        us = (ctypes.c_double * 2)()
        pq, pkv, pout, _ = self._step_ptrs(plan.n_seqs, plan.n_pool_pages, q, kv_pages, out)
        _check(load_library().taper_kernel_times(self._h, plan._h, pq, pkv, pout, warmup, iters, _stream(stream), us))
        return dict(decode_us=us[0], decode_us_min=us[1])

    def kernel_times_layers(self, plan: Plan, q_layers: Sequence, kv_layers: Sequence, out_layers: Sequence,
                            warmup: int = 5, iters: int = 20, stream=None):
        """Launch i runs on layer i mod len(layers): distinct pools, so no launch reuses cached KV of an earlier one."""
        n = len(q_layers)
        assert len(kv_layers) == n and len(out_layers) == n
        for l in range(n):
            self._step_ptrs(plan.n_seqs, plan.n_pool_pages, q_layers[l], kv_layers[l], out_layers[l])
        mk = lambda ts: (ctypes.c_void_p * n)(*[_ptr(t) for t in ts])
        us = (ctypes.c_double * 2)()
        _check(load_library().taper_kernel_times_layers(self._h, plan._h, n, mk(q_layers), mk(kv_layers), mk(out_layers),
                                                        warmup, iters, _stream(stream), us))
        return dict(decode_us=us[0], decode_us_min=us[1])

    def stream_read_probe(self, buf, pass_bytes: int, n_workgroups: int = 512, warmup: int = 2, iters: int = 8, stream=None):
        """Plain streaming read of `pass_bytes` per launch out of the device tensor `buf` (launches rotate over the
        tensor).  Returns dict(us, us_min, gbps)."""
        nbytes = buf.numel() * buf.element_size()
        us = (ctypes.c_double * 2)()
        _check(load_library().taper_stream_read_probe(self._h, _ptr(buf), nbytes, pass_bytes, n_workgroups, warmup, iters,
                                                      _stream(stream), us))
        return dict(us=us[0], us_min=us[1], gbps=pass_bytes / us[0] / 1e3)


# ----------------------------------------------------------------------------- controller side (host only)
def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def predictor_fit(n_tokens, l_context, t_ms, monotone: bool = False):
    """(a, b, c) of T = a + b n_tokens + c L_context by least squares (under b, c >= 0 if monotone), and the
    fit's MAPE in percent."""
    lib = load_library()
    n, L, t = _f64(n_tokens), _f64(l_context), _f64(t_ms)
    if not (n.shape == L.shape == t.shape and n.ndim == 1):
        raise ValueError("n_tokens, l_context, t_ms must be 1-D arrays of one length")
    p, m = taper_predictor(), ctypes.c_double()
    fit = lib.taper_predictor_fit_monotone if monotone else lib.taper_predictor_fit
    _check(fit(len(n), n.ctypes.data, L.ctypes.data, t.ctypes.data, ctypes.byref(p), ctypes.byref(m)))
    return (p.a, p.b, p.c), m.value


def predictor_eval(coef, n_tokens, l_context) -> float:
    return load_library().taper_predictor_eval(ctypes.byref(taper_predictor(*coef)), float(n_tokens), float(l_context))


def predictor_mape(coef, n_tokens, l_context, t_ms) -> float:
    lib = load_library()
    n, L, t = _f64(n_tokens), _f64(l_context), _f64(t_ms)
    m = ctypes.c_double()
    _check(lib.taper_predictor_mape(ctypes.byref(taper_predictor(*coef)), len(n), n.ctypes.data, L.ctypes.data,
                                    t.ctypes.data, ctypes.byref(m)))
    return m.value


class Window:
    """The most recent `capacity` observed steps; fit() refreshes the predictor from them."""

    def __init__(self, capacity: int = 200):
        self._lib = load_library()
        h = ctypes.c_void_p()
        _check(self._lib.taper_window_create(capacity, ctypes.byref(h)))
        self._h = h

    def push(self, n_tokens, l_context, t_ms):
        _check(self._lib.taper_window_push(self._h, float(n_tokens), float(l_context), float(t_ms)))

    def __len__(self):
        return self._lib.taper_window_size(self._h)

    def fit(self, monotone: bool = False):
        p, m = taper_predictor(), ctypes.c_double()
        fit = self._lib.taper_window_fit_monotone if monotone else self._lib.taper_window_fit
        _check(fit(self._h, ctypes.byref(p), ctypes.byref(m)))
        return (p.a, p.b, p.c), m.value

    def close(self):
        if self._h:
            self._lib.taper_window_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def admit_step(coef, base_context, slack_ms, branch_context, rho=1.0, utility="linear", weight=None, utility_table=None):
    """One planner invocation.  branch_context: per request, the context lengths of its ready branches in
    admission order.  utility_table (for utility="table"): per request u(0..ready).  Returns (granted, result dict)."""
    lib = load_library()
    R = len(base_context)
    base = np.ascontiguousarray(base_context, dtype=np.int64)
    slack = _f64(slack_ms)
    start = np.zeros(R + 1, np.int32)
    start[1:] = np.cumsum([len(b) for b in branch_context])
    flat = np.ascontiguousarray([c for b in branch_context for c in b], dtype=np.int64)
    w = _f64(weight) if weight is not None else None
    tab = _f64([u for t in utility_table for u in t]) if utility_table is not None else None
    if tab is not None and len(tab) != int(start[-1]) + R:
        raise ValueError("utility_table needs ready + 1 entries per request")
    if len(slack) != R or len(branch_context) != R or (w is not None and len(w) != R):
        raise ValueError("per-request arrays differ in length")
    granted = np.zeros(R, np.int32)
    opts = taper_admission_options(float(rho), UTILITY_KINDS[utility], 0)
    res = taper_admission_result()
    _check(lib.taper_admit_step(ctypes.byref(taper_predictor(*coef)), R, base.ctypes.data, slack.ctypes.data,
                                start.ctypes.data, flat.ctypes.data if len(flat) else None,
                                w.ctypes.data if w is not None else None, tab.ctypes.data if tab is not None else None,
                                ctypes.byref(opts), granted.ctypes.data, ctypes.byref(res)))
    return granted, {f[0]: getattr(res, f[0]) for f in taper_admission_result._fields_}


def append_slots(block_table, prefix_len, seg_start, seg_len, page_size: int, n_pool_pages: int):
    """Where each sequence's next token goes: (slots int64 [S], opens_page int32 [S])."""
    bt = _i32(block_table)
    pl, ss, sl = _i32(prefix_len), _i32(seg_start), _i32(seg_len)
    S = bt.shape[0]
    if len(pl) != S or len(ss) != S + 1 or ss[-1] != len(sl):
        raise TaperError(TAPER_EINVAL, "per-sequence arrays do not match the block table")
    slots = np.zeros(S, np.int64)
    opens = np.zeros(S, np.int32)
    _check(load_library().taper_append_slots(S, bt.ctypes.data, bt.shape[1], pl.ctypes.data, ss.ctypes.data,
                                             sl.ctypes.data if len(sl) else None, page_size, int(n_pool_pages),
                                             slots.ctypes.data, opens.ctypes.data))
    return slots, opens


def branch_blocks(branch_local_tokens: int, page_size: int = 16) -> int:
    return int(load_library().taper_branch_blocks(int(branch_local_tokens), page_size))
