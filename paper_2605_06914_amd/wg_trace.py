"""Development aid: where the time of one decode launch goes, workgroup by workgroup.

Runs workloads through a TRACE BUILD of the library (build.py --trace: the same sources with
-DTAPER_WG_TRACE, which makes every workgroup of the decode kernel record when it started,
when its shared-prefix share was done, when it left, and how long it spent merging) and
prints the launch's span, how evenly the workgroups end, and the last ones to finish.  The
trace build is a few percent slower than the product build; its figures are for comparing
workgroups with each other, not launches with the bench.

    python -m paper_2605_06914_amd.wg_trace mixed irp_off long k4 [--kw '{"pool_pct": 40}'] [--verbose]

Workloads: mixed, irp_off, long, k<K> (admission sweep at width 1+K), w<N> (the mixed shape with
N branches per parallel request), b<N>x<C> (N serial requests of C tokens).  Needs a GPU; build the trace library first (on the CPU):
    python paper_2605_06914_amd/build.py --trace
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def structure(name):
    from taper_inputs import (structure_config2, structure_config3, structure_config4, structure_config5,
                              structure_custom)
    from taper_inputs.generators import QWEN

    if name == "mixed":
        return structure_config3()
    if name == "irp_off":
        return structure_config2()
    if name == "long":
        return structure_config4()
    if name.startswith("k"):
        return structure_config5(int(name[1:]))
    if name.startswith("w"):
        from taper_inputs import structure_wide

        return structure_wide(int(name[1:]))
    if name.startswith("b"):
        n, c = name[1:].split("x")
        return structure_custom(QWEN, [(int(c), [0])] * int(n), seed=1)
    raise SystemExit(f"unknown workload {name}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workloads", nargs="+")
    ap.add_argument("--kw", default="{}", help="plan options as JSON")
    ap.add_argument("--partial-format", default="f16_scaled")
    ap.add_argument("--verbose", action="store_true", help="one line per workgroup share")
    args = ap.parse_args()
    kw = json.loads(args.kw)

    from paper_2605_06914_amd import binding
    from paper_2605_06914_amd.build import TRACE_LIB

    if not os.path.exists(TRACE_LIB):
        raise SystemExit(f"{TRACE_LIB} is missing: run `python paper_2605_06914_amd/build.py --trace` first")
    binding.LIB_PATH = TRACE_LIB
    import torch

    lib = binding.load_library()
    lib.taper_wg_trace_buffer.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    dev = torch.device("cuda:0")
    for wl in args.workloads:
        st = structure(wl)
        sh = st.shape
        n_pools = 1 if st.n_pool_pages > 100000 else 3  # rotate pools so that no launch finds its KV in the Infinity Cache
        qs = [torch.randn((st.n_seqs, sh.n_q_heads, sh.head_dim), device=dev).to(torch.bfloat16) for _ in range(n_pools)]
        kvs = [torch.empty(st.n_pool_pages * sh.page_elems, device=dev, dtype=torch.bfloat16).normal_() for _ in range(n_pools)]
        out = torch.zeros_like(qs[0])
        ctx = binding.Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, device=0, partial_format=args.partial_format)
        plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **kw)
        e = plan.export()
        n_parts = e["n_parts_shared"] + e["n_parts_private"]
        nwg = n_parts * sh.n_kv_heads
        trace = torch.zeros(4 * nwg + 64, dtype=torch.int64, device=dev)
        binding._check(lib.taper_wg_trace_buffer(ctx._h, trace.data_ptr()))
        runs = []
        for it in range(8):
            trace.zero_()
            ctx.decode_step_attention(plan, qs[it % n_pools], kvs[it % n_pools], out)
            torch.cuda.synchronize()
            t = trace.cpu().numpy()[: 4 * nwg].reshape(nwg, 4).astype(np.float64) / 100.0  # 100 MHz clock -> us
            t[:, :3] -= t[:, 0].min()
            if it >= 2:
                runs.append(t)
        t = np.mean(runs, axis=0)
        start, own, end, mrg = t[:, 0], t[:, 1], t[:, 2], t[:, 3]
        span = end.max()
        nsh = e["n_parts_shared"] * sh.n_kv_heads
        print(f"{wl} {kw}: {nwg} workgroups ({nsh} with a shared-prefix share), {e['n_pool_items']} pool items; span {span:.1f} us; "
              f"workgroups leave at min/median/max {end.min():.1f}/{np.median(end):.1f}/{end.max():.1f} us; mean busy "
              f"{np.mean(end - start) / span * 100:.0f} %; {st.kv_bytes_unique / span / 8e6 * 100:.1f} % of 8 TB/s at this span")
        last = np.argsort(-end)[:16]
        print("   last to leave: " + " ".join(
            f"[{'S' if i < nsh else 'P'}{i // sh.n_kv_heads} own {own[i]:.0f} end {end[i]:.0f} merge {mrg[i]:.0f}]" for i in last))
        print(f"   time in merges per workgroup: mean {mrg.mean():.1f} max {mrg.max():.1f} us; leave-time histogram (5 us bins from "
              f"{5 * int(end.min() // 5)}): {np.histogram(end, bins=np.arange(5 * int(end.min() // 5), span + 5, 5))[0]}")
        if nsh:
            print(f"   shared shares done at median {np.median(own[:nsh]):.1f} max {own[:nsh].max():.1f} us "
                  f"(merges of the item's branches included)")
        if args.verbose:
            F = {n: i for i, n in enumerate(e["item_fields"])}
            ps, items = e["part_start"], e["items"]
            E, M, O = (x.reshape(n_parts, sh.n_kv_heads) for x in (end, mrg, own))
            print("   mean leave time by kv head:", np.round(E.mean(axis=0), 1))
            for p in range(n_parts):
                its = items[ps[p]: ps[p + 1]]
                print(f"   share {p:3d} {'S' if p < e['n_parts_shared'] else 'P'} items {len(its):2d} tokens {int(its[:, F['n_tokens']].sum()):6d} "
                      f"branches {int(its[:, F['n_branch']].max()):2d} own done {O[p].mean():5.1f} leave mean {E[p].mean():5.1f} "
                      f"max {E[p].max():5.1f} merge {M[p].mean():4.1f}")
        binding._check(lib.taper_wg_trace_buffer(ctx._h, None))
        plan.free()
        ctx.close()
        del kvs, qs
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
