#!/usr/bin/env python3
"""Benchmark of the decode-step attention hot path on one MI355X.

A *step* is one decode step of a layer stack over one synthetic batch: the index
resolution / plan build (once per step, inside the timed region) followed by the
attention of every layer (one launch: shared-prefix work, private work, merge), each
layer reading its own KV pool.  Inputs are resident in HBM before the timed
region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixed|irp_off|long] [--layers L]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="mixed", choices=["mixed", "irp_off", "long", "tiny", "sweep"])
    ap.add_argument("--layers", type=int, default=0, help="layers per step (0 = workload default)")
    ap.add_argument("--target-workgroups", type=int, default=0)
    ap.add_argument("--shared-cost-pct", type=int, default=0)
    ap.add_argument("--no-share", action="store_true", help="every branch streams its prefix itself (for comparison)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-iters", type=int, default=50)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times: scales the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--sweep-pools", type=int, default=16, help="distinct KV pools the 64 layers of the sweep cycle through")
    return ap.parse_args()


def make_structure(name):
    from taper_inputs import structure_config1, structure_config2, structure_config3, structure_config4

    return {"tiny": structure_config1, "irp_off": structure_config2, "mixed": structure_config3,
            "long": structure_config4}[name]()


def run_sweep(args):
    """Admission sweep (paper §2.3: branch externality E(k) = T(S(k)) - T(S_0)): 96 serial + 32 parallel
    requests on a 64-layer stack; every parallel request runs its protected branch plus k opportunistic
    ones, k in {0,2,4,8,16}.  64 independent pools of this size do not fit one GPU (k=16: 64 x 5.6 GB), so
    layer l reads pool l mod --sweep-pools; each layer's working set (3-5 GB) is far beyond the 256 MB
    Infinity Cache, so reuse of a pool 16 layers later cannot hit in cache."""
    import torch

    from paper_2605_06914_amd import Context
    from taper_inputs import structure_config5

    dev = torch.device("cuda:0")
    n_layers = args.layers or 64
    sts = {k: structure_config5(k) for k in (0, 2, 4, 8, 16)}
    sh = sts[0].shape
    n_pool_pages = sts[16].n_pool_pages
    assert all(st.n_pool_pages == n_pool_pages for st in sts.values())
    gen = torch.Generator(device=dev)
    gen.manual_seed(sts[0].seed + 1000)
    pool_elems = n_pool_pages * sh.page_elems
    pools = []
    for _ in range(args.sweep_pools):
        kv = torch.empty(pool_elems, device=dev, dtype=torch.bfloat16)
        chunk = 1 << 28
        for o in range(0, pool_elems, chunk):
            n = min(chunk, pool_elems - o)
            kv[o : o + n] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        pools.append(kv)
    s_max = sts[16].n_seqs
    qs = [torch.randn((s_max, sh.n_q_heads, sh.head_dim), generator=gen, device=dev).to(torch.bfloat16)
          for _ in range(n_layers)]
    outs = [torch.zeros((s_max, sh.n_q_heads, sh.head_dim), device=dev, dtype=torch.bfloat16) for _ in range(n_layers)]
    kvs = [pools[l % args.sweep_pools] for l in range(n_layers)]
    torch.cuda.synchronize()
    ctx = Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, device=0)
    rows = []
    for k, st in sts.items():
        def step():
            plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages,
                                  target_workgroups=args.target_workgroups, shared_cost_pct=args.shared_cost_pct)
            for l in range(n_layers):
                ctx.decode_step_attention(plan, qs[l], kvs[l], outs[l])
            plan.free()

        for _ in range(max(1, args.warmup)):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        gbps = (st.kv_bytes_unique + st.qo_bytes) * n_layers / (ms * 1e-3) / 1e9
        rows.append({"k": k, "admitted_branches": 32 * k, "n_seqs": st.n_seqs, "l_context": st.logical_tokens,
                     "tokens_unique": st.unique_tokens, "ms_per_step": round(ms, 3), "gbps_unique": round(gbps, 1),
                     "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)})
    t_base = rows[0]["ms_per_step"]
    for r, st in zip(rows, sts.values()):
        r["externality_ms"] = round(r["ms_per_step"] - t_base, 3)
        if r["k"]:
            # marginal cost of one admitted branch per layer, beside the bytes it adds (its private suffix:
            # the prefix is already streamed for the protected branch)
            r["externality_us_per_branch_layer"] = round((r["ms_per_step"] - t_base) * 1e3 / (32 * r["k"]) / n_layers, 4)
            r["kv_bytes_added_per_branch_layer"] = int((st.kv_bytes_unique - sts[0].kv_bytes_unique) / (32 * r["k"]))
    ctx.close()
    return rows, n_layers, sh


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one MI355X: this build has no multi-GPU path (see DESIGN.md, 'How it would shard'); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2605_06914_amd import Context
    from taper_inputs import compact_rows, f32_from_bf16_bits

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": 5}}))
        return
    if args.workload == "sweep":
        rows, n_layers, sh = run_sweep(args)
        top = rows[-1]
        print(json.dumps({
            "metric": "decode_step_attention_effective_kv_bandwidth", "value": top["gbps_unique"], "unit": "GB/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": top["ms_per_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"config5 admission sweep x {n_layers} layers, value quoted at k=16 "
                                   f"({args.sweep_pools} distinct KV pools cycled over the layers)",
                       "n_layers": n_layers},
            "step_latency_vs_admitted_branches": rows}))
        return
    st = make_structure(args.workload)
    sh = st.shape
    # default depth: the 64-layer stack of the model the shape comes from; the long workload's pool is
    # ~30 GB per layer, so it runs a shallower stack
    n_layers = args.layers or {"mixed": 64, "irp_off": 64, "long": 4, "tiny": 64}[args.workload]
    pool_elems = st.n_pool_pages * sh.page_elems
    gen = torch.Generator(device=dev)
    gen.manual_seed(st.seed + 1000)
    qs, kvs, outs = [], [], []
    for _ in range(n_layers):
        qs.append(torch.randn((st.n_seqs, sh.n_q_heads, sh.head_dim), generator=gen, device=dev,
                              dtype=torch.float32).to(torch.bfloat16))
        kv = torch.empty(pool_elems, device=dev, dtype=torch.bfloat16)
        chunk = 1 << 28
        for o in range(0, pool_elems, chunk):
            n = min(chunk, pool_elems - o)
            kv[o : o + n] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        kvs.append(kv)
        outs.append(torch.zeros((st.n_seqs, sh.n_q_heads, sh.head_dim), device=dev, dtype=torch.bfloat16))
    torch.cuda.synchronize()

    ctx = Context(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, device=0)
    plan_kw = dict(target_workgroups=args.target_workgroups, share_prefix=not args.no_share,
                   shared_cost_pct=args.shared_cost_pct)

    def step():
        plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **plan_kw)
        for l in range(n_layers):
            ctx.decode_step_attention(plan, qs[l], kvs[l], outs[l])
        plan.free()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    bytes_step = (st.kv_bytes_unique + st.qo_bytes) * n_layers
    value = bytes_step / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel durations (HIP events on the launch stream) and the plan-free probe
    plan = ctx.plan_build(st.block_table, st.branch_group, st.prefix_len, st.suffix_len, st.n_pool_pages, **plan_kw)
    e = plan.export()
    F = {n: i for i, n in enumerate(e["item_fields"])}
    tok_shared = int(e["items"][e["items"][:, F["kind"]] == 0, F["n_tokens"]].sum())
    tok_private = int(e["items"][e["items"][:, F["kind"]] == 1, F["n_tokens"]].sum())
    kt = {"decode_us": 0.0, "decode_us_min": 0.0}
    n_kt = min(n_layers, 8)
    for l in range(n_kt):
        r = ctx.kernel_times(plan, qs[l], kvs[l], outs[l], warmup=10, iters=args.kernel_iters)
        for k in kt:
            kt[k] += r[k] / n_kt
    probe = ctx.step_latency_probe(plan, qs, kvs, outs, warmup=2, iters=max(5, args.steps))
    # algorithmic bytes of one launch: every unique KV token once (a shared prefix once per request) plus
    # q read and out written; the plan may list a prefix more than once (requests wider than one
    # workgroup's row tiles are cut into sub-groups), which is reported beside it, not counted
    dom_bytes = st.kv_bytes_unique + st.qo_bytes
    achieved = dom_bytes / (kt["decode_us"] * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": "decode_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                "bytes_per_launch": dom_bytes, "kv_bytes_listed_by_plan": (tok_shared + tok_private) * sh.kv_bytes_per_token,
                "avg_launch_us": round(kt["decode_us"], 2),
                "kernel_us": {k: round(v, 2) for k, v in kt.items()},
                "workgroups": (e["n_parts_shared"] + e["n_parts_private"]) * sh.n_kv_heads,
                "pool_items": e["n_pool_items"]}

    # HBM bytes per launch as the profiler's counters saw them (a stored profile of this kernel and workload,
    # see profiles/; counters cannot be read from inside this process)
    tf = os.path.join(ROOT, "profiles", "decode_kernel_traffic.json")
    if os.path.exists(tf) and not args.no_share and not args.target_workgroups and not args.shared_cost_pct:
        t = json.load(open(tf)).get(args.workload)
        if t:
            roofline["traffic"] = t["fetch_bytes"] + t["write_bytes"]
            roofline["traffic_detail"] = {"fetch_bytes": t["fetch_bytes"], "write_bytes": t["write_bytes"],
                                          "source": "profiles/decode_kernel_%s.md" % args.workload}

    # ---- CPU oracle on a bounded sample of the same workload (rank 0, N=1)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        # whole batch of layer 0 when it is small enough, else serial requests thinned out and the first and
        # last branch of each parallel request, capped at `budget` logical tokens (~10-30 core-seconds)
        budget = 2_000_000
        if st.logical_tokens <= budget:
            rows = np.arange(st.n_seqs)
        else:
            rows = []
            serial = [s for s in range(st.n_seqs) if np.sum(st.branch_group == st.branch_group[s]) == 1]
            rows += serial[:: max(1, len(serial) // 8)][:8]
            for g in range(st.n_groups):
                m = np.flatnonzero(st.branch_group == g)
                if len(m) > 1:
                    rows += [int(m[0]), int(m[-1])]
            rows = np.array(sorted(set(rows)))
            ctxlen = (st.prefix_len + st.suffix_len)[rows]
            keep = np.cumsum(ctxlen) <= budget
            keep[0] = True
            rows = rows[keep]
        sub, pages = compact_rows(st, rows)
        pg = torch.from_numpy(pages).to(dev)
        kv_host = kvs[0].view(st.n_pool_pages, sh.page_elems)[pg].view(torch.int16).cpu().numpy().view(np.uint16)
        q_host = qs[0][torch.from_numpy(rows).to(dev)].view(torch.int16).cpu().numpy().view(np.uint16)
        t1 = time.perf_counter()
        ref, _, _, used = oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, q_host,
                                           kv_host, sub.block_table, sub.prefix_len, sub.suffix_len, want_lse=False)
        t_cpu = time.perf_counter() - t1
        # same rows from the GPU run of layer 0 (outs[0] holds the last step's result)
        ctx.decode_step_attention(plan, qs[0], kvs[0], outs[0])
        torch.cuda.synchronize()
        got = f32_from_bf16_bits(outs[0][torch.from_numpy(rows).to(dev)].view(torch.int16).cpu().numpy().view(np.uint16))
        err = np.abs(got.astype(np.float64) - ref)
        scale_up = st.logical_tokens / sub.logical_tokens
        t_full = t_cpu * scale_up  # one layer of the full batch, no prefix sharing in the oracle
        cpu = {"value": round((st.kv_bytes_unique + st.qo_bytes) / t_full / 1e9, 4), "unit": "GB/s", "cores": int(used),
               "kind": "oracle",
               "sample": f"{len(rows)} of {st.n_seqs} sequences of layer 0 (whole batch if at most {budget} logical tokens, "
                         f"else thinned serial requests plus first and last branch of each parallel request), all heads: "
                         f"{sub.logical_tokens} logical tokens in {t_cpu:.2f} s; scaled by {scale_up:.2f} "
                         f"(logical tokens of the batch / of the sample) to one layer",
               "max_abs_err_gpu_vs_oracle": float(err.max()), "mean_abs_err_gpu_vs_oracle": float(err.mean())}
        assert err.max() <= 2e-2 and err.mean() <= 2e-3, "GPU result of the benchmarked workload is off the oracle"
    plan.free()

    line = {
        "metric": "decode_step_attention_effective_kv_bandwidth",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{st.name} x {n_layers} layers (Qwen3-32B attention shape: {sh.n_q_heads} q heads, "
                               f"{sh.n_kv_heads} kv heads, head_dim {sh.head_dim}, page {sh.page_size}; plan built once "
                               f"per step inside the timed region; one KV pool per layer)",
                   "n_layers": n_layers, "n_seqs": st.n_seqs, "n_requests": st.n_groups,
                   "admitted_branches": int(st.n_seqs - st.n_groups),
                   "tokens_unique": st.unique_tokens, "tokens_logical": st.logical_tokens,
                   "kv_bytes_unique_per_layer": st.kv_bytes_unique, "kv_bytes_logical_per_layer": st.kv_bytes_logical,
                   "share_prefix": not args.no_share},
        "us_per_layer": round(ms_per_step * 1e3 / n_layers, 2),
        "frac_of_hbm_peak_whole_step": round(value / HBM_PEAK_GBPS, 4),
        "logical_gbps": round(st.kv_bytes_logical * n_layers / (ms_per_step * 1e-3) / 1e9, 1),
        "probe": {"us_per_layer_median": round(probe.us_median / n_layers, 2),
                  "us_per_layer_min": round(probe.us_min / n_layers, 2), "gbps_unique": round(probe.gbps_unique, 1)},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    ctx.close()


if __name__ == "__main__":
    main()
