#!/usr/bin/env python3
"""Benchmark of the block-sparse video attention hot path on one MI355X.

A step is one pass of the whole path over one synthetic Wan2.1-1.3B 480p attention layer
(usv_block_scores -> usv_select_topk -> usv_block_sparse_attn, 10 % of the key blocks kept),
with Q/K/V already resident in HBM.  Prints ONE JSON line:
  value        effective TFLOP/s of a step, counting only the computed 64x64 tiles (4*64*64*d flop each)
  ms_per_step  milliseconds per step (the three calls back to back)
  roofline     the attention kernel against the bf16 MFMA peak, timed with events on the launch stream
  cpu_baseline the fp64 CPU oracle on a bounded sample of the same workload (context, not the target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "ms/call + effective TFLOP/s (computed tiles) of sparse attn, Wan-1.3B 480p, 10% keep"
PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="wan13_480p",
                    choices=["wan13_480p", "wan14_720p", "merged_ragged", "tiny",
                             "sweep100", "sweep50", "sweep25", "sweep10", "sweep5"])
    ap.add_argument("--out-dtype", default="f32", choices=["f32", "bf16"],
                    help="storage type of the attention output (inputs are the workload's dtype)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (untimed) so that a rocprofv3 --pmc run of this "
                         "command shows what FETCH_SIZE / WRITE_SIZE read for a kernel of known traffic")
    ap.add_argument("--cpu-sample-heads", type=int, default=12)
    ap.add_argument("--no-work-order", action="store_true",
                    help="ragged budgets / the 720p shape: plain usv_block_sparse_attn (query blocks in index order) instead "
                         "of usv_attn_work_order + usv_block_sparse_attn_ordered")
    ap.add_argument("--path", default="attention", choices=["attention", "reorder", "two_branch", "merge", "raster", "raster_two_branch", "raster_cubes"],
                    help="attention: the three-stage hot path (the headline metric); reorder: the raster <-> "
                         "cube-major token reorder either side of it (gather Q, K, V + scatter O); two_branch: the "
                         "hot path with the local cube forced into every list, plus the cube-level branch and the "
                         "gated fusion of the two outputs; merge: token merging (similarity, plan, merge Q/K/V, "
                         "unmerge O) with half of the tokens merged; raster: the three-stage hot path on RASTER-order Q, K, V "
                         "(usv_block_scores_raster, usv_select_topk, usv_block_sparse_attn_raster: no reordered copies); "
                         "raster_two_branch: the two_branch path on raster-order tensors")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (the three calls) in a HIP graph and time --steps replays of it; the per-stage "
                         "times then come from a second, eager pass (attention and raster paths only)")
    ap.add_argument("--merge-plan-one-workgroup", action="store_true",
                    help="--path merge: usv_merge_plan without a workspace (one workgroup per batch element instead of "
                         "the radix select spread over the chip)")
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="untimed steps run ahead of the --warmup steps until this much GPU time has passed: after an "
                         "idle period the chip takes some 50 ms of sustained load to reach its steady clock, and a short "
                         "--warmup would otherwise time the ramp; 0 switches it off")
    ap.add_argument("--no-mfma-peak", action="store_true",
                    help="skip the MFMA-only peak probe (paper_2512_05754_amd/tools/mfma_peak, ~1 s)")
    return ap.parse_args()


def settle(step, ms):
    """Run untimed steps until `ms` of GPU time have passed; returns how many ran.

    The GPU's clock governor needs tens of milliseconds of sustained load to leave its idle state (the first 25
    launches of the attention kernel after an idle second take 0.98 ms each, later ones 0.81 ms).  These steps come
    ahead of the W warm-up steps, which then run without a gap before the timed region."""
    if ms <= 0:
        return 0
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = 0
    a.record()
    while True:
        for _ in range(8):
            step()
        n += 8
        b.record()
        b.synchronize()
        if a.elapsed_time(b) >= ms:
            return n


def pick_workload(name):
    from paper_2512_05754_amd import synth

    table = {"wan13_480p": synth.WAN13_480P, "wan14_720p": synth.WAN14_720P,
             "merged_ragged": synth.MERGED_RAGGED, "tiny": synth.TINY}
    if name in table:
        return table[name]
    return synth.sweep(int(name[len("sweep"):]) / 100.0)


def cpu_baseline(w, Q, K, V, n_heads, two_branch=False):
    """Times the oracle (all three stages) on the first n_heads heads of batch 0."""
    import numpy as np

    from oracle import usv_oracle as orc
    from paper_2512_05754_amd import synth

    try:
        from threadpoolctl import threadpool_info

        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    n_heads = min(n_heads, w.heads)
    Qf, Kf, Vf = (synth.as_f32(x[:1, :n_heads]) for x in (Q, K, V))
    budgets = synth.gen_budgets(w)[:1, :n_heads] if not w.keep else None
    t0 = time.perf_counter()
    S = orc.block_scores(Qf, Kf, w.seq_valid)
    idx, cnt = orc.select_topk(S, w.keep, w.seq_valid, budgets=budgets, kmax=w.kmax, force_local=two_branch)
    fine = orc.block_sparse_attn(Qf, Kf, Vf, idx, cnt, w.seq_valid)[0]
    if two_branch:
        orc.fuse_outputs(fine, orc.coarse_attn(S, Vf, w.seq_valid), w.seq_valid, np.ones_like(fine), np.ones_like(fine))
        orc.attention_entropy(S, w.seq_valid)
    dt = time.perf_counter() - t0
    tiles = int(cnt.sum())
    flop = tiles * 4.0 * 64 * 64 * w.head_dim
    return {
        "value": flop / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{n_heads} of {w.batch * w.heads} heads (all {w.nb} query blocks each, {tiles} tiles), "
                  f"{6 if two_branch else 3} stages, numpy fp64, {dt:.2f} s; host has {len(os.sched_getaffinity(0))} usable cores",
        "seconds": dt,
        "ms_per_call_extrapolated": dt * 1e3 * (w.batch * w.heads) / n_heads,
    }


def measured_traffic(workload_name, key="attn_hbm_bytes_per_launch"):
    """{"traffic": HBM bytes per launch of the dominant kernel, "traffic_source": provenance} from the rocprofv3 --pmc
    runs summarised under profiles/; traffic is null when none was recorded or when the kernel sources changed since."""
    from paper_2512_05754_amd import traffic

    value, source = traffic.lookup(workload_name, key)
    return {"traffic": value, "traffic_source": source}


def mfma_only_peak():
    """Runs the MFMA-only probe (a child process, before this process touches the GPU); None if it is not built."""
    import subprocess

    tool = os.path.join(ROOT, "paper_2512_05754_amd", "tools", "mfma_peak")
    if not os.path.exists(tool):
        return None
    try:
        res = subprocess.run([tool], capture_output=True, text=True, timeout=60)
        return json.loads(res.stdout.strip().splitlines()[-1]) if res.returncode == 0 else None
    except (OSError, ValueError, IndexError, subprocess.TimeoutExpired):
        return None


GRIDS = {"wan1.3b_480p_keep10": (21, 30, 52), "wan14b_720p_keep5": (21, 45, 80)}


def reorder_main(args):
    """Times usv_cube_gather (Q, K, V) + usv_cube_scatter (O) at the workload's latent grid; HBM roofline."""
    import numpy as np
    import torch

    import paper_2512_05754_amd as usv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = pick_workload(args.workload)
    if w.name not in GRIDS:
        print(f"bench.py: --path reorder needs a workload with a latent grid ({sorted(GRIDS)})", file=sys.stderr)
        sys.exit(2)
    grid, cube = GRIDS[w.name], (4, 4, 4)
    B, Hh, Nv, N, d = w.batch, w.heads, w.seq_valid, w.seq_len, w.head_dim
    gen = torch.Generator(device=dev).manual_seed(w.seed)
    raster = [torch.randn((B, Hh, Nv, d), device=dev, generator=gen).to(torch.bfloat16) for _ in range(3)]
    cubes = [torch.empty((B, Hh, N, d), dtype=torch.bfloat16, device=dev) for _ in range(3)]
    o_cube = torch.randn((B, Hh, N, d), device=dev, generator=gen)  # the attention output, fp32 as in --path attention
    o_raster = torch.empty((B, Hh, Nv, d), dtype=torch.float32, device=dev)

    def step(events=None):
        if events is not None:
            events[0].record()
        for x, y in zip(raster, cubes):
            usv.cube_gather(x, grid, cube, seq_len=N, out=y)
        if events is not None:
            events[1].record()
        usv.cube_scatter(o_cube, grid, cube, out=o_raster)
        if events is not None:
            events[2].record()

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    settled = settle(step, args.settle_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    st_ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(2)] for e in evs]).mean(axis=0)
    rows = B * Hh
    gather_bytes = rows * (Nv + N) * d * 2           # one gather launch: read Nv rows, write N rows (bf16)
    scatter_bytes = rows * 2 * Nv * d * 4            # the scatter launch: read and write Nv rows (fp32)
    total = 3 * gather_bytes + scatter_bytes
    gather_ms = float(st_ms[0]) / 3
    result = {
        "metric": "GB/s of raster <-> cube-major reorder (gather Q, K, V + scatter O), algorithmic bytes",
        "value": total / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settled,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": w.name, "path": "reorder", "grid": list(grid), "cube": list(cube), "batch": B, "heads": Hh,
                   "head_dim": d, "seq_valid": Nv, "seq_len": N, "bytes_per_step": total,
                   "step": "3 x usv_cube_gather (bf16) + usv_cube_scatter (fp32)"},
        "stages_ms": {"cube_gather_x3": float(st_ms[0]), "cube_scatter": float(st_ms[1])},
        "roofline": {"kernel": "usv_cube_gather (cube_move<true, 16>)", "bound": "hbm",
                     "achieved": gather_bytes / (gather_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gather_bytes / (gather_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     **measured_traffic("reorder:" + w.name, "gather_hbm_bytes_per_launch"),
                     "avg_launch_ms": gather_ms},
    }
    if not args.no_cpu_baseline:
        from oracle import usv_oracle as orc

        xs = [x[0, :2].view(torch.int16).cpu().numpy() for x in raster]
        oc = o_cube[0, :2].cpu().numpy()
        t0 = time.perf_counter()
        for x in xs:
            orc.cube_gather(x, grid, cube, N)
        orc.cube_scatter(oc, grid, cube)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": total * 2 / rows / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"2 of {rows} heads, 3 gathers + 1 scatter, numpy indexing (incl. building the order), {dt:.2f} s"}
    print(json.dumps(result))


def merge_main(args):
    """Times token merging at the workload's latent grid with 2x2x2 merge blocks and r = N/2 (HBM roofline)."""
    import numpy as np
    import torch

    import paper_2512_05754_amd as usv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = pick_workload(args.workload)
    if w.name not in GRIDS:
        print(f"bench.py: --path merge needs a workload with a latent grid ({sorted(GRIDS)})", file=sys.stderr)
        sys.exit(2)
    grid, mb = GRIDS[w.name], (2, 2, 2)
    B, Hh, N, d = w.batch, w.heads, w.seq_valid, w.head_dim
    r = N // 2
    Nm = N - r
    Np = -(-Nm // 64) * 64
    gen = torch.Generator(device=dev).manual_seed(w.seed)
    base = torch.randn((B, 1, N, d), device=dev, generator=gen)
    q, k, v = ((torch.randn((B, Hh, N, d), device=dev, generator=gen) + 2 * base).to(torch.bfloat16) for _ in range(3))
    u = torch.empty((B, N), dtype=torch.float32, device=dev)
    blk = torch.empty((N,), dtype=torch.int32, device=dev)
    ws = torch.empty(B * N * (d + 1) * 4, dtype=torch.uint8, device=dev)
    row_of = torch.empty((B, N), dtype=torch.int32, device=dev)
    src_of = torch.empty((B, Nm), dtype=torch.int32, device=dev)
    # --merge-plan-one-workgroup: usv_merge_plan without a workspace (one workgroup per batch element)
    plan_ws = False if args.merge_plan_one_workgroup else torch.empty(usv.merge_plan_workspace_bytes(B, grid, mb, r),
                                                                       dtype=torch.uint8, device=dev)
    merged = [torch.empty((B, Hh, Np, d), dtype=torch.bfloat16, device=dev) for _ in range(3)]
    o_merged = torch.randn((B, Hh, Np, d), device=dev, generator=gen)  # stands for the fp32 attention output
    o_raster = torch.empty((B, Hh, N, d), dtype=torch.float32, device=dev)
    names = ["merge_similarity", "merge_plan", "merge_apply_x3", "unmerge_apply"]

    def step(events=None):
        rec = (lambda i: events[i].record()) if events is not None else (lambda i: None)
        rec(0)
        usv.merge_similarity(k, grid, mb, out=u, blk=blk, workspace=ws)
        rec(1)
        usv.merge_plan(u, blk, grid, mb, r, row_of=row_of, src_of=src_of, workspace=plan_ws)
        rec(2)
        for x, y in zip((q, k, v), merged):
            usv.merge_apply(x, grid, mb, row_of, src_of, seq_len=Np, out=y)
        rec(3)
        usv.unmerge_apply(o_merged, grid, mb, row_of, Nm, out=o_raster)
        rec(4)

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    settled = settle(step, args.settle_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    st_ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(4)] for e in evs]).mean(axis=0)
    rows = B * Hh
    bytes_sim = rows * N * d * 2 + B * N * (d + 1) * 4 * 2 + B * N * 4       # K once; descriptors written and read
    bytes_plan = B * N * 4 * 2 + B * (N + Nm) * 4                             # u read by search and sweep; row_of, src_of
    bytes_apply = rows * (N + Np) * d * 2                                     # per tensor: every raster row once, merged rows
    bytes_unmerge = rows * (Nm + N) * d * 4
    total = bytes_sim + bytes_plan + 3 * bytes_apply + bytes_unmerge
    apply_ms = float(st_ms[2]) / 3
    result = {
        "metric": "GB/s of token merging (similarity + plan + merge Q, K, V + unmerge O), algorithmic bytes",
        "value": total / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settled,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "path": "merge", "grid": list(grid), "merge_block": list(mb), "batch": B, "heads": Hh,
                   "head_dim": d, "tokens": N, "merged_sources": r, "merged_rows": Nm, "bytes_per_step": total,
                   "step": "usv_merge_similarity + usv_merge_plan + 3 x usv_merge_apply (bf16) + usv_unmerge_apply (fp32)"},
        "stages_ms": {n: float(t) for n, t in zip(names, st_ms)},
        "stage_hbm_gbs": {"merge_similarity": bytes_sim / (st_ms[0] * 1e-3) / 1e9, "merge_plan": bytes_plan / (st_ms[1] * 1e-3) / 1e9,
                          "merge_apply": bytes_apply / (apply_ms * 1e-3) / 1e9, "unmerge_apply": bytes_unmerge / (st_ms[3] * 1e-3) / 1e9},
        "roofline": {"kernel": "usv_merge_apply (merge_rows<bf16, 128>)", "bound": "hbm",
                     "achieved": bytes_apply / (apply_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": bytes_apply / (apply_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     **measured_traffic("merge:" + w.name, "apply_hbm_bytes_per_launch"), "avg_launch_ms": apply_ms},
    }
    if not args.no_cpu_baseline:
        from oracle import usv_oracle as orc

        hs = min(2, Hh)
        kh = k[:, :hs].float().cpu().numpy()
        t0 = time.perf_counter()
        uo = orc.merge_similarity(kh, grid, mb).astype(np.float32)
        rr, rs = orc.merge_plan(uo, grid, mb, r)
        ym = orc.merge_apply(kh, rr, rs, Np)
        orc.unmerge_apply(ym, rr)
        dt = time.perf_counter() - t0
        sample = bytes_sim * hs / Hh + bytes_plan + bytes_apply * hs / Hh + bytes_unmerge * hs / Hh
        result["cpu_baseline"] = {"value": sample / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{hs} of {Hh} heads: similarity, plan, one merge, one unmerge (numpy / python loops), {dt:.2f} s"}
    print(json.dumps(result))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.path == "reorder":
        return reorder_main(args)
    if args.path == "merge":
        return merge_main(args)

    peak_probe = None if args.no_mfma_peak else mfma_only_peak()

    import numpy as np
    import torch

    import paper_2512_05754_amd as usv
    from paper_2512_05754_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = pick_workload(args.workload)

    Q, K, V = synth.gen_qkv(w)

    def up(x):
        if x.dtype == np.uint16:
            return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)

    q, k, v = up(Q), up(K), up(V)
    budgets = None if w.keep else torch.from_numpy(synth.gen_budgets(w)).to(dev)
    two_branch = args.path in ("two_branch", "raster_two_branch")
    raster = args.path in ("raster", "raster_two_branch", "raster_cubes")
    cubes = args.path == "raster_cubes"  # one cube per block, cut cubes padded (usv_cube_order_padded + block_valid)
    bv = None
    if raster:
        if w.name not in GRIDS:
            print(f"bench.py: --path raster needs a workload with a latent grid ({sorted(GRIDS)})", file=sys.stderr)
            sys.exit(2)
        # the same tokens in raster order of the latent grid (the layout a DiT block's projections leave behind)
        r_grid, r_cube = GRIDS[w.name], (4, 4, 4)
        if cubes:
            # raster tensors whose shared per-cube vector follows the TRUE cubes of the grid, cut ones included
            q, k, v = (up(x) for x in synth.gen_raster_qkv(w, r_grid, r_cube))
            order, bv = usv.cube_order_padded(r_grid, r_cube)
        else:
            q, k, v = (usv.cube_scatter(x, r_grid, r_cube) for x in (q, k, v))
            order = usv.cube_order(r_grid, r_cube, seq_len=w.seq_len)
    out_dtype = torch.float32 if (args.out_dtype == "f32" or w.dtype == "f32") else torch.bfloat16

    # every buffer is allocated once, outside the timed region
    B, Hh, N, d, nb, kmax = w.batch, w.heads, w.seq_len, w.head_dim, w.nb, w.kmax
    keep_k, topk_valid = w.keep, w.seq_valid
    if cubes:
        nb = order.numel() // 64
        N = nb * 64
        keep_k = kmax = synth.keep_count(w.keep / w.nb, nb)  # the same keep ratio over more blocks
        topk_valid = N  # every block holds a token
    S = torch.empty((B, Hh, nb, nb), dtype=torch.float32, device=dev)
    ws = torch.empty(usv.workspace_bytes(B, Hh, N, min(w.seq_valid, N), d, w.dtype), dtype=torch.uint8, device=dev)
    idx = torch.empty((B, Hh, nb, kmax), dtype=torch.int32, device=dev)
    cnt = torch.empty((B, Hh, nb), dtype=torch.int32, device=dev)
    # the attention launch walks each head's query blocks in the order of usv_attn_work_order (longest lists first, lists
    # that lie alike next to each other) where that pays: ragged budgets, or a head's K and V many times an XCD's 4 MiB L2
    kv_head_bytes = 2 * w.seq_len * w.head_dim * (2 if w.dtype == "bf16" else 4)
    ordered = ((budgets is not None or kv_head_bytes > 8 * (4 << 20)) and not raster and not two_branch and w.dtype == "bf16"
               and not args.no_work_order)
    work_order = torch.empty((B, Hh, nb), dtype=torch.int32, device=dev) if ordered else None
    out = torch.empty((B, Hh, w.seq_valid if raster else N, d), dtype=out_dtype, device=dev)
    if two_branch:
        gen = torch.Generator(device=dev).manual_seed(w.seed)
        gates = [torch.rand((B, Hh, w.seq_valid if raster else N, d), device=dev, generator=gen).to(q.dtype) for _ in range(2)]
        coarse = torch.empty((B, Hh, nb, d), dtype=torch.float32, device=dev)
        ws_c = torch.empty(B * Hh * nb * d * 4, dtype=torch.uint8, device=dev)
        fused = torch.empty((B, Hh, w.seq_valid if raster else N, d), dtype=q.dtype, device=dev)
        ent = torch.empty((B,), dtype=torch.float32, device=dev)
        ws_e = torch.empty(B * Hh * ((nb + 31) // 32) * nb * 4, dtype=torch.uint8, device=dev)
        branch_events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    step_no = [0]

    def step(events=None):
        if events is not None:
            events[0].record()
        if raster:
            usv.block_scores_raster(q, k, order, out=S, workspace=ws, block_valid=bv)
        else:
            usv.block_scores(q, k, seq_valid=w.seq_valid, out=S, workspace=ws)
        if events is not None:
            events[1].record()
        usv.select_topk(S, k=keep_k, seq_valid=topk_valid, budgets=budgets, kmax=kmax, idx=idx, cnt=cnt,
                        force_local=two_branch)
        if ordered:  # timed with the selection
            usv.attn_work_order(cnt, kmax, idx=idx, out=work_order)
        if events is not None:
            events[2].record()
        if two_branch:  # the cube-level branch first: the attention kernel folds it and the gates into its store
            be = branch_events[step_no[0]] if events is not None else None
            if raster:
                usv.coarse_attn_raster(S, v, order, out=coarse, workspace=ws_c)
            else:
                usv.coarse_attn(S, v, seq_valid=w.seq_valid, out=coarse, workspace=ws_c)
            if be is not None:
                be[0].record()
            if raster:
                usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out=fused, coarse=coarse,
                                             gate_fine=gates[0], gate_coarse=gates[1])
            else:
                usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out=fused, coarse=coarse,
                                      gate_fine=gates[0], gate_coarse=gates[1])
            if be is not None:
                be[1].record()
        elif raster:
            usv.block_sparse_attn_raster(q, k, v, order, idx, cnt, out=out, block_valid=bv)
        else:
            usv.block_sparse_attn(q, k, v, idx, cnt, seq_valid=w.seq_valid, out=out, work_order=work_order)
        if events is not None:
            events[3].record()
        if two_branch:
            usv.attn_entropy(S, seq_valid=w.seq_valid, out=ent, workspace=ws_e)  # feeds the next step's budgets
            if be is not None:
                be[2].record()
                step_no[0] += 1

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # untimed: the settle steps, then the --warmup steps; timed: exactly --steps passes, bracketed by synchronize();
    # per-stage events are recorded on the launch stream
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    settled = settle(step, args.settle_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph and not two_branch:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        settle(graph.replay, args.settle_ms)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        for s in range(args.steps):  # eager pass for the per-stage times only
            step(evs[s])
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for s in range(args.steps):
            step(evs[s])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    st_ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in evs])  # [steps, 3]; two_branch fixes [2] below
    avg = st_ms.mean(axis=0)
    tiles = int(cnt.sum().item())
    flop = tiles * 4.0 * 64 * 64 * d
    esz = 2 if w.dtype == "bf16" else 4
    bytes_scores = 2 * B * Hh * N * d * esz + B * Hh * nb * nb * 4
    bytes_topk = B * Hh * nb * nb * 4 + B * Hh * nb * (kmax + 1) * 4

    result = {
        "metric": METRIC,
        "value": flop / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": settled,  # untimed steps ahead of the warm-up (--settle-ms of GPU time)
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": w.name, "batch": B, "heads": Hh, "head_dim": d, "seq_len": N, "seq_valid": w.seq_valid,
            "block": 64, "blocks": nb, "keep": keep_k if w.keep else f"U[{w.budget_lo},{w.budget_hi}]",
            "computed_tiles": tiles, "flop_per_step": flop, "out_dtype": args.out_dtype if w.dtype == "bf16" else "f32",
            "step": "usv_block_scores + usv_select_topk + usv_block_sparse_attn"
                    + (" + usv_coarse_attn + usv_attn_entropy; the attention is usv_block_sparse_attn_fused (local cube forced, "
                       "second branch and gates folded into its store)" if two_branch else ""),
        },
        "stages_ms": {"block_scores": float(avg[0]), "select_topk": float(avg[1]), "block_sparse_attn": float(avg[2])},
        "attn_ms_min": float(st_ms[:, 2].min()),
        "attn_ms_median": float(np.median(st_ms[:, 2])),
        "attn_tflops": flop / (avg[2] * 1e-3) / 1e12,
        "stage_hbm_gbs": {"block_scores": bytes_scores / (avg[0] * 1e-3) / 1e9,
                          "select_topk": bytes_topk / (avg[1] * 1e-3) / 1e9},
        "roofline": {
            "kernel": "usv_block_sparse_attn (attn_bf16)" if w.dtype == "bf16" else "usv_block_sparse_attn (attn_f32)",
            "bound": "mfma",  # bf16 matrix cores for bf16 inputs, fp32 matrix cores (v_mfma_f32_32x32x2_f32) for fp32 inputs
            "achieved": flop / (avg[2] * 1e-3) / 1e12,
            "peak": PEAK_BF16_TFLOPS if w.dtype == "bf16" else 157.3,
            "unit": "TFLOP/s",
            "frac": flop / (avg[2] * 1e-3) / 1e12 / (PEAK_BF16_TFLOPS if w.dtype == "bf16" else 157.3),
            **measured_traffic(w.name),
            "avg_launch_ms": float(avg[2]),
        },
    }
    if ordered:
        result["config"]["step"] = ("usv_block_scores + usv_select_topk + usv_attn_work_order (timed with the selection) + "
                                    "usv_block_sparse_attn_ordered")
    if args.graph and not two_branch:
        result["config"]["launch"] = "hip graph replay (one graph = one step)"
    if raster:
        result["config"]["path"] = "raster"
        result["config"]["grid"] = list(r_grid)
        result["config"]["step"] = ("usv_block_scores_raster + usv_select_topk + usv_block_sparse_attn_raster" if not two_branch else
                                    "usv_block_scores_raster + usv_select_topk_ex + usv_coarse_attn_raster + "
                                    "usv_block_sparse_attn_raster_fused + usv_attn_entropy")
        result["roofline"]["kernel"] = "usv_block_sparse_attn_raster (attn_bf16, raster addressing)"
        result["roofline"].update(measured_traffic(("cubes:" if cubes else "raster:") + w.name))
    if cubes:
        result["config"]["path"] = "raster_cubes"
        result["config"]["seq_len"] = N
        result["config"]["layout"] = ("one cube per block (usv_cube_order_padded): %d blocks, %d of them cut cubes padded to 64 rows; "
                                      "computed tiles count padded rows in full" % (nb, int((bv < 64).sum().item())))
        result["config"]["step"] = "usv_block_scores_raster + usv_select_topk + usv_block_sparse_attn_raster, view->block_valid set"
    if two_branch:
        c_ms = float(np.mean([evs[i][2].elapsed_time(branch_events[i][0]) for i in range(args.steps)]))
        a_ms = float(np.mean([branch_events[i][0].elapsed_time(branch_events[i][1]) for i in range(args.steps)]))
        e_ms = float(np.mean([evs[i][3].elapsed_time(branch_events[i][2]) for i in range(args.steps)]))
        result["stages_ms"]["block_sparse_attn"] = a_ms  # usv_block_sparse_attn_fused: the fusion is in its store
        fused_ms = [branch_events[i][0].elapsed_time(branch_events[i][1]) for i in range(args.steps)]
        result["attn_ms_min"], result["attn_ms_median"] = float(min(fused_ms)), float(np.median(fused_ms))
        result["attn_tflops"] = flop / (a_ms * 1e-3) / 1e12
        result["roofline"].update(achieved=result["attn_tflops"], frac=result["attn_tflops"] / PEAK_BF16_TFLOPS,
                                  avg_launch_ms=a_ms)
        result["config"]["out_dtype"] = "bf16"
        result["stages_ms"]["attn_entropy"] = e_ms
        result["stage_hbm_gbs"]["attn_entropy"] = B * Hh * nb * nb * 4 / (e_ms * 1e-3) / 1e9
        result["config"]["attn_entropy"] = [float(x) for x in ent.cpu()]
        result["config"]["path"] = args.path
        result["stages_ms"]["coarse_attn"] = c_ms
        bytes_coarse = B * Hh * (N * d * esz + 2 * nb * nb * 4 + 3 * nb * d * 4)  # V once, S twice, means + output
        result["stage_hbm_gbs"]["coarse_attn"] = bytes_coarse / (c_ms * 1e-3) / 1e9
    if peak_probe is not None:
        # context for `frac`: what an MFMA-only loop sustains on this GPU (the clock drops with operand activity)
        result["roofline"]["measured_mfma_only_tflops"] = peak_probe
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, Q, K, V, args.cpu_sample_heads, two_branch)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
