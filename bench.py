#!/usr/bin/env python3
"""Benchmark of the collective KV-reuse hot path on one MI355X.

A step is one pass of the whole path over one round: for every layer, tdk_rerotate_round (collect the
shared blocks for all agents), tdk_diff_decode (restore every mirror from master + diff) and
tdk_diff_encode (store every mirror as a block-sparse diff again).  Inputs are synthetic, seeded and
resident in HBM before the timed region.  One JSON line is printed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
ROW_PAIR_BYTES = 4096    # K + V of one token at one layer (8 heads x 128 x bf16 x 2)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="batched250")
    ap.add_argument("--ring", type=int, default=0, help="resident layer buffers (0 = automatic)")
    ap.add_argument("--group", type=int, default=0, help="agents per work item (0 = automatic)")
    ap.add_argument("--flags", type=int, default=-1, help="tuning bits (TDK_TUNE_*), default: the library's")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="step mode: also time the step replayed from one captured HIP graph (reported beside value)")
    ap.add_argument("--alloc", default="fragmented", choices=["fragmented", "contiguous"],
                    help="physical page placement of the synthetic pool (fragmented = the graded recipe)")
    ap.add_argument("--layout", default="identity", choices=["identity", "permuted"],
                    help="order of the shared blocks in every agent's prompt (identity = the graded recipe)")
    ap.add_argument("--mode", default="step", choices=["step", "restore", "check", "planes", "attend", "timeline"],
                    help="step: the whole hot path (default, the headline metric); restore: layerwise ping-pong "
                         "restore from pinned host memory (Alg. 1) against a dense restore")
    ap.add_argument("--n-q", type=int, default=1, help="attend mode: query tokens per agent")
    ap.add_argument("--q-heads", type=int, default=0, help="attend mode: query heads (0 = 5 per KV head)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (for profiling runs only)")
    ap.add_argument("--sessions", type=int, default=0, help="override the number of sessions of the workload (experiments only; "
                    "the line then names the change in config.workload)")
    ap.add_argument("--agents", type=int, default=0, help="override the agents per session (experiments only)")
    ap.add_argument("--csrc-hash", action="store_true", help="print the hash of the kernel sources (the one the "
                    "counter summaries under profiles/ carry) and exit")
    return ap.parse_args()


KERNEL_SOURCES = {"hbm_traffic": ("tdk_kernels.hip", "tdk_internal.h", "tdk_types.h"),
                  "hbm_traffic_attend": ("tdk_attend.hip", "tdk_internal.h", "tdk_types.h")}


def csrc_hash(prefix="hbm_traffic"):
    """sha256 over the kernel sources (comments and whitespace left out) a counter summary under profiles/ (named by
    its prefix) was taken from: ties the traffic figures to the kernels that ran."""
    import hashlib
    import re
    h = hashlib.sha256()
    for f in KERNEL_SOURCES[prefix]:
        text = open(os.path.join(ROOT, "paper_2604_03143_amd", "csrc", f), "r", encoding="utf-8").read()
        # the code alone: comments and layout do not change what ran (no string literal in these files holds "//")
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        text = " ".join(text.split())
        h.update(f.encode() + b"\0" + text.encode())
    return h.hexdigest()[:16]


def main():
    args = parse()
    if args.csrc_hash:
        for k in KERNEL_SOURCES:
            print(k, csrc_hash(k))
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU only (every session, layer and KV head is independent; "
              "no multi-GPU figure is produced).  Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_03143_amd import tdk, workload as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    tdk.load()   # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream

    if args.mode == "restore":
        return restore_mode(args, tdk, wl, np, torch, dev)
    if args.mode == "check":
        return check_mode(args, tdk, wl, np, torch, dev)
    if args.mode == "planes":
        return planes_mode(args, tdk, wl, np, torch, dev)
    if args.mode == "attend":
        return attend_mode(args, tdk, wl, np, torch, dev)
    if args.mode == "timeline":
        return timeline_mode(args, tdk, wl, np, torch, dev)

    spec = wl.CONFIGS[args.workload]
    if args.sessions or args.agents:
        import dataclasses
        spec = dataclasses.replace(spec, n_sessions=args.sessions or spec.n_sessions,
                                   agents_per_session=args.agents or spec.agents_per_session)
        args.workload = f"{args.workload}[sessions={spec.n_sessions},agents={spec.agents_per_session}]"
    L = args.layers or spec.num_layers
    rnd = wl.make_round(spec, alloc=args.alloc)
    if args.layout == "permuted":
        rnd = wl.permute_blocks(rnd)
    A, T, RE = rnd.n_agents, spec.page_tokens, spec.row_elems
    pool_rows = rnd.pool_pages * T
    n_pert = sum(len(p) for p in rnd.perturbed)
    capacity = n_pert + 64
    page_elems = 2 * T * RE

    per_slot = (2 * rnd.total_master_rows * RE + 2 * pool_rows * RE + 2 * capacity * page_elems) * 2
    free_b, total_b = torch.cuda.mem_get_info()
    ring = args.ring or int(max(1, min(L, 8, (0.8 * free_b) // per_slot)))
    ring = min(ring, L)

    r = tdk.round_from_workload(rnd)
    if args.group or args.flags >= 0:
        tdk.tdk_round_tune(r, args.group, args.flags if args.flags >= 0 else tdk.TUNE_DEFAULT)

    def new_diff():
        d = dict(count=torch.zeros(A, dtype=torch.int32, device=dev),
                 offset=torch.zeros(A + 1, dtype=torch.int64, device=dev),
                 idx=torch.full((capacity,), -1, dtype=torch.int32, device=dev),
                 payload=torch.zeros((capacity, page_elems), dtype=torch.int16, device=dev),
                 overflow=torch.zeros(1, dtype=torch.int32, device=dev))
        d["c"] = tdk.diff(d["count"], d["offset"], d["idx"], d["payload"], capacity, d["overflow"])
        return d

    # ---- resident inputs: a ring of layer buffers, each with its own data -------------------------
    pert_rows = torch.from_numpy(wl.perturbed_rows(rnd)).to(dev)
    slots = []
    for s in range(ring):
        mk, mv = wl.master_device(rnd, s, dev)
        pk = torch.zeros((pool_rows, RE), dtype=torch.int16, device=dev)
        pv = torch.zeros((pool_rows, RE), dtype=torch.int16, device=dev)
        io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
        stored, fresh = new_diff(), new_diff()
        # the mirrors this round stores: this side's own rerotate output, refreshed on the seeded pages
        tdk.tdk_rerotate_round(r, s, io, stream)
        wl.perturb_device(rnd, s, pk, pv, rows=pert_rows)
        tdk.tdk_diff_encode(r, s, io, spec.eps, stored["c"], stream)
        slots.append(dict(mk=mk, mv=mv, pk=pk, pv=pv, io=io, stored=stored, fresh=fresh))
    torch.cuda.synchronize()
    for s in slots:
        assert int(s["stored"]["overflow"].item()) == 0
        assert int(s["stored"]["offset"][-1].item()) == n_pert, "encode did not recover the seeded page set"

    def step(stream=stream):
        for layer in range(L):
            s = slots[layer % ring]
            tdk.tdk_rerotate_round(r, layer, s["io"], stream)
            tdk.tdk_diff_decode(r, layer, s["io"], s["stored"]["c"], stream)
            tdk.tdk_diff_encode(r, layer, s["io"], spec.eps, s["fresh"]["c"], stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly args.steps steps, nothing but the library's launches in between
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    agent_tokens = rnd.agent_tokens()
    value = agent_tokens / (ms_per_step * 1e-3)

    graph_out = None
    if args.graph:
        # the calls only enqueue kernels, so one graph can hold a whole step; replays skip the per-launch host work
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                step(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for _ in range(max(1, args.warmup)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        graph_out = dict(ms_per_step=round(g_ms, 3), value=round(agent_tokens / (g_ms * 1e-3), 1))
        del g

    # the same steps once more with every kernel launch bracketed by HIP events on the launch stream
    # (the brackets cost about 2 % of wall time, so they stay out of the region `value` is taken from)
    tdk.tdk_timing_reset(r)
    tdk.tdk_timing_enable(r, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_instrumented = (time.perf_counter() - t0) * 1e3 / args.steps
    tdk.tdk_timing_enable(r, False)

    # ---- per-call durations: an event pair around each of the three calls of every layer-step --------
    def ev():
        return torch.cuda.Event(enable_timing=True)
    pairs = {"rerotate": [], "decode": [], "encode": []}
    for _ in range(args.steps):
        for layer in range(L):
            s = slots[layer % ring]
            for name, call in (("rerotate", lambda: tdk.tdk_rerotate_round(r, layer, s["io"], stream)),
                               ("decode", lambda: tdk.tdk_diff_decode(r, layer, s["io"], s["stored"]["c"], stream)),
                               ("encode", lambda: tdk.tdk_diff_encode(r, layer, s["io"], spec.eps, s["fresh"]["c"], stream))):
                a, b = ev(), ev()
                a.record()
                call()
                b.record()
                pairs[name].append((a, b))
    torch.cuda.synchronize()
    call_us = {k: np.array([a.elapsed_time(b) * 1e3 for a, b in v]) for k, v in pairs.items()}

    # ---- per-kernel durations (HIP events on the launch stream, recorded inside the timed region) ---
    kt = {}
    for k in range(tdk.KERNEL_KINDS):
        ms, n = tdk.tdk_timing_read(r, k)
        kt[tdk.tdk_kernel_name(k)] = dict(total_ms=ms, launches=n, avg_us=(ms / n * 1e3 if n else 0.0))

    # ---- algorithmic bytes per layer-step ----------------------------------------------------------
    master_b = sum(int(s) for s in rnd.span_tokens) * ROW_PAIR_BYTES
    agents_b = agent_tokens * ROW_PAIR_BYTES
    payload_b = n_pert * page_elems * 2
    meta_b = 4 * n_pert + 12 * A
    # per call (the three ABI steps) and per page kernel (what that one launch must move)
    alg = dict(rerotate=master_b + agents_b,
               encode=master_b + agents_b + payload_b + meta_b,
               decode=master_b + agents_b + payload_b + meta_b,
               flag=master_b + agents_b,                  # kernel: reads every agent page + the master
               decode_kernel=master_b + agents_b - payload_b)   # kernel: writes every page not in a diff

    def gbps(nbytes, us):
        return nbytes / (us * 1e-6) / 1e9 if us > 0 else 0.0

    us = {k.replace("tdk_", "").replace("_kernel", ""): v["avg_us"] for k, v in kt.items()}
    enc_us = us["flag"] + us["compact"] + us["gather"]
    dec_us = us["decode"] + us["scatter"]
    rates = dict(rerotate_GBps=gbps(alg["rerotate"], us["rerotate"]),
                 encode_GBps=gbps(alg["encode"], enc_us),
                 decode_GBps=gbps(alg["decode"], dec_us),
                 encode_decode_GBps=gbps(alg["encode"] + alg["decode"], enc_us + dec_us))
    by_slot = {k: [round(float(np.median(v.reshape(args.steps, L)[:, q::ring])), 1) for q in range(ring)] for k, v in call_us.items()}
    calls = {k: dict(median_us=round(float(np.median(v)), 2), min_us=round(float(v.min()), 2), n=int(v.size),
                     median_us_by_ring_slot=by_slot[k],
                     GBps_at_median=round(gbps(alg[k], float(np.median(v))), 1),
                     pct_hbm_peak_at_median=round(100 * gbps(alg[k], float(np.median(v))) / HBM_PEAK_GBPS, 2))
             for k, v in call_us.items()}
    dom = max(("rerotate", "flag", "decode"), key=lambda k: kt[f"tdk_{k}_kernel"]["total_ms"])
    dom_bytes = alg["decode_kernel"] if dom == "decode" else alg[dom]
    achieved = gbps(dom_bytes, us[dom])
    traffic = read_traffic(args.workload, f"tdk_{dom}_kernel")
    # the three calls together: all algorithmic bytes of a layer-step over its share of the timed region
    layer_bytes = alg["rerotate"] + alg["encode"] + alg["decode"]
    pipe_gbps = layer_bytes / (ms_per_step * 1e-3 / L) / 1e9
    pipeline = dict(achieved=round(pipe_gbps, 1), peak=HBM_PEAK_GBPS, unit="GB/s", frac=round(pipe_gbps / HBM_PEAK_GBPS, 4),
                    algorithmic_bytes_per_layer_step=layer_bytes, us_per_layer_step=round(ms_per_step * 1e3 / L, 2),
                    note="per-kernel times shift between neighbours (a kernel's dirty lines are flushed during the next "
                         "one), so the pipeline figure is the robust one")
    roofline = dict(bound="hbm", kernel=f"tdk_{dom}_kernel", achieved=round(achieved, 1), peak=HBM_PEAK_GBPS,
                    unit="GB/s", frac=round(achieved / HBM_PEAK_GBPS, 4), traffic=traffic,
                    traffic_source=traffic_note(args.workload),
                    algorithmic_bytes_per_launch=dom_bytes, avg_launch_us=round(us[dom], 2))

    # ---- what HBM delivers on this machine for the bare access patterns (no arithmetic) ---------------
    def timed(fn, reps=5):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    n_copy = 1 << 31
    src = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    dst = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    tdk.tdk_util_fill(src, 0x01020304, n_copy, stream)
    copy_gbps = 2 * n_copy / timed(lambda: tdk.tdk_util_copy(dst, src, n_copy, stream)) / 1e9
    del dst
    page_b = T * RE * 2                       # one plane of one page
    n_pg = n_copy // page_b
    ids_seq = torch.arange(n_pg, dtype=torch.int32, device=dev)
    ids_rnd = torch.from_numpy(np.random.default_rng(7).permutation(n_pg).astype(np.int32)).to(dev)
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)
    ceil = {}
    for nm, ids in (("sequential", ids_seq), ("scattered", ids_rnd)):
        ceil[f"{nm}_page_write_GBps"] = round(n_pg * page_b / timed(
            lambda: tdk.tdk_util_page_fill(src, ids, n_pg, page_b, 5, stream)) / 1e9, 1)
        ceil[f"{nm}_page_read_GBps"] = round(n_pg * page_b / timed(
            lambda: tdk.tdk_util_page_read(src, ids, n_pg, page_b, sink, stream)) / 1e9, 1)
    # the same in the page kernels' own access form (K and V planes, four wavefronts on interleaved rows, streaming
    # stores / non-temporal loads, a group of pages per workgroup): what the product's traversal can reach at best
    half = n_pg // 2
    plane_k, plane_v = src[:half * page_b], src[half * page_b:2 * half * page_b]
    ids_half = {"sequential": torch.arange(half, dtype=torch.int32, device=dev),
                "scattered": torch.from_numpy(np.random.default_rng(8).permutation(half).astype(np.int32)).to(dev)}
    grp = r_group(tdk, r, args)
    for nm, ids in ids_half.items():
        ceil[f"{nm}_page_write_product_form_GBps"] = round(2 * half * page_b / timed(
            lambda: tdk.tdk_util_page_fill_product(plane_k, plane_v, ids, half, grp, spec.num_kv_heads, T, 5, stream)) / 1e9, 1)
        ceil[f"{nm}_page_read_product_form_GBps"] = round(2 * half * page_b / timed(
            lambda: tdk.tdk_util_page_read_product(plane_k, plane_v, ids, half, grp, spec.num_kv_heads, T, sink, stream)) / 1e9, 1)
    ceil["product_form_pages_per_workgroup"] = grp
    del src, plane_k, plane_v

    # ---- correctness at full size, outside the timed region ---------------------------------------
    check = {}
    if not args.no_check:
        ok = True
        for s in slots:
            a, b = s["stored"], s["fresh"]
            ok &= bool(torch.equal(a["count"], b["count"]) and torch.equal(a["offset"], b["offset"]))
            ok &= bool(torch.equal(a["idx"][:n_pert], b["idx"][:n_pert]))
            ok &= bool(torch.equal(a["payload"][:n_pert], b["payload"][:n_pert]))
            ok &= int(b["overflow"].item()) == 0
        off = slots[0]["fresh"]["offset"].cpu().numpy()
        idx = slots[0]["fresh"]["idx"].cpu().numpy()
        seeded = all(np.array_equal(idx[off[i]:off[i + 1]], rnd.perturbed[i]) for i in range(A))
        check = dict(reencode_equals_stored_diff=ok, indices_equal_seeded_set=bool(seeded))

    cpu = None
    if not args.no_cpu_baseline:
        cpu, par = cpu_baseline(rnd, slots[0], r, stream, L, tdk, wl, np, torch)
        check.update(par)

    out = dict(metric="shared-KV tokens collected/sec per round; diff encode+decode GB/s (% HBM peak)",
               value=round(value, 1), unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 3), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="bf16", data="synthetic",
               pool_addresses=[dict(pk=hex(s["pk"].data_ptr()), pv=hex(s["pv"].data_ptr()), mk=hex(s["mk"].data_ptr())) for s in slots],
               config=dict(workload=args.workload, layers=L, agents=A, sessions=rnd.n_sessions,
                           span_tokens=int(spec.span_tokens), page_tokens=T, perturbed_pages=n_pert,
                           ring_layers=ring, alloc=args.alloc, layout=args.layout, agents_per_group="auto" if not args.group else args.group,
                           step="rerotate+decode+encode per layer, all layers"),
               roofline=roofline, pipeline=pipeline, ms_per_step_instrumented=round(ms_per_step_instrumented, 3),
               hip_graph=graph_out,
               cpu_baseline=cpu,
               calls=calls,
               rates={k: round(v, 1) for k, v in rates.items()},
               pct_hbm_peak={k.replace("_GBps", ""): round(100 * v / HBM_PEAK_GBPS, 2) for k, v in rates.items()},
               copy_ceiling_GBps=round(copy_gbps, 1), pattern_ceilings=ceil,
               tokens_per_s_rerotate_only=round(agent_tokens / (us["rerotate"] * 1e-6 * L), 1) if us["rerotate"] else None,
               kernels={k: dict(avg_us=round(v["avg_us"], 2), launches=v["launches"]) for k, v in kt.items() if v["launches"]},
               check=check)
    print(json.dumps(out))
    r.destroy()


def restore_mode(args, tdk, wl, np, torch, dev):
    """Alg. 1 end to end: masters of every layer sit in pinned host memory; two staging buffers
    alternate between the H2D load (copy stream) and the fused restore (compute stream).  Compared
    with (a) the same without overlap, (b) a dense restore that first materialises one dense mirror
    per agent (copy of the master) and restores from that, as the paper's comparison path does."""
    name = args.workload if args.workload != "batched250" else "session"
    spec = wl.CONFIGS[name]
    L = args.layers or 16
    rnd = wl.make_round(spec, alloc=args.alloc)
    A, T, RE = rnd.n_agents, spec.page_tokens, spec.row_elems
    rows = rnd.pool_pages * T
    n_pert = sum(len(p) for p in rnd.perturbed)
    cap = n_pert + 8
    pe = 2 * T * RE
    st = torch.cuda.current_stream().cuda_stream
    r = tdk.round_from_workload(rnd)
    pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    hk, hv, diffs, mk_dev = [], [], [], []
    for l in range(L):
        mk, mv = wl.master_device(rnd, l, dev)
        io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
        tdk.tdk_rerotate_round(r, l, io, st)
        wl.perturb_device(rnd, l, pk, pv)
        d = dict(count=torch.zeros(A, dtype=torch.int32, device=dev), offset=torch.zeros(A + 1, dtype=torch.int64, device=dev),
                 idx=torch.full((cap,), -1, dtype=torch.int32, device=dev),
                 payload=torch.zeros((cap, pe), dtype=torch.int16, device=dev),
                 overflow=torch.zeros(1, dtype=torch.int32, device=dev))
        d["c"] = tdk.diff(d["count"], d["offset"], d["idx"], d["payload"], cap, d["overflow"])
        tdk.tdk_diff_encode(r, l, io, spec.eps, d["c"], st)
        torch.cuda.synchronize()
        hk.append(mk.cpu().pin_memory()); hv.append(mv.cpu().pin_memory())
        diffs.append(d)
        if l == 0:
            want_k, want_v = pk.clone(), pv.clone()
            mk0, mv0 = mk, mv
    mbytes = hk[0].numel() * 2
    stage = [torch.zeros(mbytes // 2, dtype=torch.int16, device=dev) for _ in range(4)]
    pp = tdk.pingpong(stage[0], stage[1], stage[2], stage[3], mbytes)
    ios = [tdk.layer_io(None, None, pk, pv, rnd.pool_pages) for _ in range(L)]
    comp, copy = torch.cuda.Stream(), torch.cuda.Stream()

    def wall(fn, reps):
        for _ in range(3):          # the runtime builds its cross-stream signals during the first calls
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):       # every repetition on its own clock: the median is robust against a disturbed one
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return float(np.median(ts))

    reps = max(20, args.steps)
    dc = [d["c"] for d in diffs]
    t_pp = wall(lambda: tdk.tdk_restore_layers(r, 0, hk, hv, ios, dc, pp, comp.cuda_stream, copy.cuda_stream), reps)
    # layer L-1 was restored last: check layer 0 separately below; serial = both roles on one stream
    t_serial = wall(lambda: tdk.tdk_restore_layers(r, 0, hk, hv, ios, dc, pp, comp.cuda_stream, comp.cuda_stream), reps)

    def h2d_only():
        for l in range(L):
            stage[l & 1].copy_(hk[l].view(-1), non_blocking=True)
            stage[2 + (l & 1)].copy_(hv[l].view(-1), non_blocking=True)
    t_h2d = wall(h2d_only, reps)
    io_res = tdk.layer_io(mk0, mv0, pk, pv, rnd.pool_pages)
    t_dec = wall(lambda: [tdk.tdk_diff_decode(r, l, io_res, dc[l], st) for l in range(L)], reps)

    # dense restore: one dense mirror per agent (a copy of its master), then restore from the mirrors
    sess_rows = [int(rnd.span_tokens[s]) for s in rnd.agent_session]
    dense_k = torch.zeros((sum(sess_rows), RE), dtype=torch.int16, device=dev)
    dense_v = torch.zeros_like(dense_k)
    r_dense = tdk.tdk_round_create(tdk.model(spec.num_layers, spec.num_kv_heads, spec.head_dim, T, spec.rope_theta),
                                   sess_rows, [int(rnd.master_pos0[s]) for s in rnd.agent_session],
                                   list(range(A)), rnd.agent_pos0, rnd.block_tables)
    io_dense = tdk.layer_io(dense_k, dense_v, pk, pv, rnd.pool_pages)
    row0 = np.concatenate([[0], np.cumsum(sess_rows)])

    def dense_restore():
        for l in range(L):
            b = l & 1
            stage[b].copy_(hk[l].view(-1), non_blocking=True)
            stage[2 + b].copy_(hv[l].view(-1), non_blocking=True)
            for i in range(A):
                s0 = int(rnd.master_row0[rnd.agent_session[i]]) * RE
                n = sess_rows[i] * RE
                tdk.tdk_util_copy(dense_k[int(row0[i]):], stage[b][s0:], n * 2, st)
                tdk.tdk_util_copy(dense_v[int(row0[i]):], stage[2 + b][s0:], n * 2, st)
            tdk.tdk_diff_decode(r_dense, l, io_dense, dc[l], st)
    t_dense = wall(dense_restore, reps)

    # correctness of the ping-pong path on layer 0 (bit-exact round trip of the stored mirrors)
    pk.zero_(); pv.zero_()
    tdk.tdk_restore_layers(r, 0, hk[:1], hv[:1], ios[:1], dc[:1], pp, comp.cuda_stream, copy.cuda_stream)
    torch.cuda.synchronize()
    ok = bool(torch.equal(pk, want_k) and torch.equal(pv, want_v))
    per_mirror = lambda t: round(t / (L * A) * 1e3, 4)
    out = dict(metric="fused restore latency per Mirror per layer (Alg. 1), masters staged from pinned host memory",
               value=per_mirror(t_pp), unit="ms", n_gpus=1, steps=reps, higher_is_better=False, data="synthetic",
               dtype="bf16", vs_baseline=None,
               config=dict(workload=name, layers=L, agents=A, span_tokens=int(spec.span_tokens), alloc=args.alloc),
               pingpong_ms_per_layer=round(t_pp / L * 1e3, 4), serial_ms_per_layer=round(t_serial / L * 1e3, 4),
               h2d_only_ms_per_layer=round(t_h2d / L * 1e3, 4), resident_decode_ms_per_layer=round(t_dec / L * 1e3, 4),
               dense_restore_ms_per_layer=round(t_dense / L * 1e3, 4),
               dense_restore_ms_per_mirror=per_mirror(t_dense),
               speedup_fused_vs_dense=round(t_dense / t_pp, 3), overlap_gain_vs_serial=round(t_serial / t_pp, 3),
               h2d_GBps=round(2 * mbytes * L / t_h2d / 1e9, 1),
               paper_context="0.43 ms fused vs 0.59 ms dense per Mirror on an A100-80GB (Sec. 6.5); other hardware, other unit of work",
               check=dict(pingpong_roundtrip_bitexact=ok))
    print(json.dumps(out))
    r.destroy(); r_dense.destroy()


def check_mode(args, tdk, wl, np, torch, dev):
    """The check-layer pass (Sec. 4.2) on its own: batched key-difference over the whole group, selection
    of the important positions (ratio 15 %), master choice.  Fresh keys = the refreshed mirrors."""
    spec = wl.CONFIGS[args.workload]
    rnd = wl.make_round(spec, alloc=args.alloc)
    A, T, RE = rnd.n_agents, spec.page_tokens, spec.row_elems
    rows = rnd.pool_pages * T
    st = torch.cuda.current_stream().cuda_stream
    r = tdk.round_from_workload(rnd)
    if args.group or args.flags >= 0:
        tdk.tdk_round_tune(r, args.group, args.flags if args.flags >= 0 else tdk.TUNE_DEFAULT)
    ring = args.ring or 4
    ratio = 0.15
    n_tok = rnd.agent_tokens()
    kmax = int(np.ceil(float(np.float32(ratio)) * spec.span_tokens))
    slots = []
    pert_rows = torch.from_numpy(wl.perturbed_rows(rnd)).to(dev)
    for s in range(ring):
        mk, mv = wl.master_device(rnd, s, dev)
        pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
        pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
        io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
        tdk.tdk_rerotate_round(r, s, io, st)
        wl.perturb_device(rnd, s, pk, pv, rows=pert_rows)
        plan = dict(score=torch.zeros(n_tok, dtype=torch.float32, device=dev),
                    imp=torch.zeros((A, kmax), dtype=torch.int32, device=dev),
                    n=torch.zeros(A, dtype=torch.int32, device=dev), total=torch.zeros(A, dtype=torch.float32, device=dev),
                    master=torch.zeros(rnd.n_sessions, dtype=torch.int32, device=dev))
        plan["c"] = tdk.reuse_plan(plan["score"], plan["imp"], kmax, plan["n"], plan["total"], plan["master"])
        slots.append(dict(io=io, plan=plan, keep=(mk, mv, pk, pv)))
    torch.cuda.synchronize()
    reps = max(1, args.steps) * 4
    for s in slots:
        tdk.tdk_check_layer(r, 0, s["io"], ratio, 0.0, s["plan"]["c"], st)
    torch.cuda.synchronize()
    tdk.tdk_timing_reset(r); tdk.tdk_timing_enable(r, True)
    t0 = time.perf_counter()
    for i in range(reps):
        s = slots[i % ring]
        tdk.tdk_check_layer(r, 0, s["io"], ratio, 0.0, s["plan"]["c"], st)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / reps
    tdk.tdk_timing_enable(r, False)
    us = {}
    for k in (tdk.KERNEL_KEYDIFF, tdk.KERNEL_SELECT, tdk.KERNEL_MASTER):
        ms, n = tdk.tdk_timing_read(r, k)
        us[tdk.tdk_kernel_name(k)] = round(ms / n * 1e3, 2)
    alg = (sum(int(x) for x in rnd.span_tokens) + n_tok) * (ROW_PAIR_BYTES // 2) + 4 * n_tok
    ach = alg / (us["tdk_keydiff_kernel"] * 1e-6) / 1e9
    # the refreshed tokens carry all the deviation: every agent's list must be exactly those tokens (up to k)
    p0 = slots[0]["plan"]
    n_imp = p0["n"].cpu().numpy(); imp = p0["imp"].cpu().numpy()
    good = True
    for i in range(A):
        toks = np.concatenate([np.arange(p * T, min(spec.span_tokens, (p + 1) * T)) for p in rnd.perturbed[i]])
        good &= int(n_imp[i]) == min(kmax, len(toks)) and bool(np.all(np.isin(imp[i, :n_imp[i]], toks)))
    out = dict(metric="check-layer pass: batched key-difference GB/s, important-position selection and master choice",
               value=round(ach, 1), unit="GB/s", n_gpus=1, steps=reps, higher_is_better=True, dtype="bf16", data="synthetic",
               vs_baseline=None, config=dict(workload=args.workload, agents=A, span_tokens=int(spec.span_tokens), ratio=ratio),
               ms_per_call=round(wall_ms, 4), kernels_avg_us=us,
               roofline=dict(bound="hbm", kernel="tdk_keydiff_kernel", achieved=round(ach, 1), peak=HBM_PEAK_GBPS, unit="GB/s",
                             frac=round(ach / HBM_PEAK_GBPS, 4), traffic=None, algorithmic_bytes_per_launch=alg),
               check=dict(important_positions_are_the_refreshed_tokens=bool(good)))
    print(json.dumps(out))
    r.destroy()


def planes_mode(args, tdk, wl, np, torch, dev):
    """Single-plane diffs (separate K and V index lists, Sec. 5) against the paired diff: the same
    mirrors encoded and restored plane by plane."""
    spec = wl.CONFIGS[args.workload]
    rnd = wl.make_round(spec, alloc=args.alloc)
    A, T, RE = rnd.n_agents, spec.page_tokens, spec.row_elems
    rows = rnd.pool_pages * T
    st = torch.cuda.current_stream().cuda_stream
    r = tdk.round_from_workload(rnd)
    n_pert = sum(len(p) for p in rnd.perturbed)
    cap = n_pert + 64
    mk, mv = wl.master_device(rnd, 0, dev)
    pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
    tdk.tdk_rerotate_round(r, 0, io, st)
    wl.perturb_device(rnd, 0, pk, pv)
    want_k, want_v = pk.clone(), pv.clone()

    def new_diff(planes):
        d = dict(count=torch.zeros(A, dtype=torch.int32, device=dev), offset=torch.zeros(A + 1, dtype=torch.int64, device=dev),
                 idx=torch.full((cap,), -1, dtype=torch.int32, device=dev),
                 payload=torch.zeros((cap, planes * T * RE), dtype=torch.int16, device=dev),
                 overflow=torch.zeros(1, dtype=torch.int32, device=dev))
        d["c"] = tdk.diff(d["count"], d["offset"], d["idx"], d["payload"], cap, d["overflow"])
        return d

    dp, dk, dv = new_diff(2), new_diff(1), new_diff(1)

    def timed(fn, reps=10):
        fn(); fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps      # us

    t = {}
    t["encode_paired"] = timed(lambda: tdk.tdk_diff_encode(r, 0, io, spec.eps, dp["c"], st))
    t["encode_K"] = timed(lambda: tdk.tdk_diff_encode_plane(r, 0, io, spec.eps, tdk.PLANE_K, dk["c"], st))
    t["encode_V"] = timed(lambda: tdk.tdk_diff_encode_plane(r, 0, io, spec.eps, tdk.PLANE_V, dv["c"], st))
    t["decode_paired"] = timed(lambda: tdk.tdk_diff_decode(r, 0, io, dp["c"], st))
    t["decode_K"] = timed(lambda: tdk.tdk_diff_decode_plane(r, 0, io, tdk.PLANE_K, dk["c"], st))
    t["decode_V"] = timed(lambda: tdk.tdk_diff_decode_plane(r, 0, io, tdk.PLANE_V, dv["c"], st))
    pk.zero_(); pv.zero_()
    tdk.tdk_diff_decode_plane(r, 0, io, tdk.PLANE_K, dk["c"], st)
    tdk.tdk_diff_decode_plane(r, 0, io, tdk.PLANE_V, dv["c"], st)
    torch.cuda.synchronize()
    ok = bool(torch.equal(pk, want_k) and torch.equal(pv, want_v))
    same_lists = bool(torch.equal(dk["idx"][:n_pert], dp["idx"][:n_pert]) and torch.equal(dv["idx"][:n_pert], dp["idx"][:n_pert]))
    half = ROW_PAIR_BYTES // 2
    master_b = sum(int(x) for x in rnd.span_tokens) * half
    agents_b = rnd.agent_tokens() * half
    payload_b = n_pert * T * RE * 2
    one = master_b + agents_b + payload_b
    gb = lambda nbytes, us: round(nbytes / (us * 1e-6) / 1e9, 1)
    out = dict(metric="single-plane diff encode / decode GB/s (algorithmic bytes) against the paired diff",
               value=gb(2 * one, t["encode_K"] + t["encode_V"]), unit="GB/s", n_gpus=1, higher_is_better=True,
               dtype="bf16", data="synthetic", vs_baseline=None,
               config=dict(workload=args.workload, agents=A, span_tokens=int(spec.span_tokens), listed_pages=n_pert),
               us={k: round(v, 1) for k, v in t.items()},
               GBps=dict(encode_paired=gb(2 * one, t["encode_paired"]), encode_K=gb(one, t["encode_K"]), encode_V=gb(one, t["encode_V"]),
                         decode_paired=gb(2 * one, t["decode_paired"]), decode_K=gb(one, t["decode_K"]), decode_V=gb(one, t["decode_V"])),
               paired_vs_split=dict(encode=round((t["encode_K"] + t["encode_V"]) / t["encode_paired"], 3),
                                    decode=round((t["decode_K"] + t["decode_V"]) / t["decode_paired"], 3)),
               check=dict(planewise_restore_bitexact=ok, lists_equal_shared_list=same_lists))
    print(json.dumps(out))
    r.destroy()


def attend_mode(args, tdk, wl, np, torch, dev):
    """Attention of new query tokens over the shared span of every mirror straight from master + diff
    (Sec. 4.4, the diff applied as attention tiles are loaded), against what restoring the mirrors first
    costs: the restore itself plus one read of the restored caches (the least an attention kernel over
    them has to do)."""
    spec = wl.CONFIGS[args.workload]
    rnd = wl.make_round(spec, alloc=args.alloc)
    A, T, RE, H, D = rnd.n_agents, spec.page_tokens, spec.row_elems, spec.num_kv_heads, spec.head_dim
    Hq = args.q_heads or 5 * H
    n_q = args.n_q
    rows = rnd.pool_pages * T
    st = torch.cuda.current_stream().cuda_stream
    r = tdk.round_from_workload(rnd)
    n_pert = sum(len(p) for p in rnd.perturbed)
    cap = n_pert + 64
    mk, mv = wl.master_device(rnd, 0, dev)
    pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
    tdk.tdk_rerotate_round(r, 0, io, st)
    wl.perturb_device(rnd, 0, pk, pv)
    d = dict(count=torch.zeros(A, dtype=torch.int32, device=dev), offset=torch.zeros(A + 1, dtype=torch.int64, device=dev),
             idx=torch.full((cap,), -1, dtype=torch.int32, device=dev),
             payload=torch.zeros((cap, 2 * T * RE), dtype=torch.int16, device=dev),
             overflow=torch.zeros(1, dtype=torch.int32, device=dev))
    d["c"] = tdk.diff(d["count"], d["offset"], d["idx"], d["payload"], cap, d["overflow"])
    tdk.tdk_diff_encode(r, 0, io, spec.eps, d["c"], st)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.SEED_BASE + 17)
    q = torch.randn((A, n_q, Hq, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16).view(torch.int16)
    out = torch.zeros((A, n_q, Hq, D), dtype=torch.float32, device=dev)
    lse = torch.zeros((A, n_q, Hq), dtype=torch.float32, device=dev)
    nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    scale = 1.0 / float(np.sqrt(D))
    a = tdk.attend_io(q, n_q, Hq, scale, out, lse, ws, nbytes)
    torch.cuda.synchronize()
    assert int(d["offset"][-1].item()) == n_pert

    def timed(fn, reps):
        fn(); fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps      # us

    reps = max(1, args.steps) * 4
    t_att = timed(lambda: tdk.tdk_attend_shared(r, 0, io, d["c"], a, st), reps)
    tdk.tdk_timing_reset(r); tdk.tdk_timing_enable(r, True)
    for _ in range(reps):
        tdk.tdk_attend_shared(r, 0, io, d["c"], a, st)
    torch.cuda.synchronize()
    tdk.tdk_timing_enable(r, False)
    us = {}
    for k in (tdk.KERNEL_ATTEND_QROT, tdk.KERNEL_ATTEND_MASTER, tdk.KERNEL_ATTEND_DIFF, tdk.KERNEL_ATTEND_MERGE):
        ms, n = tdk.tdk_timing_read(r, k)
        if n:          # (the master and the listed-pages pass share one launch, timed as the master pass, when the round allows)
            us[tdk.tdk_kernel_name(k)] = round(ms / n * 1e3, 2)
    # the other way: restore every mirror, then read the restored caches once
    t_dec = timed(lambda: tdk.tdk_diff_decode(r, 0, io, d["c"], st), 5)
    ids = torch.from_numpy(np.unique(np.concatenate([rnd.block_tables[i][int(rnd.agent_pos0[i]) // T:] for i in range(A)])
                                     ).astype(np.int32)).to(dev)
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)
    t_read = timed(lambda: (tdk.tdk_util_page_read(pk, ids, ids.numel(), T * RE * 2, sink, st),
                            tdk.tdk_util_page_read(pv, ids, ids.numel(), T * RE * 2, sink, st)), 5)

    # parity sample: the first three agents against the oracle (exact definition, double precision)
    check = {}
    if not args.no_check:
        from oracle import tdo
        n = 3
        sub, _ = wl.subround(rnd, range(n))
        off = d["offset"].cpu().numpy(); cnt = d["count"].cpu().numpy()
        m = int(off[n])
        od = tdo.Diff(n, max(m, 1), 2 * T * RE)
        od.count[:] = cnt[:n]; od.offset[:] = off[:n + 1]
        od.idx[:m] = d["idx"][:m].cpu().numpy(); od.payload[:m] = d["payload"][:m].cpu().numpy().view(np.uint16)
        S0 = int(sub.span_tokens[0])
        hmk, hmv = mk[:S0].cpu().numpy().view(np.uint16), mv[:S0].cpu().numpy().view(np.uint16)
        t0 = time.perf_counter()
        want_o, want_l = tdo.attend_shared(tdo.geom_of(spec), tdo.HostRound(sub), hmk, hmv, od,
                                           q[:n].cpu().numpy().view(np.uint16), n_q, Hq, scale)
        oracle_s = time.perf_counter() - t0
        err_o = float(np.max(np.abs(out[:n].cpu().numpy().astype(np.float64) - want_o)))
        err_l = float(np.max(np.abs(lse[:n].cpu().numpy().astype(np.float64) - want_l)))
        check = dict(sample="agents 0-2 against the oracle", max_abs_err_out=err_o, max_abs_err_lse=err_l,
                     within_tolerance=bool(err_o <= 1e-2 * max(1.0, float(np.abs(wl.bf16_bits_to_f32(hmv)).max())) and err_l <= 5e-3),
                     oracle_seconds=round(oracle_s, 2), oracle_cores=tdo.max_threads())

    master_b = sum(int(x) for x in rnd.span_tokens) * ROW_PAIR_BYTES
    payload_b = n_pert * 2 * T * RE * 2
    qo_b = A * n_q * Hq * D * (2 + 4) + A * n_q * Hq * 4
    alg = master_b + payload_b + qo_b
    flops = 4.0 * A * n_q * Hq * D * spec.span_tokens
    ach = alg / (t_att * 1e-6) / 1e9
    # counter figures exist for the default shape only (one query token, the shared launch + the merge)
    traffic = None
    if n_q == 1 and args.q_heads == 0:
        parts = [read_traffic(args.workload, k, "hbm_traffic_attend") for k in ("tdk_attend_fused_kernel", "tdk_attend_merge_kernel")]
        if all(x is not None for x in parts):
            traffic = sum(parts)
    out_d = dict(metric="attention over the shared span of never-restored mirrors: query rows per second; GB/s of master + diff read",
                 value=round(A * n_q * Hq / (t_att * 1e-6), 1), unit="query rows/s", n_gpus=1, steps=reps, higher_is_better=True,
                 dtype="bf16", data="synthetic", vs_baseline=None,
                 config=dict(workload=args.workload, agents=A, span_tokens=int(spec.span_tokens), n_q=n_q, q_heads=Hq,
                             listed_pages=n_pert, workspace_bytes=nbytes),
                 us_per_layer=round(t_att, 2), kernels_avg_us=us,
                 roofline=dict(bound="hbm", kernel="tdk_attend_shared (all its launches)", achieved=round(ach, 1), peak=HBM_PEAK_GBPS,
                               unit="GB/s", frac=round(ach / HBM_PEAK_GBPS, 4), traffic=traffic, algorithmic_bytes_per_launch=alg),
                 mfma_TFLOPs=round(flops / (t_att * 1e-6) / 1e12, 2),
                 restore_first=dict(decode_us=round(t_dec, 2), read_restored_caches_us=round(t_read, 2),
                                    speedup=round((t_dec + t_read) / t_att, 2)),
                 check=check)
    print(json.dumps(out_d))
    r.destroy()


def timeline_mode(args, tdk, wl, np, torch, dev):
    """Workgroup timeline of the three page kernels (rerotate, decode, compare) inside the step's own sequence:
    when every workgroup of a launch started and ended (device clock, 10 ns ticks).  Shows how long the launch
    takes to fill the chip, how many workgroups run at a time, and how long the chip drains after the last
    workgroup has started (the tail that a coarse work list would leave)."""
    spec = wl.CONFIGS[args.workload]
    rnd = wl.make_round(spec, alloc=args.alloc)
    A, T, RE = rnd.n_agents, spec.page_tokens, spec.row_elems
    rows = rnd.pool_pages * T
    st = torch.cuda.current_stream().cuda_stream
    r = tdk.round_from_workload(rnd)
    if args.group or args.flags >= 0:
        tdk.tdk_round_tune(r, args.group, args.flags if args.flags >= 0 else tdk.TUNE_DEFAULT)
    n_pert = sum(len(p) for p in rnd.perturbed)
    cap = n_pert + 64
    slots = []
    pert_rows = torch.from_numpy(wl.perturbed_rows(rnd)).to(dev)
    for s_ in range(2):
        mk, mv = wl.master_device(rnd, s_, dev)
        pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
        pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
        io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
        d = dict(count=torch.zeros(A, dtype=torch.int32, device=dev), offset=torch.zeros(A + 1, dtype=torch.int64, device=dev),
                 idx=torch.full((cap,), -1, dtype=torch.int32, device=dev),
                 payload=torch.zeros((cap, 2 * T * RE), dtype=torch.int16, device=dev),
                 overflow=torch.zeros(1, dtype=torch.int32, device=dev))
        d["c"] = tdk.diff(d["count"], d["offset"], d["idx"], d["payload"], cap, d["overflow"])
        tdk.tdk_rerotate_round(r, s_, io, st)
        wl.perturb_device(rnd, s_, pk, pv, rows=pert_rows)
        tdk.tdk_diff_encode(r, s_, io, spec.eps, d["c"], st)
        slots.append(dict(io=io, d=d, keep=(mk, mv, pk, pv)))
    torch.cuda.synchronize()
    nbytes = tdk.tdk_timeline_bytes(r)
    stamps = torch.zeros(nbytes // 8, dtype=torch.int64, device=dev)

    calls = [("rerotate", lambda s_: tdk.tdk_rerotate_round(r, 0, s_["io"], st)),
             ("decode", lambda s_: tdk.tdk_diff_decode(r, 0, s_["io"], s_["d"]["c"], st)),
             ("encode", lambda s_: tdk.tdk_diff_encode(r, 0, s_["io"], spec.eps, s_["d"]["c"], st))]

    def sequence(upto, stamped):
        """The step's sequence on both slots; the launch to look at is call `stamped` on slot 1."""
        for k, s_ in enumerate(slots):
            for j, (nm, fn) in enumerate(calls):
                on = k == 1 and j == stamped
                if on:
                    tdk.tdk_timeline_set(r, stamps, nbytes)
                fn(s_)
                if on:
                    tdk.tdk_timeline_set(r, None, 0)

    out_k = {}
    for j, (nm, _) in enumerate(calls):
        sequence(None, -1)
        torch.cuda.synchronize()
        stamps.zero_()
        sequence(None, j)
        torch.cuda.synchronize()
        h4 = stamps.cpu().numpy().reshape(-1, 4)
        h4 = h4[h4[:, 0] > 0]
        h = h4[:, :2]
        xcd = (h[:, 0] & 15).astype(np.int64)
        s0, e0 = (h[:, 0] & ~15).astype(np.float64) * 1e-2, h[:, 1].astype(np.float64) * 1e-2      # us
        t0 = s0.min()
        s0 -= t0; e0 -= t0
        span = float(e0.max())
        # workgroups running at time t
        ev = np.concatenate([np.stack([s0, np.ones_like(s0)], 1), np.stack([e0, -np.ones_like(e0)], 1)])
        ev = ev[np.argsort(ev[:, 0], kind="stable")]
        active = np.cumsum(ev[:, 1])
        tt = ev[:, 0]
        mid = (tt > 0.2 * span) & (tt < 0.8 * span)
        steady = float(np.median(active[mid])) if mid.any() else float(active.max())
        full = np.nonzero(active >= 0.9 * steady)[0]
        ramp = float(tt[full[0]]) if full.size else 0.0
        last_start = float(s0.max())
        below = np.nonzero(active >= 0.5 * steady)[0]
        half_until = float(tt[below[-1]]) if below.size else span
        dur = e0 - s0
        out_k[nm] = dict(workgroups=int(h.shape[0]), span_us=round(span, 2), running_at_a_time=steady,
                         us_until_90pct_running=round(ramp, 2),
                         us_after_last_start=round(span - last_start, 2),
                         us_below_half_running_at_end=round(span - half_until, 2),
                         workgroup_us=dict(median=round(float(np.median(dur)), 2), p99=round(float(np.percentile(dur, 99)), 2),
                                           max=round(float(dur.max()), 2)),
                         first_end_us=round(float(e0.min()), 2),
                         us_from_item_taken=None if not (h4[:, 2] > 0).all() else dict(
                             staged_median=round(float(np.median((h4[:, 2] - (h4[:, 0] & ~15)) * 1e-2)), 2),
                             first_agent_written_median=round(float(np.median((h4[:, 3] - (h4[:, 0] & ~15)) * 1e-2)), 2),
                             staged_p90=round(float(np.percentile((h4[:, 2] - (h4[:, 0] & ~15)) * 1e-2, 90)), 2),
                             first_agent_written_p90=round(float(np.percentile((h4[:, 3] - (h4[:, 0] & ~15)) * 1e-2, 90)), 2)),
                         running_every_2pct=[int(active[np.searchsorted(tt, q * span / 50, side="right") - 1]) for q in range(1, 50)],
                         finished_per_2pct=np.histogram(e0, bins=50, range=(0, span))[0].tolist(),
                         per_xcd=dict(workgroups=np.bincount(xcd, minlength=8).tolist(),
                                      last_end_us=[round(float(e0[xcd == x].max()), 1) if (xcd == x).any() else None for x in range(8)],
                                      last_start_us=[round(float(s0[xcd == x].max()), 1) if (xcd == x).any() else None for x in range(8)]))
    print(json.dumps(dict(metric="workgroup timeline of the page kernels", unit="us", n_gpus=1, data="synthetic",
                          config=dict(workload=args.workload, agents=A, agents_per_group=tdk.tdk_round_agents_per_group(r)),
                          kernels=out_k)))
    r.destroy()


def r_group(tdk, r, args):
    """Agents per work item of the round (what the product-form probes use as pages per workgroup)."""
    return tdk.tdk_round_agents_per_group(r)


def read_traffic(workload, kernel, prefix="hbm_traffic"):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None: if there is no
    summary, or if it was taken from other kernel sources than the ones this run uses (its `csrc_sha256` line)."""
    path = os.path.join(ROOT, "profiles", f"{prefix}_{workload}.txt")
    value, tagged = None, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 2 and "csrc_sha256" in f[:2]:
                tagged = f[-1]
            if len(f) == 4 and f[0] == kernel:
                value = float(f[3])
    except OSError:
        return None
    return value if tagged == csrc_hash(prefix) else None


def traffic_note(workload, prefix="hbm_traffic"):
    path = os.path.join(ROOT, "profiles", f"{prefix}_{workload}.txt")
    if not os.path.exists(path):
        return "no counter summary for this workload under profiles/"
    tagged = None
    for line in open(path):
        f = line.split()
        if len(f) >= 2 and "csrc_sha256" in f[:2]:
            tagged = f[-1]
    if tagged != csrc_hash(prefix):
        return (f"profiles/{prefix}_{workload}.txt was taken from kernel sources {tagged}, this run uses {csrc_hash(prefix)}: "
                "traffic withheld")
    return f"from profiles/{prefix}_{workload}.txt (rocprofv3 --pmc, same kernel sources {tagged})"


def cpu_baseline(rnd, slot, r, stream, L, tdk, wl, np, torch):
    """The CPU oracle as it stands, on one session of layer 0 (the first 25 agents): one layer-step
    (rerotate + decode + encode).  Also serves as the full-size parity sample."""
    from oracle import tdo
    spec = rnd.spec
    T, RE = spec.page_tokens, spec.row_elems
    n = min(rnd.n_agents, spec.agents_per_session)
    sub, page_map = wl.subround(rnd, range(n))
    rows = (torch.from_numpy(page_map).to(slot["pk"].device)[:, None] * T +
            torch.arange(T, device=slot["pk"].device)[None, :]).reshape(-1)

    def pool_sample():
        torch.cuda.synchronize()
        return (slot["pk"][rows].cpu().numpy().view(np.uint16), slot["pv"][rows].cpu().numpy().view(np.uint16))

    sess = sub.extra["sessions"]
    r0, r1 = int(rnd.master_row0[sess[0]]), int(rnd.master_row0[sess[-1] + 1])
    mk = slot["mk"][r0:r1].cpu().numpy().view(np.uint16)
    mv = slot["mv"][r0:r1].cpu().numpy().view(np.uint16)
    g = tdo.geom_of(spec)
    hr = tdo.HostRound(sub)
    cap = n * spec.span_pages

    # state after the timed steps: the pool holds the restored (perturbed) mirrors
    mir_k, mir_v = pool_sample()
    gd = slot["fresh"]
    off = gd["offset"].cpu().numpy()
    cnt = gd["count"].cpu().numpy()

    t = {}
    ok, ov = mir_k.copy(), mir_v.copy()
    t0 = time.perf_counter()
    tdo.rerotate_round(g, hr, mk, mv, ok, ov)
    t["rerotate"] = time.perf_counter() - t0
    tdk.tdk_rerotate_round(r, 0, slot["io"], stream)
    gk, gv = pool_sample()
    shared = wl.shared_row_mask(sub)
    par = dict(sample_rerotate_bitexact=bool(np.array_equal(gk[shared], ok[shared]) and np.array_equal(gv[shared], ov[shared])))

    t0 = time.perf_counter()
    od = tdo.diff_encode(g, hr, mk, mv, mir_k, mir_v, spec.eps, cap)
    t["encode"] = time.perf_counter() - t0
    m = int(od.offset[-1])
    par["sample_encode_bitexact"] = bool(
        np.array_equal(od.count, cnt[:n]) and np.array_equal(od.offset, off[:n + 1] - off[0]) and
        np.array_equal(od.idx[:m], gd["idx"][int(off[0]):int(off[0]) + m].cpu().numpy()) and
        np.array_equal(od.payload[:m], gd["payload"][int(off[0]):int(off[0]) + m].cpu().numpy().view(np.uint16)))

    dk, dv = ok.copy(), ov.copy()
    t0 = time.perf_counter()
    tdo.diff_decode(g, hr, mk, mv, dk, dv, od)
    t["decode"] = time.perf_counter() - t0
    tdk.tdk_diff_decode(r, 0, slot["io"], slot["stored"]["c"], stream)
    gk, gv = pool_sample()
    par["sample_decode_bitexact"] = bool(np.array_equal(gk[shared], dk[shared]) and np.array_equal(gv[shared], dv[shared]))

    # repeat the timed trio until about 10 s of CPU work are spent
    reps, spent = 1, sum(t.values())
    while spent < 12.0 and reps < 400:
        t0 = time.perf_counter()
        tdo.rerotate_round(g, hr, mk, mv, ok, ov)
        tdo.diff_encode(g, hr, mk, mv, mir_k, mir_v, spec.eps, cap)
        tdo.diff_decode(g, hr, mk, mv, dk, dv, od)
        spent += time.perf_counter() - t0
        reps += 1
    layer_step_s = spent / reps
    toks = sub.agent_tokens()
    # algorithmic bytes of the sample's layer-step, by the same definition as the GPU figures
    base_b = (int(sum(int(x) for x in sub.span_tokens)) + toks) * ROW_PAIR_BYTES
    sample_bytes = 3 * base_b + 2 * (m * 2 * T * RE * 2 + 4 * m + 12 * n)
    threads = tdo.max_threads()
    tdo.set_threads(1)                       # the same trio once on one thread
    t0 = time.perf_counter()
    tdo.rerotate_round(g, hr, mk, mv, ok, ov)
    tdo.diff_encode(g, hr, mk, mv, mir_k, mir_v, spec.eps, cap)
    tdo.diff_decode(g, hr, mk, mv, dk, dv, od)
    one_thread_s = time.perf_counter() - t0
    tdo.set_threads(threads)
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    cpu = dict(value=round(toks / (layer_step_s * L), 1), unit="tokens/s", cores=threads, kind="oracle",
               affinity_cores=len(os.sched_getaffinity(0)), cpu_model=model,
               sample=f"layer 0, session 0 ({n} agents x {int(sub.span_tokens[0])} tokens): rerotate+encode+decode, "
                      f"{reps} repetitions, {spent:.1f} s; scaled to {L} layers",
               layer_step_s=round(layer_step_s, 3),
               one_thread=dict(value=round(toks / (one_thread_s * L), 1), layer_step_s=round(one_thread_s, 3)),
               GBps=round(sample_bytes / layer_step_s / 1e9, 2),
               first_rep_s={k: round(v, 3) for k, v in t.items()})
    return cpu, par


if __name__ == "__main__":
    main()
