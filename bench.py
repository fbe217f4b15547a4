#!/usr/bin/env python3
"""Benchmark of the KV-migration hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: route (host),
plan (flatten + validate on the GPU), and the double-buffered pack -> staging ->
unpack migration, with both pools already resident in HBM.  The metric is
fragments per second (a fragment is the contiguous head slice of one
(token, layer, K|V)).  One JSON line is printed; `roofline` describes the
dominant kernel (the stage kernel that packs one chunk while unpacking the
previous one) against the 8 TB/s HBM peak, `cpu_baseline` times the CPU oracle
on a bounded sample of the same recipe.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c3|c3b|c2|c4|c3d] [--staging-mib 64]
  python bench.py --copy-calibration      # plain copies of known size, for scaling PMC byte counters
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
WORKLOAD_DESC = {
    "c5": "config 5: 720896 tokens / 704 requests of 16-bit Llama-8B KV (L=32,H=8,D=128), all 8 heads, "
          "token-granular fully fragmented pages, two 92 GiB pools, 88 GiB payload",
    "c3": "config 3 (paper's microbenchmark top point): 40960 tokens / 40 requests, 5 GiB payload, fully fragmented",
    "c3b": "config 3b (paper's microbenchmark bottom point): 4096 tokens, 0.5 GiB payload",
    "c3c": "config 3c: 40960 tokens, contiguous-per-request layout",
    "c3d": "config 3d: 40960 tokens, TP1->2 / 2->4 / 4->8 slices of 4, 2, 1 heads",
    "c2": "config 2: 16384 tokens / 16 requests, full and half slice",
    "c4": "config 4: 40960 tokens, Zipf(1.1) request lengths, Zipf(1.1) page runs, 4 destinations",
    "c3_p16": "config 3 with 16-token pages (fragmented at page granularity)",
    "c3_fp8": "config 3 with 1-byte KV elements (1 KiB fragments, 2.5 GiB payload)",
    "c3_70b": "16384 tokens of a 70B-class geometry (L=80, 8 KV heads, D=128, 16-bit): 5 GiB payload",
}

# other KV geometries: (base recipe, model shape, page size, tokens)
def _variant_cases(name):
    from workload import make_case, ModelShape, M8B
    if name == "c3_p16":
        return make_case("c3", shape=M8B, p=16)
    if name == "c3_fp8":
        return make_case("c3", shape=ModelShape(L=32, H=8, D=128, e=1))
    if name == "c3_70b":
        return make_case("c3", shape=ModelShape(L=80, H=8, D=128, e=2), tokens=16384)
    return make_case(name)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOAD_DESC))
    ap.add_argument("--staging-mib", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batch", action="store_true",
                    help="workloads with several pairs: one nts_run_migrate per pair instead of one batch call")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--linear", action="store_true",
                    help="TP-shard-selecting linear layer (Sec. 3.2.1): decode and prefill batches of the "
                         "8B model's four layers at TP 1/2/4/8, one JSON line each")
    ap.add_argument("--model", default="8b", choices=("8b", "14b"),
                    help="with --linear: whose layer shapes (the paper serves an 8B and a 14B model)")
    ap.add_argument("--layers", default="qkv,o,gate_up,down", help="with --linear: which of the block's layers")
    ap.add_argument("--tp", default="1,2,4,8", help="with --linear: which TP levels")
    ap.add_argument("--batches", default="1,16,64,256,1024,4096",
                    help="with --linear: the batch sizes M to time")
    ap.add_argument("--tune", action="store_true",
                    help="with --linear: let nts_shard_linear_tune pick each shape's configuration by timing the "
                         "candidates once, and report the default's time beside the tuned one")
    ap.add_argument("--tune-replay", action="store_true",
                    help="with --linear: time every candidate configuration (nts_shard_linear_candidates) by the same "
                         "graph replay as the result itself and keep the fastest (nts_shard_linear_remember): what a "
                         "caller with its own measurement loop gets")
    ap.add_argument("--library", action="store_true",
                    help="with --linear: also time torch.matmul (hipBLASLt) on the same shards, graph-replayed alike")
    ap.add_argument("--planner", action="store_true",
                    help="goodput-efficiency planner (Sec. 3.3.1): planning time at 128 GPUs x 4 tiers (host only)")
    ap.add_argument("--strategies", action="store_true",
                    help="latency of four migration strategies on the paper's payload sizes, one JSON line each")
    ap.add_argument("--no-memcpy", action="store_true",
                    help="with --strategies: skip the per-region memcpy baseline (keeps a profiler trace short)")
    ap.add_argument("--full-memcpy", action="store_true",
                    help="with --strategies: run the per-fragment memcpy baseline at 40960 tokens too (tens of seconds)")
    return ap.parse_args()


class Pair:
    """Device state of one (source, destination) pair case."""

    def __init__(self, b, torch, wdev, case, src_pool=None):
        sh = case.shape
        self.case, self.b = case, b
        self.src = src_pool if src_pool is not None else torch.empty(case.pool_bytes("src"), dtype=torch.uint8, device="cuda")
        if src_pool is None:
            wdev.fill_tensor(self.src, case.seed_src)
        self.dst = torch.empty(case.pool_bytes("dst"), dtype=torch.uint8, device="cuda")
        wdev.fill_tensor(self.dst, case.seed_dst)
        self.sp = b.layer_ptrs(self.src.data_ptr(), sh.L, case.S_src * case.Hs * sh.D * sh.e)
        self.dp = b.layer_ptrs(self.dst.data_ptr(), sh.L, case.S_dst * case.Hd * sh.D * sh.e)

    def plan(self, ctx, staging_bytes):
        """route + plan for this pair."""
        c, b, sh = self.case, self.b, self.case.shape
        so, do, w = b.nts_route(sh.H, c.Ns, c.rs, c.Nd, c.rd)
        return b.nts_plan_create(ctx, L=sh.L, D=sh.D, elem_bytes=sh.e, page_size=c.p, Hs=c.Hs, Hd=c.Hd,
                                 src_head_off=so, dst_head_off=do, w=w, S_src=c.S_src, S_dst=c.S_dst,
                                 ctx_len=c.ctx_len, src_pages=c.src_pages, dst_pages=c.dst_pages,
                                 staging_bytes=staging_bytes, flags=b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST)

    def step(self, ctx, staging, staging_bytes, hip_stream, ev=None):
        """route + plan + migrate + plan_free; returns the plan's info."""
        b = self.b
        plan = self.plan(ctx, staging_bytes)
        info = b.nts_plan_info(plan)
        if ev is not None:
            ev[0].record()
        b.nts_run_migrate(plan, self.sp, self.dp, staging.data_ptr(), hip_stream)
        if ev is not None:
            ev[1].record()
        b.nts_plan_free(plan)
        return info


def copy_ceiling(torch, b, ctx, stream):
    """What a plain linear copy reaches on this GPU, through the same mover: nts_run_pack with
    the identity slot list and whole rows is a straight 1 GiB copy (read once, write once)."""
    import numpy as np
    L, H, D, T = 4, 8, 128, 65536
    pool = torch.empty(L * 2 * T * H * D * 2, dtype=torch.uint8, device="cuda").fill_(7)
    out = torch.empty_like(pool)
    plan = b.nts_plan_create(ctx, L=L, D=D, elem_bytes=2, page_size=1, Hs=H, Hd=H, src_head_off=0, dst_head_off=0,
                             w=H, S_src=T, S_dst=T, ctx_len=[T], src_pages=np.arange(T, dtype=np.int32),
                             dst_pages=np.arange(T, dtype=np.int32), staging_bytes=0, flags=0)
    sp = b.layer_ptrs(pool.data_ptr(), L, T * H * D * 2)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        b.nts_run_pack(plan, sp, out.data_ptr(), stream)
    n = 20
    e0.record()
    for _ in range(n):
        b.nts_run_pack(plan, sp, out.data_ptr(), stream)
    e1.record()
    torch.cuda.synchronize()
    b.nts_plan_free(plan)
    return 2.0 * pool.numel() * n / (e0.elapsed_time(e1) * 1e-3) / 1e9


def measured_traffic(workload: str):
    """Bytes per stage-kernel launch that leave the L2s, from the committed rocprofv3 --pmc
    summary of this workload (counters cannot be read inside a timing run).  The summary
    records the hash of the kernel source it was taken with; a summary taken with another
    version of the kernel is not reported.  Returns (bytes or None, note)."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"nts_stage_kernel_{workload}_pmc.txt")
    try:
        text = open(path).read()
    except OSError:
        return None, "no rocprofv3 --pmc summary committed for this workload"
    src = os.path.join(ROOT, "paper_2605_05467_amd", "csrc", "nts_move.hip")
    sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    m_sha = re.search(r"^kernel_source_sha256:\s*([0-9a-f]{64})", text, flags=re.M)
    if not m_sha or m_sha.group(1) != sha:
        return None, f"profiles/{os.path.basename(path)} was taken with another version of nts_move.hip"
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
    return (float(m.group(1)) if m else None), (
        f"FETCH_SIZE x2 + WRITE_SIZE per dispatch from profiles/{os.path.basename(path)} (same kernel source); "
        "counted where the L2s meet the fabric, so staging bytes served by the memory-side cache are included")


def cpu_baseline(workload: str):
    """The CPU oracle timed on this host, on a bounded sample of the workload: the
    whole configuration when it has at most 40960 tokens (config 3, the headline,
    runs whole), else 40960 tokens of the same recipe (config 5); the first pair of
    a multi-pair workload.  Two figures: the plain single-thread oracle (flatten +
    pack + unpack over the whole sample in one call), and the same oracle with the
    layers dealt to all host cores (layers are independent in its loops; one
    unchanged oracle call per layer from a thread pool).  Both pools are generated
    before the clock starts."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import kvmig as orc
    from workload import fill_words_fast, make_case
    name = workload if workload in ("c5", "c3", "c3b", "c3c", "c3d", "c2", "c4") else "c3"
    full = make_case(name)[0]
    case = full if full.T <= 40960 else make_case(name, tokens=40960)[0]
    sh = case.shape
    so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[sh.e]
    src = fill_words_fast(case.seed_src, 0, case.pool_bytes("src") // 8).view(dt).reshape(sh.L, 2, case.S_src, case.Hs, sh.D)
    dst = fill_words_fast(case.seed_dst, 0, case.pool_bytes("dst") // 8).view(dt).reshape(sh.L, 2, case.S_dst, case.Hd, sh.D)
    F = case.T * sh.L * 2
    # (i) one thread
    t0 = time.perf_counter()
    sslot = orc.flatten(case.ctx_len, case.src_pages, case.p)
    dslot = orc.flatten(case.ctx_len, case.dst_pages, case.p)
    t_flat = time.perf_counter() - t0
    orc.migrate(src, dst, sslot, dslot, so, do, w)
    t_one = time.perf_counter() - t0
    # (ii) all cores: one oracle call per layer
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    workers = max(1, min(cores, sh.L))
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(lambda l: orc.migrate(src[l:l + 1], dst[l:l + 1], sslot, dslot, so, do, w), range(sh.L)))
    t_all = (time.perf_counter() - t0) / reps + t_flat
    sample = (f"{case.T} tokens of the {workload} recipe ({F} fragments of {w * sh.D * sh.e} B, "
              f"{F * w * sh.D * sh.e / 2**30:.2f} GiB payload; "
              + ("the whole configuration" if case.T == full.T else f"the configuration has {full.T} tokens") + ")")
    return {"value": F / t_all, "unit": "fragments/s", "cores": workers, "kind": "oracle",
            "sample": sample + f", flatten + pack + unpack, layers dealt to {workers} threads, "
                               f"{reps} passes of {t_all:.2f} s each",
            "host_cores": cores,
            "single_thread": {"value": F / t_one, "unit": "fragments/s", "cores": 1, "kind": "oracle",
                              "sample": sample + f", flatten + pack + unpack in one call, one pass of {t_one:.2f} s"}}


def copy_calibration(torch):
    """Plain device-to-device copies of known size (for scaling FETCH_SIZE / WRITE_SIZE)."""
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    c = torch.empty(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for _ in range(8):
        c.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "8 copy_ launches", "bytes_read_each": n, "bytes_written_each": n}))


def strategies(args, torch, b, wdev, make_case):
    """The paper's three-strategy comparison (Sec. 3.2.2, Fig. "KV-Migration Latency
    Comparison") on one MI355X, wire left out, plus the pool-to-pool kernel:
    per-fragment memcpy, aggregate-then-scatter without pipelining, the
    double-buffered pipeline, and the direct kernel; fragmented and contiguous layouts."""
    ctx = b.nts_init(0)
    stream = torch.cuda.current_stream().cuda_stream
    staging_bytes = args.staging_mib << 20
    staging = torch.empty(2 * staging_bytes, dtype=torch.uint8, device="cuda")

    def timed(fn, iters):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(iters):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return 1e3 * sorted(ts)[len(ts) // 2]

    for tokens in (4096, 40960):
        for layout, name in (("fragmented", "c3"), ("contiguous", "c3c")):
            case = make_case(name, tokens=tokens)[0]
            pr = Pair(b, torch, wdev, case)
            sh = case.shape
            so, do, w = b.nts_route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
            plan = b.nts_plan_create(ctx, L=sh.L, D=sh.D, elem_bytes=sh.e, page_size=case.p, Hs=case.Hs, Hd=case.Hd,
                                     src_head_off=so, dst_head_off=do, w=w, S_src=case.S_src, S_dst=case.S_dst,
                                     ctx_len=case.ctx_len, src_pages=case.src_pages, dst_pages=case.dst_pages,
                                     staging_bytes=staging_bytes, flags=b.NTS_VALIDATE_UNIQUE_DST)
            info = b.nts_plan_info(plan)
            whole = torch.empty(info.X, dtype=torch.uint8, device="cuda")
            res = {"strategies": True, "tokens": tokens, "layout": layout, "payload_bytes": info.X,
                   "fragments": info.F, "unit": "ms (median, host clock around enqueue + synchronise)"}
            n_copies = [0]

            def memcpy_run():
                n_copies[0] = b.nts_run_memcpy_baseline(plan, pr.sp, pr.dp, layout == "contiguous", stream)

            if not args.no_memcpy and (tokens <= 4096 or args.full_memcpy or layout == "contiguous"):
                res["memcpy_per_region"] = timed(memcpy_run, 1 if tokens > 4096 and layout == "fragmented" else 3)
                res["memcpy_calls"] = n_copies[0]

            def aggregate_run():
                b.nts_run_pack(plan, pr.sp, whole.data_ptr(), stream)
                b.nts_run_unpack(plan, whole.data_ptr(), pr.dp, stream)

            res["aggregate_unpipelined"] = timed(aggregate_run, 10)
            res["pipelined_double_buffer"] = timed(
                lambda: b.nts_run_migrate(plan, pr.sp, pr.dp, staging.data_ptr(), stream), 10)
            res["direct_pool_to_pool"] = timed(lambda: b.nts_run_migrate_direct(plan, pr.sp, pr.dp, stream), 10)
            b.nts_plan_free(plan)
            # the same kernel walking the tokens in ascending destination-slot order (plan flag)
            plan = b.nts_plan_create(ctx, L=sh.L, D=sh.D, elem_bytes=sh.e, page_size=case.p, Hs=case.Hs, Hd=case.Hd,
                                     src_head_off=so, dst_head_off=do, w=w, S_src=case.S_src, S_dst=case.S_dst,
                                     ctx_len=case.ctx_len, src_pages=case.src_pages, dst_pages=case.dst_pages,
                                     staging_bytes=staging_bytes,
                                     flags=b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST)
            res["direct_pool_to_pool_dst_order"] = timed(lambda: b.nts_run_migrate_direct(plan, pr.sp, pr.dp, stream), 10)
            b.nts_plan_free(plan)
            del whole, pr
            print(json.dumps(res), flush=True)
    del staging
    b.nts_free(ctx)


def linear_bench(args, torch, b):
    """Shard-selecting linear layer: rank tp-1 of each TP level computes with its 1/tp of the
    full weight.  Batches up to 256 rows are HBM-bound: bytes = the shard read once (+X, +Y).
    Prefill batches are matrix-core-bound: 2*M*Nn*K flops against 2.5 PFLOP/s (bf16, dense).
    Launches are captured into a HIP graph that walks through more than 3 GiB of distinct
    weight copies, so no shard is served from a cache and launch gaps do not hide the kernels."""
    from workload.linear import LAYERS
    from workload import device as wdev
    ctx = b.nts_init(0)
    # measured ceilings beside the nominal peaks: the matrix cores alone on random operands (the clock
    # they sustain is power-limited and data-dependent) and a read-only HBM stream
    mfma_ceiling = wdev.mfma_ceiling_tflops()
    read_ceiling = wdev.read_ceiling_gbs()
    print(json.dumps({"linear_ceilings": {"mfma_bf16_TFLOPs_measured": mfma_ceiling, "mfma_bf16_TFLOPs_nominal": 2500.0,
                                          "hbm_read_GBs_measured": read_ceiling, "hbm_GBs_nominal": HBM_PEAK_GBS,
                                          "how": "workload/fill_gpu.hip probes: 4 x 4 v_mfma_f32_32x32x16_bf16 tiles per "
                                                 "wavefront on pseudo-random registers, four wavefronts per CU; eight "
                                                 "16-byte non-temporal loads per lane over 1 GiB"}}), flush=True)
    for layer in [f"{args.model}_{name}" for name in args.layers.split(",")]:
        n_out, n_in, split = LAYERS[layer]
        wbytes = n_out * n_in * 2
        copies = max(2, (3 << 30) // wbytes + 1)
        W = (torch.rand(copies, n_out, n_in, device="cuda") * 0.08 - 0.04).to(torch.bfloat16)
        for tp in [int(x) for x in args.tp.split(",")]:
            for M in [int(x) for x in args.batches.split(",")]:
                k = n_in if split == "out" else n_in // tp
                nn = n_out // tp if split == "out" else n_out
                X = (torch.rand(M, k, device="cuda") * 4 - 2).to(torch.bfloat16)
                Y = torch.empty(M, nn, device="cuda", dtype=torch.bfloat16)
                kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=tp - 1,
                          split=b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN)
                wsb = b.nts_shard_linear_workspace(**kw)
                how = b.nts_shard_linear_launch(**kw)
                ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")

                def launch(i):
                    b.nts_shard_linear(ctx, X.data_ptr(), W[i % copies].data_ptr(), Y.data_ptr(),
                                       workspace=ws.data_ptr(), workspace_bytes=wsb,
                                       hip_stream=torch.cuda.current_stream().cuda_stream, **kw)

                n_launch = copies * 2 if M <= 256 else max(4, copies)

                def replay_us():
                    launch(0)
                    torch.cuda.synchronize()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph):
                        for i in range(n_launch):
                            launch(i)
                    graph.replay()
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    ts = []
                    for _ in range(5):
                        e0.record()
                        graph.replay()
                        e1.record()
                        torch.cuda.synchronize()
                        ts.append(e0.elapsed_time(e1) * 1e3 / n_launch)
                    del graph
                    return sorted(ts)[2]

                us = replay_us()
                default_us = None
                if args.tune:
                    default_us, default_how = us, how
                    wsb = max(wsb, 8 * M * nn * 4)         # room for up to eight K splits
                    ws = torch.empty(wsb + 16, dtype=torch.uint8, device="cuda")
                    how = b.nts_shard_linear_tune(ctx, X.data_ptr(), [W[i].data_ptr() for i in range(copies)], Y.data_ptr(), workspace=ws.data_ptr(),
                                                  workspace_bytes=wsb,
                                                  hip_stream=torch.cuda.current_stream().cuda_stream, **kw)
                    torch.cuda.synchronize()
                    us = replay_us()
                if args.tune_replay:
                    default_us, default_how = us, how
                    wsb = max(wsb, 32 * M * nn * 4)        # room for every candidate's K split
                    ws = torch.empty(wsb + 16, dtype=torch.uint8, device="cuda")
                    best = (us, how)
                    cand_us = [(how, us)]
                    for cand in b.nts_shard_linear_candidates(**kw)[1:]:
                        b.nts_shard_linear_remember(ctx, cand, **kw)
                        t = replay_us()
                        cand_us.append((cand, t))
                        if t < best[0]:
                            best = (t, cand)
                    b.nts_shard_linear_remember(ctx, best[1], **kw)
                    us, how = best
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                lib_us = None
                if args.library:
                    # the same shard through torch.matmul (hipBLASLt), replayed from a graph in the same way
                    # (the shard as the library's own view of the full matrix: offset, rows, columns, row stride)
                    v_off, v_rows, v_cols, v_rs = b.nts_shard_linear_view(**kw)
                    # (as_strided takes the offset from the start of the storage, so each copy's own offset is added)
                    Wv = [torch.as_strided(W, (v_rows, v_cols), (v_rs, 1), W[i].storage_offset() + v_off) for i in range(copies)]
                    torch.matmul(X, Wv[0].t(), out=Y)
                    torch.cuda.synchronize()
                    lgraph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(lgraph):
                        for i in range(n_launch):
                            torch.matmul(X, Wv[i % copies].t(), out=Y)
                    lgraph.replay()
                    torch.cuda.synchronize()
                    ts = []
                    for _ in range(5):
                        e0.record()
                        lgraph.replay()
                        e1.record()
                        torch.cuda.synchronize()
                        ts.append(e0.elapsed_time(e1) * 1e3 / n_launch)
                    lib_us = sorted(ts)[2]
                    del lgraph
                shard_bytes = nn * k * 2
                # below ~312 flop per weight byte (2.5 PFLOP/s / 8 TB/s) the layer is bound by reading the shard
                if M <= 256:
                    ach = (shard_bytes + M * k * 2 + M * nn * 2) / us / 1e3
                    roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                            "read_ceiling": read_ceiling, "frac_of_read_ceiling": ach / read_ceiling}
                else:
                    ach = 2.0 * M * nn * k / us / 1e6
                    roof = {"bound": "mfma", "achieved": ach, "peak": 2500.0, "unit": "TFLOP/s", "frac": ach / 2500.0,
                            "mfma_ceiling": mfma_ceiling, "frac_of_mfma_ceiling": ach / mfma_ceiling}
                print(json.dumps({"linear": layer, "split": split, "tp": tp, "rank": tp - 1, "M": M, "Nn": nn, "K": k,
                                  "shard_MiB": shard_bytes / 2**20, "us_per_call": us, "dtype": "bf16",
                                  "kernel": "tiled" if how.tiled else "decode" if how.tile_rows == 16 else "stream",
                                  "tile": "%dx%d" % (how.tile_rows, how.tile_cols), "k_splits": how.k_splits,
                                  "roofline": roof,
                                  **({"default_us_per_call": default_us,
                                      "default_kernel": "tiled" if default_how.tiled else "decode" if default_how.tile_rows == 16 else "stream",
                                      "default_tile": "%dx%d" % (default_how.tile_rows, default_how.tile_cols),
                                      "default_k_splits": default_how.k_splits} if default_us else {}),
                                  **({"candidates_us": [["tiled" if c_.tiled else "decode" if c_.tile_rows == 16 else "stream",
                                                         "%dx%d" % (c_.tile_rows, c_.tile_cols), c_.k_splits, c_.k_waves, t_]
                                                        for c_, t_ in cand_us]} if args.tune_replay else {}),
                                  **({"library_us_per_call": lib_us, "vs_library": us / lib_us} if lib_us else {})}),
                      flush=True)
        del W
    b.nts_free(ctx)
    if not args.no_cpu_baseline:
        # the oracle (slice, then fp64 matmul of the exact 16-bit values) timed beside it on the host
        import numpy as np
        import threadpoolctl
        from oracle import shard_linear as osl
        from workload.linear import linear_inputs
        n_out, n_in, split = LAYERS["8b_gate_up"]
        M, tp = 2048, 1
        Xh, Wh = linear_inputs(11, M, n_out, n_in, x_cols=n_in)
        X64, W64 = osl.bf16_to_f64(Xh), osl.bf16_to_f64(Wh)
        reps = 8
        t0 = time.perf_counter()
        for _ in range(reps):
            osl.shard_linear(X64, W64, tp, tp - 1, split)
        dt = (time.perf_counter() - t0) / reps
        threads = max((p_["num_threads"] for p_ in threadpoolctl.threadpool_info()), default=1)
        flops = 2.0 * 2 * M * (n_out // tp) * n_in             # the product and the error-bound product
        print(json.dumps({"linear_cpu_baseline": {"value": flops / dt / 1e12, "unit": "TFLOP/s (fp64)", "cores": threads,
                                                  "kind": "oracle", "seconds": dt,
                                                  "sample": f"8b_gate_up TP{tp} rank {tp - 1}, M = {M}: slice + two "
                                                            f"{M} x {n_out // tp} x {n_in} fp64 products, {reps} passes"}}), flush=True)


def planner_bench():
    """Planning time of one control window at the size the paper quotes (128 GPUs,
    four request groups; Sec. 4.2.3), on synthetic capacity tables; host code only."""
    from oracle import planner as op
    from paper_2605_05467_amd import binding as b
    from workload.planner import synthetic_tiers
    for n_gpus, n_tiers in ((128, 4), (1024, 8)):
        tiers = synthetic_tiers(2024, n_tiers, rps_scale=100.0 * n_gpus / 32)
        reps = 2000
        t0 = time.perf_counter()
        for _ in range(reps):
            allocs, left = b.nts_plan_cluster(n_gpus, tiers)
        dt = (time.perf_counter() - t0) / reps
        t0 = time.perf_counter()
        want, wleft = op.plan(n_gpus, [op.Tier(*t) for t in tiers])
        dt_oracle = time.perf_counter() - t0
        same = [(a.tier, a.tp_prefill, a.tp_decode, a.P, a.D) for a in allocs] == \
               [(a.tier, a.tp_prefill, a.tp_decode, a.P, a.D) for a in want] and left == wleft
        print(json.dumps({"planner": True, "n_gpus": n_gpus, "n_tiers": n_tiers, "configs_enumerated": n_tiers * 16,
                          "greedy_steps": len(allocs), "gpus_left": left, "us_per_plan": dt * 1e6,
                          "includes": "ctypes marshalling of tiers and results", "threads": 1,
                          "matches_oracle": same,
                          "cpu_baseline": {"value": dt_oracle * 1e6, "unit": "us per plan", "kind": "oracle", "cores": 1},
                          "paper_context": "2.49 ms average at 128 GPUs x 4 groups, multi-threaded Rust, other hardware"}))


def main():
    args = parse_args()
    if args.planner:
        planner_bench()
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); multi-GPU runs are not part of it",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_05467_amd import binding as b
    from workload import device as wdev
    from workload import make_case

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        copy_calibration(torch)
        return
    if args.strategies:
        strategies(args, torch, b, wdev, make_case)
        return
    if args.linear:
        linear_bench(args, torch, b)
        return

    cases = _variant_cases(args.workload)
    ctx = b.nts_init(0)
    stream = torch.cuda.current_stream().cuda_stream
    staging_bytes = args.staging_mib << 20
    staging = torch.empty(2 * staging_bytes, dtype=torch.uint8, device="cuda")
    pairs = []
    shared_src = None
    for case in cases:                       # config 4's destinations share one source pool
        share = shared_src if (shared_src is not None and args.workload == "c4") else None
        pr = Pair(b, torch, wdev, case, share)
        shared_src = pr.src
        pairs.append(pr)
    torch.cuda.synchronize()

    batch = len(pairs) > 1 and not args.no_batch

    def one_step(evs=None):
        if not batch:
            return [pr.step(ctx, staging, staging_bytes, stream, None if evs is None else evs[i])
                    for i, pr in enumerate(pairs)]
        # several pairs: plan them all, then ONE pipeline through the two staging buffers
        plans = [pr.plan(ctx, staging_bytes) for pr in pairs]
        infos = [b.nts_plan_info(p) for p in plans]
        if evs is not None:
            evs[0][0].record()
        b.nts_run_migrate_batch(plans, [pr.sp for pr in pairs], [pr.dp for pr in pairs], staging.data_ptr(), stream)
        if evs is not None:
            evs[0][1].record()
        for p in plans:
            b.nts_plan_free(p)
        return infos

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    evs = [[[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)]
            for _ in (pairs[:1] if batch else pairs)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        infos = one_step(evs[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = 1e3 * (t1 - t0) / args.steps
    # In the timed loop the planning of step k+1 runs while the GPU still executes step k's
    # launches (run calls only enqueue).  Beside it: one step at a time with the device idle before
    # and after (no overlap between steps), and the planning part alone; medians of five.
    alone, plan_alone = [], []
    for _ in range(5):
        torch.cuda.synchronize()
        ta = time.perf_counter()
        one_step()
        torch.cuda.synchronize()
        alone.append(1e3 * (time.perf_counter() - ta))
        ta = time.perf_counter()
        for p_ in [pr.plan(ctx, staging_bytes) for pr in pairs]:
            b.nts_plan_free(p_)
        plan_alone.append(1e3 * (time.perf_counter() - ta))
    F = sum(i.F for i in infos)
    X = sum(i.X for i in infos)
    T = sum(i.T for i in infos)
    # a batch chains the pairs' chunks: one launch per chunk plus one to drain the pipeline
    launches = sum(i.n_chunks for i in infos) + 1 if batch else sum(i.n_chunks + 1 for i in infos)
    kernel_ms = sum(e[0].elapsed_time(e[1]) for step in evs for e in step) / args.steps
    # algorithmic HBM bytes: each payload byte is read from the pool and written to staging
    # by the pack half, read from staging and written to the pool by the unpack half
    alg_bytes_per_launch = 4.0 * X / launches
    avg_launch_ms = kernel_ms / launches
    achieved = alg_bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    traffic, traffic_note = measured_traffic(args.workload)
    n_pairs = len(pairs)
    del pairs, staging
    torch.cuda.empty_cache()
    ceiling = copy_ceiling(torch, b, ctx, stream)

    out = {
        "metric": "hot-path items/sec on 1 MI355X (fragments/s through route+plan+pack+staging+unpack)",
        "value": F / (ms_per_step * 1e-3),
        "unit": "fragments/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOAD_DESC[args.workload]}",
                   "tokens": T, "fragments": F, "fragment_bytes": infos[0].frag_bytes,
                   "payload_bytes": X, "staging_bytes_each": infos[0].chunk_bytes,
                   "stage_launches_per_step": launches, "pairs": n_pairs,
                   "pairs_run_as": "one batch (nts_run_migrate_batch)" if batch else "one call per pair"},
        "ms_per_step_one_at_a_time": sorted(alone)[2],
        "plan_ms_alone": sorted(plan_alone)[2],
        "steps_overlap": "run calls only enqueue, so in the timed loop a step's route + plan runs while the previous "
                         "step's launches execute; ms_per_step_one_at_a_time has the device idle before and after "
                         "each step, plan_ms_alone is route + nts_plan_create + nts_plan_free by themselves",
        "tokens_per_s": T / (ms_per_step * 1e-3),
        "payload_GBps": X / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "kernel": "nts_stage_kernel<16> (pack chunk k || unpack chunk k-1)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_how": traffic_note,
                     "copy_ceiling": ceiling, "frac_of_copy_ceiling": achieved / ceiling,
                     "copy_ceiling_how": "plain 1 GiB linear copy through the same mover (identity slot list), "
                                         "measured in this run",
                     "note": "the two staging buffers (half of the algorithmic bytes) are kept in the 256 MiB "
                             "memory-side cache when together they fit it, which is why the figure can exceed copy_ceiling",
                     "algorithmic_bytes_per_launch": alg_bytes_per_launch,
                     "avg_launch_ms": avg_launch_ms, "launches_per_step": launches,
                     "timing": "HIP events on the launch stream around each step's stage launches "
                               "(includes the gaps between back-to-back launches)"},
    }
    b.nts_free(ctx)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
