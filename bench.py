#!/usr/bin/env python3
"""Benchmark of the KV page codec on one MI355X.

A step is one pass of the whole hot path over the workload, inputs resident in HBM:
    reset pool -> kvc_compress_blocks (all pages) -> kvc_decompress_blocks (all pages)
    -> kvc_gather_decompress (one decode step's predicted blocks).
`value` = uncompressed FP16 bytes processed per second over the whole step.  Per-kernel durations come
from HIP events recorded on the launch stream inside the timed region; the roofline entry is
algorithmic bytes (read + written, measured from the descriptors) over that duration against the
8 TB/s HBM3E peak.  The CPU oracle is timed on a bounded sample of the same bytes as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 70b_gqa|7b_full|7b_layer|tiny|decode_gather]
    python bench.py --workload geometry --tokens-per-block N --head-dim d    (a 2 GB slice of another page shape)
    python bench.py --workload prefetch_pipeline | prefetch_window | host_pool ;  python bench.py --ablation
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def kernel_fingerprint() -> str:
    """Identifies the kernel sources a measurement belongs to: SHA-256 over the files of csrc/ (kernels and
    the host code that launches them; names and contents), first 16 hex digits.  The profile summaries
    carry the value of the run they were taken from."""
    import hashlib

    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2512_11920_amd", "csrc")
    for path in sorted(os.path.join(csrc, f) for f in os.listdir(csrc)):
        h.update(os.path.basename(path).encode() + b"\0")
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def read_traffic(tag: str, kernel: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one
    (profiles/hbm_traffic_<tag>.txt, lines `<kernel>_traffic_bytes: <int>` and `kernel_fingerprint: <hex>`).
    -> (bytes or None, where the number comes from).  A summary taken on other kernel sources than the
    ones in the tree is not used: the number is then None and the source says why."""
    rel = os.path.join("profiles", f"hbm_traffic_{tag}.txt")
    p = os.path.join(ROOT, rel)
    if not os.path.exists(p):
        return None, {"file": None, "note": "no rocprofv3 --pmc summary is committed for this workload"}
    val, fp, name = None, None, None
    for line in open(p):
        # `kernel` is k_compress or k_decompress
        if line.startswith(kernel) and "_traffic_bytes:" in line:
            name, val = line.split("_traffic_bytes:")[0], int(float(line.split(":")[1].split()[0]))
        if line.startswith("kernel_fingerprint:"):
            fp = line.split(":")[1].strip()
    now = kernel_fingerprint()
    src = {"file": rel, "kernel": name, "profile_kernel_fingerprint": fp, "current_kernel_fingerprint": now}
    if fp != now:
        src["note"] = "summary was taken on other kernel sources: not used"
        return None, src
    return val, src


def device_info():
    """What the runtime reports about the GPU, recorded beside the pinned 8 TB/s peak."""
    import torch

    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "hbm_GB": round(p.total_memory / 1e9, 1)}
    from paper_2512_11920_amd import kvc

    ck = kvc.device_clocks()
    info.update({"arch": p.gcnArchName, "shader_clock_MHz": round(ck["shader_khz"] / 1e3), "memory_clock_MHz": round(ck["memory_khz"] / 1e3),
                 "memory_bus_bits": ck["memory_bus_bits"]})
    return info


def choose_placement(codec, blocks, pool_bytes, dev, mode):
    """Allocate the compressed pool and the output buffer.  This GPU's HBM behaves as three regions of about
    96 GB, and any kernel (a plain copy too) runs 4-7 % slower when the buffer it reads and the buffer it
    writes lie in the same region; which region an allocation lands in is the driver's choice and differs from
    process to process.  mode "search" (buffers of 8 GB and more): allocate up to three candidate pools and
    four candidate output buffers (about 120 GB in allocation order, so they straddle a region boundary), time
    compress into every pool and decompress from it into every output buffer, keep the pair with the smallest
    sum and free the rest -- what a serving process can do once at start-up.  mode "first": one of each, as
    allocated.  -> (output buffer, record of what was measured, for the bench line)."""
    import numpy as np
    import torch

    n_blocks = blocks.shape[0]
    out_bytes = blocks.numel() * 2
    desc_bytes = n_blocks * codec.cfg.pages_per_block * 16

    def new_pool():
        return (torch.empty(pool_bytes, dtype=torch.uint8, device=dev), torch.empty(desc_bytes, dtype=torch.uint8, device=dev))

    if mode != "search" or out_bytes < (8 << 30):
        codec.bind_pool(*new_pool())
        codec.reset_pool()
        return torch.empty_like(blocks), {"searched": False}
    free = torch.cuda.mem_get_info()[0] - (24 << 30)  # room for the gather output and the allocator's slack
    n_pool, n_out = 3, 4
    while n_out > 1 and n_pool * pool_bytes + n_out * out_bytes > free:
        n_out -= 1
    while n_pool > 1 and n_pool * pool_bytes + n_out * out_bytes > free:
        n_pool -= 1
    pools = [new_pool() for _ in range(n_pool)]
    outs = [torch.empty_like(blocks) for _ in range(n_out)]

    def timed(fn, reps=3):
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]))

    def comp():
        codec.reset_pool()
        codec.compress_blocks(blocks)

    codec.bind_pool(*pools[0])
    for _ in range(4):  # the shader clock ramps up over the first launches
        comp()
        codec.decompress_blocks(outs[0])
    t_c, t_d = [], []
    for pool, desc in pools:
        codec.bind_pool(pool, desc)
        t_c.append(timed(comp))
        t_d.append([timed(lambda o=o: codec.decompress_blocks(o)) for o in outs])
    i, j = min(((i, j) for i in range(n_pool) for j in range(n_out)), key=lambda ij: t_c[ij[0]] + t_d[ij[0]][ij[1]])
    pool, out = pools[i], outs[j]
    del pools, outs
    torch.cuda.empty_cache()
    codec.bind_pool(*pool)
    codec.reset_pool()
    rec = {"searched": True, "compress_ms_by_pool": [round(t, 3) for t in t_c],
           "decompress_ms_by_pool_and_output": [[round(t, 3) for t in row] for row in t_d], "chosen_pool_and_output": [i, j]}
    return out, rec


def sample_check(codec, cache_blocks, out_blocks, n_sample, N, d, ppb, scheme):
    """Compare a random sample of pages (descriptor, payload, decoded values) with the oracle."""
    import numpy as np
    import torch

    from oracle import kvc_oracle as o

    n_pages = cache_blocks.shape[0] * ppb
    g = np.random.default_rng(12345)
    ids = np.unique(g.integers(0, n_pages, n_sample))
    idt = torch.from_numpy(ids).to(cache_blocks.device)
    x = cache_blocks.view(-1, N, d)[idt].cpu().numpy().view(np.uint16)
    y = out_blocks.view(-1, N, d)[idt].cpu().numpy().view(np.uint16)
    desc = codec.desc.view(-1, 16)[idt].cpu().numpy().view(codec_desc_dtype()).ravel()
    od, op = o.compress_pages(x, N, d, scheme, n_threads=8)
    ok = (np.array_equal(desc["mode"], od["mode"]) and np.array_equal(desc["n16"], od["n16"])
          and np.array_equal(desc["scale"].view(np.uint32), od["scale"].view(np.uint32)))
    for i in range(len(ids)):
        a, n = int(desc["off"][i]), int(desc["n16"][i]) * 16
        ok = ok and codec.pool[a:a + n].cpu().numpy().tobytes() == o.page_payload(op, od[i])
        if i >= 256:
            break
    want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
    ok = ok and bad == 0 and np.array_equal(want, y)
    return bool(ok), len(ids)


def codec_desc_dtype():
    from paper_2512_11920_amd import kvc

    return kvc.DESC_DTYPE


def cpu_baseline(sample_u16, N, d, scheme, target_s=12.0):
    """Oracle compress + decompress on host cores over a bounded sample.  GB/s of uncompressed FP16
    (bytes through compress + bytes through decompress) / elapsed."""
    from oracle import kvc_oracle as o

    cores = max(1, min(16, os.cpu_count() or 1))  # threads the oracle runs on
    n_pages = sample_u16.shape[0]
    done_bytes, t_total, reps = 0, 0.0, 0
    while t_total < target_s and reps < 16:
        t0 = time.perf_counter()
        od, op = o.compress_pages(sample_u16, N, d, scheme, n_threads=cores)
        out, bad = o.decompress_pages(op, od, N, d, n_threads=cores)
        t_total += time.perf_counter() - t0
        done_bytes += 2 * sample_u16.nbytes
        reps += 1
    # the same on one thread, over a sixteenth of the sample
    one = sample_u16[: max(1, n_pages // 16)]
    t0 = time.perf_counter()
    od, op = o.compress_pages(one, N, d, scheme, n_threads=1)
    o.decompress_pages(op, od, N, d, n_threads=1)
    t_one = time.perf_counter() - t0
    return {"value": round(done_bytes / t_total / 1e9, 4), "unit": "GB/s", "cores": cores, "host_cpus": os.cpu_count(), "kind": "oracle",
            "sample": f"{n_pages} pages ({sample_u16.nbytes / 2**20:.0f} MiB of the same seeded cache), "
                      f"compress+decompress x{reps}, {t_total:.1f} s",
            "single_thread_value": round(2 * one.nbytes / t_one / 1e9, 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 10; decode_gather: 1000, as the config is stated)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="70b_gqa")
    ap.add_argument("--scheme", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (quick runs; not the headline)")
    ap.add_argument("--tokens-per-block", type=int, default=16, help="workload geometry: tokens per page (N)")
    ap.add_argument("--head-dim", type=int, default=128, help="workload geometry: channels per token (d)")
    ap.add_argument("--prefetch-policy", type=int, default=1, help="prefetch_pipeline: 0 positional slots, 1 slot reuse")
    ap.add_argument("--ablation", action="store_true", help="ratio and speed per scheme (Table 9 analogue)")
    ap.add_argument("--placement", choices=("search", "first"), default="search",
                    help="pool and output buffer: the best of a few candidate allocations (see choose_placement), or the first")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 1000 if args.workload == "decode_gather" else 10
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (pages are independent; no collective exists "
              "on the path). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2512_11920_amd import kvc, synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.ablation:
        return bench_ablation(args)
    if args.workload == "decode_gather":
        return bench_decode_gather(args)
    if args.workload == "prefetch_pipeline":
        return bench_prefetch_pipeline(args)
    if args.workload == "host_pool":
        return bench_host_pool(args)
    if args.workload == "prefetch_window":
        return bench_prefetch_window(args)
    if args.workload == "geometry":
        # a slice of about 2 GB with the 70B config's layout (8 KV heads, 4096-token sequences) and another page shape
        gN, gd = args.tokens_per_block, args.head_dim
        shape = synth.KVShape(f"geometry_{gN}x{gd}", 8, 8, gd, 4096, max(1, round(16 * 128 / gd)), tokens_per_block=gN)
    else:
        shape = synth.CONFIGS[args.workload]
    if args.layers:
        import dataclasses

        shape = dataclasses.replace(shape, n_layers=args.layers, name=f"{shape.name}[{args.layers} layers]")
    N, d, H = shape.tokens_per_block, shape.head_dim, shape.n_kv_heads
    ppb = H
    E = N * d
    log(f"[bench] building {shape.name}: {shape.n_pages} pages, {shape.nbytes / 1e9:.2f} GB fp16")
    pool_bytes = (shape.n_pages * (E if args.scheme else 2 * E) + 4096) // 16 * 16
    codec = kvc.Codec(N, d, ppb, args.scheme)
    cache = synth.cache_torch(shape, dev)
    blocks = cache.view(-1, ppb, N, d)
    out, placement = choose_placement(codec, blocks, pool_bytes, dev, args.placement)
    log(f"[bench] placement: {placement}")
    n_blocks = blocks.shape[0]

    # decode-step pattern over the same pool: each (sequence, K|V) is a table row of its blocks
    bps = shape.seq_len // N
    rows = 2 * shape.batch
    table = (torch.arange(rows, dtype=torch.int32, device=dev)[:, None] * bps
             + torch.arange(bps, dtype=torch.int32, device=dev)[None, :])
    # kv-major layout: pool block of (kv, seq, blk) within a layer = (kv*batch + seq)*bps + blk = row*bps + blk
    table = table.contiguous()
    k = min(8, bps)
    gen = torch.Generator(device=dev)
    gen.manual_seed(shape.seed + 99)
    pred = torch.randint(0, bps, (rows, k), generator=gen, device=dev, dtype=torch.int32)
    g_out = torch.empty((shape.n_layers * rows * k, ppb, N, d), dtype=torch.float16, device=dev)
    pbpl = 2 * shape.blocks_per_layer

    stream = torch.cuda.current_stream()

    def step(ev=None):
        codec.reset_pool()
        if ev:
            ev[0].record()
        codec.compress_blocks(blocks)
        if ev:
            ev[1].record()
        codec.decompress_blocks(out)
        if ev:
            ev[2].record()
        codec.gather_decompress(g_out, table, pred, shape.n_layers, pbpl)
        if ev:
            ev[3].record()

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # statistics and the parity sample come from the last timed step's pool and output (host work: kept
    # out of the way of the timed region, which therefore follows the warm-up steps directly)
    st = codec.stats()
    assert st["rc"] == 0, st
    n_live = sum(st["pages"])
    payload = st["payload_bytes"]
    ratio = codec.ratio()
    check_ok, n_checked = sample_check(codec, blocks, out, 512, N, d, ppb, args.scheme)
    log(f"[bench] modes {st['pages']} ratio {ratio:.4f} sample parity vs oracle on {n_checked} pages: {check_ok}")
    ms_step = (t1 - t0) * 1e3 / args.steps
    per_step = {"compress": [e[0].elapsed_time(e[1]) for e in evs], "decompress": [e[1].elapsed_time(e[2]) for e in evs],
                "gather_decompress": [e[2].elapsed_time(e[3]) for e in evs]}
    t_c, t_d, t_g = (sum(per_step[k_]) / args.steps for k_ in ("compress", "decompress", "gather_decompress"))

    unc = shape.nbytes
    g_pages = g_out.numel() // E
    g_unc = g_out.numel() * 2
    # algorithmic bytes: page in + payload + descriptor out (compress); the reverse (decompress);
    # gather reads its pages' payloads (mean payload size) + descriptors + 4 B of ids per block
    alg_c = unc + payload + 16 * n_live
    alg_d = alg_c
    alg_g = g_unc + g_pages * (payload / n_live + 16) + 8 * (g_pages // ppb)
    kern = {
        "compress": {"ms": t_c, "uncompressed_GBps": unc / t_c / 1e6, "hbm_GBps": alg_c / t_c / 1e6, "alg_bytes": alg_c},
        "decompress": {"ms": t_d, "uncompressed_GBps": unc / t_d / 1e6, "hbm_GBps": alg_d / t_d / 1e6, "alg_bytes": alg_d},
        "gather_decompress": {"ms": t_g, "uncompressed_GBps": g_unc / t_g / 1e6, "hbm_GBps": alg_g / t_g / 1e6,
                              "alg_bytes": alg_g},
    }
    for k_, v in kern.items():
        v["frac_of_peak"] = v["hbm_GBps"] / HBM_PEAK_GBS
        v["ms_min"], v["ms_max"], v["ms_p50"] = min(per_step[k_]), max(per_step[k_]), float(np.median(per_step[k_]))
    # same-run yardstick: plain 128-bit copy of the cache
    cp = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    src8, dst8 = blocks.view(torch.uint8).view(-1), out.view(torch.uint8).view(-1)
    for _ in range(3):
        kvc.copy_bytes(dst8, src8)
    cp[0].record()
    for _ in range(3):
        kvc.copy_bytes(dst8, src8)
    cp[1].record()
    torch.cuda.synchronize()
    t_copy = cp[0].elapsed_time(cp[1]) / 3
    copy_gbps = 2 * unc / t_copy / 1e6
    for v in kern.values():
        v["frac_of_copy"] = v["hbm_GBps"] / copy_gbps

    dom = "compress" if t_c >= t_d else "decompress"
    tag = shape.name + (f"_scheme{args.scheme}" if args.scheme != 3 else "")
    traffic, traffic_source = (None, {"file": None, "note": "layer count overridden"}) if args.layers else read_traffic(tag, "k_" + dom)
    # the kernel behind the entry point; the committed profile of the workload names it
    kname = traffic_source.get("kernel") or f"k_{dom}"
    res = {
        "metric": "KV codec GB/s (uncompressed fp16) compress+decompress; % of HBM peak",
        "value": round((2 * unc + g_unc) / (ms_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{shape.name}: {shape.n_layers} layers x {H} KV heads x {d}, seq {shape.seq_len}, "
                               f"batch {shape.batch}, {N}-token blocks, K+V {unc / 1e9:.2f} GB fp16, scheme {args.scheme}",
                   "pages": shape.n_pages, "ratio": round(ratio, 4), "pages_per_mode": st["pages"],
                   "gather": f"{rows} rows x {k} predicted blocks x {shape.n_layers} layers = {g_pages} pages"},
        "roofline": {"bound": "hbm", "kernel": kname, "achieved": round(kern[dom]["hbm_GBps"], 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(kern[dom]["frac_of_peak"], 4),
                     "traffic": traffic, "traffic_source": traffic_source, "alg_bytes_per_launch": int(kern[dom]["alg_bytes"]),
                     "launch_ms": round(kern[dom]["ms"], 4)},
        "kernel_fingerprint": kernel_fingerprint(),
        "kernels": {k_: {a: (round(b, 4) if isinstance(b, float) else b) for a, b in v.items()} for k_, v in kern.items()},
        "copy_kernel_GBps": round(copy_gbps, 1),
        "sample_parity_vs_oracle": check_ok,
        "device": device_info(),
        "placement": placement,
    }
    if not args.no_cpu_baseline:
        # the first layers of the same cache, moved to the host
        per_layer = shape.pages_per_layer
        n_layers_s = max(1, min(shape.n_layers, (1 << 30) // (per_layer * E * 2) or 1))
        sample = cache[:n_layers_s].reshape(-1, N, d).cpu().numpy().view(np.uint16)
        res["cpu_baseline"] = cpu_baseline(sample, N, d, args.scheme, args.cpu_seconds)
    print(json.dumps(res), flush=True)


def bench_decode_gather(args):
    """Decode-step prefetch pattern, 70B shape: 64 sequences with lengths ~U[512, 8192], block tables
    permuted in the pool, 8 predicted blocks per sequence per layer per step.  The pool is built
    layer by layer (one layer of raw KV at a time)."""
    import numpy as np
    import torch

    from paper_2512_11920_amd import kvc, synth

    dev = "cuda:0"
    shape = synth.KVShape("decode_gather", 80, 8, 128, 0, 0)
    N, d, H = 16, 128, 8
    ppb, E = 2 * H, N * d
    pat = synth.gather_pattern(64, 8, 512, 8192, N, seed=0)
    pbl = pat.pool_blocks_per_layer
    n_pool_blocks = shape.n_layers * pbl
    log(f"[bench] decode_gather: {pbl} blocks/layer, pool of {n_pool_blocks * ppb} pages "
        f"({n_pool_blocks * ppb * E * 2 / 1e9:.1f} GB raw)")
    codec = kvc.Codec(N, d, ppb, args.scheme)
    codec.alloc_pool(n_pool_blocks, n_pool_blocks * ppb * E + 4096, dev)
    ids = torch.arange(pbl, dtype=torch.int32, device=dev)
    for l in range(shape.n_layers):
        layer = synth.gather_layer_torch(shape, pat, l, dev)
        codec.compress_blocks(layer.view(-1, ppb, N, d), pool_ids=ids + l * pbl)
    torch.cuda.synchronize()
    st = codec.stats()
    assert st["rc"] == 0, st
    table = torch.from_numpy(pat.block_table).to(dev)
    n_out = shape.n_layers * pat.n_seq * pat.k
    preds = [torch.from_numpy(pat.predictions(s)).to(dev) for s in range(args.steps + args.warmup)]
    placement = {"searched": False}
    if args.placement == "search":
        # the output buffer in another HBM region than the pool, if one of three candidates about 48 GB apart
        # in allocation order is (see choose_placement): the step is timed into each, the fastest is kept
        cands, spacers = [], []
        for c in range(3):
            cands.append(torch.empty((n_out, ppb, N, d), dtype=torch.float16, device=dev))
            if c < 2:
                spacers.append(torch.empty(45 << 30, dtype=torch.uint8, device=dev))
        t_cand = []
        for o in cands:
            for _ in range(3):
                codec.gather_decompress(o, table, preds[0], shape.n_layers, pbl)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
            ev[0].record()
            for i in range(5):
                codec.gather_decompress(o, table, preds[0], shape.n_layers, pbl)
                ev[i + 1].record()
            torch.cuda.synchronize()
            t_cand.append(float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(5)])))
        best = int(np.argmin(t_cand))
        out = cands[best]
        del cands, spacers
        torch.cuda.empty_cache()
        placement = {"searched": True, "step_ms_by_output": [round(t, 4) for t in t_cand], "chosen_output": best}
        log(f"[bench] placement: {placement}")
    else:
        out = torch.empty((n_out, ppb, N, d), dtype=torch.float16, device=dev)
    for s in range(args.warmup):
        codec.gather_decompress(out, table, preds[s], shape.n_layers, pbl)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for s in range(args.steps):
        codec.gather_decompress(out, table, preds[args.warmup + s], shape.n_layers, pbl)
        evs[s + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ts = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)])
    unc = out.numel() * 2
    n_pages = n_out * ppb
    mean_payload = st["payload_bytes"] / sum(st["pages"])
    alg = unc + n_pages * (mean_payload + 16) + 8 * n_out
    ms = (t1 - t0) * 1e3 / args.steps
    dg_traffic, dg_source = read_traffic("decode_gather" + (f"_scheme{args.scheme}" if args.scheme != 3 else ""), "k_decompress")
    res = {
        "metric": "KV codec GB/s (uncompressed fp16) gather-decompress; % of HBM peak",
        "value": round(unc / (ms * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"decode_gather: 80 layers x 8 KV heads x 128, 64 sequences U[512,8192], "
                               f"8 predicted blocks/seq/layer, {n_pages} pages = {unc / 1e9:.2f} GB out per step",
                   "ratio": round(codec.ratio(), 4)},
        "roofline": {"bound": "hbm", "kernel": "k_decompress", "achieved": round(alg / ts.mean() / 1e6, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(alg / ts.mean() / 1e6 / HBM_PEAK_GBS, 4),
                     "traffic": dg_traffic, "traffic_source": dg_source, "alg_bytes_per_launch": int(alg),
                     "launch_ms": round(float(ts.mean()), 4)},
        "kernel_fingerprint": kernel_fingerprint(),
        "step_ms": {"mean": round(float(ts.mean()), 4), "p50": round(float(np.percentile(ts, 50)), 4),
                    "p99": round(float(np.percentile(ts, 99)), 4)},
        "placement": placement,
    }
    print(json.dumps(res), flush=True)


def bench_prefetch_pipeline(args):
    """Algorithm 1 around the gather, 70B decode shape: per decode step and layer, the predicted blocks
    that are not already in the double-buffered L2 prefetch buffer are decoded into it
    (kvc_prefetch_layers), two layers ahead of a stand-in for the layer's compute on a second stream
    (Section 3.4.4: T_eff = T_compute + max(T_prefetch - 2 T_layer, 0)).  Predictions slide over each
    sequence's blocks (positions pos+1..pos+k, one new token per step)."""
    import numpy as np
    import torch

    from paper_2512_11920_amd import kvc, synth

    dev = "cuda:0"
    n_layers = args.layers or 80
    shape = synth.KVShape("prefetch_pipeline", n_layers, 8, 128, 0, 0)
    N, d, H = 16, 128, 8
    ppb, E = 2 * H, N * d
    pat = synth.gather_pattern(64, 8, 512, 8192, N, seed=0)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    codec = kvc.Codec(N, d, ppb, args.scheme)
    codec.alloc_pool(n_layers * pbl, n_layers * pbl * ppb * E + 4096, dev)
    ids = torch.arange(pbl, dtype=torch.int32, device=dev)
    for l in range(n_layers):
        codec.compress_blocks(synth.gather_layer_torch(shape, pat, l, dev).view(-1, ppb, N, d), pool_ids=ids + l * pbl)
    n_slots = n_layers * n_seq * k
    codec.set_prefetch_policy(args.prefetch_policy)
    l2 = torch.zeros((2 * n_slots, ppb, N, d), dtype=torch.float16, device=dev)
    tags = torch.empty(2 * n_slots, dtype=torch.int32, device=dev)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=dev)
    loc = torch.empty(n_slots, dtype=torch.int32, device=dev)
    table = torch.from_numpy(pat.block_table).to(dev)
    steps = args.steps + args.warmup

    def preds(pattern, t):
        if pattern == "uniform":
            return pat.predictions(t)
        pos = (t // N + np.arange(n_seq) * 7) % pat.n_blocks  # block of the current token, one token per step
        return ((pos[:, None] + 1 + np.arange(k)[None, :]) % pat.n_blocks[:, None]).astype(np.int32)

    # stand-ins for one layer's compute, each about 100 us: an HBM-bound copy (competes with the prefetch
    # for bandwidth) and an MFMA-bound bf16 GEMM (leaves HBM to the prefetch)
    work_bytes = 256 << 20
    wa = torch.empty(work_bytes, dtype=torch.uint8, device=dev)
    wb = torch.empty_like(wa)
    ga = torch.randn((4096, 4096), device=dev, dtype=torch.bfloat16)
    gb = torch.randn((4096, 4096), device=dev, dtype=torch.bfloat16)
    gc = torch.empty((4096, 4096), device=dev, dtype=torch.bfloat16)
    torch.mm(ga, gb, out=gc)
    compute_kind = ["copy"]

    def compute(st):
        if compute_kind[0] == "copy":
            kvc.copy_bytes(wb, wa, stream=st)
        else:
            with torch.cuda.stream(st):
                torch.mm(ga, gb, out=gc)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    pred_buf = torch.zeros((n_seq, k), dtype=torch.int32, device=dev)  # static input of the captured graphs

    def issue_step(mode, fill, pred_t):
        """Enqueue one decode step: per layer, the prefetch of its predicted blocks and the compute stand-in."""
        pf = lambda l, st: codec.prefetch_layers(l2, tags, fetch, loc, table, pred_t, n_layers, pbl, fill,
                                                 layer_begin=l, layer_end=l + 1, stream=st)
        if mode == "pipelined":
            done = [torch.cuda.Event() for _ in range(n_layers)]
            side.wait_stream(main)
            for l in range(min(2, n_layers)):
                pf(l, side)
                done[l].record(side)
            for l in range(n_layers):
                main.wait_event(done[l])
                started = torch.cuda.Event()
                started.record(main)
                compute(main)
                if l + 2 < n_layers:
                    side.wait_event(started)
                    pf(l + 2, side)
                    done[l + 2].record(side)
            main.wait_stream(side)
        elif mode in ("batched", "batched_prefetch_only"):
            # one planner + one decode launch for all layers, then the layers' compute
            codec.prefetch_layers(l2, tags, fetch, loc, table, pred_t, n_layers, pbl, fill, stream=main)
            if mode == "batched":
                for l in range(n_layers):
                    compute(main)
        else:
            for l in range(n_layers):
                if mode != "compute_only":
                    pf(l, main)
                if mode != "prefetch_only":
                    compute(main)

    out = {}
    for kind, pattern in (("copy", "sliding"), ("copy", "uniform"), ("gemm", "sliding"), ("gemm", "uniform")):
        compute_kind[0] = kind
        pr = [torch.from_numpy(preds(pattern, t)).to(dev) for t in range(steps)]
        res = {}
        for mode in ("compute_only", "prefetch_only", "serial", "pipelined", "batched_prefetch_only", "batched"):
            # eager launches are bound by host-side issue (about 400 calls per step), so the step is
            # also captured once per buffer half into a HIP graph and replayed
            for graphed in (False, True):
                codec.prefetch_reset(tags, n_seq, k, n_layers)
                graphs = []
                if graphed:
                    cap = torch.cuda.Stream()
                    for fill in (0, 1):
                        g = torch.cuda.CUDAGraph()
                        torch.cuda.synchronize()
                        with torch.cuda.stream(cap):
                            main = cap
                            g.capture_begin()
                            issue_step(mode, fill, pred_buf)
                            g.capture_end()
                        graphs.append(g)
                    main = torch.cuda.current_stream()
                    codec.prefetch_reset(tags, n_seq, k, n_layers)
                torch.cuda.synchronize()
                n_fetched = 0
                for t in range(steps):
                    if t == args.warmup:
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                    if graphed:
                        pred_buf.copy_(pr[t])
                        graphs[t % 2].replay()
                    else:
                        issue_step(mode, t % 2, pr[t])
                    if mode == "prefetch_only" and not graphed and t >= args.warmup:
                        n_fetched += int((fetch >= 0).sum())
                torch.cuda.synchronize()
                res[mode + ("_graph" if graphed else "")] = (time.perf_counter() - t0) * 1e3 / args.steps
                if mode == "prefetch_only" and not graphed:
                    res["blocks_fetched_per_step"] = n_fetched / args.steps
                del graphs
        res["blocks_predicted_per_step"] = n_slots
        for sfx in ("", "_graph"):
            res["hidden_fraction" + sfx] = round(1.0 - (res["pipelined" + sfx] - res["compute_only" + sfx])
                                                 / max(res["serial" + sfx] - res["compute_only" + sfx], 1e-9), 3)
        out[f"{kind}/{pattern}"] = {a: (round(b, 4) if isinstance(b, float) else b) for a, b in res.items()}
        log(f"[prefetch] compute={kind} predictions={pattern}: {out[f'{kind}/{pattern}']}")
    st = codec.stats()
    assert st["status"] == 0, st
    print(json.dumps({"metric": "decode-step time with speculative prefetch (ms per step)", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "data": "synthetic", "unit": "ms", "higher_is_better": False,
                      "config": {"workload": f"prefetch_pipeline: {n_layers} layers x 8 KV heads x 128, 64 sequences "
                                             f"U[512,8192], k=8, slot policy {args.prefetch_policy}, per-layer prefetch two layers ahead of the layer's compute "
                                             f"stand-in ({work_bytes >> 20} MiB copy, or 4096^3 bf16 GEMM)"},
                      "patterns": out}), flush=True)


def bench_prefetch_window(args):
    """Algorithm 1's outstanding-request window on the 70B decode shape (80 layers, 64 sequences, k = 8): one
    kvc_prefetch_layers_window call per decode step for all layers, with at most omega transfers in flight,
    against the unbounded kvc_prefetch_layers.  Per omega: time of the call alone, when the first layer and
    when all layers were ready (the call's own ready stamps), and the step time when the call runs beside
    a stand-in for the step's compute (80 x 256 MiB copies, HBM-bound) on another stream."""
    import numpy as np
    import torch

    from paper_2512_11920_amd import kvc, synth

    dev = "cuda:0"
    n_layers = args.layers or 80
    shape = synth.KVShape("prefetch_window", n_layers, 8, 128, 0, 0)
    N, d, H = 16, 128, 8
    ppb, E = 2 * H, N * d
    pat = synth.gather_pattern(64, 8, 512, 8192, N, seed=0)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    codec = kvc.Codec(N, d, ppb, args.scheme)
    codec.alloc_pool(n_layers * pbl, n_layers * pbl * ppb * E + 4096, dev)
    ids = torch.arange(pbl, dtype=torch.int32, device=dev)
    for l in range(n_layers):
        codec.compress_blocks(synth.gather_layer_torch(shape, pat, l, dev).view(-1, ppb, N, d), pool_ids=ids + l * pbl)
    n_slots = n_layers * n_seq * k
    codec.set_prefetch_policy(args.prefetch_policy)
    l2 = torch.zeros((2 * n_slots, ppb, N, d), dtype=torch.float16, device=dev)
    tags = torch.empty(2 * n_slots, dtype=torch.int32, device=dev)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=dev)
    loc = torch.empty(n_slots, dtype=torch.int32, device=dev)
    notify = torch.zeros(n_layers + 4, dtype=torch.int64, device=dev)
    work = torch.empty(kvc.window_workspace(n_slots, n_layers), dtype=torch.uint8, device=dev)
    table = torch.from_numpy(pat.block_table).to(dev)
    khz = kvc.wall_clock_khz()
    steps = args.steps + args.warmup
    wa = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    wb = torch.empty_like(wa)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()

    def preds(pattern, t):
        if pattern == "uniform":
            return pat.predictions(t)
        # a window sliding over consecutive blocks, at the steps where it moves (every 16th token of a decode):
        # one new block per sequence and layer, 5,120 transfers per step
        pos = (t + np.arange(n_seq) * 7) % pat.n_blocks
        return ((pos[:, None] + 1 + np.arange(k)[None, :]) % pat.n_blocks[:, None]).astype(np.int32)

    def prefetch(omega, fill, pred_t, st):
        if omega:
            codec.prefetch_layers_window(l2, tags, fetch, loc, table, pred_t, n_layers, pbl, fill, omega, notify, work, stream=st)
        else:
            codec.prefetch_layers(l2, tags, fetch, loc, table, pred_t, n_layers, pbl, fill, stream=st)

    # the compute stand-in alone
    for _ in range(3):
        for l in range(n_layers):
            kvc.copy_bytes(wb, wa)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for l in range(n_layers):
            kvc.copy_bytes(wb, wa)
    torch.cuda.synchronize()
    compute_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    out = {"compute_only_ms": round(compute_ms, 4)}
    for pattern in ("uniform", "sliding"):
        pr = [torch.from_numpy(preds(pattern, t)).to(dev) for t in range(steps)]
        rows = []
        for omega in (16, 64, 256, 1024, 4096, 0):
            row = {"omega": omega or "unbounded"}
            # (1) the call alone
            codec.prefetch_reset(tags, n_seq, k, n_layers)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            t_call, first, half, allr, high, issued = [], [], [], [], [], []
            for t in range(steps):
                ev[0].record()
                prefetch(omega, t % 2, pr[t], main)
                ev[1].record()
                torch.cuda.synchronize()
                if t >= args.warmup:
                    t_call.append(ev[0].elapsed_time(ev[1]))
                    if omega:
                        nt = notify.cpu().numpy()
                        opened = nt[n_layers]
                        first.append((nt[0] - opened) / khz * 1e3)
                        half.append((nt[n_layers // 2] - opened) / khz * 1e3)
                        allr.append((nt[n_layers + 3] - opened) / khz * 1e3)
                        issued.append(int(nt[n_layers + 1]))
                        high.append(int(nt[n_layers + 2]))
            row["call_ms"] = round(float(np.mean(t_call)), 4)
            if omega:
                row.update({"first_layer_ready_us": round(float(np.mean(first)), 1), "half_layers_ready_us": round(float(np.mean(half)), 1),
                            "all_ready_us": round(float(np.mean(allr)), 1), "blocks_issued": round(float(np.mean(issued)), 1),
                            "max_in_flight": int(max(high))})
            # (2) beside the step's compute on another stream
            codec.prefetch_reset(tags, n_seq, k, n_layers)
            torch.cuda.synchronize()
            for t in range(steps):
                if t == args.warmup:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                side.wait_stream(main)
                prefetch(omega, t % 2, pr[t], side)
                for l in range(n_layers):
                    kvc.copy_bytes(wb, wa, stream=main)
                main.wait_stream(side)
            torch.cuda.synchronize()
            row["step_ms_beside_compute"] = round((time.perf_counter() - t0) * 1e3 / args.steps, 4)
            rows.append(row)
            log(f"[window] {pattern}: {row}")
        out[pattern] = rows
    assert codec.stats()["status"] == 0
    print(json.dumps({"metric": "prefetch step under an outstanding-request window (ms, us)", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "data": "synthetic", "higher_is_better": False,
                      "config": {"workload": f"prefetch_window: {n_layers} layers x 8 KV heads x 128, 64 sequences U[512,8192], k=8, "
                                             f"slot policy {args.prefetch_policy}; compute stand-in {n_layers} x 256 MiB copies"},
                      "wall_clock_khz": khz, "window": out}), flush=True)


def bench_host_pool(args):
    """Slow-tier emulation: the compressed pool in pinned host memory, reached over the host link, as the
    paper's pool sits behind a 64 GB/s CXL link (Sections 3.2, 4.4.2).  Per scheme: uncompressed GB/s
    the codec sustains and the bytes that actually cross the link."""
    import torch

    from paper_2512_11920_amd import kvc, synth

    dev = "cuda:0"
    N, d, ppb = 16, 128, 8
    shape = synth.KVShape("70b_gqa_slice", args.layers or 4, 8, 128, 4096, 16)
    blocks = synth.cache_torch(shape, dev).view(-1, ppb, N, d)
    out = torch.empty_like(blocks)
    unc = blocks.numel() * 2
    rows = []
    for scheme, label in ((0, "None (FP16)"), (1, "INT8 only"), (3, "INT8 + Delta + RLE"),
                          (5, "INT8 + pack over channel-pair groups (extension)")):
        codec = kvc.Codec(N, d, ppb, scheme)
        codec.alloc_pool(blocks.shape[0], unc + 4096, dev, host_pool=True)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        tc = td = 0.0
        for rep in range(args.warmup + args.steps):
            codec.reset_pool()
            ev[0].record()
            codec.compress_blocks(blocks)
            ev[1].record()
            codec.decompress_blocks(out)
            ev[2].record()
            torch.cuda.synchronize()
            if rep >= args.warmup:
                tc += ev[0].elapsed_time(ev[1])
                td += ev[1].elapsed_time(ev[2])
        st = codec.stats()
        assert st["rc"] == 0
        tc, td = tc / args.steps, td / args.steps
        rows.append({"scheme": label, "ratio": round(codec.ratio(), 4), "compress_ms": round(tc, 3), "decompress_ms": round(td, 3),
                     "compress_GBps_unc": round(unc / tc / 1e6, 1), "decompress_GBps_unc": round(unc / td / 1e6, 1),
                     "link_GBps_write": round(st["payload_bytes"] / tc / 1e6, 1),
                     "link_GBps_read": round(st["payload_bytes"] / td / 1e6, 1)})
        log(f"[host_pool] {rows[-1]}")
        del codec
    print(json.dumps({"metric": "codec GB/s (uncompressed fp16) with the pool behind the host link", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": f"host_pool: {shape.n_layers} layers of the 70B shape, {unc / 1e9:.2f} GB fp16, "
                                             "compressed pool in pinned host memory"}, "rows": rows}), flush=True)


def bench_ablation(args):
    """Compression-scheme ablation in the manner of the paper's Table 9 (None / INT8 / +Delta / +RLE):
    ratio and kernel speed per scheme on two synthetic inputs -- the LLaMA-shaped i.i.d.-channel cache
    and channel-correlated AR(1) pages.  Perplexity cannot be reproduced here."""
    import torch

    from paper_2512_11920_amd import kvc, synth

    dev = "cuda:0"
    N, d, ppb = 16, 128, 8
    n_layers = args.layers or 8
    shape = synth.KVShape("70b_gqa_slice", n_layers, 8, 128, 4096, 16)
    inputs = {"llama_iid": synth.cache_torch(shape, dev).view(-1, ppb, N, d)}
    inputs["ar1_rho0.95"] = synth.ar1_pages_torch(inputs["llama_iid"].shape[0] * ppb, dev).view(-1, ppb, N, d)
    rows = []
    for name, blocks in inputs.items():
        out = torch.empty_like(blocks)
        unc = blocks.numel() * 2
        for scheme, label in ((0, "None (FP16)"), (1, "INT8 only"), (2, "INT8 + Delta"), (3, "INT8 + Delta + RLE"),
                              (4, "INT8 + pack, no delta (extension)"),
                              (5, "INT8 + pack over channel-pair groups (extension)")):
            codec = kvc.Codec(N, d, ppb, scheme)
            codec.alloc_pool(blocks.shape[0], unc + 4096, dev)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            tc = td = 0.0
            for rep in range(args.warmup + args.steps):
                codec.reset_pool()
                ev[0].record()
                codec.compress_blocks(blocks)
                ev[1].record()
                codec.decompress_blocks(out)
                ev[2].record()
                torch.cuda.synchronize()
                if rep >= args.warmup:
                    tc += ev[0].elapsed_time(ev[1])
                    td += ev[1].elapsed_time(ev[2])
            st = codec.stats()
            assert st["rc"] == 0
            err = (out.float() - blocks.float()).pow(2).mean().sqrt() / blocks.float().pow(2).mean().sqrt()
            rows.append({"input": name, "scheme": label, "ratio": round(codec.ratio(), 4),
                         "payload_ratio": round(unc / st["payload_bytes"], 4), "pages_per_mode": st["pages"],
                         "compress_GBps_unc": round(unc / (tc / args.steps) / 1e6, 1),
                         "decompress_GBps_unc": round(unc / (td / args.steps) / 1e6, 1),
                         "rel_rmse": round(float(err), 5)})
            log(f"[ablation] {name:12s} {label:34s} ratio {rows[-1]['ratio']:.3f} (payload {rows[-1]['payload_ratio']:.3f}) "
                f"C {rows[-1]['compress_GBps_unc']:.0f} D {rows[-1]['decompress_GBps_unc']:.0f} GB/s rel-rmse {rows[-1]['rel_rmse']:.4f}")
            del codec
    print(json.dumps({"metric": "compression ratio and codec GB/s (uncompressed fp16) per scheme", "n_gpus": 1,
                      "data": "synthetic", "config": {"workload": f"ablation: {n_layers} layers of the 70B shape "
                                                      f"({inputs['llama_iid'].shape[0] * ppb} pages per input)"},
                      "ablation": rows}), flush=True)


if __name__ == "__main__":
    main()
