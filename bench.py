#!/usr/bin/env python3
"""Benchmark of the MoSKA decode-attention hot path on one MI355X.

A step is one pass of the whole path (route -> bucket -> shared attention -> unique attention ->
merge) over one batch of synthetic requests, inputs resident in HBM.  Default workload: the
configuration the headline metric is quoted on (batch 256, 1M shared tokens, bf16).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i] [--no-cpu-baseline] [--no-extra-configs]

Prints one JSON line: decode queries/s (value), shared-attention TFLOP/s, per-call times with
their roofline fractions, the roofline object of the slowest call, the CPU oracle's rate on a
bounded sample of the same workload and, under "configs", a short measurement of the two larger
benchmark configurations (3: 4M shared tokens, Zipf popularity; 4: fp8 store, 64 query heads).

    python bench.py --calibrate      a plain 1 GiB device copy, for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def algorithmic_work(p, bucket_off):
    """Bytes each call must move and flops it must do, from the problem and the actual bucket
    occupancy (a bucket's K and V are counted once, however many rows it has)."""
    esz_q = 4 if p.q_dtype == "f32" else 2
    esz_kv = {"f32": 4, "bf16": 2, "fp8": 1}[p.kv_dtype]
    sizes = (bucket_off[1:] - bucket_off[:-1])
    nonempty = int((sizes > 0).sum())
    Bq = p.B * p.T                      # query tokens; only the unique K/V are per request
    rows_q = Bq * p.Hq
    shared_rows = rows_q * p.k
    w = {}
    w["route"] = dict(bytes=Bq * p.Hq * p.D * esz_q + p.Hkv * p.C * p.D * esz_q + Bq * p.Hkv * p.k * 4,
                      flops=2.0 * Bq * p.Hkv * p.C * p.D)
    w["bucket"] = dict(bytes=Bq * p.Hkv * p.k * 4 * 4 + (p.Hkv * p.C + 1) * 4, flops=0.0)
    w["shared_attn"] = dict(bytes=nonempty * 2 * p.L * p.D * esz_kv + shared_rows * p.D * esz_q
                            + shared_rows * (p.D + 1) * 4,
                            flops=4.0 * p.D * shared_rows * p.L)
    w["unique_attn"] = dict(bytes=2 * p.B * p.Hkv * p.U * p.D * esz_q + rows_q * p.D * esz_q + rows_q * (p.D + 1) * 4,
                            flops=4.0 * p.D * rows_q * p.U)
    w["merge"] = dict(bytes=rows_q * ((p.k + 1) * (p.D + 1) * 4 + p.D * esz_q + 4), flops=0.0)
    return w


def shared_attainable_s(p, bucket_off):
    """Roofline time of the shared attention for this bucket occupancy: each bucket costs the larger
    of its HBM time (K and V once, queries in, partials out) and its MFMA time."""
    esz_q = 4 if p.q_dtype == "f32" else 2
    esz_kv = {"f32": 4, "bf16": 2, "fp8": 1}[p.kv_dtype]
    rows = (bucket_off[1:] - bucket_off[:-1]).double() * p.G
    rows = rows[rows > 0]
    t_mem = (2 * p.L * p.D * esz_kv + rows * (p.D * esz_q + (p.D + 1) * 4)) / (HBM_PEAK_GBS * 1e9)
    t_mfma = 4.0 * p.D * rows * p.L / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    return float(t_mem.clamp_min(t_mfma).sum())


def read_traffic(name):
    """HBM traffic per launch measured offline with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE),
    kept as `kernel workload bytes` lines in profiles/hbm_traffic.txt; None if not recorded."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split("#")[0].split()
        if len(f) == 3 and (f[0], f[1]) == name:
            return float(f[2])
    return None


def paper_sweep(steps, warmup, full_scale=False):
    """Second workload: the paper's operating point (Sec. IV: fp8 store, 75 % routing sparsity,
    batch growing to 256) -- shared and unique attention utilisation against batch size, the measured
    counterpart of the paper's modelled Fig. 5.  One JSON line per batch.
    full_scale: the paper's own sizes as far as one GPU holds them: a 16M-token shared context (4096
    chunks of 4096 tokens, top-k = 1024) and 64K unique tokens per request; otherwise a 256K-token
    context (64 chunks, top-k = 16) and 8K unique tokens.  The store is generated once, for the
    largest batch; smaller batches use its first requests."""
    import torch
    import paper_2511_06010_amd as moska
    from moska_inputs import Inputs, Problem, generate
    shape = dict(C=4096, L=4096, k=1024, U=65536) if full_scale else dict(C=64, L=4096, k=16, U=8192)
    tag = "paper-point-16M" if full_scale else "paper-point"
    batches = (1, 4, 16, 64, 256)
    pmax = Problem(B=batches[-1], Hq=32, Hkv=8, D=128, kv_dtype="fp8", name=f"{tag}-b{batches[-1]}", **shape)
    full = generate(pmax, seed=20251106, device="cuda")
    for B in batches:
        p = pmax.with_(B=B, name=f"{tag}-b{B}")
        inp = Inputs(p, full.Q[:B], full.E, full.Ks, full.Vs, full.scale_k, full.scale_v, full.Ku[:B], full.Vu[:B],
                     full.unique_len[:B], full.cstar[:B])
        buf = moska.Buffers(p)

        def timed(fn):
            for _ in range(warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps
        ms_r = timed(lambda: moska.route(p, inp.Q, inp.E, buf.ids, None, buf.ws))
        ms_b = timed(lambda: moska.bucket(p, buf.ids, buf.bucket_off, buf.bucket_items, buf.ws))
        ms_s = timed(lambda: moska.shared_attn(p, inp.Q, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, buf.ids,
                                               buf.bucket_off, buf.bucket_items, buf.part_O, buf.part_LSE, buf.ws))
        ms_u = timed(lambda: moska.unique_attn(p, inp.Q, inp.Ku, inp.Vu, inp.unique_len, buf.part_O, buf.part_LSE,
                                               buf.ws))
        ms_m = timed(lambda: moska.merge(p, buf.part_O, buf.part_LSE, buf.O, buf.LSE))
        w = algorithmic_work(p, buf.bucket_off.cpu())
        rows = (buf.bucket_off[1:] - buf.bucket_off[:-1]).float() * p.G
        print(json.dumps({
            "workload": p.name, "B": B, "rows_per_bucket_mean": round(float(rows.mean()), 1),
            "route_ms": round(ms_r, 4), "bucket_ms": round(ms_b, 4), "merge_ms": round(ms_m, 4),
            "merge_GBs": round(w["merge"]["bytes"] / ms_m / 1e6, 1),
            "shared_ms": round(ms_s, 4), "shared_TFLOPs": round(w["shared_attn"]["flops"] / ms_s / 1e9, 1),
            "shared_mfma_frac": round(w["shared_attn"]["flops"] / ms_s / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
            "shared_GBs": round(w["shared_attn"]["bytes"] / ms_s / 1e6, 1),
            "shared_hbm_frac": round(w["shared_attn"]["bytes"] / ms_s / 1e6 / HBM_PEAK_GBS, 4),
            "unique_ms": round(ms_u, 4), "unique_GBs": round(w["unique_attn"]["bytes"] / ms_u / 1e6, 1),
            "unique_hbm_frac": round(w["unique_attn"]["bytes"] / ms_u / 1e6 / HBM_PEAK_GBS, 4),
            "unique_mfma_frac": round(w["unique_attn"]["flops"] / ms_u / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
            "step_ms": round(ms_r + ms_b + ms_s + ms_u + ms_m, 4)}), flush=True)
        del inp, buf
        torch.cuda.empty_cache()


def reuse_sweep(steps, warmup, stores=("bf16", "fp8"), chunks=16):
    """Shared attention against query rows per bucket at the chunk shape of configs 2-4 (L = 4096,
    D = 128, 8 KV heads, G = 4).  chunks = 16 (default): every request attends all 16 chunks (k = C), so
    each of the 128 buckets holds exactly 4*B rows, 16 .. 4096: where the path leaves the HBM roofline for
    the MFMA one (ridge: 313 rows for a bf16 store on its K/V bytes alone, 353 with the rows' own bytes;
    fp8: 156 / 177).  chunks = 1024: a 4M-token store of 8192 buckets, top-k = 256 of uniform popularity,
    8 .. 192 rows per bucket on average: the region round the ridge with the chip filled many times over.
    One JSON line per point."""
    import torch
    import paper_2511_06010_amd as moska
    from moska_inputs import Inputs, Problem, generate
    if chunks != 16:
        batches = (8, 16, 32, 48, 64, 96, 128, 192)
        for kv in stores:
            pmax = Problem(B=batches[-1], Hq=32, Hkv=8, D=128, C=chunks, L=4096, k=chunks // 4, U=64, kv_dtype=kv,
                           name=f"reuse-{kv}-c{chunks}")
            full = generate(pmax, seed=20251106, device="cuda")
            for B in batches:
                p = pmax.with_(B=B, name=f"reuse-{kv}-c{chunks}-b{B}")
                inp = Inputs(p, full.Q[:B], full.E, full.Ks, full.Vs, full.scale_k, full.scale_v, full.Ku[:B],
                             full.Vu[:B], full.unique_len[:B], full.cstar[:B])
                _reuse_point(p, inp, float(B) * p.k * p.G / p.C, steps, warmup)
            del full
            torch.cuda.empty_cache()
        return
    for kv in stores:
        for B in (4, 8, 16, 32, 64, 128, 256, 512, 1024):
            p = Problem(B=B, Hq=32, Hkv=8, D=128, C=16, L=4096, k=16, U=64, kv_dtype=kv, name=f"reuse-{kv}-m{4 * B}")
            _reuse_point(p, generate(p, seed=20251106, device="cuda"), 4 * B, steps, warmup)


def _reuse_point(p, inp, rows_per_bucket, steps, warmup):
    """One point of the reuse sweep: moska_shared_attn on problem p, timed with HIP events."""
    import torch
    import paper_2511_06010_amd as moska
    buf = moska.Buffers(p)
    moska.route(p, inp.Q, inp.E, buf.ids, None, buf.ws)
    moska.bucket(p, buf.ids, buf.bucket_off, buf.bucket_items, buf.ws)
    fn = lambda: moska.shared_attn(p, inp.Q, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, buf.ids, buf.bucket_off,
                                   buf.bucket_items, buf.part_O, buf.part_LSE, buf.ws)
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    off = buf.bucket_off.cpu()
    w = algorithmic_work(p, off)["shared_attn"]
    att = shared_attainable_s(p, off)
    print(json.dumps({
        "workload": p.name, "rows_per_bucket": rows_per_bucket, "shared_ms": round(ms, 4),
        "TFLOPs": round(w["flops"] / ms / 1e9, 1), "mfma_frac": round(w["flops"] / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
        "GBs": round(w["bytes"] / ms / 1e6, 1), "hbm_frac": round(w["bytes"] / ms / 1e6 / HBM_PEAK_GBS, 4),
        "roofline_ms": round(att * 1e3, 4), "of_roofline": round(att * 1e3 / ms, 4)}), flush=True)
    del buf
    torch.cuda.empty_cache()


def time_step(moska, torch, p, inp, buf, steps, warmup):
    """W warm-up and K timed passes of the five calls on torch's current stream (the stream every call
    is enqueued on), with HIP events between the calls.  Returns (ms per step, {call: sorted ms})."""
    calls = ["route", "bucket", "shared_attn", "unique_attn", "merge"]

    def step(events=None):
        rec = (lambda i: events[i].record()) if events is not None else (lambda i: None)
        rec(0)
        moska.route(p, inp.Q, inp.E, buf.ids, None, buf.ws)
        rec(1)
        moska.bucket(p, buf.ids, buf.bucket_off, buf.bucket_items, buf.ws)
        rec(2)
        moska.shared_attn(p, inp.Q, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, buf.ids, buf.bucket_off,
                          buf.bucket_items, buf.part_O, buf.part_LSE, buf.ws)
        rec(3)
        moska.unique_attn(p, inp.Q, inp.Ku, inp.Vu, inp.unique_len, buf.part_O, buf.part_LSE, buf.ws)
        rec(4)
        moska.merge(p, buf.part_O, buf.part_LSE, buf.O, buf.LSE)
        rec(5)

    for _ in range(warmup):
        step()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    samples = {c: sorted(e[i].elapsed_time(e[i + 1]) for e in evs) for i, c in enumerate(calls)}
    return (t1 - t0) * 1e3 / steps, samples


def kernel_table(p, bucket_off, samples):
    """Per call: mean / median / min time, achieved GB/s and TFLOP/s of ALGORITHMIC work, roofline fractions."""
    work = algorithmic_work(p, bucket_off)
    kernels = {}
    for c, v in samples.items():
        ms = sum(v) / len(v)
        gbs = work[c]["bytes"] / (ms * 1e-3) / 1e9
        tfl = work[c]["flops"] / (ms * 1e-3) / 1e12
        kernels[c] = {"ms": round(ms, 5), "ms_median": round(v[len(v) // 2], 5), "ms_min": round(v[0], 5),
                      "GB/s": round(gbs, 1), "TFLOP/s": round(tfl, 2), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4),
                      "mfma_frac": round(tfl / MFMA_BF16_PEAK_TFLOPS, 4)}
    att_s = shared_attainable_s(p, bucket_off)
    kernels["shared_attn"]["roofline_ms"] = round(att_s * 1e3, 5)          # sum over buckets of max(HBM, MFMA) time
    kernels["shared_attn"]["of_roofline"] = round(att_s * 1e3 / kernels["shared_attn"]["ms"], 4)
    return kernels, work


def extra_config(moska, torch, idx, steps, warmup):
    """A short measurement of another benchmark configuration, for the "configs" object."""
    from moska_inputs import config, generate
    p = config(idx)
    inp = generate(p, seed=20251106 + idx, device="cuda")
    buf = moska.Buffers(p)
    torch.cuda.synchronize()
    ms, samples = time_step(moska, torch, p, inp, buf, steps, warmup)
    kernels, _ = kernel_table(p, buf.bucket_off.cpu(), samples)
    sh, un = kernels["shared_attn"], kernels["unique_attn"]
    out = {"workload": p.name, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4),
           "queries_per_s": round(p.Bq / (ms * 1e-3), 1),
           "shared_ms": sh["ms"], "shared_TFLOPs": sh["TFLOP/s"], "shared_mfma_frac": sh["mfma_frac"],
           "shared_of_attainable": sh["of_roofline"], "shared_GBs": sh["GB/s"], "shared_hbm_frac": sh["hbm_frac"],
           "unique_ms": un["ms"], "unique_GBs": un["GB/s"], "unique_hbm_frac": un["hbm_frac"],
           "route_ms": kernels["route"]["ms"], "bucket_ms": kernels["bucket"]["ms"], "merge_ms": kernels["merge"]["ms"]}
    del inp, buf
    torch.cuda.empty_cache()
    return out


def offline(steps, warmup):
    """The two cache-construction kernels (Sec. III-A/B: pre-computed shared store and chunk
    embeddings) at the store of configuration 4 (512 chunks x 8 KV heads x 4096 tokens x 128):
    quantisation of a bf16 store to fp8 and the chunk embeddings of the bf16 and of the fp8 store.
    One JSON line per kernel; bytes are the algorithmic ones (every input element read once, every
    output element written once)."""
    import torch
    import paper_2511_06010_amd as moska
    from moska_inputs import config
    p = config(4)
    n = p.C * p.Hkv * p.L * p.D
    g = torch.Generator(device="cuda").manual_seed(20251110)
    X = torch.randn((p.C, p.Hkv, p.L, p.D), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    X8 = torch.empty(X.shape, dtype=torch.float8_e4m3fn, device="cuda")
    sc = torch.empty((p.C, p.Hkv), dtype=torch.float32, device="cuda")
    E = torch.empty((p.Hkv, p.C, p.D), dtype=torch.bfloat16, device="cuda")
    pb = p.with_(kv_dtype="bf16")

    def timed(fn):
        for _ in range(warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps
    for name, fn, nbytes in (
            ("moska_quantize_shared bf16->fp8", lambda: moska.quantize_shared(p, X, X8, sc), 3 * n),
            ("moska_chunk_embeddings bf16 store", lambda: moska.chunk_embeddings(pb, X, None, E), 2 * n),
            ("moska_chunk_embeddings fp8 store", lambda: moska.chunk_embeddings(p, X8, sc, E), n)):
        ms = timed(fn)
        print(json.dumps({"kernel": name, "store": f"{p.C}x{p.Hkv}x{p.L}x{p.D}", "ms": round(ms, 4),
                          "algorithmic_GB": round(nbytes / 1e9, 3), "GB/s": round(nbytes / ms / 1e6, 1),
                          "hbm_frac": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}), flush=True)


def calibrate():
    """A plain device-to-device copy of 1 GiB (torch's copy kernel), 10 times: its FETCH_SIZE and
    WRITE_SIZE under `rocprofv3 --pmc` against the known 1 GiB each way give the factors by which the
    counters of the attention kernels are scaled; also prints the copy's own rate."""
    import torch
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    print(json.dumps({"calibration_copy_bytes": n, "ms": round(ms, 4), "GB/s_each_way": round(n / ms / 1e6, 1)}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload index (2 = the headline configuration)")
    ap.add_argument("--q-len", type=int, default=1,
                    help="query tokens per request: the same number of query tokens from B/q_len requests")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="skip the short measurement of configurations 3 and 4 that follows the headline one")
    ap.add_argument("--cpu-sample", type=int, default=0, help="requests in the oracle's sample (0 = auto)")
    ap.add_argument("--reuse-sweep", action="store_true",
                    help="shared attention against rows per bucket (16..4096) instead of the decode step")
    ap.add_argument("--sweep-store", choices=["bf16", "fp8"], help="restrict --reuse-sweep to one store dtype")
    ap.add_argument("--sweep-chunks", type=int, choices=[16, 1024], default=16,
                    help="--reuse-sweep over 16 chunks (16..4096 rows per bucket) or 1024 chunks (8..192 rows)")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="instead of the benchmark line: utilisation against batch size at the paper's operating point")
    ap.add_argument("--paper-scale", choices=["256K", "16M"], default="256K",
                    help="--paper-sweep: shared context of 64 chunks (top-16, 8K unique tokens) or of 4096 chunks "
                         "(top-1024, 64K unique tokens)")
    ap.add_argument("--offline", action="store_true",
                    help="time the cache-construction kernels (quantisation, chunk embeddings) at config 4's store")
    ap.add_argument("--calibrate", action="store_true", help="run the 1 GiB calibration copy and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_06010_amd as moska
    from moska_inputs import config, generate

    moska.load_library()                       # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate:
        calibrate()
        return
    if args.offline:
        offline(args.steps, args.warmup)
        return
    if args.reuse_sweep:
        reuse_sweep(args.steps, args.warmup, (args.sweep_store,) if args.sweep_store else ("bf16", "fp8"),
                    args.sweep_chunks)
        return
    if args.paper_sweep:
        paper_sweep(args.steps, args.warmup, args.paper_scale == "16M")
        return
    p = config(args.config)
    if args.q_len > 1:
        assert p.B % args.q_len == 0, "q_len must divide the batch size"
        p = p.with_(T=args.q_len, B=p.B // args.q_len, name=p.name + f"-qlen{args.q_len}")
    inp = generate(p, seed=20251106 + args.config, device="cuda")
    buf = moska.Buffers(p)
    torch.cuda.synchronize()

    ms_per_step, samples = time_step(moska, torch, p, inp, buf, args.steps, args.warmup)
    per_call_ms = {c: sum(v) / len(v) for c, v in samples.items()}

    # the same step through the single entry point (the same five launches in the same order)
    def fused():
        moska.decode_step(p, inp.Q, inp.E, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, inp.Ku, inp.Vu, inp.unique_len,
                          buf.ids, buf.bucket_off, buf.bucket_items, buf.part_O, buf.part_LSE, buf.O, buf.LSE, buf.ws)
    for _ in range(args.warmup):
        fused()
    torch.cuda.synchronize()
    f0 = time.perf_counter()
    for _ in range(args.steps):
        fused()
    torch.cuda.synchronize()
    decode_step_ms = (time.perf_counter() - f0) * 1e3 / args.steps

    # and replayed from a HIP graph (one capture of the entry point; launch overhead off the host)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fused()
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - g0) * 1e3 / args.steps

    # the five calls again on two streams (same priority): the latency-bound routing and bucketing run
    # beside unique attention, which does not depend on them; shared attention waits for both.  The side
    # stream has a workspace of its own (calls on different streams must not share one).
    side = torch.cuda.Stream()
    fork, join = torch.cuda.Event(), torch.cuda.Event()
    side_ws = torch.empty_like(buf.ws)

    def two_streams():
        fork.record()
        with torch.cuda.stream(side):
            side.wait_event(fork)
            moska.route(p, inp.Q, inp.E, buf.ids, None, side_ws)
            moska.bucket(p, buf.ids, buf.bucket_off, buf.bucket_items, side_ws)
            join.record()
        moska.unique_attn(p, inp.Q, inp.Ku, inp.Vu, inp.unique_len, buf.part_O, buf.part_LSE, buf.ws)
        torch.cuda.current_stream().wait_event(join)
        moska.shared_attn(p, inp.Q, inp.Ks, inp.Vs, inp.scale_k, inp.scale_v, buf.ids, buf.bucket_off,
                          buf.bucket_items, buf.part_O, buf.part_LSE, buf.ws)
        moska.merge(p, buf.part_O, buf.part_LSE, buf.O, buf.LSE)
    for _ in range(args.warmup):
        two_streams()
    torch.cuda.synchronize()
    s0 = time.perf_counter()
    for _ in range(args.steps):
        two_streams()
    torch.cuda.synchronize()
    two_stream_ms = (time.perf_counter() - s0) * 1e3 / args.steps
    del side_ws

    kernels, work = kernel_table(p, buf.bucket_off.cpu(), samples)
    dom = max(("shared_attn", "unique_attn"), key=lambda c: per_call_ms[c])
    # both attention calls are bound by the bytes the method itself must stream at this workload
    # (arithmetic intensity ~ rows per bucket flop/B, far left of the 315 flop/B ridge)
    ach = work[dom]["bytes"] / (per_call_ms[dom] * 1e-3) / 1e9
    roofline = {"kernel": "moska_" + dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": read_traffic(("moska_" + dom, p.name))}

    out = {
        "metric": "shared-attn TFLOP/s + decode queries/s, B=256, 1M shared tokens, 1 GPU",
        "value": round(p.Bq / (ms_per_step * 1e-3), 1), "unit": "queries/s",
        "shared_attn_tflops": kernels["shared_attn"]["TFLOP/s"],
        "unique_attn_gbs": kernels["unique_attn"]["GB/s"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if p.q_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": p.name, "B": p.B, "Hq": p.Hq, "Hkv": p.Hkv, "D": p.D, "C": p.C, "L": p.L,
                   "k": p.k, "U": p.U, "q_len": p.T, "shared_kv_dtype": p.kv_dtype, "popularity": p.popularity,
                   "layers": 1},
        "kernels": kernels,
        "decode_step_ms": round(decode_step_ms, 5),
        "decode_step_graph_ms": round(graph_ms, 5),
        "two_stream_ms": round(two_stream_ms, 5),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        import oracle
        from moska_inputs import Inputs
        # bounded sample: the first nb requests (all heads) against the full shared store
        rows_per_s_guess = 60.0 * oracle.threads()                 # ~17 ms per row per core at this size
        nb = args.cpu_sample or max(1, min(p.B, int(15.0 * rows_per_s_guess * (36864.0 / (p.k * p.L + p.U)) / p.Hq) // p.T))
        sp = p.with_(B=nb)
        nq = nb * p.T                                               # query tokens of the sampled requests
        cpu = lambda t: None if t is None else t.cpu()
        sub = Inputs(sp, inp.Q[:nq].cpu(), inp.E.cpu(), inp.Ks.cpu(), inp.Vs.cpu(), cpu(inp.scale_k), cpu(inp.scale_v),
                     inp.Ku[:nb].cpu(), inp.Vu[:nb].cpu(), inp.unique_len[:nb].cpu(), inp.cstar[:nb].cpu())
        c0 = time.perf_counter()
        ids, _ = oracle.route(sp, sub.Q, sub.E)
        oracle.bucket(sp, ids)
        pO, pL = oracle.partials(sub, ids)
        O, _ = oracle.merge(pO, pL)
        c1 = time.perf_counter()
        err = float((buf.O[:nq].double().cpu() - O).abs().max())
        out["cpu_baseline"] = {"value": round(nq / (c1 - c0), 3), "unit": "queries/s", "cores": oracle.threads(),
                               "kind": "oracle", "seconds": round(c1 - c0, 2),
                               "sample": f"first {nb} of {p.B} requests, all {p.Hq} heads, full shared store; "
                                         f"max |GPU-oracle| on the sample {err:.2e}"}
    if not args.no_extra_configs and args.config == 2 and args.q_len == 1:
        # free the headline workload, then a few steps of the two larger configurations
        del inp, buf
        torch.cuda.empty_cache()
        out["configs"] = {f"cfg{i}": extra_config(moska, torch, i, 5, 2) for i in (3, 4)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
