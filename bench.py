#!/usr/bin/env python3
"""Benchmark of the KV compress / decompress hot path on one MI355X.

One step = one pass of the whole path over one request of synthetic KV that is already
resident in HBM: kvc_compress (tables, quantize + pack + Huffman encode + offset scan for
K and V) followed by kvc_decompress (table set-up, decode + unpack + dequantize).
Workload: the Llama-3.1-70B shape (80 layers, 8 KV heads, head_dim 128,
32768 tokens, fp16, 10.74 GB), strategy 4-bit / group 32 followed by the lossless stage.

Prints ONE JSON line.  `value` is the paper's effective throughput s_p = V / (t_enc + t_dec)
(section 3.1: harmonic combination of encode and decode throughput over uncompressed bytes).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

WORKLOADS = {
    # name: (layers, heads, tokens, dtype, bits_k, bits_v, group_k, group_v, codec[, transform[, widths]])
    # transform: 0 none, 1 Hadamard, (2, anchor period) delta
    "llama70b_32k_fp16_int4g32_huff8": (80, 8, 32768, "f16", 4, 4, 32, 32, 1),
    "llama70b_32k_fp16_int4g32": (80, 8, 32768, "f16", 4, 4, 32, 32, 0),
    "llama70b_32k_fp16_hadamard_int4g32_huff8": (80, 8, 32768, "f16", 4, 4, 32, 32, 1, 1),
    "llama70b_32k_fp16_hadamard_int4g32": (80, 8, 32768, "f16", 4, 4, 32, 32, 0, 1),
    "llama70b_32k_fp16_delta32_int4g32_huff8": (80, 8, 32768, "f16", 4, 4, 32, 32, 1, (2, 32)),
    "llama70b_32k_fp16_delta32_int4g32": (80, 8, 32768, "f16", 4, 4, 32, 32, 0, (2, 32)),
    # per-head widths: a seeded random half of the heads at 8 bits, the other half at 2 (the paper's
    # MixHQ takes the split from trained head masks, which are not available here)
    "llama70b_32k_fp16_mixhq_8_2_g32": (80, 8, 32768, "f16", 4, 4, 32, 32, 0, 0, (8, 2)),
    "llama8b_8k_bf16_int4g32": (32, 8, 8192, "bf16", 4, 4, 32, 32, 0),
    "llama8b_8k_bf16_int2g64": (32, 8, 8192, "bf16", 2, 2, 64, 64, 0),
    "tiny_fp16_int4g32": (1, 8, 1024, "f16", 4, 4, 32, 32, 0),
}


def cpu_baseline(x_dev, layers, heads, tokens, dt, bits_k, bits_v, gk, gv, codec, transform, sample_layers,
                 head_bits=None, anchor_period=0):
    """The oracle as it stands, single-threaded, on the first `sample_layers` layers."""
    import numpy as np
    from oracle import ref
    from paper_2605_13734_amd import kvgen
    xs = x_dev[:sample_layers].cpu()
    xu = kvgen.as_u16(xs)
    cfg = ref.config(dtype=dt, layers=sample_layers, heads=heads, bits_k=bits_k, bits_v=bits_v,
                     group_k=gk, group_v=gv, codec=codec, transform=transform, anchor_period=anchor_period,
                     head_bits_k=head_bits[0][:sample_layers * heads] if head_bits else None,
                     head_bits_v=head_bits[1][:sample_layers * heads] if head_bits else None)
    lay = ref.contiguous_layout(heads, tokens, 128)
    t0 = time.perf_counter()
    payload = ref.compress(cfg, xu[0, 0], xu[0, 1], lay, tokens)
    t1 = time.perf_counter()
    out = np.zeros_like(xu)
    rc = ref.decompress(payload, out[0, 0], out[0, 1], lay, cfg)
    t2 = time.perf_counter()
    assert rc == 0
    nbytes = xu.nbytes
    return {"value": round(nbytes / (t2 - t0) / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d layers (%.0f MB of fp16 KV), compress %.2f s + decompress %.2f s"
                      % (sample_layers, layers, nbytes / 1e6, t1 - t0, t2 - t1),
            "s_enc": round(nbytes / (t1 - t0) / 1e9, 5), "s_dec": round(nbytes / (t2 - t1) / 1e9, 5)}


POLICY_STRATEGIES = [
    # name, bits_k, bits_v, group_k, group_v, codec, transform (0 none, 1 Hadamard, (2, anchor period) delta)
    ("int8g32", 8, 8, 32, 32, 0, 0),
    ("int4g32", 4, 4, 32, 32, 0, 0),
    ("int4g32_huff8", 4, 4, 32, 32, 1, 0),
    ("hadamard_int4g32", 4, 4, 32, 32, 0, 1),
    ("delta32_int4g32", 4, 4, 32, 32, 0, (2, 32)),
    ("delta128_int2g64", 2, 2, 64, 64, 0, (2, 128)),
    ("k4v2g64", 4, 2, 64, 64, 0, 0),
    ("int3g64", 3, 3, 64, 64, 0, 0),
    ("int2g64", 2, 2, 64, 64, 0, 0),
    ("int2g128_huff8", 2, 2, 128, 128, 1, 0),
]


def policy_table(x, y, dt, L, H, T, steps):
    """Measures (cr, s_enc, s_dec) of several strategies on the same tensor and turns them into the
    piecewise policy of section 6.1 (kvc_policy_build): which strategy to use below which bandwidth."""
    import ctypes
    import torch
    from paper_2605_13734_amd import kvc
    V = x.numel() * 2
    stream = torch.cuda.current_stream().cuda_stream
    profiles, rows = [], []
    for name, bk, bv, gk, gv, codec, tr in POLICY_STRATEGIES:
        tr, period = tr if isinstance(tr, tuple) else (tr, 0)
        plan = kvc.Plan(dt, L, H, 128, bk, bv, gk, gv, codec, max_tokens=T, transform=tr, anchor_period=period)
        buf = kvc.Buffers(plan, [T], "cuda:0")
        src, dst = [kvc.contiguous_request(x)], [kvc.contiguous_request(y)]
        buf.compress(src, stream)
        buf.decompress(dst, stream)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        for _ in range(steps):
            buf.compress(src, stream)
        ev[1].record()
        for _ in range(steps):
            buf.decompress(dst, stream)
        ev[2].record()
        torch.cuda.synchronize()
        assert int(buf.status[0]) == 0
        t_enc, t_dec = ev[0].elapsed_time(ev[1]) / steps, ev[1].elapsed_time(ev[2]) / steps
        cr = V / int(buf.out_bytes[0])
        prof = (cr, V / t_enc / 1e6, V / t_dec / 1e6)                       # GB/s of fp16 KV
        profiles.append(prof)
        rows.append({"name": name, "cr": round(cr, 4), "s_enc_GBps": round(prof[1], 1), "s_dec_GBps": round(prof[2], 1),
                     "s_p_GBps": round(kvc.profile_throughput(*prof), 1),
                     "break_even_bandwidth_GBps": round(kvc.benefit_threshold(*prof), 1)})
        del buf, plan
    rc, table = kvc.policy_build(profiles)
    assert rc == 0
    segs = []
    for k, (x_from, prof) in enumerate(table):
        segs.append({"profile": rows[prof]["name"] if prof >= 0 else "uncompressed",
                     "bandwidth_below_GBps": None if x_from == 0 else round(1.0 / x_from, 1)})
    return {"profiles": rows, "table": segs}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama70b_32k_fp16_int4g32_huff8", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--policy", action="store_true",
                    help="also measure a set of strategies and print the analytic policy table")
    ap.add_argument("--cpu-sample-layers", type=int, default=4)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is the single-GPU hot path (one process, one MI355X); "
              "--gpus %d is not supported. Each GPU would compress the KV heads it holds, "
              "with no exchange step." % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2605_13734_amd import kvc, kvgen
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    kvc.load()                                    # fails loudly if the HIP library is missing

    L, H, T, dtn, bk, bv, gk, gv, codec = WORKLOADS[args.workload][:9]
    transform = WORKLOADS[args.workload][9] if len(WORKLOADS[args.workload]) > 9 else 0
    transform, anchor_period = transform if isinstance(transform, tuple) else (transform, 0)
    mix = WORKLOADS[args.workload][10] if len(WORKLOADS[args.workload]) > 10 else None
    head_bits = None
    if mix:
        import numpy as np
        rng = np.random.default_rng(0)
        head_bits = [np.where(rng.permutation(L * H) < L * H // 2, mix[0], mix[1]).astype(np.uint8) for _ in range(2)]
    dtype, dt = (torch.float16, kvc.F16) if dtn == "f16" else (torch.bfloat16, kvc.BF16)
    dev = "cuda:0"
    x = kvgen.make_kv(0, L, H, 128, T, dtype, dev)
    y = torch.empty_like(x)
    plan = kvc.Plan(dt, L, H, 128, bk, bv, gk, gv, codec, max_tokens=T, transform=transform, anchor_period=anchor_period,
                    head_bits_k=head_bits[0] if mix else None, head_bits_v=head_bits[1] if mix else None)
    buf = kvc.Buffers(plan, [T], dev)
    src, dst = [kvc.contiguous_request(x)], [kvc.contiguous_request(y)]
    stream = torch.cuda.current_stream().cuda_stream
    V = x.numel() * 2

    # plain-copy reference with a known size (16-bit pass-through of the first 8 layers): the
    # kernel copy_rows_kernel<true> reads and writes exactly ref_bytes per launch, which is
    # what the rocprofv3 byte counters are scaled by
    ref_layers = min(8, L)
    ref_plan = kvc.Plan(dt, ref_layers, H, 128, 16, 16, 32, 32, 0, max_tokens=T)
    ref_buf = kvc.Buffers(ref_plan, [T], dev)
    ref_buf.compress([kvc.contiguous_request(x[:ref_layers])], stream)
    torch.cuda.synchronize()
    ref_bytes = ref_layers * H * T * 128 * 2
    del ref_buf

    def step():
        buf.compress(src, stream)
        buf.decompress(dst, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert int(buf.status[0]) == 0, "device status %d" % int(buf.status[0])
    payload_bytes = int(buf.out_bytes[0])

    # events between the kernels of every timed step (recorded by the library on `stream`)
    n_ev = 8 * args.steps
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev)]
    for e in evs:
        e.record()                                # instantiates the underlying hipEvent_t
    torch.cuda.synchronize()
    import ctypes
    handles = (ctypes.c_void_p * n_ev)(*[e.cuda_event for e in evs])
    kvc.trace(plan, handles, n_ev)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    recorded = kvc.trace(plan, None, 0)
    assert recorded == n_ev, recorded
    assert int(buf.status[0]) == 0

    def avg(i, j):
        return sum(evs[8 * s + i].elapsed_time(evs[8 * s + j]) for s in range(args.steps)) / args.steps

    t_enc_setup, t_enc_k, t_enc_v = avg(0, 1), avg(1, 2), avg(2, 3)
    t_dec_setup, t_dec_k, t_dec_v = avg(4, 5), avg(5, 6), avg(6, 7)
    t_enc, t_dec = avg(0, 3), avg(4, 7)
    ms_step = wall * 1e3 / args.steps

    # algorithmic bytes of each main kernel: 2 B/element on the fp16 side, actual code bytes,
    # 4 B of metadata per group and 4 B of directory per chunk on the payload side
    hdr = buf.payload[:128].cpu().numpy()
    rc, _, _, _, total, sec = kvc.payload_inspect(hdr)
    assert rc == 0 and total == payload_bytes
    n_half = x.numel() // 2
    chunks = L * H * -(-T // 128) if codec else 0
    # (delta transform: plus the anchor rows, 16 bits per element, written or read once)
    anchors = 2 * L * H * -(-T // anchor_period) * 128 if anchor_period else 0
    alg = {"k": 2 * n_half + sec[7] + sec[1] + 4 * chunks + (anchors if bk != 16 else 0),
           "v": 2 * n_half + sec[9] + sec[3] + 4 * chunks + (anchors if bv != 16 else 0)}
    kernels = {
        "compress_k": (t_enc_k, alg["k"]), "compress_v": (t_enc_v, alg["v"]),
        "decompress_k": (t_dec_k, alg["k"]), "decompress_v": (t_dec_v, alg["v"]),
    }
    dom = max(kernels, key=lambda k: kernels[k][0])
    dom_ms, dom_bytes = kernels[dom]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(args.workload, {}).get(dom)
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(dom_bytes / dom_ms / 1e6, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom_bytes / dom_ms / 1e6 / HBM_PEAK_GBS, 4),
                "traffic": traffic, "avg_ms": round(dom_ms, 4), "algorithmic_bytes": dom_bytes}
    per_kernel = {k: {"avg_ms": round(ms, 4), "GBps_rw": round(b / ms / 1e6, 1),
                      "frac_hbm": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)} for k, (ms, b) in kernels.items()}

    # reference: a plain device copy of the same tensor (reads V bytes, writes V bytes)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    y.copy_(x)
    c0.record()
    for _ in range(3):
        y.copy_(x)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * V * 3 / c0.elapsed_time(c1) / 1e6

    s_enc, s_dec = V / t_enc / 1e6, V / t_dec / 1e6          # GB/s of uncompressed KV
    s_p = V / (ms_step * 1e-3) / 1e9
    cr = V / payload_bytes
    out = {
        "metric": "KV compress+decompress GB/s of fp16 KV (s_p = V/(t_enc+t_dec)), 1 MI355X",
        "value": round(s_p, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": L, "kv_heads": H, "head_dim": 128, "tokens": T,
                   "kv_dtype": dtn, "bits_k": bk, "bits_v": bv, "group_k": gk, "group_v": gv,
                   "codec": "huff8" if codec else "none", "transform": ("none", "hadamard", "delta%d" % anchor_period)[transform],
                   "kv_bytes": V, "payload_bytes": payload_bytes},
        "s_enc_GBps": round(s_enc, 1), "s_dec_GBps": round(s_dec, 1), "cr": round(cr, 4),
        "break_even_bandwidth_GBps": round((1 - 1 / cr) * s_p, 1),
        "compress_ms": round(t_enc, 4), "decompress_ms": round(t_dec, 4),
        "compress_setup_ms": round(t_enc_setup, 4), "decompress_setup_ms": round(t_dec_setup, 4),
        "hbm_frac_compress": round((alg["k"] + alg["v"]) / t_enc / 1e6 / HBM_PEAK_GBS, 4),
        "hbm_frac_decompress": round((alg["k"] + alg["v"]) / t_dec / 1e6 / HBM_PEAK_GBS, 4),
        "device_copy_GBps_rw": round(copy_gbps, 1), "copy_rows_reference_bytes_per_launch": ref_bytes,
        "kernels": per_kernel, "roofline": roofline,
    }
    if args.policy:
        out["policy"] = policy_table(x, y, dt, L, H, T, max(2, args.steps // 3))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x, L, H, T, dt, bk, bv, gk, gv, codec, transform,
                                           min(args.cpu_sample_layers, L), head_bits, anchor_period)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
