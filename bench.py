#!/usr/bin/env python3
"""Throughput of the whole compression hot path (score -> allocate -> select+gather) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config long_32k] [--path auto]

One "step" is one pass of the whole path over one batch of synthetic KV resident in HBM.  The
default workload is the 28-layer, 32768-token Qwen2.5-VL-7B-shaped cache the target is quoted
on.  Prints ONE JSON line: KV tokens compressed per second (a KV token = one (sequence, layer,
token) entry with all its heads' K and V), the roofline record of the dominant kernel measured
with HIP events inside the timed region, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP32_MFMA_PEAK_TFLOPS = 157.3
FP32_VALU_PEAK_TFLOPS = 157.3  # 256 CU x 128 lanes x 2 flop x 2.4 GHz with packed issue (78.6 without)


def algorithmic_bytes(cfg, T):
    """Bytes the method must move: K,V once, scores written and re-read, kept rows read+written."""
    e = cfg.elem_bytes
    units = cfg.batch * cfg.layers * cfg.kv_heads
    score = units * (2 * cfg.n_tokens * cfg.head_dim * e + 4 * cfg.n_tokens)
    select = units * 4 * cfg.n_tokens
    gather = cfg.batch * cfg.kv_heads * T * (4 * cfg.head_dim * e + 4)
    return {"score": score, "select_gather": select + gather, "total": score + select + gather}


def read_traffic(kernel, workload, path):
    """HBM bytes per launch of `kernel` as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (two runs of this script, scaled by the counters' reading for a plain copy of known size);
    taken from the committed summary of those runs, None if there is none for this kernel."""
    fname = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_traffic.txt")
    if not os.path.exists(fname):
        return None
    vals = {}
    with open(fname) as f:
        for ln in f:
            if "=" in ln and not ln.startswith("#"):
                k, v = ln.split("=", 1)
                vals[k.strip()] = v.strip()
    if vals.get("path") != path:
        return None
    try:
        return {"read_bytes": float(vals["read_bytes_per_launch"]),
                "write_bytes": float(vals["write_bytes_per_launch"]),
                "total_bytes": float(vals["read_bytes_per_launch"]) + float(vals["write_bytes_per_launch"])}
    except (KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="long_32k")
    ap.add_argument("--path", default="auto", choices=["auto", "dense", "fft"])
    ap.add_argument("--gamma", type=float, default=None, help="override the config's cut-off factor")
    ap.add_argument("--rho", type=float, default=None, help="override the config's retention ratio")
    ap.add_argument("--n-tokens", type=int, default=None,
                    help="override the token count (image blocks are added or dropped to fit)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--decode", action="store_true",
                    help="also time one decode-step attention over the compacted and over the full cache")
    ap.add_argument("--q-heads-per-kv", type=int, default=7, help="query heads per KV head for --decode")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference point for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (units are independent: a batch shards by "
              "sequence, a sequence by layer and head); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import kvsynth
    import paper_2511_16786_amd as fc
    from paper_2511_16786_amd import binding
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import parity_util as pu

    cfg = kvsynth.get_config(args.config)
    if args.gamma is not None:
        cfg = cfg.scaled(gamma=args.gamma)
    if args.rho is not None:
        cfg = cfg.scaled(rho=args.rho)
    if args.n_tokens is not None:
        nb = cfg.n_blocks
        if cfg.layout == "blocks":
            nb = max(1, (args.n_tokens - 2 * cfg.visual_start) // cfg.block_len)
        cfg = cfg.scaled(n_tokens=args.n_tokens, n_blocks=nb)
    workers = min(16, os.cpu_count() or 1)
    t0 = time.time()
    from kvsynth.generate import generate
    K, V = generate(cfg, workers=workers)
    t_gen = time.time() - t0
    print(f"[bench] generated {args.config}: K,V {K.shape} {cfg.dtype} in {t_gen:.1f}s", file=sys.stderr, flush=True)

    torch.cuda.set_device(0)
    t0 = time.time()
    Kt, Vt = pu.to_torch(K, cfg.dtype), pu.to_torch(V, cfg.dtype)
    torch.cuda.synchronize()
    t_upload = time.time() - t0

    r = fc.cutoff_r(cfg.n_tokens, cfg.gamma)
    T = fc.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    t0 = time.time()
    comp = fc.Compressor(Kt, r, T, path=args.path)      # includes the one-time table build (A1)
    torch.cuda.synchronize()
    t_prepare = time.time() - t0
    path_name = {binding.FC_PATH_DENSE: "dense", binding.FC_PATH_FFT: "fft"}[comp.path]

    if args.copy_calibration:
        # one elementwise copy kernel that reads 1 GiB and writes 1 GiB: what FETCH_SIZE and
        # WRITE_SIZE report for it gives the factor that turns counter units into bytes
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        comp.run(Kt, Vt)
    torch.cuda.synchronize()
    fc.binding.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        comp.run(Kt, Vt)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = fc.binding.profile_read()
    fc.binding.profile_enable(False)
    assert fc.workspace_error(comp.workspace) == 0

    tokens = cfg.batch * cfg.layers * cfg.n_tokens
    ms_per_step = 1e3 * elapsed / args.steps
    value = tokens / (elapsed / args.steps)
    ab = algorithmic_bytes(cfg, T)

    # dominant kernel = the one with the largest summed event time
    kern = {k: (n, ms / n) for k, (n, ms) in prof.items() if n > 0}
    dom = max(kern, key=lambda k: kern[k][0] * kern[k][1])
    dom_ms = kern[dom][1]
    units = cfg.batch * cfg.layers * cfg.kv_heads
    n, d = cfg.n_tokens, cfg.head_dim
    if dom.startswith("dense"):
        # each dense product is 2*r*N*d flop per tensor, two tensors per unit
        flops = 4.0 * r * n * d * units
        roofline = {"kernel": dom, "bound": "mfma", "achieved": flops / (dom_ms * 1e-3) / 1e12,
                    "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s"}
    elif dom.startswith("fft"):
        # bound by vector-ALU issue, not by HBM.  Algorithmic flops: a forward and an inverse
        # fast transform of the 2d real columns of a unit, packed in pairs = 10*N*log2(N)*d.
        flops = 10.0 * n * math.log2(n) * d * units
        roofline = {"kernel": dom, "bound": "alu", "achieved": flops / (dom_ms * 1e-3) / 1e12,
                    "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s"}
        # the same launch against the HBM roof: read K and V once, write one fp32 score per token
        gbs = ab["score"] / (dom_ms * 1e-3) / 1e9
        roofline["hbm"] = {"achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": ab["select_gather"] / (dom_ms * 1e-3) / 1e9,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["avg_launch_ms"] = dom_ms
    # the stored traffic figures belong to the named workload as configured, not to overridden ones
    overridden = args.gamma is not None or args.rho is not None or args.n_tokens is not None
    roofline["traffic"] = None if overridden else read_traffic(dom, args.config, path_name)
    roofline["kernels_ms"] = {k: round(v[1], 4) for k, v in kern.items()}

    decode = None
    if args.decode:
        # decode-step attention (one new token per sequence) over the compacted cache this run just
        # produced and over the uncompressed cache (same kernel, b_l = N): the traffic ratio is 1/rho
        G = args.q_heads_per_kv
        Hq = G * cfg.kv_heads
        gq = torch.Generator(device="cuda").manual_seed(1234)
        Qt = torch.randn((cfg.batch, cfg.layers, Hq, d), device="cuda", generator=gq).to(Kt.dtype)
        scale = 1.0 / math.sqrt(d)
        full_b = torch.full((cfg.batch, cfg.layers), n, dtype=torch.int32, device="cuda")
        full_off = (torch.arange(cfg.layers + 1, device="cuda", dtype=torch.int64) * (cfg.kv_heads * n)
                    ).repeat(cfg.batch, 1).contiguous()
        full_rows = cfg.layers * cfg.kv_heads * n
        Kfull, Vfull = Kt.reshape(cfg.batch, full_rows, d), Vt.reshape(cfg.batch, full_rows, d)
        out_c = torch.empty((cfg.batch, cfg.layers, Hq, d), dtype=torch.float32, device="cuda")
        out_f = torch.empty_like(out_c)
        ws = torch.empty(max(16, int(binding._lib.flashcache_decode_workspace_bytes(
            cfg.batch, cfg.layers, cfg.kv_heads, Hq, d))), dtype=torch.uint8, device="cuda")

        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0) / reps

        ms_c = timed(lambda: fc.decode_attention(Qt, comp.K_out, comp.V_out, cfg.kv_heads, comp.budgets,
                                                 comp.layer_offsets, comp.rows_per_seq, scale, out_c, ws))
        ms_f = timed(lambda: fc.decode_attention(Qt, Kfull, Vfull, cfg.kv_heads, full_b, full_off,
                                                 full_rows, scale, out_f, ws))
        bytes_c = 2 * cfg.batch * comp.rows_per_seq * d * cfg.elem_bytes
        bytes_f = 2 * cfg.batch * full_rows * d * cfg.elem_bytes
        decode = {"q_heads": Hq, "compacted_ms": ms_c, "full_cache_ms": ms_f, "speedup": ms_f / ms_c,
                  "compacted_GBps": bytes_c / ms_c / 1e6, "full_cache_GBps": bytes_f / ms_f / 1e6,
                  "hbm_frac_full_cache": bytes_f / ms_f / 1e6 / HBM_PEAK_GBS}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import flashcache_ref as ref
        threads = workers
        # bounded sample: whole layers of sequence 0 (all heads), scored, allocated over the
        # sampled layers at the same keep ratio, selected and gathered by the oracle
        n_layers, spent, done_tokens = 1, 0.0, 0
        l0 = 0
        while spent < args.cpu_seconds and l0 < cfg.layers:
            ls = list(range(l0, min(cfg.layers, l0 + n_layers)))
            Ts = ref.total_budget(len(ls), cfg.n_tokens, cfg.rho)
            t0 = time.perf_counter()
            ref.compress(K[:1, ls], V[:1, ls], cfg.dtype, r, Ts, route="fast", workers=threads)
            dt = time.perf_counter() - t0
            spent += dt
            done_tokens += len(ls) * cfg.n_tokens
            l0 += len(ls)
            n_layers = max(1, min(cfg.layers - l0, int(n_layers * 2)))
        cpu_baseline = {"value": done_tokens / spent, "unit": "KV tokens/s", "cores": threads,
                        "kind": "oracle",
                        "sample": f"{l0} of {cfg.layers} layers of sequence 0 ({done_tokens} KV tokens, "
                                  f"{spent:.1f}s), fp64 scipy DCT route"}

    line = {
        "metric": "KV tokens compressed/sec (score+select+gather)",
        "value": value,
        "unit": "KV tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.config, "batch": cfg.batch, "layers": cfg.layers,
                   "kv_heads": cfg.kv_heads, "n_tokens": cfg.n_tokens, "head_dim": cfg.head_dim,
                   "storage": cfg.dtype, "gamma": cfg.gamma, "rho": cfg.rho, "r": r,
                   "total_budget": T, "path": path_name, "seed": cfg.seed},
        "sequence_tokens_per_s": cfg.batch * cfg.n_tokens / (ms_per_step * 1e-3),
        "hbm_frac_whole_path": ab["total"] / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBS,
        "algorithmic_bytes": ab,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "decode": decode,
        "setup_s": {"generate": round(t_gen, 2), "upload": round(t_upload, 2), "prepare_tables": round(t_prepare, 3)},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
