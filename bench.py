#!/usr/bin/env python3
"""Benchmark of the SwiftKV prefill hot path on one MI355X.

One "step" = one swiftkv_prefill call over the whole batch of the workload
(layers 1..l on all prompt tokens, fused KV projection of the later layers,
last-token tail, logits), inputs resident in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
# HBM-side bytes per launch of the dominant kernel (gate/up GEMM): NOT measured in this run (rocprofv3 cannot run
# inside the bench) but taken from the committed counter run of the same command, FETCH_SIZE / WRITE_SIZE scaled
# on a 1 GiB copy: profiles/bench_8b_l16_b8x2048_hbm_traffic.txt
PROFILED_TRAFFIC_BYTES = {("8b_l16_b8x2048", "gateup_gemm"): 5829.6 * 2 ** 20}
PROFILED_TRAFFIC_SOURCE = "profiles/bench_8b_l16_b8x2048_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, copy-calibrated)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="8b_l16_b8x2048")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the per-launch HIP events (roofline is then null)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=256)
    ap.add_argument("--no-mfma-rate", action="store_true",
                    help="skip the measurement of the matrix-instruction rate on random operands")
    ap.add_argument("--kv-scales", choices=("per_head", "per_token"), default="per_head",
                    help="FP8-cache workloads: one scale per (cache layer, K|V, KV head) or one per token")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first copy 1 GiB device-to-device (a plain copy of known size, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as WL
    from paper_2410_03960_amd import binding as B

    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.zeros(1 << 29, dtype=torch.bfloat16, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    wl = WL.get_workload(args.workload)
    sh = wl.shape
    t0 = time.time()
    store = WL.WeightStore(sh, wl.seed, device="cuda", keep=True).materialize()
    dev_w = dict(store._cache)
    torch.cuda.synchronize()
    t_gen = time.time() - t0
    batch = WL.build_batch(wl)
    T, nseq = batch.n_tokens, batch.n_seqs
    ctx = B.Context(sh, dev_w, wl.l, wl.g)
    kvd = B.SWIFTKV_KV_FP8_E4M3 if wl.kv_fp8 else B.SWIFTKV_KV_BF16
    per_token = wl.kv_fp8 and args.kv_scales == "per_token"
    scale_mode = B.SWIFTKV_SCALE_PER_TOKEN if per_token else B.SWIFTKV_SCALE_COMPUTE_ABSMAX
    cache = B.KVCache(ctx.n_cache_layers, batch.n_blocks, sh.n_kv_heads, sh.head_dim, batch.block_tables,
                      batch.context_lens.tolist(), fp8=wl.kv_fp8, scale_mode=scale_mode)
    has_ctx = bool((batch.context_lens > 0).any())
    if wl.kv_fp8 and has_ctx:
        # pre-existing contexts: seeded codes under fixed scales
        if not per_token:
            cache.scale_mode = B.SWIFTKV_SCALE_USE_GIVEN
        cache.scales.fill_(0.02)
        cache.data.random_(0, 0x77, generator=torch.Generator(device="cuda").manual_seed(wl.seed))
    elif has_ctx:
        # pre-existing contexts: seeded values of the size K/V rows have on these models
        cache.data.normal_(0.0, 0.5, generator=torch.Generator(device="cuda").manual_seed(wl.seed))
    prefix = sum(int(c) for c, n in zip(batch.context_lens.tolist(), batch.seq_lens.tolist()) if n > 1)
    ws = torch.empty(ctx.workspace_bytes(T, nseq, kvd, prefix), dtype=torch.uint8, device="cuda")
    logits = torch.empty((nseq, sh.vocab), dtype=torch.float32, device="cuda")
    ids = batch.token_ids.cuda()
    lens = batch.seq_lens.tolist()
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        ctx.prefill(ids, lens, cache, logits, ws, stream)
    torch.cuda.synchronize()
    # Inside the timed region only the launches of the roofline's kernel (the gate/up GEMM, the largest share of a
    # prefill step) are bracketed by HIP events: an event pair costs a few microseconds on the stream, and around
    # every launch that is 1 % of a prefill step and 10 % of a decode step.  A decode step's roofline is the whole
    # step, so nothing is bracketed there.  The other classes are timed in a separate pass after the timed region.
    prefill_like = T >= 1024
    ctx.set_timing(prefill_like and not args.no_kernel_timing, classes=("gateup_gemm",))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # step boundaries on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record(stream)
        ctx.prefill(ids, lens, cache, logits, ws, stream)
    marks[args.steps].record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    tok_s = T * args.steps / dt
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    assert torch.isfinite(logits).all(), "non-finite logits"

    gemm_fl, attn_fl = ctx.flops(lens, batch.context_lens.tolist())
    # the same tokens through all L layers of the unmodified model (what the paper normalises its TFLOPS
    # figures to: footnote of the introduction, Sec. 4.2), next to the parameter-count form 2 * params * tokens
    d, qd, kvdim, f, L = sh.hidden, sh.q_dim, sh.kv_dim, sh.ffn, sh.n_layers
    layer_gemm = 2.0 * d * (qd + 2 * kvdim) + 2.0 * d * qd + 6.0 * d * f
    pairs = sum(n * c + n * (n + 1) / 2.0 for c, n in zip(batch.context_lens.tolist(), lens))
    base_fl = T * L * layer_gemm + nseq * 2.0 * d * sh.vocab + L * 4.0 * qd * pairs
    n_params = L * (d * (qd + 2 * kvdim) + d * qd + 3 * d * f + 2 * d) + 2 * sh.vocab * d + d
    out = {
        "metric": ("prefill tokens/s, 8B-shape SwiftKV-50%; GEMM MFMA TFLOPS as % of bf16 peak" if T >= 1024
                   else "decode-step tokens/s (one new token per sequence over its cached context)"),
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "n_seqs": nseq, "n_tokens": T, "l": wl.l, "acrosskv_group": wl.g,
                   "kv_cache": ("fp8_e4m3/" + args.kv_scales) if wl.kv_fp8 else "bf16", "n_layers": sh.n_layers,
                   "hidden": sh.hidden},
        "ms_per_step_median": step_ms[len(step_ms) // 2], "ms_per_step_min": step_ms[0],
        "executed_flops_per_step": gemm_fl + attn_fl,
        "executed_tflops": (gemm_fl + attn_fl) / (ms_per_step * 1e-3) / 1e12,
        "executed_frac_of_bf16_peak": (gemm_fl + attn_fl) / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "normalised_to_baseline_model": {      # NOT executed work: what the unmodified L-layer model would have done
            "flops_per_step": base_fl, "tflops": base_fl / (ms_per_step * 1e-3) / 1e12,
            "two_params_tokens_tflops": 2.0 * n_params * T / (ms_per_step * 1e-3) / 1e12,
            "executed_over_baseline": (gemm_fl + attn_fl) / base_fl},
        "weight_gen_s": t_gen,
    }

    roof = None
    if not args.no_kernel_timing:
        tim_roof = ctx.get_timing() if prefill_like else None       # events of the timed region
        class_steps = min(args.steps, 5)
        ctx.set_timing(True)                                         # every class: a pass of its own, after the timed region
        for _ in range(class_steps):
            ctx.prefill(ids, lens, cache, logits, ws, stream)
        tim = ctx.get_timing()
        ctx.set_timing(False)
        P = (sh.n_layers - wl.l) // wl.g
        per_launch_flops = {"qkv_gemm": 2.0 * T * d * (qd + 2 * kvdim), "o_gemm": 2.0 * T * d * qd,
                            "gateup_gemm": 4.0 * T * d * f, "down_gemm": 2.0 * T * d * f,
                            "fused_kv_gemm": 2.0 * T * d * P * 2 * kvdim,
                            "attn_prefill": attn_fl / max(wl.l, 1) if wl.l else 0.0}
        # algorithmic HBM bytes per step of the bandwidth-bound classes: the normalising passes (one pass over
        # the fp32 embeddings writing bf16 rows, then only per-row sums: 64 partial sums read, one value written),
        # and the KV commit (reads K and V rows, writes them to their paged slots and V once more transposed)
        esz = 1 if wl.kv_fp8 else 2
        per_step_bytes = {
            "norm": T * d * 6.0 + 2 * wl.l * T * (d // 64 + 1) * 4.0 if T >= 1024 else None,
            "kv_commit": wl.l * T * kvdim * (2 * 2 + 2 * esz + 2.0) + (P * T * kvdim * 2 * (2 + esz) if wl.kv_fp8 else 0.0),
        }
        classes, gemm_ms, gemm_flops = {}, 0.0, 0.0
        for name, (ms, n) in tim.items():
            ent = {"ms_per_step": ms / class_steps, "launches_per_step": n / class_steps}
            if per_step_bytes.get(name) and ms > 0:
                ent["algorithmic_gbytes_per_step"] = per_step_bytes[name] / 1e9
                ent["achieved_gb_s"] = per_step_bytes[name] / (ms / class_steps * 1e-3) / 1e9
                ent["frac_of_hbm_peak"] = ent["achieved_gb_s"] / 8000.0
            if name in per_launch_flops and n:
                avg_ms = ms / n
                ent["avg_launch_ms"] = avg_ms
                ent["tflops"] = per_launch_flops[name] / (avg_ms * 1e-3) / 1e12
                if name.endswith("_gemm"):
                    gemm_ms += ms
                    gemm_flops += per_launch_flops[name] * n
            classes[name] = ent
        out["kernel_classes"] = classes
        out["kernel_classes_source"] = (f"separate pass of {class_steps} steps after the timed region, HIP events "
                                        "around every launch (those steps run ~1 ms longer)")
        if gemm_ms > 0:
            out["gemm_tflops"] = gemm_flops / (gemm_ms * 1e-3) / 1e12
            out["gemm_frac_of_bf16_peak"] = out["gemm_tflops"] / PEAK_BF16_TFLOPS
        if tim_roof and tim_roof["gateup_gemm"][1]:
            ms, n = tim_roof["gateup_gemm"]
            avg_ms = ms / n
            tf = per_launch_flops["gateup_gemm"] / (avg_ms * 1e-3) / 1e12
            roof = {"bound": "mfma", "kernel": "gemm_wreg_kernel / gemm_dlds5_kernel (gateup_gemm)", "achieved": tf,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS,
                    "avg_launch_ms": avg_ms, "launches_timed": n,
                    "measured": "HIP events on the launch stream around each of its launches inside the timed region",
                    "flops_per_launch": per_launch_flops["gateup_gemm"],
                    "traffic": PROFILED_TRAFFIC_BYTES.get((wl.name, "gateup_gemm")),
                    "traffic_source": PROFILED_TRAFFIC_SOURCE if (wl.name, "gateup_gemm") in PROFILED_TRAFFIC_BYTES else None}
    if T < 1024:
        # a decode step streams every weight once and each sequence's cached K/V of every cache layer once: HBM-bound
        n_par = 2 * sh.vocab * sh.hidden + sh.n_layers * (2 * sh.hidden * sh.q_dim + 3 * sh.hidden * sh.ffn) \
            + ctx.n_cache_layers * 2 * sh.hidden * sh.kv_dim
        n_par -= (sh.vocab - T) * sh.hidden if T < sh.vocab else 0     # embedding: only the rows of the T tokens
        keys = float((batch.context_lens + batch.seq_lens).sum())
        kv_bytes = keys * ctx.n_cache_layers * 2 * sh.kv_dim * (1 if wl.kv_fp8 else 2)
        alg = 2.0 * n_par + kv_bytes
        roof = {"bound": "hbm", "kernel": "whole decode step (weight-streaming GEMMs + paged single-query attention)",
                "achieved": alg / (ms_per_step * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                "frac": alg / (ms_per_step * 1e-3) / 1e9 / 8000.0, "bytes_per_step": alg, "traffic": None}
    out["roofline"] = roof
    if not args.no_mfma_rate and T >= 1024:
        # what the matrix unit alone sustains on operand data like the model's (the chip is power-limited;
        # the data-sheet peak assumes nothing toggles): A-like N(0,1) and W-like N(0,0.02) fragments
        g = torch.Generator(device="cuda").manual_seed(wl.seed)
        ops = torch.cat([torch.randn(8192, generator=g, device="cuda"), 0.02 * torch.randn(8192, generator=g, device="cuda")])
        ops = ops.view(2, 4, 4, 512).transpose(0, 1).contiguous().view(-1).to(torch.bfloat16)   # per wave: 4 A-like, 4 W-like fragments
        rate = B.op_mfma_rate(ops, 40000)
        out["mfma_only_tflops"] = rate
        if "gemm_tflops" in out:
            out["gemm_frac_of_mfma_only"] = out["gemm_tflops"] / rate

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, store, ctx, args.cpu_sample_tokens)
    print(json.dumps(out))


def cpu_baseline(wl, store, ctx, n_sample):
    """Time the CPU oracle (float32, as it stands) on a bounded sample of the same
    workload: the first `n_sample` tokens of sequence 0 as one prompt, all steps
    of the path.  Also reports how far the GPU result for that prompt is from it."""
    import torch
    import workloads as WL
    from oracle import swiftkv_oracle as O
    from paper_2410_03960_amd import binding as B
    sh = wl.shape
    full = WL.build_batch(wl)
    n = min(n_sample, int(full.seq_lens[0]))
    sub = WL.build_batch(wl, lens=[n], ctx=[0], shuffled=False)
    sub.token_ids = full.token_ids[:n].clone()
    host = {}

    def wfn(name, j0=None):
        key = name if j0 is None else f"{name}.{j0}"
        if key not in host:
            host[key] = store.get(name, j0).cpu()
        return host[key]
    # bring the needed weights to the host before the clock starts
    for nm in ("embed", "final_norm", "lm_head"):
        wfn(nm)
    leaders = set(j - 1 for j in O.leader_layers(sh.n_layers, wl.l, wl.g))
    for j in range(sh.n_layers):
        for nm in ("norm1", "wq", "wo", "norm2", "wgate", "wup", "wdown"):
            wfn(nm, j)
        if j < wl.l or j in leaders:
            wfn("wk", j), wfn("wv", j)
    osh = O.Shape(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn, sh.vocab,
                  sh.rope_theta, sh.rms_eps)
    ocache = O.PagedKVCache(ctx.n_cache_layers, sub.n_blocks, sh.n_kv_heads, sh.head_dim, sub.block_tables,
                            dtype=torch.float32, fp8=wl.kv_fp8)
    t0 = time.perf_counter()
    ologits, _ = O.swiftkv_prefill(osh, wfn, sub.token_ids, [n], [0], wl.l, wl.g, ocache, dtype=torch.float32)
    dt = time.perf_counter() - t0
    # untimed: the same prompt with the oracle rounding every matrix-product input to bf16 (what bf16 matrix
    # instructions force on any implementation): the error floor the GPU figure below is to be read against
    def bf16(x):
        return x.to(torch.bfloat16).to(x.dtype)
    fcache = O.PagedKVCache(ctx.n_cache_layers, sub.n_blocks, sh.n_kv_heads, sh.head_dim, sub.block_tables,
                            dtype=torch.float32, fp8=wl.kv_fp8)
    flogits, _ = O.swiftkv_prefill(osh, wfn, sub.token_ids, [n], [0], wl.l, wl.g, fcache, dtype=torch.float32,
                                   act_round={p: bf16 for p in ("a", "qkv", "p", "o", "z")})
    # same prompt through the HIP path, for a parity figure at this shape
    cache = B.KVCache(ctx.n_cache_layers, sub.n_blocks, sh.n_kv_heads, sh.head_dim, sub.block_tables, [0],
                      fp8=wl.kv_fp8)
    kvd = B.SWIFTKV_KV_FP8_E4M3 if wl.kv_fp8 else B.SWIFTKV_KV_BF16
    ws = torch.empty(ctx.workspace_bytes(n, 1, kvd), dtype=torch.uint8, device="cuda")
    logits = torch.empty((1, sh.vocab), dtype=torch.float32, device="cuda")
    ctx.prefill(sub.token_ids.cuda(), [n], cache, logits, ws)
    torch.cuda.synchronize()
    a, b, fl = logits[0].double().cpu(), ologits[0].double(), flogits[0].double()
    rel = float((a - b).abs().max() / b.abs().max())
    cos = float((a @ b) / (a.norm() * b.norm()))
    return {"value": n / dt, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"first {n} tokens of sequence 0 of {wl.name} as one prompt, whole path, float32",
            "seconds": dt, "gpu_vs_oracle_logits_rel_err": rel, "gpu_vs_oracle_logits_cosine": cos,
            "bf16_matrix_input_floor_logits_rel_err": float((fl - b).abs().max() / b.abs().max()),
            "bf16_matrix_input_floor_logits_cosine": float((fl @ b) / (fl.norm() * b.norm()))}


if __name__ == "__main__":
    main()
