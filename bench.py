#!/usr/bin/env python3
"""Benchmark of the deduplicated prefill hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic batch that is already resident in
HBM: radix_build_index (trie index maps, including its one 8-byte device-to-host read of N')
followed by radix_prefill_forward (compact-space position-wise ops + full-layout attention).
The headline value is uncompressed tokens per second, N / step time.

Prints ONE JSON line: metric, value (tokens/s), ms_per_step, config, the roofline of the dominant kernel,
the CPU oracle baseline and context fields (per-kernel times, speedup over the no-dedup path).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}



def measured_traffic_bytes(key):
    """HBM-side bytes of one gate/up GEMM launch (fetched + written) from the two rocprofv3 --pmc runs of this
    command (FETCH_SIZE, WRITE_SIZE, each scaled by what the counter reads for the 256 MiB row copy this program
    launches as the reference dispatch): the figure is kept in the profile summary of the workload, in a line
    "traffic_bytes_per_launch = <integer>", so that the bench line and the committed summary cannot drift apart.
    None where no such summary exists."""
    import re
    path = os.path.join(ROOT, "profiles", f"gemm_gateup_{key}_hbm_traffic.md")
    try:
        m = re.search(r"traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read())
    except OSError:
        return None
    return int(m.group(1)) if m else None


WORKLOAD_TEXT = {
    "C1": "C1: tiny Qwen3-style decoder fp32, 8 seqs = 32 shared + 16 own tokens",
    "C2": "C2: Qwen3-0.6B shape, reranking batch of 64 seqs = 48-token shared prefix + suffix U[64,192]",
    "C3": "C3: Qwen3-4B shape, 128 seqs = 256 shared + 8 query groups x 32 + suffix U[64,192]",
    "C4": "C4: Qwen3-8B shape, reranking batch of 256 seqs = 64 shared + suffix U[96,256]",
    "C5": "C5: Qwen3-0.6B shape, 128 seqs = 2048-token shared prefix + 32 own tokens",
    "C5ctl": "C5 control: Qwen3-0.6B shape, 128 x 2080 tokens, no sharing, dedup forced on",
    "SWEEP": "paper's synthetic sweep point (Experiments, forward-pass benchmark): B = 32 sequences = one shared prefix + "
             "distinct fixed-length suffixes",
}
SWEEP_SEED = 2001
WORKLOAD_TEXT["SWEEPTABLE"] = ("all rows of the paper's forward-pass sweep for one model shape (Appendix, forward-pass latency "
                              "table: B = 32, prefix {1..2048} x suffix {256, 1024}), forward time only, both attention modes")
WORKLOAD_TEXT["INDEXBUILD"] = ("radix_build_index at the shapes of the paper's index-construction benchmark (Appendix, index "
                              "construction: 16 384 tokens at several prefix ratios, 2048 x 512, identical / no-overlap 32 x 512, one "
                              "sequence) and on tries that branch at every level")
# (prefix, suffix) rows of the paper's sweep table
SWEEP_ROWS = [(1, 256), (16, 256), (32, 256), (128, 256), (256, 256), (512, 256), (1024, 256), (2048, 256),
              (1, 1024), (32, 1024), (128, 1024), (256, 1024), (512, 1024), (1024, 1024), (2048, 1024)]
WORKLOAD_TEXT["INDEXSELECT"] = "row index-select at the shapes of the paper's gather/scatter kernel benchmark (Appendix, index-select kernel)"
# (source rows, row elements, selected rows)
INDEX_SELECT_SHAPES = [(16000, 1024, 12000), (16000, 1024, 70000), (100000, 2048, 500000), (2000, 64 * 256, 10000)]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=sorted(WORKLOAD_TEXT),
                    help="default: C4, the largest of the named single-GPU configurations")
    ap.add_argument("--three-kernel-attention", action="store_true",
                    help="time the scatter -> attention over all N rows -> gather sequence as Algorithm 1 writes it "
                         "(default: the library's default, one attention kernel that indexes the compact buffer; same "
                         "values bit for bit)")
    ap.add_argument("--hilo-layers", type=int, default=0,
                    help="radix_model_config.hilo_layers: 0 = decided by the library from the weights (what the parity "
                         "tests run with), k > 0 = the first k layers, -1 = none")
    ap.add_argument("--fold-norms", action="store_true",
                    help="radix_model_config.fold_norms = 1: RMSNorms folded into the GEMMs around them (default: norm kernels)")
    ap.add_argument("--sweep-model", choices=["0.6B", "4B", "8B"], default="0.6B", help="--workload SWEEP: model shape")
    ap.add_argument("--sweep-prefix", type=int, default=2048, help="--workload SWEEP: shared prefix length")
    ap.add_argument("--sweep-suffix", type=int, default=256, help="--workload SWEEP: suffix length")
    ap.add_argument("--lm-head", action="store_true",
                    help="also time the LM head (tied to the embedding) on the last token of every sequence, outside "
                         "the timed steps; reported as lm_head_last_token")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default run (C4) only: skip the short runs of C2, C3, C5 and C5ctl that are reported beside "
                         "the headline as other_workloads")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="rough budget of the oracle timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2601_15013_amd import binding, harness, synth

    binding.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    key = args.workload
    if key == "INDEXSELECT":
        return index_select_bench(args, torch, np, binding)
    if key == "INDEXBUILD":
        return index_build_bench(args, torch, np, binding, synth)
    if key == "SWEEPTABLE":
        return sweep_table_bench(args, torch, np, binding, harness, synth)
    if key == "SWEEP":
        model_cfg = {"0.6B": synth.QWEN3_0_6B, "4B": synth.QWEN3_4B, "8B": synth.QWEN3_8B}[args.sweep_model]
        batch = synth.shared_prefix_batch(SWEEP_SEED, 32, args.sweep_prefix, args.sweep_suffix, args.sweep_suffix,
                                          model_cfg.vocab, name="sweep")
        weights = synth.SynthWeights(model_cfg, SWEEP_SEED)
    else:
        batch = synth.make_batch(key)
        weights = synth.make_weights(key)
    cfg = weights.cfg
    model = harness.upload_model(weights, hilo_layers=args.hilo_layers, lm_head_mode=1 if args.lm_head else 0,
                                 fold_norms=int(args.fold_norms))
    compute_dtype, hilo = model.compute_dtype, model.hilo_layers
    run = harness.Runner(model, batch.N, batch.B)
    tok, cu = harness.upload_batch(batch)
    N, B, max_len = batch.N, batch.B, batch.max_seqlen
    out = torch.empty((N, cfg.d), dtype=torch.float32, device="cuda")
    I_s = torch.empty(N, dtype=torch.int32, device="cuda")
    I_g = torch.empty(N, dtype=torch.int32, device="cuda")
    n_dev = torch.empty(1, dtype=torch.int32, device="cuda")
    force = key == "C5ctl"

    can_fuse = compute_dtype != "f32"          # the fused kernel is the 16-bit MFMA one
    fused = can_fuse and not args.three_kernel_attention

    def step(fused_attention=fused):
        maps = binding.radix_build_index(tok, None, cu, run.ws, I_s, I_g, n_dev)
        binding.radix_prefill_forward(model, tok, None, cu, max_len, maps[0], maps[1], maps[3], run.ws, out=out,
                                      force_dedup=force, fused_attention=fused_attention)
        return maps[3]

    def timed(fn, iters):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iters

    # ---- headline: W warm-up steps, then exactly K timed steps; the dominant kernel (gate/up
    # GEMM + SwiGLU) is bracketed by HIP events on the launch stream inside the timed region
    for _ in range(args.warmup):
        n_c = step()
    dominant = "gemm_gateup"        # launches of the layers without (hi, lo) inputs: one size, one flop count
    # an event pair idles the GPU for a few microseconds around the launch it brackets: sample sparsely where a
    # launch is short, bracket every launch where that gap is below a thousandth of it
    sparse = 2.0 * batch.N * (2 * cfg.d_int) * cfg.d < 2e12
    binding.radix_timing_enable([dominant], every_nth=4 if sparse else 1)
    ms_per_step = timed(step, args.steps)
    t_dom, n_dom = binding.radix_timing_collect()[dominant]
    binding.radix_timing_enable([])
    assert run.status() == 0
    n_c = int(n_dev.item())

    # ---- context numbers (outside the timed region)
    maps = (I_s, I_g, n_dev, n_c)
    k2 = max(3, min(args.steps, 10))
    t_build = timed(lambda: binding.radix_build_index(tok, None, cu, run.ws, I_s, I_g, n_dev), k2)
    t_fwd = timed(lambda: binding.radix_prefill_forward(model, tok, None, cu, max_len, I_s, I_g, n_c, run.ws, out=out,
                                                        force_dedup=force, fused_attention=fused), k2)
    # the other attention mode, for context: whole step and forward alone
    other = (not fused) if can_fuse else False
    t_step_other = timed(lambda: step(other), k2)
    t_fwd_other = timed(lambda: binding.radix_prefill_forward(model, tok, None, cu, max_len, I_s, I_g, n_c, run.ws,
                                                              out=out, force_dedup=force, fused_attention=other), k2)
    t_nodedup = timed(lambda: binding.radix_prefill_forward_nodedup(model, tok, None, cu, max_len, run.ws, out=out), k2)
    binding.radix_timing_enable(binding.TIMING_CATEGORIES)
    binding.radix_prefill_forward(model, tok, None, cu, max_len, I_s, I_g, n_c, run.ws, out=out, force_dedup=force,
                                  fused_attention=fused)
    per_kernel = binding.radix_timing_collect()
    binding.radix_timing_enable(["attention"])
    binding.radix_prefill_forward(model, tok, None, cu, max_len, I_s, I_g, n_c, run.ws, out=out, force_dedup=force,
                                  fused_attention=other)
    attn_other_ms = binding.radix_timing_collect()["attention"][0]
    binding.radix_timing_enable([])

    # one plain row copy of known size (256 MiB read + 256 MiB written): the reference dispatch that
    # the rocprofv3 FETCH_SIZE / WRITE_SIZE readings of the other kernels are scaled by
    cal_rows, cal_row_bytes = 65536, 4096
    cal_src = torch.empty(cal_rows * cal_row_bytes, dtype=torch.uint8, device="cuda").view(cal_rows, cal_row_bytes)
    cal_idx = torch.arange(cal_rows, dtype=torch.int32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    binding.radix_index_select_rows(cal_src, cal_idx, out=cal_dst)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    d, di, dq, dkv = cfg.d, cfg.d_int, cfg.dq, cfg.dkv
    flops_dom = 2.0 * n_c * (2 * di) * d                      # one gate/up GEMM launch
    avg_dom_s = t_dom / max(n_dom, 1) * 1e-3
    achieved = flops_dom / avg_dom_s / 1e12
    peak = PEAK_TFLOPS[compute_dtype]
    gemm_flops_layer = n_c * (2.0 * d * (dq + 2 * dkv) + 2.0 * dq * d + 6.0 * d * di)
    gemm_ms = sum(per_kernel[k][0] for k in ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "gemm_hilo_layers"))
    lens = np.diff(batch.cu_seqlens).astype(np.float64)
    attn_flops = float(np.sum(2.0 * cfg.n_q_heads * cfg.head_dim * (lens * lens + lens))) * cfg.n_layers
    attn_flops_all_rows = attn_flops
    if fused and n_c < N:
        # the fused kernel computes the rows the gather keeps: per sequence the positions from its first
        # representative on (in a trie the representatives of a sequence are a suffix of it)
        g = I_g[:n_c].cpu().numpy().astype(np.int64)
        per_seq = np.bincount(np.searchsorted(batch.cu_seqlens[1:], g, side="right"), minlength=batch.B).astype(np.float64)
        first = lens - per_seq
        attn_flops = float(np.sum(2.0 * cfg.n_q_heads * cfg.head_dim * ((lens * lens + lens) - (first * first + first)))) * cfg.n_layers
    es = 2 if cfg.dtype != "f32" else 4
    scatter_bytes = (n_c + N) * (dq + 2 * dkv) * es
    gather_bytes = 2 * n_c * dq * es

    result = {
        "metric": "prefill tokens/s (uncompressed)",
        "value": N / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": compute_dtype,
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[key] + (f" - Qwen3-{args.sweep_model} shape, prefix {args.sweep_prefix}, "
                                                     f"suffix {args.sweep_suffix}" if key == "SWEEP" else ""), "B": B, "N": N, "N_compact": n_c,
                   "compression_r": N / max(n_c, 1), "layers": cfg.n_layers, "seed": SWEEP_SEED if key == "SWEEP" else synth.WORKLOADS[key].seed,
                   "weights": cfg.dtype, "operands": compute_dtype, "accumulate": "f32",
                   "hilo_layers": hilo, "fold_norms": int(args.fold_norms),
                   "attention_mode": "fused (indexed q/k/v, representative rows only)" if fused
                   else "scatter -> attention over N rows -> gather"},
        "step_breakdown_ms": {"build_index": t_build, "forward_dedup": t_fwd, "forward_nodedup": t_nodedup},
        "speedup_vs_nodedup": t_nodedup / t_fwd,
        "speedup_vs_nodedup_incl_build": t_nodedup / (t_fwd + t_build),
        "amdahl_model": amdahl_model(gemm_flops_layer / max(n_c, 1) * cfg.n_layers, N, n_c, attn_flops_all_rows, attn_flops),
        "nodedup_tokens_per_s": N / (t_nodedup * 1e-3),
        "other_attention_mode": {"mode": "scatter -> attention -> gather" if fused else "fused",
                                 "ms_per_step": t_step_other, "value": N / (t_step_other * 1e-3),
                                 "forward_ms": t_fwd_other, "speedup_vs_nodedup": t_nodedup / t_fwd_other,
                                 "attention_ms_per_forward": attn_other_ms},
        "kernel_ms_per_forward": {k: v[0] for k, v in per_kernel.items()},
        "compact_gemm_tflops": gemm_flops_layer * cfg.n_layers / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else None,
        "compact_gemm_frac_of_peak": (gemm_flops_layer * cfg.n_layers / (gemm_ms * 1e-3) / 1e12 / peak) if gemm_ms > 0 else None,
        "attention_tflops_note": "algorithmic flop of the query rows the running attention mode computes (all N rows, or the representative rows in the fused mode) over the attention kernel time",
        "attention_tflops": attn_flops / (per_kernel["attention"][0] * 1e-3) / 1e12 if per_kernel["attention"][0] > 0 else None,
        "scatter_GBps": scatter_bytes * cfg.n_layers / (per_kernel["scatter"][0] * 1e-3) / 1e9 if per_kernel["scatter"][0] > 0 else None,
        "gather_GBps": gather_bytes * cfg.n_layers / (per_kernel["gather"][0] * 1e-3) / 1e9 if per_kernel["gather"][0] > 0 else None,
        "roofline": {"kernel": "gate/up GEMM + SwiGLU (M=N', N=2*d_int, K=d)", "bound": "mfma", "achieved": achieved,
                     "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": measured_traffic_bytes(key),
                     "launches_timed": n_dom, "avg_launch_us": avg_dom_s * 1e6, "flops_per_launch": flops_dom},
    }

    if args.lm_head:
        last = (cu[1:] - 1).to(torch.int32).contiguous()
        ws_head = binding.alloc_workspace(binding.radix_lm_head_workspace_bytes(model, B))
        logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
        t_head = timed(lambda: binding.radix_lm_head(model, out, last, ws_head, out=logits), max(k2, 10))
        w_bytes = cfg.vocab * d * (2 if cfg.dtype != "f32" else 4)
        result["lm_head_last_token"] = {"rows": B, "vocab": cfg.vocab, "ms": t_head,
                                        "weight_GBps": w_bytes / (t_head * 1e-3) / 1e9,
                                        "tflops": 2.0 * B * cfg.vocab * d / (t_head * 1e-3) / 1e12}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(batch, weights, args.cpu_seconds)

    others = key == "C4" and not args.no_other_workloads and not args.three_kernel_attention and not args.fold_norms \
        and args.hilo_layers == 0
    if others:
        del run, out, I_s, I_g, tok, cu
        torch.cuda.empty_cache()
        result["paper_sweep_2048_256"] = paper_sweep_point(model, cfg, torch, binding, harness, synth)   # 8B shape
    model.close()
    if others:
        del model, weights, batch
        torch.cuda.empty_cache()
        result["other_workloads"] = {k: short_run(k, torch, binding, harness, synth) for k in ("C2", "C3", "C5", "C5ctl")}
    print(json.dumps(result))
    return 0


def amdahl_model(pw_flops_per_row, N, n_c, attn_flops_all_rows, attn_flops_computed):
    """The paper's speedup model (Experiments, theoretical speedup model: speedup = 1 / ((1 - f_c) + f_c / r), f_c the
    position-wise share of the flop) with the exact flop counts of this model shape and batch; and the same with
    the attention flop of the rows the running attention mode computes (fewer than all rows in the fused mode)."""
    pw_full, pw_compact = pw_flops_per_row * N, pw_flops_per_row * n_c
    f_c = pw_full / (pw_full + attn_flops_all_rows)
    r = N / max(n_c, 1)
    return {"f_c": f_c, "expected_speedup": 1.0 / ((1.0 - f_c) + f_c / r),
            "expected_speedup_this_attention_mode": (pw_full + attn_flops_all_rows) / (pw_compact + attn_flops_computed)}


def paper_sweep_point(model, cfg, torch, binding, harness, synth, prefix=2048, suffix=256):
    """One point of the paper's sweep (Experiments, forward-pass benchmark: B = 32, shared prefix + distinct suffixes;
    2048 / 256 is the point its speedup-model table quotes) on a model that is already uploaded: forward time with the
    library's defaults, with Algorithm 1's three-kernel attention, and without deduplication; index build not
    counted, as in the paper."""
    batch = synth.shared_prefix_batch(SWEEP_SEED, 32, prefix, suffix, suffix, cfg.vocab, name="sweep")
    run = harness.Runner(model, batch.N, batch.B)
    tok, cu = harness.upload_batch(batch)
    out = torch.empty((batch.N, cfg.d), dtype=torch.float32, device="cuda")
    I_s, I_g, _, n_c = binding.radix_build_index(tok, None, cu, run.ws)
    fwd = lambda mode: binding.radix_prefill_forward(model, tok, None, cu, batch.max_seqlen, I_s, I_g, n_c, run.ws,
                                                     out=out, fused_attention=mode)
    t_nd = _time_ms(torch, lambda: binding.radix_prefill_forward_nodedup(model, tok, None, cu, batch.max_seqlen, run.ws,
                                                                          out=out), 3, 1)
    t_def = _time_ms(torch, lambda: fwd(None), 3, 1)
    t_3k = _time_ms(torch, lambda: fwd(False), 3, 1) if model.compute_dtype != "f32" else t_def
    assert run.status() == 0
    return {"prefix": prefix, "suffix": suffix, "N": batch.N, "N_compact": n_c, "nodedup_ms": t_nd, "dedup_ms": t_def,
            "speedup": t_nd / t_def, "three_kernel_attention_ms": t_3k, "three_kernel_attention_speedup": t_nd / t_3k}


def short_run(key, torch, binding, harness, synth):
    """A named workload with the library's defaults, timed briefly: the same step as the headline (index build +
    deduplicated forward) and the no-dedup forward on the same batch."""
    batch, weights = synth.make_batch(key), synth.make_weights(key)
    cfg = weights.cfg
    model = harness.upload_model(weights)
    run = harness.Runner(model, batch.N, batch.B)
    tok, cu = harness.upload_batch(batch)
    N, max_len = batch.N, batch.max_seqlen
    out = torch.empty((N, cfg.d), dtype=torch.float32, device="cuda")
    I_s = torch.empty(N, dtype=torch.int32, device="cuda")
    I_g = torch.empty(N, dtype=torch.int32, device="cuda")
    n_dev = torch.empty(1, dtype=torch.int32, device="cuda")
    force = key == "C5ctl"
    n_c = [0]

    def step():
        maps = binding.radix_build_index(tok, None, cu, run.ws, I_s, I_g, n_dev)
        binding.radix_prefill_forward(model, tok, None, cu, max_len, maps[0], maps[1], maps[3], run.ws, out=out,
                                      force_dedup=force)
        n_c[0] = maps[3]

    def timed(fn, iters):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iters

    step()
    iters = 20 if N * cfg.n_layers * cfg.d * cfg.d_int < 3e15 else 4
    ms = timed(step, iters)
    ms_nd = timed(lambda: binding.radix_prefill_forward_nodedup(model, tok, None, cu, max_len, run.ws, out=out),
                  max(2, iters // 4))
    assert run.status() == 0
    res = {"workload": WORKLOAD_TEXT[key], "N": N, "N_compact": n_c[0], "compression_r": N / max(n_c[0], 1),
           "steps": iters, "ms_per_step": ms, "tokens_per_s": N / (ms * 1e-3), "forward_nodedup_ms": ms_nd,
           "speedup_vs_nodedup_incl_build": ms_nd / ms, "hilo_layers": model.hilo_layers}
    if key in ("C2", "C3"):          # the 0.6B and 4B model shapes are on the GPU now
        del out, I_s, I_g, run
        res["paper_sweep_2048_256"] = paper_sweep_point(model, cfg, torch, binding, harness, synth)
    model.close()
    return res


def index_select_bench(args, torch, np, binding):
    """out[r] = src[idx[r]] with seeded uniform indices: time per call and moved bytes (read + written) per second."""
    rows = []
    rng = np.random.Generator(np.random.Philox(key=[3001, 0x1D5E]))
    for n_src, width, n_out in INDEX_SELECT_SHAPES:
        for dt, name in ((torch.float16, "f16"), (torch.float32, "f32")):
            src = torch.empty((n_src, width), dtype=dt, device="cuda").normal_()
            idx = torch.from_numpy(rng.integers(0, n_src, size=n_out, dtype=np.int64).astype(np.int32)).cuda()
            out = torch.empty((n_out, width), dtype=dt, device="cuda")
            for _ in range(args.warmup):
                binding.radix_index_select_rows(src, idx, out=out)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                binding.radix_index_select_rows(src, idx, out=out)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) * 1e6 / args.steps
            moved = 2.0 * n_out * width * src.element_size()
            rows.append({"src_rows": n_src, "row_elems": width, "out_rows": n_out, "dtype": name, "us": us,
                         "GBps": moved / us / 1e3})
            del src, idx, out
    big = rows[-3]      # [100000, 2048] -> 500000 rows, f32: the largest transfer
    print(json.dumps({"metric": "index-select throughput (bytes read + written)", "value": big["GBps"], "unit": "GB/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": big["us"] * 1e-3,
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
                      "data": "synthetic", "config": {"workload": WORKLOAD_TEXT["INDEXSELECT"]}, "shapes": rows,
                      "roofline": {"bound": "hbm", "achieved": big["GBps"], "peak": 8000.0, "unit": "GB/s",
                                   "frac": big["GBps"] / 8000.0, "traffic": None}}))
    return 0


def _time_ms(torch, fn, iters, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / iters


def sweep_table_bench(args, torch, np, binding, harness, synth):
    """Every (prefix, suffix) row of the paper's sweep for one model shape, one model upload: forward time without
    deduplication, with the library's defaults (fused attention kernel, gated by the library's cost model; and with
    deduplication forced) and with Algorithm 1's three-kernel attention (gated, and forced).
    Timings exclude the index build, as the paper's do."""
    model_cfg = {"0.6B": synth.QWEN3_0_6B, "4B": synth.QWEN3_4B, "8B": synth.QWEN3_8B}[args.sweep_model]
    weights = synth.SynthWeights(model_cfg, SWEEP_SEED)
    model = harness.upload_model(weights, hilo_layers=args.hilo_layers, fold_norms=int(args.fold_norms))
    n_max = max(32 * (p + s) for p, s in SWEEP_ROWS)
    run = harness.Runner(model, n_max, 32)
    out = torch.empty((n_max, model_cfg.d), dtype=torch.float32, device="cuda")
    rows = []
    for prefix, suffix in SWEEP_ROWS:
        batch = synth.shared_prefix_batch(SWEEP_SEED, 32, prefix, suffix, suffix, model_cfg.vocab, name="sweep")
        tok, cu = harness.upload_batch(batch)
        I_s, I_g, _, n_c = binding.radix_build_index(tok, None, cu, run.ws)
        assert n_c == batch.expected_n_compact
        o = out[:batch.N]
        fwd = lambda mode, force=False: binding.radix_prefill_forward(model, tok, None, cu, batch.max_seqlen, I_s, I_g, n_c,
                                                                      run.ws, out=o, fused_attention=mode, force_dedup=force)
        t_nd = _time_ms(torch, lambda: binding.radix_prefill_forward_nodedup(model, tok, None, cu, batch.max_seqlen,
                                                                              run.ws, out=o), args.steps, args.warmup)
        t_def = _time_ms(torch, lambda: fwd(None), args.steps, args.warmup)
        t_forced = _time_ms(torch, lambda: fwd(None, True), args.steps, args.warmup)
        t_3k = _time_ms(torch, lambda: fwd(False), args.steps, args.warmup)           # gated by the library's cost model
        t_3k_forced = _time_ms(torch, lambda: fwd(False, True), args.steps, args.warmup)
        assert run.status() == 0
        rows.append({"prefix": prefix, "suffix": suffix, "N": batch.N, "N_compact": n_c, "gamma": n_c / batch.N,
                     "nodedup_ms": t_nd, "dedup_ms": t_def, "speedup": t_nd / t_def,
                     "forced_ms": t_forced, "forced_speedup": t_nd / t_forced,
                     "three_kernel_ms": t_3k, "three_kernel_speedup": t_nd / t_3k,
                     "three_kernel_forced_ms": t_3k_forced, "three_kernel_forced_speedup": t_nd / t_3k_forced})
        print(f"{args.sweep_model} {prefix}/{suffix}: N {batch.N} N' {n_c} no-dedup {t_nd:.1f} ms, default {t_def:.1f} ms "
              f"({t_nd / t_def:.2f}x; deduplication forced: {t_forced:.1f} ms, {t_nd / t_forced:.2f}x), three-kernel attention {t_3k:.1f} ms ({t_nd / t_3k:.2f}x; deduplication forced: "
              f"{t_3k_forced:.1f} ms, {t_nd / t_3k_forced:.2f}x)", file=sys.stderr, flush=True)
    head = next(r for r in rows if (r["prefix"], r["suffix"]) == (2048, 256))
    model.close()
    print(json.dumps({"metric": "prefill tokens/s (uncompressed), forward only", "value": head["N"] / (head["dedup_ms"] * 1e-3),
                      "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": head["dedup_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                      "dtype": model.compute_dtype, "data": "synthetic",
                      "config": {"workload": WORKLOAD_TEXT["SWEEPTABLE"] + f" - Qwen3-{args.sweep_model} shape; headline = "
                                 "prefix 2048 / suffix 256", "B": 32, "seed": SWEEP_SEED},
                      "rows": rows}))
    return 0


def index_build_bench(args, torch, np, binding, synth):
    """radix_build_index alone (maps + the 8-byte read-back of N'), microseconds per call."""
    vocab = 151936
    rng = np.random.Generator(np.random.Philox(key=[4001, 0x1B1D]))

    def branching(depth, seg):
        # 2^depth sequences over a binary trie: at every level a sequence takes one of two distinct seg-token segments
        segs = [[rng.integers(0, vocab, size=seg, dtype=np.int64).astype(np.int32) for _ in range(2)] for _ in range(depth)]
        for pair in segs:
            while pair[1][0] == pair[0][0]:
                pair[1][0] = rng.integers(0, vocab)
        seqs = [np.concatenate([segs[l][(i >> (depth - 1 - l)) & 1] for l in range(depth)]) for i in range(1 << depth)]
        n_c = sum((2 << l) * seg for l in range(depth))
        return synth._assemble(f"binary trie depth {depth}", seqs, n_c)

    one = synth.shared_prefix_batch(4002, 1, 0, 512, 512, vocab)
    same = synth._assemble("32 identical x 512", [one.tok.copy() for _ in range(32)], 512)
    cases = [("16 384 tokens = 32 x 512, prefix ratio 0.0", synth.no_sharing_batch(4003, 32, 512, vocab)),
             ("16 384 tokens = 32 x 512, prefix ratio 0.5", synth.shared_prefix_batch(4004, 32, 256, 256, 256, vocab)),
             ("16 384 tokens = 32 x 512, prefix ratio 1.0 (identical sequences)", same),
             ("one sequence of 512", one),
             ("2048 x 512, prefix ratio 0.5", synth.shared_prefix_batch(4005, 2048, 256, 256, 256, vocab)),
             ("2048 x 512, no sharing", synth.no_sharing_batch(4006, 2048, 512, vocab)),
             ("2048 sequences on a binary trie of depth 11 (32-token segments: a branching at every level)", branching(11, 32)),
             ("4096 x 64, prefix ratio 0.5", synth.shared_prefix_batch(4007, 4096, 32, 32, 32, vocab))]
    rows = []
    for name, b in cases:
        tok = torch.from_numpy(b.tok.astype(np.int32)).cuda()
        cu = torch.from_numpy(b.cu_seqlens.astype(np.int32)).cuda()
        ws = binding.alloc_workspace(binding.radix_index_workspace_bytes(b.B))
        I_s = torch.empty(b.N, dtype=torch.int32, device="cuda")
        I_g = torch.empty(b.N, dtype=torch.int32, device="cuda")
        n_dev = torch.empty(1, dtype=torch.int32, device="cuda")
        n_c = binding.radix_build_index(tok, None, cu, ws, I_s, I_g, n_dev)[3]
        assert n_c == b.expected_n_compact, (name, n_c, b.expected_n_compact)
        us = _time_ms(torch, lambda: binding.radix_build_index(tok, None, cu, ws, I_s, I_g, n_dev), max(args.steps, 20),
                      args.warmup) * 1e3
        rows.append({"case": name, "B": b.B, "N": b.N, "N_compact": n_c, "us": us, "Mtok_per_s": b.N / us})
        print(f"{name}: B {b.B} N {b.N} N' {n_c}: {us:.1f} us ({b.N / us:.1f} M tok/s)", file=sys.stderr, flush=True)
    big = rows[4]
    print(json.dumps({"metric": "index build tokens/s", "value": big["N"] / (big["us"] * 1e-6), "unit": "tokens/s",
                      "n_gpus": 1, "steps": max(args.steps, 20), "warmup": args.warmup, "ms_per_step": big["us"] * 1e-3,
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
                      "config": {"workload": WORKLOAD_TEXT["INDEXBUILD"] + "; headline = 2048 x 512, prefix ratio 0.5"},
                      "rows": rows}))
    return 0


def cpu_baseline(batch, weights, budget_s):
    """The oracle as it stands (fp64, no deduplication), timed on the host cores on a bounded sample of whole
    sequences of the same batch.  The weights are drawn layer by layer while the oracle consumes them; the time
    spent drawing them is measured and taken off the clock."""
    import torch
    from oracle import forward as oracle_forward
    cfg = weights.cfg
    embed, gf = weights.embed, weights.gf
    lens = [int(batch.cu_seqlens[s + 1] - batch.cu_seqlens[s]) for s in range(batch.B)]
    # sample size from a rough rate (fp64 matmuls on ~16 cores: a few hundred GFLOP/s), at least one sequence
    flops_tok = cfg.n_layers * (2.0 * cfg.d * (cfg.dq + 2 * cfg.dkv) + 2.0 * cfg.dq * cfg.d + 6.0 * cfg.d * cfg.d_int)
    want_tokens = budget_s * 4e11 / flops_tok
    seqs, tokens = [], 0
    for s in range(batch.B):
        if tokens >= want_tokens:
            break
        if lens[s] > 0:
            seqs.append(s)
            tokens += lens[s]
    drawing = [0.0]

    def layers():
        for l in range(cfg.n_layers):
            t0 = time.perf_counter()
            lw = weights.layer(l)
            drawing[0] += time.perf_counter() - t0
            yield lw

    t0 = time.perf_counter()
    oracle_forward.forward_nodedup(cfg, embed, layers(), gf, batch.tok, batch.cu_seqlens, sequences=seqs)
    total_t = time.perf_counter() - t0 - drawing[0]
    return {"value": tokens / total_t, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"fp64 no-dedup oracle on the first {len(seqs)} whole sequences ({tokens} tokens) of the same "
                      f"batch, all {cfg.n_layers} layers, {total_t:.1f} s (drawing the weights, {drawing[0]:.1f} s, "
                      f"not counted)"}


if __name__ == "__main__":
    sys.exit(main())
